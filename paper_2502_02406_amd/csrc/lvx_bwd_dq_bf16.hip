// bf16 backward kernels.  The attention probabilities are recomputed from the saved statistic:
// p_ij = exp(scale <Q_i, K_j> - L_i) (Section 3.2 of the paper saves only x, O and L), and
// dS_ij = p_ij (<dO_i, V_j> - delta_i) with delta_i = sum_d dO_id O_id.
//
// Two kernels, no atomics in the inner loops and no round trip of P or dS through memory:
//   dq kernel   -- query-stationary (same structure as the forward kernel): transposed tiles
//                  S^T = K Q^T and dP^T = V dO^T put one query per lane, dS^T (bf16) is then the
//                  B operand of dQ^T += K^T dS^T, K^T coming from transposing LDS reads.
//   dkdv kernel -- key-stationary: a wave keeps its keys of K in registers (V in LDS) and streams the
//                  query rows of every head that shares this K/V head.  S = Q K^T and
//                  dP = dO V^T put one KEY per lane, so P and dS (bf16) are the B operands of
//                  dV^T += dO^T P and dK^T += Q^T dS, with dO^T / Q^T from transposing reads.
// S and dP are therefore formed twice (7 matrix products for the 5 that Table 1 counts); the
// alternative, one kernel that scatters dQ with float atomics, is bounded by the L2 atomic rate
// (about one float per channel per clock), far below the matrix cores for long key ranges.
#include "lvx_internal.h"
#include "lvx_mfma.h"

namespace lvx {

namespace {

constexpr float LOG2E = 1.4426950408889634f;

// ------------------------------------------------------------------------------------------
// dQ kernel
// ------------------------------------------------------------------------------------------
constexpr int QM = 128;      // query rows per workgroup
constexpr int QN = 64;       // keys per tile

template <int D> struct DqSmem {
  static constexpr int P = (D + 8) * 2;        // row pitch (bytes) of the V tile (b128 reads only)
  static constexpr int K_BYTES = ILV_ROWS * P; // K tile: row-interleaved, read both ways
  static constexpr int V_BYTES = QN * P;
  static constexpr int STAGE = K_BYTES + V_BYTES;
  static constexpr int TOTAL = 2 * STAGE;
};

template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
bwd_dq_bf16_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  using SM = DqSmem<D>;
  constexpr int KS = D / 16, DB = D / 32, CPR = D / 8, RPP = 256 / CPR, NPASS = QN / RPP;

  const Dims& d = a.d;
  const int G = d.Hq / d.Hkv;
  const int n_qt = (d.Sq + QM - 1) / QM;
  HeadWork hw;
  if (!xcd_decode(blockIdx.x, d.B * d.Hkv, a.n_split_dq * G * n_qt, &hw)) return;
  const int b = hw.head / d.Hkv, hk = hw.head % d.Hkv;
  const int split = hw.item / (G * n_qt);
  const int hq = hk * G + (hw.item % (G * n_qt)) / n_qt;
  const int qt = hw.item % n_qt;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ql = lane & 31;
  const int i_wave0 = qt * QM + wave * 32;
  const int i_lane = i_wave0 + ql;
  const bool row_ok = i_lane < d.Sq;

  const int n_tiles = (d.Skv + QN - 1) / QN;
  const int tps = (n_tiles + a.n_split_dq - 1) / a.n_split_dq;
  const int t_begin = split * tps;
  const int t_end = min(n_tiles, t_begin + tps);

  bf16x8 qf[KS], gf[KS];
  {
    const long off = b * d.q_sb + hq * d.q_sh + (long)i_lane * d.q_ss;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 x = {0, 0, 0, 0}, y = {0, 0, 0, 0};
      if (row_ok) {
        x = *(const u32x4*)((const uint16_t*)a.q + off + 16 * ks + 8 * g);
        y = *(const u32x4*)((const uint16_t*)a.d_o + off + 16 * ks + 8 * g);
      }
      qf[ks] = __builtin_bit_cast(bf16x8, x);
      gf[ks] = __builtin_bit_cast(bf16x8, y);
    }
  }
  const long row = ((long)b * d.Hq + hq) * d.Sq + i_lane;
  float lse2 = INFINITY, delta = 0.f;       // +inf makes p = exp2(-inf) = 0 for dead rows
  if (row_ok) {
    const long slot = (((long)b * d.Hq + hq) * a.sq_pad + (i_lane & ~31)) * 2 + (i_lane & 31);
    lse2 = a.stats[slot];
    delta = -a.stats[slot + 32];
  }
  const float c2 = d.scale * LOG2E;

  const uint16_t* kbase = (const uint16_t*)a.k + b * d.kv_sb + hk * d.kv_sh;
  const uint16_t* vbase = (const uint16_t*)a.v + b * d.kv_sb + hk * d.kv_sh;
  const int ld_row = tid / CPR, ld_col = (tid % CPR) * 8;
  const int i_wg0 = qt * QM, i_wg1 = min(d.Sq, i_wg0 + QM) - 1;
  auto next_tile = [&](int t) -> int {
    if (a.mask.allow)
      while (t < t_end && mask_rect(a.mask, b, i_wg0, i_wg1, t * QN, min(d.Skv, t * QN + QN) - 1) == 0) ++t;
    return t;
  };
  u32x4 kreg[NPASS], vreg[NPASS];
  auto load_tile = [&](int t) {
#pragma unroll
    for (int p = 0; p < NPASS; ++p) {
      const int j = t * QN + p * RPP + ld_row;
      u32x4 zk = {0, 0, 0, 0}, zv = {0, 0, 0, 0};
      if (j < d.Skv) {
        zk = *(const u32x4*)(kbase + (long)j * d.kv_ss + ld_col);
        zv = *(const u32x4*)(vbase + (long)j * d.kv_ss + ld_col);
      }
      kreg[p] = zk;
      vreg[p] = zv;
    }
  };
  auto store_tile = [&](int stage) {
    char* ks = smem + stage * SM::STAGE;
    char* vs = ks + SM::K_BYTES;
#pragma unroll
    for (int p = 0; p < NPASS; ++p) {
      const int r = p * RPP + ld_row;
      *(u32x4*)(ks + ilv_off<D>(ld_row, p * RPP, ld_col)) = kreg[p];
      *(u32x4*)(vs + r * SM::P + ld_col * 2) = vreg[p];
    }
  };

  f32x16 dq[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i) dq[i] = zero16();

  int cur = next_tile(t_begin);
  if (cur < t_end) { load_tile(cur); store_tile(0); }
  __syncthreads();
  int stage = 0;
  while (cur < t_end) {
    const int nxt = next_tile(cur + 1);
    if (nxt < t_end) load_tile(nxt);
    const char* ks_ = smem + stage * SM::STAGE;
    const char* vs_ = ks_ + SM::K_BYTES;
    const int j0 = cur * QN;
    int cls = 1;
    if (a.mask.allow)
      cls = mask_rect(a.mask, b, i_wave0, min(d.Sq - 1, i_wave0 + 31), j0, min(d.Skv, j0 + QN) - 1);
    if (i_wave0 >= d.Sq) cls = 0;
    if (cls != 0) {
      f32x16 sacc[2], pacc[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        sacc[kb] = zero16();
        pacc[kb] = zero16();
        const char* vrow = vs_ + (kb * 32 + ql) * SM::P + g * 16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          sacc[kb] = mfma32(*(const bf16x8*)(ks_ + ilv_off<D>(ql, kb * 32, 16 * ks + 8 * g)), qf[ks], sacc[kb]);
          pacc[kb] = mfma32(*(const bf16x8*)(vrow + ks * 32), gf[ks], pacc[kb]);
        }
      }
      const bool need_mask = (j0 + QN > d.Skv) || cls == 2;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][v], c2, -lse2));
          if (need_mask) {
            const int j = j0 + kb * 32 + 8 * (v / 4) + 4 * g + (v % 4);
            bool ok = j < d.Skv;
            if (ok && cls == 2) ok = row_ok && mask_elem(a.mask, b, i_lane, j);
            if (!ok) p = 0.f;
          }
          sacc[kb][v] = p * (pacc[kb][v] - delta);      // dS^T
        }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const bf16x8 sf = cvt_operand(sacc[t >> 1], 8 * (t & 1));
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 kt = load_tr_operand_ilv<D>(ks_, 16 * t, 32 * db, lane);
          dq[db] = mfma32(kt, sf, dq[db]);
        }
      }
    }
    if (nxt < t_end) store_tile(stage ^ 1);
    __syncthreads();
    stage ^= 1;
    cur = nxt;
  }
  if (!row_ok) return;
  float* out = a.dq_accum + row * D;
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v)
      unsafeAtomicAdd(out + 32 * db + 8 * (v / 4) + 4 * g + (v % 4), dq[db][v] * d.scale);
}

template <typename F>
hipError_t set_smem_once(F* fn, int bytes, bool* done) {
  if (*done) return hipSuccess;
  hipError_t e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) *done = true;
  return e;
}

}  // namespace

int bwd_bf16_pick_split(const Dims& d, int n_cu) {
  const long base = (long)d.B * d.Hq * ((d.Sq + QM - 1) / QM);
  const int n_tiles = (d.Skv + QN - 1) / QN;
  long want = (2L * n_cu + base - 1) / base;
  if (want < 1) want = 1;
  long cap = n_tiles / 8;
  if (cap < 1) cap = 1;
  if (want > cap) want = cap;
  if (want > 64) want = 64;
  return (int)want;
}

hipError_t launch_bwd_dq_bf16(const BwdArgs& a, hipStream_t s) {
  const Dims& d = a.d;
  const int G = d.Hq / d.Hkv;
  const int n_qt = (d.Sq + QM - 1) / QM;
  const long grid_q = xcd_grid(d.B * d.Hkv, a.n_split_dq * G * n_qt);
  hipError_t e;
  if (d.D == 64) {
    static bool once = false;
    if ((e = set_smem_once(bwd_dq_bf16_kernel<64>, DqSmem<64>::TOTAL, &once)) != hipSuccess) return e;
    bwd_dq_bf16_kernel<64><<<(unsigned)grid_q, 256, DqSmem<64>::TOTAL, s>>>(a);
  } else {
    static bool once = false;
    if ((e = set_smem_once(bwd_dq_bf16_kernel<128>, DqSmem<128>::TOTAL, &once)) != hipSuccess) return e;
    bwd_dq_bf16_kernel<128><<<(unsigned)grid_q, 256, DqSmem<128>::TOTAL, s>>>(a);
  }
  return hipGetLastError();
}

hipError_t launch_bwd_bf16(const BwdArgs& a, unsigned stages, hipStream_t s) {
  hipError_t e = hipSuccess;
  if (stages & 2) e = launch_bwd_dkdv_bf16(a, s);
  if (e == hipSuccess && (stages & 4)) e = launch_bwd_dq_bf16(a, s);
  return e;
}

}  // namespace lvx
