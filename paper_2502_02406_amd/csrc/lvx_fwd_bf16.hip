// bf16 forward kernel: the FlashAttention call of Algorithm 1 for a short query block against a
// long local K/V block, on the gfx950 matrix cores.
//
// Workgroup = 4 wavefronts = 128 query rows of one (batch, query head); each wave owns 32 rows
// whose Q operands stay in registers for the whole kernel.  K/V tiles of 64 keys are staged
// through LDS (double buffered, coalesced 16-byte global reads) and shared by the four waves.
// Per tile a wave computes S^T = K Q^T (keys in registers, one query column per lane), the online
// softmax in that layout (row statistics are per-lane scalars; the two half-waves exchange one
// value per tile), and O^T += V^T P^T with P^T taken straight from the score registers and V^T
// fetched by transposing LDS reads.  The grid is cut along the KV axis (split-KV) when the query
// block alone cannot fill the chip; partial (O, L) pairs are combined by the merge kernel.
#include "lvx_internal.h"
#include "lvx_mfma.h"

namespace lvx {

namespace {

constexpr int BM = 128;       // query rows per workgroup
constexpr int BN = 64;        // keys per tile
constexpr float LOG2E = 1.4426950408889634f;

template <int D> struct FwdSmem {
  static constexpr int KP = (D + 8) * 2;     // K row pitch in bytes (conflict-free b128 reads)
  static constexpr int VP = (D + 32) * 2;    // V row pitch in bytes (transposing reads)
  static constexpr int K_BYTES = BN * KP;
  static constexpr int V_BYTES = BN * VP;
  static constexpr int STAGE = K_BYTES + V_BYTES;
  static constexpr int TOTAL = 2 * STAGE;
};

template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
fwd_bf16_kernel(FwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  using SM = FwdSmem<D>;
  constexpr int KS = D / 16;            // k-steps of the QK^T product
  constexpr int DB = D / 32;            // 32-row blocks of O^T
  constexpr int CPR = D / 8;            // 16-byte chunks per K/V row
  constexpr int RPP = 256 / CPR;        // rows per load pass
  constexpr int NPASS = BN / RPP;       // load passes per tile

  const Dims& d = a.d;
  const int G = d.Hq / d.Hkv;
  const int n_qt = (d.Sq + BM - 1) / BM;
  HeadWork hw;
  if (!xcd_decode(blockIdx.x, d.B * d.Hkv, a.n_split * G * n_qt, &hw)) return;
  const int b = hw.head / d.Hkv, hk = hw.head % d.Hkv;
  const int split = hw.item / (G * n_qt);
  const int hq = hk * G + (hw.item % (G * n_qt)) / n_qt;
  const int qt = hw.item % n_qt;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ql = lane & 31;
  const int i_wave0 = qt * BM + wave * 32;          // first query row of this wave
  const int i_lane = i_wave0 + ql;                  // this lane's query row (column of S^T)

  // KV range of this split, in tiles
  const int n_tiles = (d.Skv + BN - 1) / BN;
  const int tps = (n_tiles + a.n_split - 1) / a.n_split;
  const int t_begin = split * tps;
  const int t_end = min(n_tiles, t_begin + tps);

  // Q operands (B of S^T = K Q^T): lane holds row i_lane, columns 16 ks + 8 g + 0..7
  bf16x8 qf[KS];
  {
    const uint16_t* qrow = (const uint16_t*)a.q + b * d.q_sb + hq * d.q_sh + (long)i_lane * d.q_ss;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 x = {0, 0, 0, 0};
      if (i_lane < d.Sq) x = *(const u32x4*)(qrow + 16 * ks + 8 * g);
      qf[ks] = __builtin_bit_cast(bf16x8, x);
    }
  }

  const uint16_t* kbase = (const uint16_t*)a.k + b * d.kv_sb + hk * d.kv_sh;
  const uint16_t* vbase = (const uint16_t*)a.v + b * d.kv_sb + hk * d.kv_sh;
  const int ld_row = tid / CPR, ld_col = (tid % CPR) * 8;

  // which tiles does this workgroup need at all (media mask)?
  const int i_wg0 = qt * BM, i_wg1 = min(d.Sq, i_wg0 + BM) - 1;
  auto tile_needed = [&](int t) -> bool {
    if (!a.mask.allow) return true;
    return mask_rect(a.mask, b, i_wg0, i_wg1, t * BN, min(d.Skv, t * BN + BN) - 1) != 0;
  };
  auto next_tile = [&](int t) -> int {
    while (t < t_end && !tile_needed(t)) ++t;
    return t;
  };

  u32x4 kreg[NPASS], vreg[NPASS];
  auto load_tile = [&](int t) {
#pragma unroll
    for (int p = 0; p < NPASS; ++p) {
      const int j = t * BN + p * RPP + ld_row;
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
      *(u32x4*)(ks + r * SM::KP + ld_col * 2) = kreg[p];
      *(u32x4*)(vs + r * SM::VP + ld_col * 2) = vreg[p];
    }
  };

  f32x16 oacc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i) oacc[i] = zero16();
  float m_run = -INFINITY;     // running max of raw scores (q.k, unscaled)
  float l_run = 0.f;           // this lane's share of the running sum of exp
  const float c2 = d.scale * LOG2E;

  int cur = next_tile(t_begin);
  if (cur < t_end) {
    load_tile(cur);
    store_tile(0);
  }
  __syncthreads();
  int stage = 0;
  while (cur < t_end) {
    const int nxt = next_tile(cur + 1);
    if (nxt < t_end) load_tile(nxt);          // global loads in flight during the math below

    const char* ks_ = smem + stage * SM::STAGE;
    const char* vs_ = ks_ + SM::K_BYTES;
    const int j0 = cur * BN;
    int cls = 1;
    if (a.mask.allow)
      cls = mask_rect(a.mask, b, i_wave0, min(d.Sq - 1, i_wave0 + 31), j0, min(d.Skv, j0 + BN) - 1);
    if (i_wave0 >= d.Sq) cls = 0;
    if (cls != 0) {
      // ---- S^T = K Q^T : two 32-key blocks
      f32x16 sacc[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        sacc[kb] = zero16();
        const char* krow = ks_ + (kb * 32 + ql) * SM::KP + g * 16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          bf16x8 kf = *(const bf16x8*)(krow + ks * 32);
          sacc[kb] = mfma32(kf, qf[ks], sacc[kb]);
        }
      }
      // ---- masking: key tail and mixed mask tiles
      if (j0 + BN > d.Skv || cls == 2) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int j = j0 + kb * 32 + 8 * (v / 4) + 4 * g + (v % 4);
            bool ok = j < d.Skv;
            if (ok && cls == 2) ok = (i_lane < d.Sq) && mask_elem(a.mask, b, i_lane, j);
            if (!ok) sacc[kb][v] = -INFINITY;
          }
      }
      // ---- online softmax (one query column per lane)
      float tmax = sacc[0][0];
#pragma unroll
      for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, sacc[0][v]);
#pragma unroll
      for (int v = 0; v < 16; ++v) tmax = fmaxf(tmax, sacc[1][v]);
      tmax = xhalf_max(tmax);
      const float m_new = fmaxf(m_run, tmax);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_safe) * c2);     // m_run = -inf -> 0
      const float mc = m_safe * c2;
      m_run = m_new;
      float psum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][v], c2, -mc));
          sacc[kb][v] = p;
          psum += p;
        }
      l_run = l_run * alpha + psum;
      if (!__all(alpha == 1.f)) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;
      }
      // ---- O^T += V^T P^T : four k-steps of 16 keys
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const bf16x8 pf = cvt_operand(sacc[t >> 1], 8 * (t & 1));
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 vf = load_tr_operand(vs_, SM::VP, 16 * t, 32 * db, lane);
          oacc[db] = mfma32(vf, pf, oacc[db]);
        }
      }
    }
    if (nxt < t_end) store_tile(stage ^ 1);
    __syncthreads();
    stage ^= 1;
    cur = nxt;
  }

  // ---- epilogue: O = acc / l, L = m * scale + ln l
  const float l_tot = xhalf_sum(l_run);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  const float lse = l_tot > 0.f ? m_run * d.scale + logf(l_tot) : -INFINITY;
  if (i_lane >= d.Sq) return;
  const long row = ((long)b * d.Hq + hq) * d.Sq + i_lane;
  if (a.n_split > 1) {
    float* o = a.o_part + ((long)split * d.B * d.Hq * d.Sq + row) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 y = {oacc[db][4 * q4] * inv, oacc[db][4 * q4 + 1] * inv, oacc[db][4 * q4 + 2] * inv,
                   oacc[db][4 * q4 + 3] * inv};
        *(f32x4*)(o + 32 * db + 8 * q4 + 4 * g) = y;
      }
    if (g == 0) a.lse_part[(long)split * d.B * d.Hq * d.Sq + row] = lse;
    return;
  }
  const long off = b * d.q_sb + hq * d.q_sh + (long)i_lane * d.q_ss;
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const float y0 = oacc[db][4 * q4] * inv, y1 = oacc[db][4 * q4 + 1] * inv,
                  y2 = oacc[db][4 * q4 + 2] * inv, y3 = oacc[db][4 * q4 + 3] * inv;
      const int col = 32 * db + 8 * q4 + 4 * g;
      if (a.o_is_f32) {
        f32x4 y = {y0, y1, y2, y3};
        *(f32x4*)((float*)a.o + off + col) = y;
      } else {
        u32x2 y = {pack2_bf16(y0, y1), pack2_bf16(y2, y3)};
        *(u32x2*)((uint16_t*)a.o + off + col) = y;
      }
    }
  if (g == 0) a.lse[row] = lse;
}

}  // namespace

int fwd_bf16_pick_split(const Dims& d, int n_cu) {
  // two workgroups per CU; split the KV axis until the grid covers the chip about twice over
  const long base = (long)d.B * d.Hq * ((d.Sq + BM - 1) / BM);
  const int n_tiles = (d.Skv + BN - 1) / BN;
  long want = (4L * n_cu + base - 1) / base;
  if (want < 1) want = 1;
  long cap = n_tiles / 8;                 // keep at least 8 tiles (512 keys) per split
  if (cap < 1) cap = 1;
  if (want > cap) want = cap;
  if (want > 64) want = 64;
  return (int)want;
}

hipError_t launch_fwd_bf16(const FwdArgs& a, hipStream_t s) {
  const Dims& d = a.d;
  const int G = d.Hq / d.Hkv;
  const int n_qt = (d.Sq + BM - 1) / BM;
  const long grid = xcd_grid(d.B * d.Hkv, a.n_split * G * n_qt);
  if (d.D == 64) {
    static bool once = false;
    if (!once) {
      hipError_t e = hipFuncSetAttribute((const void*)fwd_bf16_kernel<64>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, FwdSmem<64>::TOTAL);
      if (e != hipSuccess) return e;
      once = true;
    }
    fwd_bf16_kernel<64><<<(unsigned)grid, 256, FwdSmem<64>::TOTAL, s>>>(a);
  } else {
    static bool once = false;
    if (!once) {
      hipError_t e = hipFuncSetAttribute((const void*)fwd_bf16_kernel<128>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, FwdSmem<128>::TOTAL);
      if (e != hipSuccess) return e;
      once = true;
    }
    fwd_bf16_kernel<128><<<(unsigned)grid, 256, FwdSmem<128>::TOTAL, s>>>(a);
  }
  return hipGetLastError();
}

}  // namespace lvx
