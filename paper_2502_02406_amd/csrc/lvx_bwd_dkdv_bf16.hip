// bf16 backward, key-stationary kernel: dK and dV of one K/V block (Table 1 of the paper counts
// the backward as five products; this kernel performs four of them: S, dP, dV, dK).
// A wave keeps its keys of K in registers (V in LDS) and streams the query rows of every head
// that shares this K/V head.  S = Q K^T and dP = dO V^T put one KEY per lane, so P and dS (bf16)
// are the B operands of dV^T += dO^T P and dK^T += Q^T dS, with dO^T / Q^T from transposing reads.
#include "lvx_internal.h"
#include "lvx_mfma.h"

namespace lvx {

namespace {

constexpr float LOG2E = 1.4426950408889634f;

// ------------------------------------------------------------------------------------------
// dK/dV kernel
// ------------------------------------------------------------------------------------------
constexpr int KVB = 1;                 // 32-key blocks per wave
constexpr int KN = 4 * 32 * KVB;       // keys per workgroup (4 waves)
constexpr int KM = 32;                 // query rows per step

template <int D> struct DkvSmem {
  static constexpr int P = (D + 8) * 2;        // row pitch (bytes) of the resident V rows
  static constexpr int T_BYTES = ILV_ROWS * P; // [Q; dO] as ONE 64-row interleaved tile (rows 0..31 Q, 32..63 dO)
  static constexpr int STAT = KM * 4;          // one float per row
  static constexpr int STAGE = T_BYTES + 2 * STAT;
  static constexpr int V_BYTES = KN * P;       // this workgroup's V rows, resident for the kernel
  static constexpr int TOTAL = 2 * STAGE + V_BYTES;
};

template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
bwd_dkdv_bf16_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  using SM = DkvSmem<D>;
  constexpr int KS = D / 16, DB = D / 32, CPR = D / 8;
  constexpr int CHUNKS = KM * CPR;                 // 16-byte chunks per Q (or dO) tile
  constexpr int NLD = (CHUNKS + 255) / 256;        // chunks per thread

  const Dims& d = a.d;
  const int G = d.Hq / d.Hkv;
  const int n_kt = (d.Skv + KN - 1) / KN;
  HeadWork hw;
  if (!xcd_decode(blockIdx.x, d.B * d.Hkv, n_kt, &hw)) return;
  const int b = hw.head / d.Hkv, hk = hw.head % d.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, kl = lane & 31;
  const int j_wg0 = hw.item * KN;
  const int j_wave0 = j_wg0 + wave * 32 * KVB;

  // K operands of this wave's keys stay in registers: lane holds key j_wave0 + 32 kb + kl,
  // columns 16 ks + 8 g ..; the V rows of the workgroup stay in LDS (registers are spent on the
  // two accumulators).
  bf16x8 kf[KVB][KS];
#pragma unroll
  for (int kb = 0; kb < KVB; ++kb) {
    const int j = j_wave0 + 32 * kb + kl;
    const long off = b * d.kv_sb + hk * d.kv_sh + (long)j * d.kv_ss;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 x = {0, 0, 0, 0};
      if (j < d.Skv) x = *(const u32x4*)((const uint16_t*)a.k + off + 16 * ks + 8 * g);
      kf[kb][ks] = __builtin_bit_cast(bf16x8, x);
    }
  }
  char* const vres = smem + 2 * SM::STAGE;
  for (int c = tid; c < KN * CPR; c += 256) {
    const int r = c / CPR, col = (c % CPR) * 8, j = j_wg0 + r;
    u32x4 y = {0, 0, 0, 0};
    if (j < d.Skv)
      y = *(const u32x4*)((const uint16_t*)a.v + b * d.kv_sb + hk * d.kv_sh + (long)j * d.kv_ss + col);
    *(u32x4*)(vres + r * SM::P + col * 2) = y;
  }
  const char* const vwave = vres + (wave * 32 * KVB + kl) * SM::P + g * 16;
  const float c2 = d.scale * LOG2E;

  f32x16 dk[KVB][DB], dv[KVB][DB];
#pragma unroll
  for (int kb = 0; kb < KVB; ++kb)
#pragma unroll
    for (int i = 0; i < DB; ++i) { dk[kb][i] = zero16(); dv[kb][i] = zero16(); }

  // query steps: the G heads of the group, KM rows at a time
  const int spH = (d.Sq + KM - 1) / KM;
  const int n_steps = G * spH;
  const int j_wg1 = min(d.Skv, j_wg0 + KN) - 1;
  auto next_step = [&](int s) -> int {
    if (a.mask.allow)
      while (s < n_steps) {
        const int i0 = (s % spH) * KM;
        if (mask_rect(a.mask, b, i0, min(d.Sq, i0 + KM) - 1, j_wg0, j_wg1) != 0) break;
        ++s;
      }
    return s;
  };
  u32x4 qreg[NLD], greg[NLD];
  float sreg = 0.f;
  auto load_step = [&](int s) {
    const int hq = hk * G + s / spH, i0 = (s % spH) * KM;
    const long base = b * d.q_sb + hq * d.q_sh;
#pragma unroll
    for (int p = 0; p < NLD; ++p) {
      const int c = p * 256 + tid;
      const int r = c / CPR, col = (c % CPR) * 8;
      u32x4 x = {0, 0, 0, 0}, y = {0, 0, 0, 0};
      if (c < CHUNKS && i0 + r < d.Sq) {
        x = *(const u32x4*)((const uint16_t*)a.q + base + (long)(i0 + r) * d.q_ss + col);
        y = *(const u32x4*)((const uint16_t*)a.d_o + base + (long)(i0 + r) * d.q_ss + col);
      }
      qreg[p] = x;
      greg[p] = y;
    }
    if (tid < 2 * KM) {                      // threads 0..31: L * log2(e); 32..63: delta
      const int r = tid % KM;
      const long row = ((long)b * d.Hq + hq) * d.Sq + i0 + r;
      float x = tid < KM ? INFINITY : 0.f;
      if (i0 + r < d.Sq) {
        if (tid < KM) { const float L = a.lse[row]; if (L != -INFINITY) x = L * LOG2E; }
        else x = a.delta[row];
      }
      sreg = x;
    }
  };
  auto store_step = [&](int stage) {
    char* qs = smem + stage * SM::STAGE;
#pragma unroll
    for (int p = 0; p < NLD; ++p) {
      const int c = p * 256 + tid;
      if (c < CHUNKS) {
        const int r = c / CPR, col = (c % CPR) * 8;
        (void)r;
        *(u32x4*)(qs + ilv_off<D>(tid / CPR, p * (256 / CPR), col)) = qreg[p];
        *(u32x4*)(qs + ilv_off<D>(tid / CPR, KM + p * (256 / CPR), col)) = greg[p];
      }
    }
    if (tid < 2 * KM) *(float*)(qs + SM::T_BYTES + tid * 4) = sreg;
  };

  int cur = next_step(0);
  if (cur < n_steps) { load_step(cur); store_step(0); }
  __syncthreads();
  int stage = 0;
  while (cur < n_steps) {
    const int nxt = next_step(cur + 1);
    if (nxt < n_steps) load_step(nxt);
    const char* qs_ = smem + stage * SM::STAGE;
    const float* lse_s = (const float*)(qs_ + SM::T_BYTES);
    const float* del_s = lse_s + KM;
    const int i0 = (cur % spH) * KM;
    int cls = 1;
    if (a.mask.allow)
      cls = mask_rect(a.mask, b, i0, min(d.Sq, i0 + KM) - 1, j_wave0,
                      min(d.Skv - 1, j_wave0 + 32 * KVB - 1));
    if (j_wave0 >= d.Skv) cls = 0;
    if (cls != 0) {
      // ---- S = Q K^T and dP = dO V^T: lane = key column, registers = query rows
      f32x16 sacc[KVB], pacc[KVB];
#pragma unroll
      for (int kb = 0; kb < KVB; ++kb) { sacc[kb] = zero16(); pacc[kb] = zero16(); }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 qa = *(const bf16x8*)(qs_ + ilv_off<D>(kl, 0, 16 * ks + 8 * g));
        const bf16x8 ga = *(const bf16x8*)(qs_ + ilv_off<D>(kl, KM, 16 * ks + 8 * g));
#pragma unroll
        for (int kb = 0; kb < KVB; ++kb) {
          sacc[kb] = mfma32(qa, kf[kb][ks], sacc[kb]);
          pacc[kb] = mfma32(ga, *(const bf16x8*)(vwave + kb * 32 * SM::P + ks * 32), pacc[kb]);
        }
      }
      // ---- P and dS in place
      const bool need_mask = (j_wave0 + 32 * KVB > d.Skv) || cls == 2;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4 l4 = *(const f32x4*)(lse_s + 8 * q4 + 4 * g);
        const f32x4 d4 = *(const f32x4*)(del_s + 8 * q4 + 4 * g);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int v = 4 * q4 + e;
#pragma unroll
          for (int kb = 0; kb < KVB; ++kb) {
            float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][v], c2, -l4[e]));
            if (need_mask) {
              const int j = j_wave0 + 32 * kb + kl, i = i0 + 8 * q4 + 4 * g + e;
              bool ok = j < d.Skv;
              if (ok && cls == 2) ok = i < d.Sq && mask_elem(a.mask, b, i, j);
              if (!ok) p = 0.f;
            }
            sacc[kb][v] = p;
            pacc[kb][v] = p * (pacc[kb][v] - d4[e]);
          }
        }
      }
      // ---- dV^T += dO^T P,  dK^T += Q^T dS  (two k-steps of 16 query rows)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        bf16x8 pf[KVB], sf[KVB];
#pragma unroll
        for (int kb = 0; kb < KVB; ++kb) {
          pf[kb] = cvt_operand(sacc[kb], 8 * t);
          sf[kb] = cvt_operand(pacc[kb], 8 * t);
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 gt = load_tr_operand_ilv<D>(qs_, KM + 16 * t, 32 * db, lane);
          const bf16x8 qtr = load_tr_operand_ilv<D>(qs_, 16 * t, 32 * db, lane);
#pragma unroll
          for (int kb = 0; kb < KVB; ++kb) {
            dv[kb][db] = mfma32(gt, pf[kb], dv[kb][db]);
            dk[kb][db] = mfma32(qtr, sf[kb], dk[kb][db]);
          }
        }
      }
    }
    if (nxt < n_steps) store_step(stage ^ 1);
    __syncthreads();
    stage ^= 1;
    cur = nxt;
  }

  // ---- write dK = scale * acc, dV = acc (transposed accumulators: lane = key row)
#pragma unroll
  for (int kb = 0; kb < KVB; ++kb) {
    const int j = j_wave0 + 32 * kb + kl;
    if (j >= d.Skv) continue;
    const long off = b * d.kv_sb + hk * d.kv_sh + (long)j * d.kv_ss;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int col = 32 * db + 8 * q4 + 4 * g;
        u32x2 yk = {pack2_bf16(dk[kb][db][4 * q4] * d.scale, dk[kb][db][4 * q4 + 1] * d.scale),
                    pack2_bf16(dk[kb][db][4 * q4 + 2] * d.scale, dk[kb][db][4 * q4 + 3] * d.scale)};
        u32x2 yv = {pack2_bf16(dv[kb][db][4 * q4], dv[kb][db][4 * q4 + 1]),
                    pack2_bf16(dv[kb][db][4 * q4 + 2], dv[kb][db][4 * q4 + 3])};
        *(u32x2*)((uint16_t*)a.dk + off + col) = yk;
        *(u32x2*)((uint16_t*)a.dv + off + col) = yv;
      }
  }
}

template <typename F>
hipError_t set_smem_once(F* fn, int bytes, bool* done) {
  if (*done) return hipSuccess;
  hipError_t e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) *done = true;
  return e;
}

}  // namespace

hipError_t launch_bwd_dkdv_bf16(const BwdArgs& a, hipStream_t s) {
  const Dims& d = a.d;
  const long grid_k = xcd_grid(d.B * d.Hkv, (d.Skv + KN - 1) / KN);
  hipError_t e;
  if (d.D == 64) {
    static bool once = false;
    if ((e = set_smem_once(bwd_dkdv_bf16_kernel<64>, DkvSmem<64>::TOTAL, &once)) != hipSuccess) return e;
    bwd_dkdv_bf16_kernel<64><<<(unsigned)grid_k, 256, DkvSmem<64>::TOTAL, s>>>(a);
  } else {
    static bool once = false;
    if ((e = set_smem_once(bwd_dkdv_bf16_kernel<128>, DkvSmem<128>::TOTAL, &once)) != hipSuccess) return e;
    bwd_dkdv_bf16_kernel<128><<<(unsigned)grid_k, 256, DkvSmem<128>::TOTAL, s>>>(a);
  }
  return hipGetLastError();
}

}  // namespace lvx
