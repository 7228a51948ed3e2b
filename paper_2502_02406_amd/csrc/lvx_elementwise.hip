// HBM-bound kernels of the path: the Rescale/merge of Algorithm 1 (also used to combine the
// forward kernel's KV splits), the backward's delta = rowsum(dO * O), and the dQ conversion.
#include "lvx_internal.h"

namespace lvx {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

__device__ __forceinline__ float bf16_lo(unsigned u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(unsigned u) { return __uint_as_float(u & 0xffff0000u); }
__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  bf16x2 r;
  r[0] = (__bf16)a;   // round to nearest even
  r[1] = (__bf16)b;
  return *(unsigned*)&r;
}

// One thread owns VEC consecutive elements of one (b,h,i) row: VEC = 4 floats or 8 bf16 (16 bytes).
// L' = ln sum_k exp(L_k), O' = sum_k exp(L_k - L') O_k.  A row's threads sit in one wavefront, so
// every lane has read lse_parts[*][row] before lane 0 of the row stores lse_out[row]; this is
// what makes lse_out == lse_parts[0] (in-place update of the running state) safe.  (A row takes a
// power-of-two number of lanes, the next one up when D / VEC is none: the spare lanes idle.)
__host__ __device__ inline int merge_lanes_per_row(int n) {   // smallest power of two >= n (n <= 64)
  int p = 1;
  while (p < n) p <<= 1;
  return p;
}

constexpr int MERGE_UNITS = 1;        // 16-byte pieces of rows that one thread merges (2: measured, no faster)

template <bool PART_F32, bool OUT_F32>
__global__ void __launch_bounds__(256) merge_kernel(MergeArgs a) {
  constexpr int VEC_IN = PART_F32 ? 4 : 8;
  constexpr int VEC_OUT = OUT_F32 ? 4 : 8;
  constexpr int VEC = VEC_IN < VEC_OUT ? VEC_IN : VEC_OUT;   // elements per piece
  constexpr int U = MERGE_UNITS, GRP = 4;
  const int vpr = merge_lanes_per_row(a.D / VEC);             // lanes per row
  // Piece u of a thread lies a whole grid further on (a multiple of 64 lanes, so rows still sit in
  // one wavefront).  The parts' elements are fetched four parts at a time, the first four of
  // every piece before anything else: they are on their way while the rows' statistics are read
  // and turned into weights, so a thread waits for memory once, not twice.  (A part without keys
  // still has a buffer; what it holds is fetched and dropped.)
  const long t0 = (long)blockIdx.x * 256 + threadIdx.x, stride = (long)gridDim.x * 256;
  long row[U];
  int c[U];
  bool on[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const long t = t0 + u * stride;
    row[u] = t / vpr;
    c[u] = (int)(t % vpr) * VEC;
    on[u] = row[u] < a.rows && c[u] < a.D;
  }
  auto load_part = [&](int u, int k) __attribute__((always_inline)) -> u32x4 {
    if (PART_F32) return *(const u32x4*)((const float*)a.o_parts[k] + row[u] * a.D + c[u]);
    const uint16_t* src = (const uint16_t*)a.o_parts[k] + row[u] * a.D + c[u];
    if (VEC == 8) return *(const u32x4*)src;
    const unsigned x0 = ((const unsigned*)src)[0], x1 = ((const unsigned*)src)[1];
    return u32x4{x0, x1, 0u, 0u};
  };
  const int n = a.n_parts;
  u32x4 buf[U][GRP];
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int g = 0; g < GRP; ++g)
      if (on[u] && g < n) buf[u][g] = load_part(u, g);

  float acc[U][VEC], Lout[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[u][e] = 0.f;
    Lout[u] = -INFINITY;
    if (!on[u]) continue;
    auto add_part = [&](const u32x4& x, float w) __attribute__((always_inline)) {
      if (PART_F32) {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[u][e] += w * __uint_as_float(x[e]);
      } else {
#pragma unroll
        for (int e = 0; e < VEC / 2; ++e) {
          acc[u][2 * e] += w * bf16_lo(x[e]);
          acc[u][2 * e + 1] += w * bf16_hi(x[e]);
        }
      }
    };
    // The statistics of the first LG parts (all of them, as a rule) are read once, together, and
    // kept: read part by part inside the loops below, each would wait for the one before it.
    constexpr int LG = 8;
    float lk[LG];
#pragma unroll
    for (int k = 0; k < LG; ++k) {
      const float x = a.lse_parts[k < n ? k : n - 1][row[u]];
      lk[k] = k < n ? x : -INFINITY;
    }
    float M = -INFINITY;
#pragma unroll
    for (int k = 0; k < LG; ++k) M = fmaxf(M, lk[k]);
    for (int k = LG; k < n; ++k) M = fmaxf(M, a.lse_parts[k][row[u]]);
    if (M == -INFINITY) continue;
    float z = 0.f;
#pragma unroll
    for (int k = 0; k < LG; ++k) z += expf(lk[k] - M);               // (exp(-inf) = 0: parts that are not there)
    for (int k = LG; k < n; ++k) z += expf(a.lse_parts[k][row[u]] - M);
    Lout[u] = M + logf(z);
#pragma unroll
    for (int k0 = 0; k0 < LG; k0 += GRP) {
      if (k0 >= n) break;
      if (k0 > 0) {
#pragma unroll
        for (int g = 0; g < GRP; ++g)
          if (k0 + g < n) buf[u][g] = load_part(u, k0 + g);
      }
#pragma unroll
      for (int g = 0; g < GRP; ++g)
        if (k0 + g < n && lk[k0 + g] != -INFINITY) add_part(buf[u][g], expf(lk[k0 + g] - Lout[u]));
    }
    for (int k0 = LG; k0 < n; k0 += GRP) {
#pragma unroll
      for (int g = 0; g < GRP; ++g)
        if (k0 + g < n) buf[u][g] = load_part(u, k0 + g);
#pragma unroll
      for (int g = 0; g < GRP; ++g)
        if (k0 + g < n) {
          const float l = a.lse_parts[k0 + g][row[u]];
          if (l != -INFINITY) add_part(buf[u][g], expf(l - Lout[u]));
        }
    }
  }
  // (every load of the statistics above precedes every store below: lse_out may be lse_parts[0])
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (!on[u]) continue;
    const long i = row[u] % a.Sq, h = (row[u] / a.Sq) % a.Hq, b = row[u] / ((long)a.Sq * a.Hq);
    const long off = b * a.o_sb + h * a.o_sh + i * a.o_ss + c[u];
    if (OUT_F32) {
      const f32x4 y = {acc[u][0], acc[u][1], acc[u][2], acc[u][3]};
      *(f32x4*)((float*)a.o_out + off) = y;
    } else {
      unsigned* dst = (unsigned*)((uint16_t*)a.o_out + off);
      if (VEC == 8) {
        const u32x4 y = {pack_bf16(acc[u][0], acc[u][1]), pack_bf16(acc[u][2], acc[u][3]),
                         pack_bf16(acc[u][4], acc[u][5]), pack_bf16(acc[u][6], acc[u][7])};
        *(u32x4*)dst = y;
      } else {
        dst[0] = pack_bf16(acc[u][0], acc[u][1]);
        dst[1] = pack_bf16(acc[u][2], acc[u][3]);
      }
    }
    if (c[u] == 0) a.lse_out[row[u]] = Lout[u];
  }
}

hipError_t launch_merge(const MergeArgs& a, int part_is_f32, int out_is_f32, hipStream_t s) {
  const int vec = (part_is_f32 || out_is_f32) ? 4 : 8;
  const long threads = a.rows * merge_lanes_per_row(a.D / vec);
  const unsigned blocks = (unsigned)((threads + 256 * MERGE_UNITS - 1) / (256 * MERGE_UNITS));
  if (part_is_f32 && out_is_f32) merge_kernel<true, true><<<blocks, 256, 0, s>>>(a);
  else if (part_is_f32) merge_kernel<true, false><<<blocks, 256, 0, s>>>(a);
  else if (out_is_f32) merge_kernel<false, true><<<blocks, 256, 0, s>>>(a);
  else merge_kernel<false, false><<<blocks, 256, 0, s>>>(a);
  return hipGetLastError();
}

// delta[b,h,i] = sum_d dO[b,h,i,d] * O[b,h,i,d].  16 lanes per row.  The bf16 kernels read the
// row statistics 32 rows at a time with aligned copies, so a padded, grouped copy is written as
// well: stats[B,Hq,sq_pad/32][2][32] (sq_pad a multiple of 32) holds, per group of 32 rows, 32
// values of -L * log2(e) -- -inf for rows without keys and for pad rows, which makes their
// probabilities exp2(-inf) = 0 -- followed by the 32 values of -delta (0 in pad rows).
// stats_ovl (optional, [B,Hq][2][32]): the same for rows Sq-32 .. Sq-1, with -inf for those of them
// that belong to a full group of 32.
template <bool F32>
__global__ void __launch_bounds__(256) delta_kernel(Dims d, const void* o, const void* d_o,
                                                    const float* lse, float* delta, float* stats,
                                                    int sq_pad, float* stats_ovl) {
  const long rows = (long)d.B * d.Hq * sq_pad;
  const long rowp = ((long)blockIdx.x * 256 + threadIdx.x) / 16;
  const int c = threadIdx.x % 16;
  if (rowp >= rows) return;                 // whole 16-lane groups leave together
  const long i = rowp % sq_pad, h = (rowp / sq_pad) % d.Hq, b = rowp / ((long)sq_pad * d.Hq);
  float s = 0.f;
  if (i < d.Sq) {
    const long off = b * d.q_sb + h * d.q_sh + i * d.q_ss;
    if (F32) {
      const float* po = (const float*)o + off;
      const float* pg = (const float*)d_o + off;
      for (int e = c * 4; e < d.D; e += 64) {
        f32x4 x = *(const f32x4*)(po + e), y = *(const f32x4*)(pg + e);
        s += x[0] * y[0] + x[1] * y[1] + x[2] * y[2] + x[3] * y[3];
      }
    } else {
      const uint16_t* po = (const uint16_t*)o + off;
      const uint16_t* pg = (const uint16_t*)d_o + off;
      for (int e = c * 8; e < d.D; e += 128) {
        u32x4 x = *(const u32x4*)(po + e), y = *(const u32x4*)(pg + e);
#pragma unroll
        for (int k = 0; k < 4; ++k) s += bf16_lo(x[k]) * bf16_lo(y[k]) + bf16_hi(x[k]) * bf16_hi(y[k]);
      }
    }
  }
#pragma unroll
  for (int m = 8; m >= 1; m >>= 1) s += __shfl_xor(s, m, 16);
  if (c != 0) return;
  float nl2 = -INFINITY;
  if (i < d.Sq) {
    const long row = (b * d.Hq + h) * d.Sq + i;
    delta[row] = s;
    const float L = lse[row];
    if (L != -INFINITY) nl2 = -L * 1.4426950408889634f;
  }
  const long slot = (rowp / 32) * 64 + rowp % 32;     // sq_pad is a multiple of 32
  stats[slot] = nl2;
  stats[slot + 32] = -s;
  if (stats_ovl && i >= d.Sq - 32 && i < d.Sq) {
    const long j = (b * d.Hq + h) * 64 + (i - (d.Sq - 32));
    stats_ovl[j] = i >= (d.Sq & ~31) ? nl2 : -INFINITY;
    stats_ovl[j + 32] = -s;
  }
}

hipError_t launch_delta(const Dims& d, const void* o, const void* d_o, int is_f32, const float* lse,
                        float* delta, float* stats, int sq_pad, float* stats_ovl, hipStream_t s) {
  const long rows = (long)d.B * d.Hq * sq_pad;
  const unsigned blocks = (unsigned)((rows * 16 + 255) / 256);
  if (is_f32) delta_kernel<true><<<blocks, 256, 0, s>>>(d, o, d_o, lse, delta, stats, sq_pad, stats_ovl);
  else delta_kernel<false><<<blocks, 256, 0, s>>>(d, o, d_o, lse, delta, stats, sq_pad, stats_ovl);
  return hipGetLastError();
}

// dq_accum += sum of the KV splits' partial dQ (float32, contiguous).  One thread per 4 elements.
__global__ void __launch_bounds__(256) dq_reduce_kernel(const float* parts, int n_parts, long n, float* acc) {
  const long i = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= n) return;
  f32x4 x = *(const f32x4*)(acc + i);
  for (int k = 0; k < n_parts; ++k) x += *(const f32x4*)(parts + (long)k * n + i);
  *(f32x4*)(acc + i) = x;
}

hipError_t launch_dq_reduce(const float* parts, int n_parts, long n, float* dq_accum, hipStream_t s) {
  const unsigned blocks = (unsigned)((n / 4 + 255) / 256);
  dq_reduce_kernel<<<blocks, 256, 0, s>>>(parts, n_parts, n, dq_accum);
  return hipGetLastError();
}

// dq (input dtype, Q's strides) = dq_accum (float32, contiguous).  One thread per 8 elements.
template <bool F32>
__global__ void __launch_bounds__(256) dq_finalize_kernel(Dims d, const float* acc, void* dq) {
  const int vpr = d.D / 8;
  const long t = (long)blockIdx.x * 256 + threadIdx.x;
  const long row = t / vpr;
  if (row >= (long)d.B * d.Hq * d.Sq) return;
  const int c = (int)(t % vpr) * 8;
  const long i = row % d.Sq, h = (row / d.Sq) % d.Hq, b = row / ((long)d.Sq * d.Hq);
  const long off = b * d.q_sb + h * d.q_sh + i * d.q_ss + c;
  const f32x4 x0 = *(const f32x4*)(acc + row * d.D + c), x1 = *(const f32x4*)(acc + row * d.D + c + 4);
  if (F32) {
    *(f32x4*)((float*)dq + off) = x0;
    *(f32x4*)((float*)dq + off + 4) = x1;
  } else {
    u32x4 y = {pack_bf16(x0[0], x0[1]), pack_bf16(x0[2], x0[3]), pack_bf16(x1[0], x1[1]),
               pack_bf16(x1[2], x1[3])};
    *(u32x4*)((uint16_t*)dq + off) = y;
  }
}

hipError_t launch_dq_finalize(const Dims& d, const float* dq_accum, void* dq, int is_f32,
                              hipStream_t s) {
  const long threads = (long)d.B * d.Hq * d.Sq * (d.D / 8);
  const unsigned blocks = (unsigned)((threads + 255) / 256);
  if (is_f32) dq_finalize_kernel<true><<<blocks, 256, 0, s>>>(d, dq_accum, dq);
  else dq_finalize_kernel<false><<<blocks, 256, 0, s>>>(d, dq_accum, dq);
  return hipGetLastError();
}

}  // namespace lvx
