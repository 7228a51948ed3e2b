// float32 instantiation of the forward and backward passes: LDS-tiled, plain FMA arithmetic.
// It exists so that float32 workloads (the tiny exact check) are computed in float32 end to end
// instead of being rounded to bf16 for the matrix cores; it is not the performance path.
//
// Thread layout shared by the three kernels: 256 threads = 16 "owner" rows x 16 lanes.  The 16
// lanes of a row split the columns of the opposite sequence (score phase) and then the head
// dimension (accumulation phase).
#include "lvx_internal.h"

namespace lvx {

namespace {

constexpr int R = 16;    // owner rows per workgroup
constexpr int T = 32;    // rows of the streamed tile

__device__ __forceinline__ bool visible(const MaskDev& m, int b, int i, int j) {
  if (!m.allow) return true;
  return m.allow[b * m.stride_b + (long)(i / m.q_chunk) * m.stride_q + (j / m.kv_block)] != 0;
}

// Forward: workgroup owns R query rows of one (b, hq); streams K/V tiles of T rows.
template <int D>
__global__ void __launch_bounds__(256) fwd_f32_kernel(FwdArgs a) {
  __shared__ float Qs[R][D];
  __shared__ float Ks[T][D + 1];
  __shared__ float Vs[T][D];
  __shared__ float Ps[R][T];
  const Dims& d = a.d;
  const int tid = threadIdx.x, r = tid / 16, c = tid % 16;
  const int b = blockIdx.z, hq = blockIdx.y, hk = hq / (d.Hq / d.Hkv);
  const int i = blockIdx.x * R + r;
  const bool row_ok = i < d.Sq;
  const float* q = (const float*)a.q + b * d.q_sb + hq * d.q_sh;
  const float* k = (const float*)a.k + b * d.kv_sb + hk * d.kv_sh;
  const float* v = (const float*)a.v + b * d.kv_sb + hk * d.kv_sh;
  for (int e = c; e < D; e += 16) Qs[r][e] = row_ok ? q[(long)i * d.q_ss + e] : 0.f;

  float m = -INFINITY, l = 0.f;
  float acc[D / 16];
#pragma unroll
  for (int e = 0; e < D / 16; ++e) acc[e] = 0.f;

  for (int j0 = 0; j0 < d.Skv; j0 += T) {
    __syncthreads();
    for (int e = tid; e < T * D; e += 256) {
      const int jj = e / D, dd = e % D;
      const bool ok = j0 + jj < d.Skv;
      Ks[jj][dd] = ok ? k[(long)(j0 + jj) * d.kv_ss + dd] : 0.f;
      Vs[jj][dd] = ok ? v[(long)(j0 + jj) * d.kv_ss + dd] : 0.f;
    }
    __syncthreads();
    float s[T / 16];
    float tmax = -INFINITY;
#pragma unroll
    for (int t = 0; t < T / 16; ++t) {
      const int jj = c + 16 * t, j = j0 + jj;
      float x = 0.f;
      for (int e = 0; e < D; ++e) x = fmaf(Qs[r][e], Ks[jj][e], x);
      x *= d.scale;
      if (!row_ok || j >= d.Skv || !visible(a.mask, b, i, j)) x = -INFINITY;
      s[t] = x;
      tmax = fmaxf(tmax, x);
    }
#pragma unroll
    for (int w = 8; w >= 1; w >>= 1) tmax = fmaxf(tmax, __shfl_xor(tmax, w, 16));
    const float m_new = fmaxf(m, tmax);
    float alpha = 1.f, psum = 0.f;
    if (m_new != -INFINITY) {
      alpha = expf(m - m_new);                  // m = -inf -> 0
#pragma unroll
      for (int t = 0; t < T / 16; ++t) {
        const float p = expf(s[t] - m_new);     // s = -inf -> 0
        Ps[r][c + 16 * t] = p;
        psum += p;
      }
    } else {
#pragma unroll
      for (int t = 0; t < T / 16; ++t) Ps[r][c + 16 * t] = 0.f;
    }
#pragma unroll
    for (int w = 8; w >= 1; w >>= 1) psum += __shfl_xor(psum, w, 16);
    l = l * alpha + psum;
    m = m_new;
    __syncthreads();
#pragma unroll
    for (int e = 0; e < D / 16; ++e) {
      float x = acc[e] * alpha;
      for (int jj = 0; jj < T; ++jj) x = fmaf(Ps[r][jj], Vs[jj][c + 16 * e], x);
      acc[e] = x;
    }
  }
  if (!row_ok) return;
  const long row = ((long)b * d.Hq + hq) * d.Sq + i;
  const float inv = l > 0.f ? 1.f / l : 0.f;
  float* o = (float*)a.o + b * d.q_sb + hq * d.q_sh + (long)i * d.q_ss;
#pragma unroll
  for (int e = 0; e < D / 16; ++e) o[c + 16 * e] = acc[e] * inv;
  if (c == 0) a.lse[row] = l > 0.f ? m + logf(l) : -INFINITY;
}

// Backward, dQ part: workgroup owns R query rows; streams K/V tiles; p = exp(s - L).
template <int D>
__global__ void __launch_bounds__(256) bwd_dq_f32_kernel(BwdArgs a) {
  __shared__ float Qs[R][D];
  __shared__ float Gs[R][D];
  __shared__ float Ks[T][D + 1];
  __shared__ float Vs[T][D + 1];
  __shared__ float Ss[R][T];
  const Dims& d = a.d;
  const int tid = threadIdx.x, r = tid / 16, c = tid % 16;
  const int b = blockIdx.z, hq = blockIdx.y, hk = hq / (d.Hq / d.Hkv);
  const int i = blockIdx.x * R + r;
  const bool row_ok = i < d.Sq;
  const long qoff = b * d.q_sb + hq * d.q_sh + (long)i * d.q_ss;
  const float* k = (const float*)a.k + b * d.kv_sb + hk * d.kv_sh;
  const float* v = (const float*)a.v + b * d.kv_sb + hk * d.kv_sh;
  for (int e = c; e < D; e += 16) {
    Qs[r][e] = row_ok ? ((const float*)a.q)[qoff + e] : 0.f;
    Gs[r][e] = row_ok ? ((const float*)a.d_o)[qoff + e] : 0.f;
  }
  const long row = ((long)b * d.Hq + hq) * d.Sq + i;
  const float L = row_ok ? a.lse[row] : -INFINITY;
  const float delta = row_ok ? a.delta[row] : 0.f;
  float acc[D / 16];
#pragma unroll
  for (int e = 0; e < D / 16; ++e) acc[e] = 0.f;

  for (int j0 = 0; j0 < d.Skv; j0 += T) {
    __syncthreads();
    for (int e = tid; e < T * D; e += 256) {
      const int jj = e / D, dd = e % D;
      const bool ok = j0 + jj < d.Skv;
      Ks[jj][dd] = ok ? k[(long)(j0 + jj) * d.kv_ss + dd] : 0.f;
      Vs[jj][dd] = ok ? v[(long)(j0 + jj) * d.kv_ss + dd] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < T / 16; ++t) {
      const int jj = c + 16 * t, j = j0 + jj;
      float x = 0.f, g = 0.f;
      for (int e = 0; e < D; ++e) {
        x = fmaf(Qs[r][e], Ks[jj][e], x);
        g = fmaf(Gs[r][e], Vs[jj][e], g);
      }
      float ds = 0.f;
      if (row_ok && j < d.Skv && L != -INFINITY && visible(a.mask, b, i, j))
        ds = expf(x * d.scale - L) * (g - delta);
      Ss[r][jj] = ds;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < D / 16; ++e) {
      float x = acc[e];
      for (int jj = 0; jj < T; ++jj) x = fmaf(Ss[r][jj], Ks[jj][c + 16 * e], x);
      acc[e] = x;
    }
  }
  if (!row_ok) return;
  float* dq = a.dq_accum + row * D;
#pragma unroll
  for (int e = 0; e < D / 16; ++e) dq[c + 16 * e] += acc[e] * d.scale;   // rows are owned exclusively
}

// Backward, dK/dV part: workgroup owns R key rows of one (b, hkv); streams the query rows of
// every head in the group.
template <int D>
__global__ void __launch_bounds__(256) bwd_dkdv_f32_kernel(BwdArgs a) {
  __shared__ float Ks[R][D];
  __shared__ float Vs[R][D];
  __shared__ float Qs[T][D + 1];
  __shared__ float Gs[T][D + 1];
  __shared__ float Ps[R][T];
  __shared__ float Ss[R][T];
  __shared__ float Ls[T], Ds[T];
  const Dims& d = a.d;
  const int tid = threadIdx.x, r = tid / 16, c = tid % 16;
  const int b = blockIdx.z, hk = blockIdx.y, G = d.Hq / d.Hkv;
  const int j = blockIdx.x * R + r;
  const bool row_ok = j < d.Skv;
  const long koff = b * d.kv_sb + hk * d.kv_sh + (long)j * d.kv_ss;
  for (int e = c; e < D; e += 16) {
    Ks[r][e] = row_ok ? ((const float*)a.k)[koff + e] : 0.f;
    Vs[r][e] = row_ok ? ((const float*)a.v)[koff + e] : 0.f;
  }
  float dk[D / 16], dv[D / 16];
#pragma unroll
  for (int e = 0; e < D / 16; ++e) { dk[e] = 0.f; dv[e] = 0.f; }

  for (int hq = hk * G; hq < (hk + 1) * G; ++hq) {
    const float* q = (const float*)a.q + b * d.q_sb + hq * d.q_sh;
    const float* g = (const float*)a.d_o + b * d.q_sb + hq * d.q_sh;
    const long row0 = ((long)b * d.Hq + hq) * d.Sq;
    for (int i0 = 0; i0 < d.Sq; i0 += T) {
      __syncthreads();
      for (int e = tid; e < T * D; e += 256) {
        const int ii = e / D, dd = e % D;
        const bool ok = i0 + ii < d.Sq;
        Qs[ii][dd] = ok ? q[(long)(i0 + ii) * d.q_ss + dd] : 0.f;
        Gs[ii][dd] = ok ? g[(long)(i0 + ii) * d.q_ss + dd] : 0.f;
      }
      if (tid < T) {
        const bool ok = i0 + tid < d.Sq;
        Ls[tid] = ok ? a.lse[row0 + i0 + tid] : -INFINITY;
        Ds[tid] = ok ? a.delta[row0 + i0 + tid] : 0.f;
      }
      __syncthreads();
#pragma unroll
      for (int t = 0; t < T / 16; ++t) {
        const int ii = c + 16 * t, i = i0 + ii;
        float x = 0.f, gv = 0.f;
        for (int e = 0; e < D; ++e) {
          x = fmaf(Qs[ii][e], Ks[r][e], x);
          gv = fmaf(Gs[ii][e], Vs[r][e], gv);
        }
        float p = 0.f;
        if (row_ok && i < d.Sq && Ls[ii] != -INFINITY && visible(a.mask, b, i, j))
          p = expf(x * d.scale - Ls[ii]);
        Ps[r][ii] = p;
        Ss[r][ii] = p * (gv - Ds[ii]);
      }
      __syncthreads();
#pragma unroll
      for (int e = 0; e < D / 16; ++e) {
        float x = dv[e], y = dk[e];
        for (int ii = 0; ii < T; ++ii) {
          x = fmaf(Ps[r][ii], Gs[ii][c + 16 * e], x);
          y = fmaf(Ss[r][ii], Qs[ii][c + 16 * e], y);
        }
        dv[e] = x; dk[e] = y;
      }
    }
  }
  if (!row_ok) return;
#pragma unroll
  for (int e = 0; e < D / 16; ++e) {
    ((float*)a.dk)[koff + c + 16 * e] = dk[e] * d.scale;
    ((float*)a.dv)[koff + c + 16 * e] = dv[e];
  }
}

}  // namespace

hipError_t launch_fwd_f32(const FwdArgs& a, hipStream_t s) {
  dim3 grid((a.d.Sq + R - 1) / R, a.d.Hq, a.d.B);
  if (a.d.D == 64) fwd_f32_kernel<64><<<grid, 256, 0, s>>>(a);
  else if (a.d.D == 96) fwd_f32_kernel<96><<<grid, 256, 0, s>>>(a);
  else fwd_f32_kernel<128><<<grid, 256, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_bwd_f32(const BwdArgs& a, unsigned stages, hipStream_t s) {
  dim3 gq((a.d.Sq + R - 1) / R, a.d.Hq, a.d.B);
  dim3 gk((a.d.Skv + R - 1) / R, a.d.Hkv, a.d.B);
  if (a.d.D == 64) {
    if (stages & 4) bwd_dq_f32_kernel<64><<<gq, 256, 0, s>>>(a);
    if (stages & 2) bwd_dkdv_f32_kernel<64><<<gk, 256, 0, s>>>(a);
  } else if (a.d.D == 96) {
    if (stages & 4) bwd_dq_f32_kernel<96><<<gq, 256, 0, s>>>(a);
    if (stages & 2) bwd_dkdv_f32_kernel<96><<<gk, 256, 0, s>>>(a);
  } else {
    if (stages & 4) bwd_dq_f32_kernel<128><<<gq, 256, 0, s>>>(a);
    if (stages & 2) bwd_dkdv_f32_kernel<128><<<gk, 256, 0, s>>>(a);
  }
  return hipGetLastError();
}

}  // namespace lvx
