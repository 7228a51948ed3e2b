// Device helpers shared by the bf16 MFMA kernels (gfx950 only).
//
// Register layouts of v_mfma_f32_32x32x16_bf16 (wave64), lane l, g = l / 32:
//   A (32 x 16): row m = l % 32, k = 8 g + e, e = 0..7   (8 bf16 per lane)
//   B (16 x 32): col n = l % 32, k = 8 g + e
//   C (32 x 32): col n = l % 32, row m = 8 (v / 4) + 4 g + (v % 4), v = 0..15
// All kernels compute TRANSPOSED score tiles S^T = K Q^T, so that a lane holds one query column
// and 16 key rows per 32x32 block: the softmax statistics of a query are per-lane scalars, and
// the C registers, converted to bf16, already ARE the B operand of the next product over keys
// (k index = key), with key order  key = 16 t + 8 (e / 4) + 4 g + (e % 4)  for k-step t, slot e.
// The matching A operand (V^T or K^T) is fetched with the transposing LDS read, two per operand.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lvx {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

#define LVX_LDS(ptr, type) ((type __attribute__((address_space(3)))*)(ptr))

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.f;
  return z;
}

// Transposing LDS read.  Within each group of 16 lanes, lane j supplies the address of 4
// consecutive bf16; lane i receives element i of the 4 quads supplied by lanes 4r..4r+3 taken as
// row r, i.e. result[r] = row_r[i].  With lanes 4r..4r+3 pointing at 16 consecutive columns of
// row k0 + r of a row-major tile, lane i gets the column (k0..k0+3, n0 + i).
__device__ __forceinline__ s16x4 lds_read_tr(const void* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(uintptr_t)(p));
}

// A operand (32 rows n x 16 k) of a product over k taken from a ROW-MAJOR LDS tile X[k][n]
// (pitch in bytes): rows n0 + l%32, k slots e -> k = kbase + 8 (e / 4) + 4 g + (e % 4).
__device__ __forceinline__ bf16x8 load_tr_operand(const char* tile, int pitch_b, int kbase, int n0,
                                                  int lane) {
  const int j = lane & 15, half = (lane >> 4) & 1, g = lane >> 5;
  const char* p = tile + (kbase + 4 * g + (j >> 2)) * pitch_b + (n0 + 16 * half + 4 * (j & 3)) * 2;
  s16x4 lo = lds_read_tr(p);
  s16x4 hi = lds_read_tr(p + 8 * pitch_b);
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  s16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// Row-interleaved tile: up to 64 logical rows of D bf16 at pitch (D + 8) * 2 bytes, logical row r
// stored in physical row (r % 4) * 20 + r / 4.  With D = 128 (pitch 272 = 16 mod 256) BOTH access
// patterns of a tile are free of LDS bank conflicts and need no address arithmetic beyond an
// immediate offset: b128 reads of one 16-byte column by 16 consecutive logical rows land in 16
// distinct 16-byte bank groups, and a transposing read of 4 consecutive logical rows x 64 bytes
// lands in four disjoint 64-byte groups (20 * 272 = 64 mod 256).
constexpr int ILV_ROWS = 80;                       // physical rows of a 64-row interleaved tile
__device__ __forceinline__ int ilv_row(int r) { return (r & 3) * 20 + (r >> 2); }
// Byte offset of logical row (rc + rl), column col: rc is a compile-time multiple of 4 (so that it
// becomes an immediate offset), rl the lane-dependent part.
template <int D> __device__ __forceinline__ int ilv_off(int rl, int rc, int col) {
  return ilv_row(rl) * ((D + 8) * 2) + (rc >> 2) * ((D + 8) * 2) + col * 2;
}
// A operand via transposing reads from an interleaved tile (same contract as load_tr_operand;
// kbase is the first logical row, a multiple of 16).
template <int D>
__device__ __forceinline__ bf16x8 load_tr_operand_ilv(const char* tile, int kbase, int n0, int lane) {
  const int j = lane & 15, half = (lane >> 4) & 1, g = lane >> 5;
  const char* p = tile + ilv_off<D>(4 * g + (j >> 2), 0, 16 * half + 4 * (j & 3));   // lane part
  s16x4 lo = lds_read_tr(p + ilv_off<D>(0, kbase, n0));
  s16x4 hi = lds_read_tr(p + ilv_off<D>(0, kbase + 8, n0));
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  s16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// Direct global -> LDS copy of 16 bytes per lane (no staging registers): lane l's 16 bytes land at
// lds_dst + 16 l, where lds_dst must be wave-uniform.  Completion is tracked by vmcnt; the
// compiler does not order later LDS reads against it, so callers wait with wait_vmcnt<N>() and
// then cross a barrier before reading.
__device__ __forceinline__ void dma16(const void* gsrc, void* lds_dst) {
  __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)gsrc,
                                   (void __attribute__((address_space(3)))*)lds_dst, 16, 0, 0);
}
// The same copy written out as an instruction, with a wave-uniform 64-bit base and a 32-bit byte
// offset per lane (dma4s: 4 bytes per lane, landing at lds_dst + 4 l).  The compiler does not see
// a memory instruction here: it neither counts the copy in vmcnt nor lets it force the waits of
// unrelated LDS reads to zero, which it does for the builtin above while any copy is in flight.
// The caller orders everything by hand: wait_vmcnt<N>() + barrier before the data is read, a
// barrier before a stage is overwritten.  m0 (declared clobbered) carries the LDS address; one wait
// state separates its write from the copy.
__device__ __forceinline__ unsigned lds_addr_uniform(void* p) {
  // wave-uniform LDS byte address in a scalar register (a no-op when the compiler already keeps it there)
  return (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(uintptr_t)LVX_LDS(p, char));
}
__device__ __forceinline__ const void* ptr_uniform(const void* p) {
  // wave-uniform pointer in scalar registers (a no-op when the compiler already keeps it there)
  const unsigned long long x = (unsigned long long)(uintptr_t)p;
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)x);
  const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(x >> 32));
  return (const void*)(uintptr_t)(((unsigned long long)hi << 32) | lo);
}
// (the forms that take an LDS byte address save the null test that a cast from a generic pointer
// carries -- two scalar instructions per copy, which a kernel with one wave per SIMD pays for in
// issue slots; lds_base gives the address of the dynamic LDS array once per kernel)
__device__ __forceinline__ unsigned lds_base(void* smem) { return lds_addr_uniform(smem); }
__device__ __forceinline__ void dma16u(const void* base, unsigned voff, unsigned lds_addr) {
  base = ptr_uniform(base);
  const unsigned l = (unsigned)__builtin_amdgcn_readfirstlane((int)lds_addr);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(voff), "s"(base), "s"(l) : "memory", "m0");
}
__device__ __forceinline__ void dma4u(const void* base, unsigned voff, unsigned lds_addr) {
  base = ptr_uniform(base);
  const unsigned l = (unsigned)__builtin_amdgcn_readfirstlane((int)lds_addr);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
               :: "v"(voff), "s"(base), "s"(l) : "memory", "m0");
}
__device__ __forceinline__ void dma16s(const void* base, unsigned voff, void* lds_dst) {
  base = ptr_uniform(base);
  const unsigned l = lds_addr_uniform(lds_dst);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(voff), "s"(base), "s"(l) : "memory", "m0");
}
__device__ __forceinline__ void dma4s(const void* base, unsigned voff, void* lds_dst) {
  base = ptr_uniform(base);
  const unsigned l = lds_addr_uniform(lds_dst);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
               :: "v"(voff), "s"(base), "s"(l) : "memory", "m0");
}
// s_waitcnt vmcnt(N) only (expcnt and lgkmcnt left at "no wait").
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}
// Workgroup barrier without the memory fences of __syncthreads (which would drain vmcnt and so
// serialise the DMA pipeline).  LDS traffic of the calling wave must already be waited for.
__device__ __forceinline__ void wg_barrier() { __builtin_amdgcn_s_barrier(); }

// Two floats -> packed bf16 (round to nearest even), low half = a.
__device__ __forceinline__ unsigned pack2_bf16(float a, float b) {
  bf16x2 r;
  r[0] = (__bf16)a;
  r[1] = (__bf16)b;
  return __builtin_bit_cast(unsigned, r);
}

// 8 consecutive C registers (v0..v0+7) of one 32x32 block -> B operand of the next product.
__device__ __forceinline__ bf16x8 cvt_operand(const f32x16& c, int v0) {
  u32x4 r = {pack2_bf16(c[v0], c[v0 + 1]), pack2_bf16(c[v0 + 2], c[v0 + 3]),
             pack2_bf16(c[v0 + 4], c[v0 + 5]), pack2_bf16(c[v0 + 6], c[v0 + 7])};
  return __builtin_bit_cast(bf16x8, r);
}

// max / sum across the two half-waves (lanes l and l ^ 32 hold the same query column).
__device__ __forceinline__ float xhalf_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Media-mask classification of the rectangle query rows [i0, i1] x key rows [j0, j1]:
// 0 = nothing visible, 1 = everything visible, 2 = mixed.  Wave-uniform arguments.
__device__ __forceinline__ int mask_rect(const MaskDev& m, int b, int i0, int i1, int j0, int j1) {
  if (!m.allow) return 1;
  const uint8_t* base = m.allow + b * m.stride_b;
  bool any = false, all = true;
  for (int c = i0 / m.q_chunk; c <= i1 / m.q_chunk; ++c)
    for (int f = j0 / m.kv_block; f <= j1 / m.kv_block; ++f) {
      const bool on = base[(long)c * m.stride_q + f] != 0;
      any |= on;
      all &= on;
    }
  return all ? 1 : (any ? 2 : 0);
}

// mask_rect for rectangles that may span many chunks (planning: a workgroup's rows against one key
// tile, a different tile in every lane; the loops: a wave's rows when chunks are a few rows): the
// same probes and the same answer, the bitmap's rows taken eight at a time so that their round
// trips overlap when the bitmap is in global memory (the rows past the last chunk repeat the last
// one).
__device__ inline int mask_rect_tall(const MaskDev& m, int b, int i0, int i1, int j0, int j1) {
  if (!m.allow) return 1;
  const uint8_t* base = m.allow + b * m.stride_b;
  const int ca = i0 / m.q_chunk, cb = i1 / m.q_chunk;
  if (cb - ca < 4) return mask_rect(m, b, i0, i1, j0, j1);
  unsigned any = 0, all = 1;
  for (int f = j0 / m.kv_block; f <= j1 / m.kv_block; ++f)
    for (int c = ca; c <= cb; c += 8) {
      uint8_t v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = base[(long)min(c + u, cb) * m.stride_q + f];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        any |= v[u];
        all &= v[u] != 0 ? 1u : 0u;
      }
    }
  return all ? 1 : (any ? 2 : 0);
}

__device__ __forceinline__ bool mask_elem(const MaskDev& m, int b, int i, int j) {
  return m.allow[b * m.stride_b + (long)(i / m.q_chunk) * m.stride_q + (j / m.kv_block)] != 0;
}

// ---- media mask, staged for a workgroup -----------------------------------------------------
// Reading the bitmap from global memory costs a round trip per probe, and a workgroup probes it
// once per tile or step.  Two helpers take that off the critical path (every thread of the
// workgroup, nthreads of them, must call them; both end with a barrier):
//  * mask_to_lds copies the window [c0, c1] x [f0, f1] of batch b's bitmap into LDS when it fits
//    in `cap` bytes and returns a MaskDev that addresses the copy (mask_rect / mask_elem work
//    unchanged: the pointer is generic); otherwise it returns the mask as it is.
//  * build_bits evaluates pred(i), i in [0, n), with all threads at once and leaves bit i in the
//    word array bits[2 ..] (bits[0] = number of set bits); next_bit then finds the next set bit.
//  * class_of reads a three-way classification back from two such planes: the query-stationary
//    kernels keep one pair per wave, so that inside the loop the class of a (wave, tile) pair is
//    two LDS words away and only mixed tiles ever touch the bitmap.
__device__ inline MaskDev mask_to_lds(const MaskDev& m, int b, int c0, int c1, int f0, int f1,
                                      uint8_t* lds, int cap, int tid, int nthreads) {
  if (!m.allow) return m;
  const int w = f1 - f0 + 1, h = c1 - c0 + 1;
  if (w <= 0 || h <= 0 || (long)w * h > cap) return m;               // workgroup-uniform
  for (int i = tid; i < w * h; i += nthreads)
    lds[i] = m.allow[b * m.stride_b + (long)(c0 + i / w) * m.stride_q + f0 + i % w];
  __syncthreads();
  MaskDev r = m;
  r.allow = lds - ((long)c0 * w + f0);
  r.stride_b = 0;
  r.stride_q = w;
  return r;
}
template <typename Pred>
__device__ inline int build_bits(unsigned* bits, int n, int tid, int nthreads, Pred pred) {
  if (tid == 0) bits[0] = 0;
  __syncthreads();
  for (int base = 0; base < n; base += nthreads) {   // workgroup-uniform trip count
    const int i = base + tid;
    const bool on = i < n && pred(i);
    const unsigned long long m = __ballot(on);
    if ((tid & 63) == 0 && i < n) {
      *(unsigned long long*)(bits + 2 + i / 32) = m;
      atomicAdd(&bits[0], (unsigned)__popcll(m));
    }
  }
  __syncthreads();
  return __builtin_amdgcn_readfirstlane((int)bits[0]);
}
// Class of item i from two bit planes laid out like build_bits' (words from [2]): bit i of `any`
// = something visible, of `all` = everything visible.
__device__ inline int class_of(const unsigned* any, const unsigned* all, int i) {   // wave-uniform i
  const unsigned a = (unsigned)__builtin_amdgcn_readfirstlane((int)any[2 + (i >> 5)]) >> (i & 31);
  const unsigned l = (unsigned)__builtin_amdgcn_readfirstlane((int)all[2 + (i >> 5)]) >> (i & 31);
  return (l & 1) ? 1 : ((a & 1) ? 2 : 0);
}
constexpr __host__ __device__ int bit_plane_words(int n) { return 2 + ((n + 63) / 64) * 2; }   // words one plane of n bits takes
__device__ inline int next_bit(const unsigned* bits, int i, int n) {    // first set bit >= i, or n
  // (wave-uniform argument and result: the words are read through the vector path, so say so)
  while (i < n) {
    const unsigned w = (unsigned)__builtin_amdgcn_readfirstlane((int)bits[2 + (i >> 5)]) >> (i & 31);
    if (w) return __builtin_amdgcn_readfirstlane(min(n, i + __ffs(w) - 1));
    i = (i | 31) + 1;
  }
  return __builtin_amdgcn_readfirstlane(n);
}

__device__ inline int nth_bit(const unsigned* bits, int k, int n) {     // index of the k-th set bit (k >= 0), or n
  for (int w0 = 0; w0 < n; w0 += 32) {
    unsigned w = (unsigned)__builtin_amdgcn_readfirstlane((int)bits[2 + (w0 >> 5)]);
    const int c = __popc(w);
    if (k < c) {
      for (; k > 0; --k) w &= w - 1;
      return __builtin_amdgcn_readfirstlane(min(n, w0 + __ffs(w) - 1));
    }
    k -= c;
  }
  return __builtin_amdgcn_readfirstlane(n);
}

// XCD-aware decode of a 1-D grid.  Workgroup ids are dealt round-robin to the 8 XCDs, each with
// its own L2.  All work items that share a K/V head are placed on one XCD (or, when there are
// fewer heads than XCDs, a head is cut into equal parts) so that one HBM fetch of a K/V tile
// feeds every workgroup that needs it.  Returns false for padding workgroups.
struct HeadWork { int head; int item; };
__host__ __device__ inline int xcd_parts(int n_heads) {   // parts a head is cut into
  int g = n_heads % 8 == 0 ? 8 : (n_heads % 4 == 0 ? 4 : (n_heads % 2 == 0 ? 2 : 1));
  return 8 / g;
}
__host__ __device__ inline long xcd_grid(int n_heads, int items_per_head) {
  const int S = xcd_parts(n_heads);
  const int per_vh = (items_per_head + S - 1) / S;
  const long n_vh = (long)n_heads * S;                    // multiple of 8
  return n_vh * per_vh;
}
__device__ __forceinline__ bool xcd_decode(long pid, int n_heads, int items_per_head, HeadWork* w) {
  const int S = xcd_parts(n_heads);
  const int per_vh = (items_per_head + S - 1) / S;
  const int xcd = (int)(pid % 8);
  const long slot = pid / 8;
  const long vh = (slot / per_vh) * 8 + xcd;
  const int item = (int)(vh % S) * per_vh + (int)(slot % per_vh);
  w->head = (int)(vh / S);
  w->item = item;
  return item < items_per_head;
}

}  // namespace lvx
