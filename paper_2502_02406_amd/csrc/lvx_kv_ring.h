// Shared by the query-stationary kernels (dense forward, and the dQ kernel of the backward): a
// workgroup of four wavefronts, one per SIMD, each owning 64 query rows (two 32-row blocks), and a
// ring of K/V tiles of 64 keys in LDS.  The mask planner at the end serves the dQ kernel.
#pragma once
#include "lvx_mfma.h"

namespace lvx {
namespace kvring {

constexpr float LOG2E = 1.4426950408889634f;
constexpr int QB = 2;                  // 32-row query blocks per wave
constexpr int NWV = 4;                 // waves per workgroup
constexpr int QM = NWV * 32 * QB;      // query rows per workgroup
constexpr int TN = 64;                 // keys per tile (two halves of 32)
constexpr int NSTG = 4;                // ring stages

// LDS tile of 64 rows x D bf16, rows interleaved: logical row r lives in group r % 4 at row r / 4;
// a group is 16 rows of pitch (D + 8) * 2 bytes plus 64 bytes, which puts the four groups 64 bytes
// apart modulo 256.  Both access patterns are then free of bank conflicts: b128 reads of one
// column chunk by 16 consecutive logical rows, and transposing reads of 4 consecutive logical
// rows x 64 bytes.
template <int D> struct KvSmem {
  static constexpr int CPR = D / 8;                 // 16-byte chunks of data per row
  static constexpr int P = (D + 8) * 2;             // row pitch in bytes
  static constexpr int SPR = P / 16;                // 16-byte slots per row
  static constexpr int GS = 16 * P + 64;            // group stride in bytes
  static constexpr int TILE = 4 * GS;
  static constexpr int STAGE = 2 * TILE;            // K tile, then V tile
  static constexpr int RING = NSTG * STAGE;
  static constexpr int BITS_BYTES = 4096;           // visibility bits of up to 32704 tiles (media mask only)
  static constexpr int WIN_BYTES = 16384;           // window of the mask bitmap (media mask only)
  static constexpr int TOTAL = RING + BITS_BYTES + WIN_BYTES;
  static constexpr int RUN = 16 * SPR;              // slots of one group (contiguous)
  static constexpr int NCR = (RUN + 63) / 64;       // wave-level copies (64 slots) per group
  static_assert(GS % 256 == 64, "groups must sit 64 bytes apart modulo 256");
};
// byte offset of logical row rl + rc (rc a compile-time multiple of 4), byte column colb
template <int D> __device__ __forceinline__ int tile_off(int rl, int rc, int colb) {
  return (rl & 3) * KvSmem<D>::GS + ((rl >> 2) + (rc >> 2)) * KvSmem<D>::P + colb;
}
// A operand (32 rows n x 16 k) of a product over k from the row-major logical tile X[k][n]:
// rows n0 + l % 32, k slots e -> logical row kbase + 8 (e / 4) + 4 g + (e % 4)
template <int D>
__device__ __forceinline__ bf16x8 tile_tr_operand(const char* tile, int kbase, int n0, int lane) {
  const int j = lane & 15, half = (lane >> 4) & 1, g = lane >> 5;
  const char* p = tile + tile_off<D>(4 * g + (j >> 2), 0, (16 * half + 4 * (j & 3)) * 2);
  s16x4 lo = lds_read_tr(p + tile_off<D>(0, kbase, n0 * 2));
  s16x4 hi = lds_read_tr(p + tile_off<D>(0, kbase + 8, n0 * 2));
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  s16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// Matrix instructions written out, so that the operand files are fixed by construction: the
// stationary B operands (Q, dO) and the dQ accumulators sit in the accumulation registers, scores
// in ordinary registers where the vector ALU reads them.  The compiler does not know these are
// matrix instructions; the distances it would otherwise enforce between a matrix result and its
// first reader are kept by the order of the code (a result is read at least two matrix
// instructions and a wait after it was issued).
__device__ __forceinline__ void mfma_first(f32x16& c, bf16x8 a, bf16x8 b_acc) {     // c = a b
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(c) : "v"(a), "a"(b_acc));
}
__device__ __forceinline__ void mfma_from(f32x16& c, bf16x8 a, bf16x8 b_acc, const f32x16& c0) {   // c = a b + c0
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(c) : "v"(a), "a"(b_acc), "v"(c0));
}
__device__ __forceinline__ void mfma_next(f32x16& c, bf16x8 a, bf16x8 b_acc) {      // c += a b
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "a"(b_acc));
}
__device__ __forceinline__ void mfma_acc(f32x16& c_acc, bf16x8 a, bf16x8 b) {       // c += a b, c in acc regs
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c_acc) : "v"(a), "v"(b));
}

// Media mask, analysed once per workgroup (all 256 threads call this; it ends with a barrier).
// The window of the bitmap that the workgroup's rows can touch -- chunks c0 .. c0 + h - 1, every
// key block -- is copied to LDS; from it one word per key block is made (bit c: chunk c0 + c sees
// the block), and from those words, for every key tile, nine bits: visible to the workgroup at
// all, and for each wave whether its rows see something / everything of the tile.  They are left
// as bit planes of bit_plane_words(n_tiles) words each from `bits` on: plane 0 the workgroup's
// (bits[0] = number of visible tiles), planes 1 + 2 w and 2 + 2 w wave w's `any` and `all`.
// Every read of the window and of the words is an LDS read; nothing here goes through the generic
// pointer of MaskDev, whose every probe costs a round trip of the flat path.
// Returns false, having done nothing, when the shapes do not fit (more than 32 chunks per
// workgroup, window and words beyond win_cap bytes, planes beyond bits_cap bytes: the test is
// plan_fits below, which the host can evaluate too); on success *mk
// addresses the LDS copy of the window and *seen_out the per-block words, which is what the loop
// probes for mixed tiles: (seen[j / kv_block] >> (i / q_chunk - c0)) & 1 says whether row i sees key j.
// (h: chunks the rows of a workgroup can touch, w: key blocks, n_tiles: key tiles)
__host__ __device__ inline bool plan_fits(int h, int w, int n_tiles, int bits_cap, int win_cap) {
  return h <= 32 && (long)h * w + 4L * w + 4 <= win_cap && (1 + 2 * NWV) * bit_plane_words(n_tiles) * 4 <= bits_cap;
}
template <int D>
__device__ inline bool plan_masked_tiles(const MaskDev& m, int b, int i_wg0, int i_wg1, int Sq, int Skv,
                                         int n_tiles, unsigned* bits, int bits_cap, uint8_t* win,
                                         int win_cap, int tid, MaskDev* mk, const unsigned** seen_out,
                                         bool skip_full = false) {
  const int c0 = i_wg0 / m.q_chunk, h = i_wg1 / m.q_chunk - c0 + 1;
  const int w = (Skv - 1) / m.kv_block + 1;
  const int pw = bit_plane_words(n_tiles);
  const int win_bytes = (h * w + 3) & ~3;
  if (!plan_fits(h, w, n_tiles, bits_cap, win_cap)) return false;
  for (int i = tid; i < w * h; i += 256)
    win[i] = m.allow[b * m.stride_b + (long)(c0 + i / w) * m.stride_q + i % w];
  if (tid == 0) bits[0] = 0;
  __syncthreads();
  unsigned* const seen = (unsigned*)(win + win_bytes);     // seen[f]: bit c = chunk c0 + c sees block f
  for (int f = tid; f < w; f += 256) {
    unsigned x = 0;
    for (int c = 0; c < h; ++c) x |= (win[c * w + f] != 0 ? 1u : 0u) << c;
    seen[f] = x;
  }
  __syncthreads();
  unsigned wmask[NWV];                                       // chunk bits of each wave's rows (0: no rows)
#pragma unroll
  for (int wv = 0; wv < NWV; ++wv) {
    const int r0 = i_wg0 + 32 * QB * wv, r1 = min(Sq, r0 + 32 * QB) - 1;
    wmask[wv] = 0;
    if (r0 <= r1) {
      const int a = r0 / m.q_chunk - c0, z = r1 / m.q_chunk - c0;           // 0 <= a <= z < h <= 32
      wmask[wv] = (z - a == 31 ? ~0u : ((1u << (z - a + 1)) - 1u)) << a;
    }
  }
  const unsigned wgm = wmask[0] | wmask[1] | wmask[2] | wmask[3];
  static_assert(NWV == 4, "wgm above names the four waves");
  for (int base = 0; base < n_tiles; base += 256) {          // workgroup-uniform trip count
    const int t = base + tid;
    unsigned any = 0, all = ~0u;
    if (t < n_tiles) {
      const int fa = (t * TN) / m.kv_block, fb = (min(Skv, t * TN + TN) - 1) / m.kv_block;
      for (int f = fa; f <= fb; ++f) { any |= seen[f]; all &= seen[f]; }
    } else {
      all = 0;
    }
    // (skip_full: tiles that every row of the workgroup sees are left to another pass)
    const unsigned long long vis = __ballot(any != 0 && !(skip_full && (all & wgm) == wgm));
    unsigned long long wa[NWV], wl[NWV];
#pragma unroll
    for (int wv = 0; wv < NWV; ++wv) {
      wa[wv] = __ballot((any & wmask[wv]) != 0);
      wl[wv] = __ballot(wmask[wv] != 0 && (all & wmask[wv]) == wmask[wv]);
    }
    if ((tid & 63) == 0 && t < n_tiles) {              // (a wave wholly past the end has no words in the planes)
      *(unsigned long long*)(bits + 2 + t / 32) = vis;
      atomicAdd(&bits[0], (unsigned)__popcll(vis));
#pragma unroll
      for (int wv = 0; wv < NWV; ++wv) {
        *(unsigned long long*)(bits + (1 + 2 * wv) * pw + 2 + t / 32) = wa[wv];
        *(unsigned long long*)(bits + (2 + 2 * wv) * pw + 2 + t / 32) = wl[wv];
      }
    }
  }
  __syncthreads();
  *seen_out = seen;
  *mk = m;
  mk->allow = win - ((long)c0 * w);
  mk->stride_b = 0;
  mk->stride_q = w;
  return true;
}

}  // namespace kvring
}  // namespace lvx
