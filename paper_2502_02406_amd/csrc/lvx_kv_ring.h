// Shared by the query-stationary kernels (forward, and the dQ kernel of the backward): a workgroup
// of four wavefronts, one per SIMD, each owning 64 query rows (two 32-row blocks), and a ring of
// K/V tiles of 64 keys in LDS.
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

}  // namespace kvring
}  // namespace lvx
