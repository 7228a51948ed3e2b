// Projection kernels: the products of Section 2 that make the attention operands from the token
// features, Q = x W_Q and K, V = y W_K, y W_V, which Section 3.2 has the backward pass compute
// again from the single saved copy of the visual tokens instead of keeping K and V per layer.
//
// out[o][b, h, s, c] = sum_e x[b, s, e] * w[(o H + h) D + c, e]: x is [M = B S tokens, E], w holds
// the projection matrices transposed and stacked ([n_out H D, E], the layout of a linear layer's
// weight), and the result is written head-major, which is the layout the attention kernels read.
//
// bf16: one workgroup = 4 wavefronts (one per SIMD, the whole register file each) makes a
// 256-token x 256-column tile; a wave owns 128 x 128 of it as 4 x 4 blocks of 32 x 32 whose
// accumulators fill the accumulation registers, so each operand read from LDS feeds four matrix
// instructions.  The product is formed transposed (columns of w as the A operand, tokens as B):
// a lane then holds ONE token and, per block, groups of four consecutive columns.
// x and w tiles of 64 features travel HBM -> LDS by direct copies, whole 128-byte lines per row
// (half lines cost as many entries of the memory pipeline as whole ones and halve its
// throughput), into two slots of 64 KB that alternate; the copies of a tile pair go out while
// the pair before it is being multiplied, spread over the matrix instructions.  The eight
// 16-byte chunks of a tile row are stored permuted (perm_of) so that the rows a quarter-wave
// reads together cover all banks.  The one barrier per 64 matrix instructions sits before the
// last quarter of a tile pair, when its last operands are already in registers: behind it the
// first operands of the next pair are read and the slot is free for the pair after that.
// The epilogue turns the tile around in LDS (rounded to bf16) and writes whole 256-byte rows.
#include "lvx_internal.h"
#include "lvx_mfma.h"
#include "lvx_kv_ring.h"

#include <type_traits>

namespace lvx {

namespace {

constexpr int TM = 256, TN = 256;      // tokens x columns per workgroup
constexpr int BK = 64;                 // features per tile pair
constexpr int NSLOT = 2;               // LDS slots
constexpr int ROWB = BK * 2;           // bytes of a tile row: one 128-byte line
constexpr int TILE_B = 256 * ROWB;     // one operand's tile
constexpr int SLOT_B = 2 * TILE_B;     // x tile, then w tile
constexpr int RING_B = NSLOT * SLOT_B;
constexpr int TB_PITCH = 128 * 2 + 16; // epilogue: a wave's 128 tokens x 128 columns of bf16, padded rows
constexpr int TB_WAVE = 128 * TB_PITCH;
constexpr int SMEM_B = RING_B > 4 * TB_WAVE ? RING_B : 4 * TB_WAVE;
constexpr int NPART = 16;              // copies per wave and tile pair: 8 of x, 8 of w (8 rows each)

// Position permutation of a tile row's eight chunks: chunk c of row r sits at position
// c ^ perm_of(r).  Eight consecutive rows get eight different values, and two rows eight apart
// differ too, so the 16-byte reads of 8 or of 16 consecutive rows at one chunk never meet in a
// bank (rows are 128 bytes apart).
__device__ __forceinline__ int perm_of(int r) { return (r & 7) ^ ((r >> 3) & 1); }

__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
project_bf16_kernel(ProjArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int n_mt = (int)((a.M + TM - 1) / TM), n_nt = a.N / TN;
  HeadWork hw;                                       // the column tiles of a token tile share an XCD (and its L2)
  if (!xcd_decode(blockIdx.x, n_mt, n_nt, &hw)) return;
  const long m0 = (long)hw.head * TM;
  const int n0 = hw.item * TN;
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, l31 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;           // this wave's 128 tokens / 128 columns of the tile
  const int nk = a.E / BK;

  // ---- copies: one instruction moves 8 rows x 128 bytes; lane l fills slot l of them, i.e. row
  // l / 8, position l % 8, which holds chunk (l % 8) ^ perm_of(row).  A wave copies rows
  // 64 wave + 8 j + l / 8 of both tiles, j = 0 .. 7.  Rows past the last token re-read the last
  // one (their results are never stored).
  const unsigned xrow_b = (unsigned)(a.ldx * 2), wrow_b = (unsigned)(a.E * 2);
  const long m_last = a.M - 1 - m0;
  unsigned xo[8], wo[2];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int r = 64 * wave + 8 * j + (lane >> 3);
    const unsigned swz = 16u * (unsigned)((lane & 7) ^ perm_of(8 * j + (lane >> 3)));
    xo[j] = (unsigned)(r < m_last ? r : (int)m_last) * xrow_b + swz;
    if (j < 2) wo[j] = (unsigned)(lane >> 3) * wrow_b + swz;      // (the permutation repeats every 16 rows)
  }
  const char* const xg = (const char*)a.x + m0 * (long)xrow_b;
  const char* const wg = (const char*)a.w + ((long)n0 + 64 * wave) * wrow_b;
  auto issue_part = [&](int kt, int part) __attribute__((always_inline)) {
    char* const st = smem + (kt % NSLOT) * SLOT_B;
    const int j = part & 7;
    char* const dst = st + (part >> 3) * TILE_B + (64 * wave + 8 * j) * ROWB;
    if (part < 8) dma16s(xg + (long)kt * ROWB, xo[j], dst);
    else dma16s(wg + (long)(8 * j) * wrow_b + (long)kt * ROWB, wo[j & 1], dst);
  };

  // ---- operands: block i of this wave's tokens / block j of its columns, k-step q = 0 .. 3 of a
  // tile pair.  Lane l reads row l % 32, chunk 2 q + g, at position chunk ^ perm_of(row).
  int rd[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) rd[q] = l31 * ROWB + 16 * ((2 * q + g) ^ perm_of(l31));
  const int xbase = wm * 128 * ROWB, wbase = TILE_B + wn * 128 * ROWB;
  auto x_op = [&](const char* st, int q, int i) __attribute__((always_inline)) -> bf16x8 {
    return *(const bf16x8*)(st + xbase + 32 * i * ROWB + rd[q]);
  };
  auto w_op = [&](const char* st, int q, int j) __attribute__((always_inline)) -> bf16x8 {
    return *(const bf16x8*)(st + wbase + 32 * j * ROWB + rd[q]);
  };

  f32x16 acc[4][4];                                  // [column block j][token block i], transposed blocks
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i) { acc[j][i] = zero16(); asm volatile("" : "+a"(acc[j][i])); }

  // 16 matrix instructions of one k-step; hook(u) is other work issued after instruction u
  auto mma16 = [&](const bf16x8 (&xv)[4], const bf16x8 (&wv)[4], auto&& hook) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        kvring::mfma_acc(acc[j][i], wv[j], xv[i]);
        hook(4 * j + i);
        __builtin_amdgcn_sched_barrier(0);
      }
  };

  // ---- pipeline: pairs 0 and 1 go out whole; later, pair P + 2 goes out in two batches, the
  // first during the last k-step of pair P (right behind the barrier that frees its slot), the
  // second during the first k-step of pair P + 1
#pragma unroll
  for (int q = 0; q < NSLOT; ++q)
    if (q < nk) {
#pragma unroll
      for (int part = 0; part < NPART; ++part) issue_part(q, part);
    }
  if (nk > 1) wait_vmcnt<NPART>();
  else wait_vmcnt<0>();
  wg_barrier();
  bf16x8 xa[4], wa[4], xb[4], wb[4];                 // operands of even / odd k-steps
#pragma unroll
  for (int i = 0; i < 4; ++i) { xa[i] = x_op(smem, 0, i); wa[i] = w_op(smem, 0, i); }

  // fetches the operands of k-step q of the pair in slot st, one per matrix instruction
  auto fetch = [&](const char* st, int q, int u, bf16x8 (&xv)[4], bf16x8 (&wv)[4]) __attribute__((always_inline)) {
    if (u < 4) xv[u] = x_op(st, q, u);
    else if (u < 8) wv[u - 4] = w_op(st, q, u - 4);
  };
  auto pair = [&](int P, auto steady, bool send2, bool send1, bool more) __attribute__((always_inline)) {
    constexpr bool STEADY = decltype(steady)::value;   // send2, send1 and more are all true
    const char* const st = smem + (P % NSLOT) * SLOT_B;
    const char* const sn = smem + ((P + 1) % NSLOT) * SLOT_B;
    mma16(xa, wa, [&](int u) __attribute__((always_inline)) {
      fetch(st, 1, u, xb, wb);
      if ((STEADY || send2) && u % 2 == 1) issue_part(P + 1, 8 + u / 2);
    });
    mma16(xb, wb, [&](int u) __attribute__((always_inline)) { fetch(st, 2, u, xa, wa); });
    mma16(xa, wa, [&](int u) __attribute__((always_inline)) { fetch(st, 3, u, xb, wb); });
    // Pair P + 1 has landed when none of this wave's copies is outstanding, and this wave's last
    // reads of pair P have returned; behind the barrier that holds for every wave: pair P + 1 can
    // be read, and the slot of pair P be overwritten.
    if (STEADY || more) {
      __builtin_amdgcn_s_waitcnt(0x0070);              // vmcnt(0) and lgkmcnt(0)
      wg_barrier();
    }
    mma16(xb, wb, [&](int u) __attribute__((always_inline)) {
      if (STEADY || more) fetch(sn, 0, u, xa, wa);
      if ((STEADY || send1) && u % 2 == 1) issue_part(P + 2, u / 2);
    });
  };
  int P = 0;
  if (nk > 0) { pair(0, std::false_type{}, false, 2 < nk, 1 < nk); P = 1; }
  for (; P + 2 < nk; ++P) pair(P, std::true_type{}, true, true, true);
  for (; P < nk; ++P) pair(P, std::false_type{}, P + 1 < nk, false, P + 1 < nk);

  // ---- epilogue.  Every wave has left the ring (its slots become the turn-around buffers) and
  // the last matrix instructions have retired before their registers are read.
  wg_barrier();
#pragma unroll
  for (int j = 0; j < 4; ++j)
    asm volatile("s_nop 15\n\ts_nop 15" : "+a"(acc[j][0]), "+a"(acc[j][1]), "+a"(acc[j][2]), "+a"(acc[j][3]));
  char* const tb = smem + wave * TB_WAVE;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {                  // registers 4 q .. 4 q + 3: columns 32 j + 8 q + 4 g + (0..3)
        const u32x2 y = {pack2_bf16(acc[j][i][4 * q], acc[j][i][4 * q + 1]),
                         pack2_bf16(acc[j][i][4 * q + 2], acc[j][i][4 * q + 3])};
        *(u32x2*)(tb + (32 * i + l31) * TB_PITCH + (32 * j + 8 * q + 4 * g) * 2) = y;
      }
  // (the buffer is this wave's own: its reads below are ordered after its writes by the compiler)
  const int nw = n0 + wn * 128;                      // first column of this wave, all in one output
  const int HD = a.H * a.D;
  uint16_t* const out = (uint16_t*)a.out[nw / HD];
  const int nn = nw % HD;
#pragma unroll 4
  for (int it = 0; it < 32; ++it) {
    const int row = 4 * it + (lane >> 4), ch = lane & 15;
    const long m = m0 + wm * 128 + row;
    const u32x4 y = *(const u32x4*)(tb + row * TB_PITCH + ch * 16);
    if (m < a.M) {
      const int col = nn + 8 * ch;
      const long b = m / a.S, s = m % a.S;
      *(u32x4*)(out + ((b * a.H + col / a.D) * a.S + s) * a.D + col % a.D) = y;
    }
  }
}

// float32 tensors: one thread per output element, plain FMA in the order of the definition
__global__ void __launch_bounds__(256) project_f32_kernel(ProjArgs a) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= a.M * a.N) return;
  const long m = idx / a.N;
  const int n = (int)(idx % a.N);
  const float* xr = (const float*)a.x + m * a.ldx;
  const float* wr = (const float*)a.w + (long)n * a.E;
  float acc = 0.f;
  for (int e = 0; e < a.E; ++e) acc = fmaf(xr[e], wr[e], acc);
  const int HD = a.H * a.D, nn = n % HD;
  const long b = m / a.S, s = m % a.S;
  ((float*)a.out[n / HD])[((b * a.H + nn / a.D) * a.S + s) * a.D + nn % a.D] = acc;
}

}  // namespace

bool project_bf16_supported(const ProjArgs& a) {
  return a.E % BK == 0 && a.N % TN == 0 && (a.H * a.D) % 128 == 0 && a.D % 8 == 0;
}

hipError_t launch_project(const ProjArgs& a, int is_f32, hipStream_t s) {
  if (is_f32) {
    const long n = a.M * a.N;
    project_f32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(a);
    return hipGetLastError();
  }
  static SmemOnce once;
  const hipError_t e = ensure_dynamic_lds((const void*)project_bf16_kernel, SMEM_B, &once);
  if (e != hipSuccess) return e;
  const long grid = xcd_grid((int)((a.M + TM - 1) / TM), a.N / TN);
  project_bf16_kernel<<<(unsigned)grid, 256, SMEM_B, s>>>(a);
  return hipGetLastError();
}

}  // namespace lvx
