// Gradients of the projections: the chain rule through the linear maps of Section 2 that Section
// 3.2 has the backward pass evaluate again.  With g[o] = d loss / d out[o], head-major like out,
//     dx[b, s, e]            = sum_{o, h, c} g[o][b, h, s, c] * w[(o H + h) D + c, e]
//     dw[(o H + h) D + c, e] += sum_{b, s}   g[o][b, h, s, c] * x[b, s, e]
// dx is rounded once to the tensors' type; dw is float32 and ACCUMULATED, because the weights of
// K and V meet one gradient per K/V block and those add up.
//
// bf16: both products run on the matrix cores with the tiling of the forward projection: one
// workgroup = 4 wavefronts (one per SIMD) makes a 256 x 256 tile of the result, a wave owns
// 128 x 128 of it as 4 x 4 blocks of 32 x 32 in the accumulation registers, tile pairs of 64
// contraction steps travel HBM -> LDS by direct copies into two 64 KB slots that alternate.
// What differs is where the contraction index lies in memory:
//   dx = G W    contraction over the columns n of the projection.  G is read like x in the
//               forward (rows = tokens, the 64 columns of a step contiguous: a 128-byte line
//               inside one head); W has n along its ROWS, so its tile is kept as [n][e] and
//               its operand taken with the transposing LDS read.
//   dw = G^T X  contraction over the tokens.  Both G ([token][n]) and x ([token][e]) have the
//               contraction index along their rows: both tiles are [token][256 columns] and both
//               operands come from transposing reads.
// A [k][256] tile has rows of 512 bytes; chunk c (16 bytes) of row r sits at position
// c ^ 4 (r % 4): the four rows that a transposing read of 16 lanes touches then lie in four
// different 64-byte bank groups.  A transposing read hands a lane four contraction steps, the
// four rows its group of 16 lanes points at; a lane's two reads per operand take rows 4 g .. 4 g + 3
// and 8 + 4 g .. in dw (g = lane / 32), and rows 8 g .. 8 g + 7 in dx, whose G operand then is one
// plain 16-byte read of the same eight steps.
// Rows past the last token are never stored (dx) and are cleared in LDS before they are
// multiplied (dw, where they would otherwise enter every sum).
// dw of a narrow projection (K and V of a model with few K/V heads) has fewer 256 x 256 tiles
// than the chip has compute units.  Its token range is then cut into parts, one workgroup per
// (tile, part), and the parts of a tile add their sums to dw ONE AFTER THE OTHER in the order of
// their numbers: a turn word per tile says whose turn it is, the data travels with agent-scope
// loads and stores (the L2 caches of the XCDs are not coherent with each other), and the last part
// sets the word back to zero.  The order is fixed, so results repeat bit for bit; a part only ever
// waits for a workgroup with a lower number, which was started before it, so the waits end (they
// are bounded all the same).  Calls that overlap in time on one GPU would share the turn words and
// must not be made.  (Without that, tiles 128 rows high: a wave owns 64 x 128, the G tile is
// [token][128 columns] with rows of 256 bytes, same permutation.)
#include "lvx_internal.h"
#include "lvx_mfma.h"
#include "lvx_kv_ring.h"

#include <type_traits>

namespace lvx {

namespace {

constexpr int T = 256;                 // edge of a workgroup's tile of the result
constexpr int BK = 64;                 // contraction steps per tile pair
constexpr int NSLOT = 2;
constexpr int KR_ROWB = T * 2;         // [k][256] tile: bytes of a row
constexpr int RK_ROWB = BK * 2;        // [256][k] tile: bytes of a row (one 128-byte line)
constexpr int TILE_B = BK * KR_ROWB;   // either kind: 32 KB
static_assert(TILE_B == T * RK_ROWB, "both tile kinds take the same room");
constexpr int SLOT_B = 2 * TILE_B;     // A-side tile ([k][256 columns e]), then B-side tile (up to as large)
constexpr int RING_B = NSLOT * SLOT_B;
// Measurement builds only (python -m paper_2502_02406_amd.build --define LVX_PROJ_PROBE=1; results
// are wrong): the dw kernel copies the first four tile pairs of its tokens over and over, so every
// copy after the first finds its lines in the nearest cache -- what is left is the kernel's own pace.
#ifdef LVX_PROJ_PROBE
#define PROBE_PAIR(p) ((p) & 3)
#else
#define PROBE_PAIR(p) (p)
#endif
constexpr int MAX_TURNS = 512;         // tiles of dw that can take turns (8 turn words each)
constexpr int SPIN_LIMIT = 1 << 22;    // tries (with a short sleep each) before a part stops waiting for its turn
constexpr int TB_PITCH = 128 * 2 + 16; // dx epilogue: a wave's 128 tokens x 128 columns of bf16, padded rows
constexpr int TB_WAVE = 128 * TB_PITCH;
constexpr int SMEM_B = RING_B > 4 * TB_WAVE ? RING_B : 4 * TB_WAVE;

__device__ __forceinline__ int perm_of(int r) { return (r & 7) ^ ((r >> 3) & 1); }

// whose turn it is to add to tile t of dw (0 between launches)
__device__ int dw_turn[MAX_TURNS * 8];
typedef int __attribute__((address_space(1))) gint;

// floor(m / S) and the remainder for 0 <= m < 2^24 (exact: the float quotient is off by at most one)
__device__ __forceinline__ void div_tokens(int m, int S, float inv_S, int* b, int* s) {
  // (without branches: this runs between the matrix instructions of the dw kernel's loop, which
  // a conditional would cut into pieces)
  const int q = (int)((float)m * inv_S);
  const int r = m - q * S;
  const int fix = (r >= S ? 1 : 0) - (r < 0 ? 1 : 0);
  *b = q + fix;
  *s = r - fix * S;
}

// MODE 0: dx = G W (rows = tokens, columns = features e, contraction over n)
// MODE 1: dw += G^T X (rows = columns n of the projection, columns = e, contraction over tokens)
// RB: 32-row blocks of the result per wave (4: tiles of 256 rows; 2: of 128 rows, MODE 1 only)
// GA (MODE 0): heads are multiples of 64 wide, so that a tile pair's 64 columns of G are one line
template <int MODE, int RB, bool GA = true>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
project_bwd_bf16_kernel(ProjBwdArgs a) {
  static_assert(RB == 4 || (RB == 2 && MODE == 1), "tile heights");
  constexpr int TR = 64 * RB;                        // rows of a workgroup's tile
  constexpr int BROWB = TR * 2;                      // MODE 1: bytes of a row of the G tile [k][TR]
  constexpr int RPI = 1024 / BROWB;                  // ... rows that one copy instruction moves (2 or 4)
  constexpr int NB = MODE == 0 ? 8 : 16 / RPI;       // copies per wave and tile pair: B side,
  constexpr int NPART = 8 + NB;                      // and with the 8 of the A side
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int n_rt = MODE == 0 ? (int)((a.M + TR - 1) / TR) : a.N / TR;   // row tiles of the result
  const int n_ct = a.E / T;
  HeadWork hw;
  // (dw: workgroups part * dw_tiles_grid + i, i = 0 .. dw_tiles_grid - 1, are part `part` of the token range)
  const unsigned wg = MODE == 1 ? blockIdx.x % a.dw_tiles_grid : blockIdx.x;
  const int tpart = MODE == 1 ? (int)(blockIdx.x / a.dw_tiles_grid) : 0;
  if (MODE == 1 && n_rt % 2 == 0 && n_ct % 4 == 0) {
    // dw streams a [tokens][TR] panel of G per row tile and a [tokens][256] panel of x per column
    // tile, and each XCD has an L2 of its own: the XCDs (workgroup number mod 8) are laid out 2 x 4
    // over the tile grid, so that each reads half of G and a quarter of x instead of an eighth of
    // G and all of x.
    const int xcd = wg % 8, slot = wg / 8, pc = n_ct / 4;
    hw.head = (xcd / 4) * (n_rt / 2) + slot / pc;
    hw.item = (xcd % 4) * pc + slot % pc;
    if (hw.head >= ((xcd / 4) + 1) * (n_rt / 2)) return;
  } else if (!xcd_decode(wg, n_rt, n_ct, &hw)) {   // the column tiles of a row tile share an XCD
    return;
  }
  const long r0 = (long)hw.head * TR;                // first token (MODE 0) / first column n (MODE 1)
  const int e0 = hw.item * T;
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, l31 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;           // this wave's 128 rows / 128 columns of the tile
  // tile pairs: all of them (dx), or this part's share of the token range (dw): k0 .. k0 + nk - 1
  const int nk_all = MODE == 0 ? a.N / BK : (int)((a.M + BK - 1) / BK);
  const int k0 = MODE == 1 ? (int)((long)tpart * nk_all / a.dw_parts) : 0;
  const int nk = MODE == 1 ? (int)((long)(tpart + 1) * nk_all / a.dw_parts) - k0 : nk_all;
  const int HD = a.H * a.D;
  const float inv_S = 1.0f / (float)a.S;
  const long head_b = (long)a.S * a.D * 2;           // bytes of one head of one batch in g

  // ---- copies into a [k][256] tile: one instruction moves 2 rows x 512 bytes; lane l fills
  // position l % 32 of row l / 32, which holds chunk (l % 32) ^ 4 (row % 4).  A wave copies rows
  // 16 wave + 2 j + l / 32, j = 0 .. 7; (row % 4) = 2 (j % 2) + l / 32.
  const int lh = lane >> 5, pos = lane & 31;
  unsigned kr_chunk[2];                              // byte offset of the lane's chunk inside a row, j even / odd
#pragma unroll
  for (int par = 0; par < 2; ++par) kr_chunk[par] = 16u * (unsigned)(pos ^ (4 * ((2 * par + lh) & 3)));

  // MODE 0: rows of the G tile ([256 tokens][64 n], the forward's x layout): one instruction
  // moves 8 rows x 128 bytes; a wave copies rows 64 wave + 8 j + l / 8.  Tokens past the last
  // one re-read it (their results are never stored).
  unsigned g_row[8];
  // MODE 1: the G tile [64 tokens][TR columns]: one instruction moves RPI rows; lane l fills
  // position l % (64 / RPI) of row l / (64 / RPI); a wave copies rows 16 wave + RPI j + that.
  // g_col: the lane's column part of a G address, j even / odd (the columns of the tile lie in
  // one output)
  const int b_rin = lane / (64 / RPI), b_pos = lane % (64 / RPI);
  unsigned g_col[2];
  const char* g_tile_base = nullptr;                 // MODE 1: the output's gradient
  if (MODE == 0) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int r = 64 * wave + 8 * j + (lane >> 3);
      const long m = r0 + r < a.M ? r0 + r : a.M - 1;
      int b, s;
      div_tokens((int)m, a.S, inv_S, &b, &s);
      g_row[j] = (unsigned)(((long)b * a.H * a.S + s) * a.D * 2);
      // (heads that are multiples of 64 wide: the 64 columns of a tile pair are one 128-byte line,
      // and the lane's chunk of it is a fixed offset; otherwise see g_lane below)
      if (GA) g_row[j] += 16u * (unsigned)((lane & 7) ^ perm_of(8 * j + (lane >> 3)));
    }
  } else {
    const int o = (int)(r0 / HD), nn0 = (int)(r0 % HD);
    g_tile_base = (const char*)a.g[o];
#pragma unroll
    for (int par = 0; par < 2; ++par) {
      const int n = nn0 + 8 * (b_pos ^ (4 * ((RPI * par + b_rin) & 3)));
      g_col[par] = (unsigned)((long)(n / a.D) * head_b + (long)(n % a.D) * 2);
    }
  }
  const unsigned wrow_b = (unsigned)(a.E * 2), xrow_b = (unsigned)(a.ldx * 2);
  const unsigned smem_u = lds_base(smem);

  // MODE 0: the head and column that tile pair kt of G starts at, advanced pair by pair (the G
  // copies of the pairs are issued in ascending order, copy 8 of a pair first)
  int g_o = 0, g_h = 0, g_c = 0;
  const char* g_pair_base = nullptr;
  // ... and for heads that are no multiple of 64 wide (96): a tile pair's 64 columns may lie in two
  // heads, so each lane works out where ITS 8 columns are: chunk (l % 8) ^ (l / 8) ^ (j % 2) of
  // the pair, i.e. column g_c + 8 chunk of the output, in head / at column (that / D, that % D)
  unsigned g_lane0 = 0u, g_lane1 = 0u;               // (j even / odd)
  const float inv_D = 1.0f / (float)a.D;

  auto issue_part = [&](int kt, int part) __attribute__((always_inline)) {
    const unsigned st = smem_u + (unsigned)((kt % NSLOT) * SLOT_B);
    const int j = part & 7;
    if (part < 8) {                                  // A side: rows kt * 64 + 16 wave + 2 j + lh of w (MODE 0) or x (MODE 1)
      const unsigned dst = st + (unsigned)((16 * wave + 2 * j) * KR_ROWB);
      if (MODE == 0) {
        const char* base = (const char*)a.w + ((long)(kt * BK + 16 * wave + 2 * j) * a.E + e0) * 2;
        dma16u(base, (unsigned)lh * wrow_b + kr_chunk[j & 1], dst);
      } else {
        const long m_first = (long)PROBE_PAIR(k0 + kt) * BK;
        const int last = (int)(a.M - 1 - m_first);   // rows past it re-read it, and are cleared in LDS
        const int r = 16 * wave + 2 * j + lh;
        const char* base = (const char*)a.x + (m_first * a.ldx + e0) * 2;
        dma16u(base, (unsigned)(r < last ? r : last) * xrow_b + kr_chunk[j & 1], dst);
      }
    } else if (MODE == 0) {                          // B side: G, 256 tokens x 64 columns
      if (part == 8) {
        if constexpr (GA) {
          g_pair_base = (const char*)a.g[g_o] + (long)g_h * head_b + (long)g_c * 2;
          g_c += BK;
          if (g_c == a.D) { g_c = 0; if (++g_h == a.H) { g_h = 0; ++g_o; } }
        } else {                                     // g_c counts the columns of the output here
          g_pair_base = (const char*)a.g[g_o];
          int h, cc;
          div_tokens(g_c + 8 * ((lane & 7) ^ (lane >> 3)), a.D, inv_D, &h, &cc);
          g_lane0 = (unsigned)((long)h * head_b + (long)cc * 2);
          div_tokens(g_c + 8 * ((lane & 7) ^ (lane >> 3) ^ 1), a.D, inv_D, &h, &cc);
          g_lane1 = (unsigned)((long)h * head_b + (long)cc * 2);
          g_c += BK;
          if (g_c == HD) { g_c = 0; ++g_o; }
        }
      }
      dma16u(g_pair_base, g_row[j] + (GA ? 0u : (j & 1) ? g_lane1 : g_lane0),
             st + (unsigned)(TILE_B + (64 * wave + 8 * j) * RK_ROWB));
    } else {                                         // B side: G, 64 tokens x TR columns
      const int jb = part - 8;
      const long m_first = (long)PROBE_PAIR(k0 + kt) * BK;
      const int r = 16 * wave + RPI * jb + b_rin;
      const long m = m_first + r < a.M ? m_first + r : a.M - 1;
      int b, s;
      div_tokens((int)m, a.S, inv_S, &b, &s);
      const unsigned row = (unsigned)(((long)b * a.H * a.S + s) * a.D * 2);
      dma16u(g_tile_base, row + g_col[jb & 1], st + (unsigned)(TILE_B + (16 * wave + RPI * jb) * BROWB));
    }
  };

  // ---- operands.  From a [k][256] tile: block jj of the wave's 128 columns, k-step q (16 rows);
  // lane l supplies the address of 8 bytes of row KG g + (l % 16) / 4 (+ 16 q, + KH for the second
  // read), byte column 64 jj' + 32 ((l / 16) % 2) + 8 (l % 4), where jj' is the block's position
  // after the permutation: (4 wcol + jj) ^ (row % 4).  Which rows a lane asks for decides which
  // contraction steps it holds, and both operands must agree: dw (both from such tiles) takes steps
  // 4 g .. 4 g + 3 and 8 + 4 g .. 8 + 4 g + 3; dx takes 8 g .. 8 g + 7, the order in which its other
  // operand lies in ONE 16-byte chunk of a [256][64] tile (two 8-byte reads of half chunks, which
  // the other order needs, use half the banks and cost 9 % of the kernel's cycles in conflicts).
  const int j16 = lane & 15, jr = j16 >> 2;
  const int tr_col = 32 * ((lane >> 4) & 1) + 8 * (j16 & 3);
  int ka[4], kb[RB];
  constexpr int KG = MODE == 0 ? 8 : 4, KH = MODE == 0 ? 4 : 8;
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) ka[jj] = (KG * g + jr) * KR_ROWB + tr_col + 64 * ((4 * wn + jj) ^ jr);
#pragma unroll
  for (int i = 0; i < RB; ++i) kb[i] = TILE_B + (4 * g + jr) * BROWB + tr_col + 64 * ((RB * wm + i) ^ jr);
  auto tr_op = [&](const char* p, auto pitch) __attribute__((always_inline)) -> bf16x8 {
    const s16x4 lo = lds_read_tr(p), hi = lds_read_tr(p + KH * decltype(pitch)::value);
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    const s16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, r);
  };
  // From the [256][64] tile (MODE 0): row 32 i + l % 32 of the wave's tokens, k-step q: chunk
  // 2 q + g (steps 8 g .. 8 g + 7), which lies at position (2 q + g) ^ perm_of(row)
  int rk[4];
#pragma unroll
  for (int q = 0; q < 4; ++q)
    rk[q] = TILE_B + (wm * 128 + l31) * RK_ROWB + 16 * ((2 * q + g) ^ perm_of(l31));
  auto a_op = [&](const char* st, int q, int jj) __attribute__((always_inline)) -> bf16x8 {
    return tr_op(st + ka[jj] + 16 * q * KR_ROWB, std::integral_constant<int, KR_ROWB>{});
  };
  auto b_op = [&](const char* st, int q, int i) __attribute__((always_inline)) -> bf16x8 {
    if (MODE == 1) return tr_op(st + kb[i] + 16 * q * BROWB, std::integral_constant<int, BROWB>{});
    return __builtin_bit_cast(bf16x8, *(const u32x4*)(st + rk[q] + 32 * i * RK_ROWB));
  };

  f32x16 acc[4][RB];                                 // [column block jj][row block i]: lane = row, registers = columns
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < RB; ++i) { acc[j][i] = zero16(); asm volatile("" : "+a"(acc[j][i])); }

  // the 4 RB matrix instructions of one k-step; hook(u) is other work issued after instruction u
  constexpr int NU = 4 * RB;
  auto mma16 = [&](const bf16x8 (&bv)[RB], const bf16x8 (&av)[4], auto&& hook) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int i = 0; i < RB; ++i) {
        kvring::mfma_acc(acc[j][i], av[j], bv[i]);
        hook(RB * j + i);
        __builtin_amdgcn_sched_barrier(0);
      }
  };

  // dw: the rows of the last tile pair that lie past the last token are cleared, in both tiles,
  // once the pair has landed (every thread calls this behind the barrier that says so)
  const int tail_rows = (int)(a.M - (long)(nk_all - 1) * BK);  // rows of the last pair that exist
  auto settle = [&](int kt) __attribute__((always_inline)) {
    if (MODE == 1 && k0 + kt == nk_all - 1 && tail_rows < BK) {
      char* const st = smem + (kt % NSLOT) * SLOT_B;
      const u32x4 z = {0u, 0u, 0u, 0u};
      for (int c = tid; c < (BK - tail_rows) * (KR_ROWB / 16); c += 256)
        *(u32x4*)(st + tail_rows * KR_ROWB + c * 16) = z;
      for (int c = tid; c < (BK - tail_rows) * (BROWB / 16); c += 256)
        *(u32x4*)(st + TILE_B + tail_rows * BROWB + c * 16) = z;
      __builtin_amdgcn_s_waitcnt(0xc07f);            // lgkmcnt(0)
      wg_barrier();
    }
  };

  // ---- pipeline (the forward projection's): pairs 0 and 1 go out whole; later, pair P + 2 goes
  // out in two batches, the first during the last k-step of pair P (right behind the barrier
  // that frees its slot), the second during the first k-step of pair P + 1
#pragma unroll
  for (int q = 0; q < NSLOT; ++q)
    if (q < nk) {
#pragma unroll
      for (int part = 0; part < NPART; ++part) issue_part(q, part);
    }
  if (nk > 1) wait_vmcnt<NPART>();
  else wait_vmcnt<0>();
  wg_barrier();
  settle(0);
  bf16x8 ba[RB], aa[4], bb[RB], ab[4];               // operands of even / odd k-steps
#pragma unroll
  for (int i = 0; i < RB; ++i) ba[i] = b_op(smem, 0, i);
#pragma unroll
  for (int i = 0; i < 4; ++i) aa[i] = a_op(smem, 0, i);

  auto fetch = [&](const char* st, int q, int u, bf16x8 (&bv)[RB], bf16x8 (&av)[4]) __attribute__((always_inline)) {
    if (u < RB) bv[u] = b_op(st, q, u);
    else if (u < RB + 4) av[u - RB] = a_op(st, q, u - RB);
  };
  // the B-side copies of a pair go out during one k-step, the A-side copies during another: one
  // every NU / NB (NU / 8) matrix instructions
  constexpr int EB = NU / NB, EA = NU / 8;
  auto pair = [&](int P, auto steady, bool send2, bool send1, bool more) __attribute__((always_inline)) {
    constexpr bool STEADY = decltype(steady)::value;   // send2, send1 and more are all true
    const char* const st = smem + (P % NSLOT) * SLOT_B;
    const char* const sn = smem + ((P + 1) % NSLOT) * SLOT_B;
    mma16(ba, aa, [&](int u) __attribute__((always_inline)) {
      fetch(st, 1, u, bb, ab);
      if ((STEADY || send2) && u % EB == EB - 1) issue_part(P + 1, 8 + u / EB);
    });
    mma16(bb, ab, [&](int u) __attribute__((always_inline)) { fetch(st, 2, u, ba, aa); });
    mma16(ba, aa, [&](int u) __attribute__((always_inline)) { fetch(st, 3, u, bb, ab); });
    // Pair P + 1 has landed when none of this wave's copies is outstanding, and this wave's last
    // reads of pair P have returned; behind the barrier that holds for every wave.
    if (STEADY || more) {
      __builtin_amdgcn_s_waitcnt(0x0070);              // vmcnt(0) and lgkmcnt(0)
      wg_barrier();
      if constexpr (!STEADY) settle(P + 1);          // (a steady pair is never followed by the last one)
    }
    mma16(bb, ab, [&](int u) __attribute__((always_inline)) {
      if (STEADY || more) fetch(sn, 0, u, ba, aa);
      if ((STEADY || send1) && u % EA == EA - 1) issue_part(P + 2, u / EA);
    });
  };
  int P = 0;
  if (nk > 0) { pair(0, std::false_type{}, false, 2 < nk, 1 < nk); P = 1; }
  for (; P + 2 < nk; ++P) pair(P, std::true_type{}, true, true, true);
  for (; P < nk; ++P) pair(P, std::false_type{}, P + 1 < nk, false, P + 1 < nk);

  // ---- epilogue.  Every wave has left the ring and the last matrix instructions have retired
  // before their registers are read.
  wg_barrier();
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < RB; i += 2)
      asm volatile("s_nop 15\n\ts_nop 15" : "+a"(acc[j][i]), "+a"(acc[j][i + 1]));
  if constexpr (MODE == 0) {
    // turn the tile around in LDS (rounded to bf16) and write whole 256-byte row segments
    char* const tb = smem + wave * TB_WAVE;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {                // registers 4 q .. 4 q + 3: columns 32 j + 8 q + 4 g + (0..3)
          const u32x2 y = {pack2_bf16(acc[j][i][4 * q], acc[j][i][4 * q + 1]),
                           pack2_bf16(acc[j][i][4 * q + 2], acc[j][i][4 * q + 3])};
          *(u32x2*)(tb + (32 * i + l31) * TB_PITCH + (32 * j + 8 * q + 4 * g) * 2) = y;
        }
    uint16_t* const out = (uint16_t*)a.dx + e0 + wn * 128;
#pragma unroll 4
    for (int it = 0; it < 32; ++it) {
      const int row = 4 * it + (lane >> 4), ch = lane & 15;
      const long m = r0 + wm * 128 + row;
      const u32x4 y = *(const u32x4*)(tb + row * TB_PITCH + ch * 16);
      if (m < a.M) *(u32x4*)(out + m * a.ldx + 8 * ch) = y;
    }
  } else {
    if constexpr (RB != 4) {
      // (128-row tiles: never divided) this workgroup alone owns its tile of dw: add in place, 16
      // bytes per lane and register group, the sixteen old values of a row block read before the
      // first sum is stored (a store between two loads would make the second wait for the first)
      float* const out = a.dw + (r0 + wm * (32 * RB) + l31) * (long)a.E + e0 + wn * 128 + 4 * g;
#pragma unroll
      for (int i = 0; i < RB; ++i) {
        f32x4 v[4][4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) v[j][q] = *(const f32x4*)(out + (long)(32 * i) * a.E + 32 * j + 8 * q);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int t = 0; t < 4; ++t) v[j][q][t] += acc[j][i][4 * q + t];
            *(f32x4*)(out + (long)(32 * i) * a.E + 32 * j + 8 * q) = v[j][q];
          }
      }
    } else {
      // A tile whose tokens are divided (dw_parts > 1): the parts take turns, in the order of their
      // numbers; an undivided tile goes the same way without the waiting.  Every wave owns a quarter
      // of the tile and passes it on in two halves of 64 rows, each with a turn word of its own,
      // so a part starts on a half as soon as the part before it has left that half.  A half is
      // turned through LDS (64 rows x 128 floats per wave, 16-byte chunks permuted by the row)
      // so that every load and store covers two whole 512-byte row segments, and the old values
      // come in sixteen rows at a time: a turn costs a few trips to memory, not one per register.
      int* const turn = dw_turn + (a.dw_parts > 1 ? ((hw.head * n_ct + hw.item) * 4 + wave) * 2 : 0);
      float* const tb = (float*)(smem + wave * 32768);
      constexpr int AGENT = 16;                      // cache policy sc1: the L2s of different XCDs do not see each other's lines
      const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
          (char*)(a.dw + r0 * (long)a.E + e0), 0, (int)(((long)TR * a.E - e0) * 4), 0x00020000);
      const int rrow = lane >> 5, rch = lane & 31;
      const int two_rows = __builtin_amdgcn_readfirstlane(2 * a.E * 4);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
          for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const f32x4 v = {acc[j][2 * h + ii][4 * q], acc[j][2 * h + ii][4 * q + 1],
                               acc[j][2 * h + ii][4 * q + 2], acc[j][2 * h + ii][4 * q + 3]};
              *(f32x4*)(tb + (32 * ii + l31) * 128 + (((8 * j + 2 * q + g) ^ l31) * 4)) = v;
            }
        int tries = 0;
        while (a.dw_parts > 1 && __builtin_amdgcn_readfirstlane(__hip_atomic_load(
                                     (gint*)(turn + h), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) != tpart) {
          if (++tries > SPIN_LIMIT) break;
          __builtin_amdgcn_s_sleep(8);
        }
        asm volatile("" ::: "memory");               // the old values are read after the turn has come
        // (a wait that gave up -- the part before never came, which takes a fault elsewhere -- must
        // not pass for a result: this half of the tile becomes NaN)
        const float poison = tries > SPIN_LIMIT ? __builtin_nanf("") : 0.f;
        const int voff = ((wm * 128 + 64 * h + rrow) * a.E + wn * 128 + 4 * rch) * 4;
#pragma unroll
        for (int b0 = 0; b0 < 32; b0 += 16) {
          u32x4 old[16];
#pragma unroll
          for (int t = 0; t < 16; ++t)
            old[t] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, (b0 + t) * two_rows, AGENT);
#pragma unroll
          for (int t = 0; t < 16; ++t) {
            const int row = 2 * (b0 + t) + rrow;
            const f32x4 v = *(const f32x4*)(tb + row * 128 + ((rch ^ (row & 31)) * 4));
            const u32x4 y = {__float_as_uint(__uint_as_float(old[t][0]) + (v[0] + poison)),
                             __float_as_uint(__uint_as_float(old[t][1]) + (v[1] + poison)),
                             __float_as_uint(__uint_as_float(old[t][2]) + (v[2] + poison)),
                             __float_as_uint(__uint_as_float(old[t][3]) + (v[3] + poison))};
            __builtin_amdgcn_raw_buffer_store_b128(y, rs, voff, (b0 + t) * two_rows, AGENT);
          }
        }
        if (a.dw_parts > 1) {
          wait_vmcnt<0>();                           // this wave's stores have been acknowledged: the next part may come
          asm volatile("" ::: "memory");
          __hip_atomic_store((gint*)(turn + h), tpart + 1 == a.dw_parts ? 0 : tpart + 1, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    }
  }
}

// Any shape and both types: one thread per element of the result, the sum in float32 in the order
// of the definition.
template <typename TIn> __device__ __forceinline__ float to_f32(TIn v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<__bf16>(__bf16 v) { return (float)v; }

template <typename TIn>
__global__ void __launch_bounds__(256) project_bwd_x_plain_kernel(ProjBwdArgs a) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= a.M * a.E) return;
  const long m = idx / a.E;
  const int e = (int)(idx % a.E);
  const long b = m / a.S, s = m % a.S;
  const int HD = a.H * a.D;
  float acc = 0.f;
  for (int n = 0; n < a.N; ++n) {
    const int nn = n % HD;
    const TIn* gp = (const TIn*)a.g[n / HD] + ((b * a.H + nn / a.D) * a.S + s) * a.D + nn % a.D;
    acc = fmaf(to_f32<TIn>(*gp), to_f32<TIn>(((const TIn*)a.w)[(long)n * a.E + e]), acc);
  }
  ((TIn*)a.dx)[m * a.ldx + e] = (TIn)acc;
}

template <typename TIn>
__global__ void __launch_bounds__(256) project_bwd_w_plain_kernel(ProjBwdArgs a) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)a.N * a.E) return;
  const int n = (int)(idx / a.E), e = (int)(idx % a.E);
  const int HD = a.H * a.D, nn = n % HD;
  const TIn* gh = (const TIn*)a.g[n / HD] + (long)(nn / a.D) * a.S * a.D + nn % a.D;
  float acc = 0.f;
  for (long m = 0; m < a.M; ++m) {
    const long b = m / a.S, s = m % a.S;
    acc = fmaf(to_f32<TIn>(gh[(b * a.H * a.S + s) * a.D]), to_f32<TIn>(((const TIn*)a.x)[m * a.ldx + e]), acc);
  }
  a.dw[idx] += acc;
}

}  // namespace

namespace {
// what both matrix-core kernels need: 16-byte chunks inside one head, a tile of 256 columns inside
// one output, tokens countable in a float, and every G offset inside 32 bits
bool mfma_common(const ProjBwdArgs& a) {
  return a.E % T == 0 && (a.H * a.D) % T == 0 && a.D % 8 == 0 &&
         a.M < (1L << 24) && a.M * a.H * a.D * 2 < (1L << 31) && 64 * a.ldx * 2 < (1L << 31) &&
         2L * a.E * 2 < (1L << 31);
}
}  // namespace
bool project_bwd_bf16_supported(const ProjBwdArgs& a) { return mfma_common(a); }

hipError_t launch_project_bwd(const ProjBwdArgs& a, int is_f32, hipStream_t s) {
  const bool mfma_w = !is_f32 && mfma_common(a), mfma_x = mfma_w;
  static SmemOnce once_x, once_xu, once_w, once_w2;
  ProjBwdArgs rest = a;                              // what is left for the plain kernels
  if (mfma_x) rest.dx = nullptr;
  if (mfma_w) rest.dw = nullptr;
  if (mfma_w) {
    if (a.dx && mfma_x) {
      const long grid = xcd_grid((int)((a.M + T - 1) / T), a.E / T);
      if (a.D % BK == 0) {
        const hipError_t e = ensure_dynamic_lds((const void*)project_bwd_bf16_kernel<0, 4, true>, SMEM_B, &once_x);
        if (e != hipSuccess) return e;
        project_bwd_bf16_kernel<0, 4, true><<<(unsigned)grid, 256, SMEM_B, s>>>(a);
      } else {
        const hipError_t e = ensure_dynamic_lds((const void*)project_bwd_bf16_kernel<0, 4, false>, SMEM_B, &once_xu);
        if (e != hipSuccess) return e;
        project_bwd_bf16_kernel<0, 4, false><<<(unsigned)grid, 256, SMEM_B, s>>>(a);
      }
    }
    if (a.dw) {
      // Fewer 256 x 256 tiles than three quarters of the compute units: the token range is cut
      // into parts (at least 8 tile pairs each) until the grid covers the chip; where that cannot
      // be (very few tokens, more tiles than turn words), tiles of 128 rows instead.
      const long tiles = (long)(a.N / T) * (a.E / T);
      const long pairs = (a.M + BK - 1) / BK;
      ProjBwdArgs w = a;
      w.dw_parts = 1;
      if (tiles * 4 <= (long)a.n_cu * 3 && tiles <= MAX_TURNS) {
        long parts = a.n_cu / tiles;
        if (parts > 32) parts = 32;
        if (parts > pairs / 8) parts = pairs / 8;
        if (parts >= 2) w.dw_parts = (int)parts;
      }
      if (tiles * 4 > (long)a.n_cu * 3 || w.dw_parts > 1) {
        const hipError_t e = ensure_dynamic_lds((const void*)project_bwd_bf16_kernel<1, 4>, SMEM_B, &once_w);
        if (e != hipSuccess) return e;
        w.dw_tiles_grid = (unsigned)xcd_grid(a.N / T, a.E / T);
        project_bwd_bf16_kernel<1, 4><<<w.dw_tiles_grid * (unsigned)w.dw_parts, 256, SMEM_B, s>>>(w);
      } else {
        const hipError_t e = ensure_dynamic_lds((const void*)project_bwd_bf16_kernel<1, 2>, SMEM_B, &once_w2);
        if (e != hipSuccess) return e;
        w.dw_tiles_grid = (unsigned)xcd_grid(a.N / 128, a.E / T);
        project_bwd_bf16_kernel<1, 2><<<w.dw_tiles_grid, 256, SMEM_B, s>>>(w);
      }
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (rest.dx) {
    const unsigned grid = (unsigned)((a.M * a.E + 255) / 256);
    if (is_f32) project_bwd_x_plain_kernel<float><<<grid, 256, 0, s>>>(rest);
    else project_bwd_x_plain_kernel<__bf16><<<grid, 256, 0, s>>>(rest);
  }
  if (rest.dw) {
    const unsigned grid = (unsigned)(((long)a.N * a.E + 255) / 256);
    if (is_f32) project_bwd_w_plain_kernel<float><<<grid, 256, 0, s>>>(rest);
    else project_bwd_w_plain_kernel<__bf16><<<grid, 256, 0, s>>>(rest);
  }
  return hipGetLastError();
}

}  // namespace lvx
