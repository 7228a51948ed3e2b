// bf16 backward, key-stationary kernel: dK and dV of one K/V block.  Table 1 of the paper counts
// the backward as five matrix products; this kernel performs four of them (S, dP, dV, dK) with
// the probabilities recomputed from the saved statistic L (Section 3.2 saves only x, O and L):
//   p_ij = exp(scale <Q_i, K_j> - L_i),   dS_ij = p_ij (<dO_i, V_j> - delta_i).
//
// Workgroup = 4 wavefronts = 256 keys of one (batch, K/V head), one wave per SIMD with the whole
// register file: a wave owns 64 keys (two 32-key blocks), keeps their K operands in registers and
// their dK^T / dV^T accumulators (2 x 2 x D/32 MFMA blocks = 256 registers at D = 128) in the
// accumulation registers; V of the workgroup stays in LDS.  Owning two key blocks halves the LDS
// traffic: every Q / dO operand fetched from LDS feeds two matrix instructions.
// The query rows of all heads that share this K/V head are streamed 32 at a time: [Q; dO] tiles
// (plus the 32 row statistics L log2(e) and delta) travel HBM -> LDS by direct global-to-LDS
// copies into a ring of four stages, issued three steps ahead, one barrier per step.
// S = Q K^T and dP = dO V^T put one KEY per lane and 16 query rows in a lane's registers, so P and
// dS, rounded to bf16, are already the B operands of dV^T += dO^T P and dK^T += Q^T dS, with
// dO^T / Q^T fetched by transposing LDS reads: nothing goes back through LDS or memory.
// The loop is software pipelined inside each wave: while the matrix core contracts step i
// (dV, dK), the vector ALU turns the scores of step i+1 into P and dS; then the scores of step
// i+2 are formed.
#include "lvx_internal.h"
#include "lvx_mfma.h"

#include <type_traits>

namespace lvx {

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr int NWV = 4;                 // waves per workgroup
// 32-key blocks per wave: two in the dense kernel; one in the general kernel, whose mask code needs
// registers and must leave the accumulation file half empty (see mfma32_acc)
constexpr int kvb_of(bool general) { return general ? 1 : 2; }
constexpr int KM = 32;                 // query rows per step
constexpr int NSTG = 4;                // ring stages

// dK^T / dV^T accumulation: the sixteen 32x32 accumulator blocks of a wave fill the accumulation
// register file exactly, and only matrix instructions touch them until the epilogue.  The
// instruction is written out so that the accumulator stays in that file by construction.
// The compiler does not know that this is a matrix instruction, so it would not wait for the
// result before a register move of its own.  The dense kernel has no such move inside its loops
// (checked in the generated code: the accumulators never leave their file); the general kernel
// is under more register pressure and the allocator may park an accumulator elsewhere between
// uses, so there (SETTLE) the instruction is followed by enough idle states for the result to land.
template <bool SETTLE>
__device__ __forceinline__ void mfma32_acc(f32x16& acc, bf16x8 a, bf16x8 b) {
  if (SETTLE)
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0\n\ts_nop 15\n\ts_nop 15\n\ts_nop 7"
                 : "+a"(acc) : "v"(a), "v"(b));
  else
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

template <int D, int KVB> struct DkvSmem;
// entries the step list of the STEPS variant can hold (the mask areas of the dense layout, less
// one word for the length)
template <int D> constexpr int dkdv_step_list_cap();

template <int D, int KVB> struct DkvSmem {
  static constexpr int KN = NWV * 32 * KVB;         // keys per workgroup
  static constexpr int CPR = D / 8;                 // 16-byte chunks of data per row
  static constexpr int P = (D + 8) * 2;             // row pitch in bytes
  static constexpr int SPR = P / 16;                // 16-byte slots per row
  static constexpr int RUN = 8 * SPR;               // slots of one run: 8 consecutive physical rows
  static constexpr int NCR = (RUN + 63) / 64;       // wave-level copies (64 slots) per run
  static constexpr int STAT_OFF = ILV_ROWS * P;     // 32 x L log2(e), then 32 x delta
  static constexpr int STAGE = STAT_OFF + 256;      // [Q; dO] as one 64-row interleaved tile + statistics
  static constexpr int V_BYTES = KN * P;            // V rows of the workgroup, resident
  static constexpr int RING = NSTG * STAGE + V_BYTES;
  static constexpr int BITS_BYTES = 2048;           // visibility bits of up to 16320 steps (media mask only)
  static constexpr int WIN_BYTES = 2048;            // window of the mask bitmap (media mask only)
  static constexpr int TOTAL = RING + BITS_BYTES + WIN_BYTES;
  static_assert(RUN >= 64, "a run must hold at least one full copy");
};
template <int D> constexpr int dkdv_step_list_cap() {
  return (DkvSmem<D, 2>::BITS_BYTES + DkvSmem<D, 2>::WIN_BYTES) / 4 - 1;
}

// GENERAL = false: dense attention (no mask code, so that the steady-state loop is one basic
// block; when Sq is no multiple of 32, the last step of a head takes rows Sq-32 .. Sq-1 with the
// statistics of BwdArgs::stats_ovl instead of a short tile -- Sq >= 32 then); GENERAL = true:
// everything else.
// STEPS (with GENERAL = false): a media mask whose chunks are multiples of the 32 query rows of a
// step and whose key blocks are multiples of a workgroup's 256 keys.  A step is then either
// visible to all of a workgroup's keys or to none, so the mask only selects WHICH steps a
// workgroup performs: the dense kernel runs over a list of them and nothing inside a step
// changes.
// Measurement builds only (python -m paper_2502_02406_amd.build --define LVX_DKDV_PROBE=1): every
// workgroup with steps to run adds the clocks of its three phases (set-up until the first tiles and
// K, V are in place; the loop; the epilogue until its stores have been acknowledged), a count and
// its number of steps to dkdv_probe, which lvx_debug_dkdv_probe copies out and clears.
#ifdef LVX_DKDV_PROBE
__device__ unsigned long long dkdv_probe[8];
#define DKDV_STAMP(x) const unsigned long long x = __builtin_readcyclecounter()
#else
#define DKDV_STAMP(x)
#endif

template <int D, bool GENERAL, bool STEPS = false>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
bwd_dkdv_bf16_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  static_assert(!(GENERAL && STEPS), "the step list is a variant of the dense kernel");
  constexpr int KVB = kvb_of(GENERAL);
  constexpr int XE = 16 * KVB;     // all elements of a step are converted during the contraction
                                   // (measured: no gain from moving some of them to the scoring)
  using SM = DkvSmem<D, KVB>;
  constexpr int KN = SM::KN;
  constexpr int KS = D / 16, DB = D / 32, CPR = SM::CPR, NCR = SM::NCR;

  const Dims& d = a.d;
  const int G = d.Hq / d.Hkv;
  const int n_kt = (d.Skv + KN - 1) / KN;
  HeadWork hw;
  if (!xcd_decode(blockIdx.x, d.B * d.Hkv, n_kt, &hw)) return;
  DKDV_STAMP(stamp0);
  const int b = hw.head / d.Hkv, hk = hw.head % d.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, kl = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j_wg0 = hw.item * KN;
  const int j_wave0 = j_wg0 + wave * 32 * KVB;

  // ---- query steps: the G heads of the group, KM rows at a time.  With a media mask, steps whose
  // rows see none of this workgroup's keys are skipped: the window of the bitmap that the
  // workgroup can touch is copied to LDS and the visibility of the spH row tiles (the same for
  // every head) is worked out by all threads at once into a bit array.
  const int spH = (d.Sq + KM - 1) / KM;
  const int n_all = G * spH;
  const int j_wg1 = min(d.Skv, j_wg0 + KN) - 1;
  MaskDev mk = a.mask;
  unsigned* const bits = (unsigned*)(smem + SM::RING);
  bool have_bits = false;
  int per_head = spH;
  if (GENERAL && mk.allow) {
    mk = mask_to_lds(a.mask, b, 0, (d.Sq - 1) / mk.q_chunk, j_wg0 / mk.kv_block, j_wg1 / mk.kv_block,
                     (uint8_t*)smem + SM::RING + SM::BITS_BYTES, SM::WIN_BYTES, tid, 256);
    if (spH <= (SM::BITS_BYTES - 16) * 8) {
      have_bits = true;
      per_head = build_bits(bits, spH, tid, 256, [&](int t) {
        return mask_rect_tall(mk, b, t * KM, min(d.Sq, t * KM + KM) - 1, j_wg0, j_wg1) != 0;
      });
    }
  }
  // STEPS: the row tiles that see this workgroup's keys (the same for every head), compacted
  // into a list by one wave; its length goes into the last word of the area.
  constexpr int LIST_CAP = dkdv_step_list_cap<D>();
  int* const tl = (int*)(smem + SM::RING);
  if (STEPS) {
    const uint8_t* const col = a.mask.allow + b * a.mask.stride_b + j_wg0 / a.mask.kv_block;
    if (wave == 0) {
      int count = 0;
      for (int base = 0; base < spH; base += 64) {     // (wave-uniform trip count)
        const int t = base + lane;
        const bool on = t < spH && col[(long)((t * KM) / a.mask.q_chunk) * a.mask.stride_q] != 0;
        const unsigned long long m = __ballot(on);
        if (on) tl[count + __popcll(m & ((1ull << lane) - 1ull))] = t;
        count += (int)__popcll(m);
      }
      if (lane == 0) tl[LIST_CAP] = count;
    }
    __syncthreads();
    per_head = __builtin_amdgcn_readfirstlane(tl[LIST_CAP]);
  }
  // cursor over the steps in issue order: step id s = head * spH + tile, kept with its head and
  // first row so that no division is needed per step (STEPS: k = position in the list, tp = the
  // list entry after it, fetched a step ahead so that nothing waits for it)
  // (dense variant: hb, lb and lo are running addresses of the cursor's step -- the byte offset of
  // this wave's first row of the head, the step's statistics, the head's overlay statistics -- so
  // that a step costs a handful of scalar additions instead of the 64-bit products of its tile
  // address: with one wave per SIMD every scalar instruction takes an issue slot from the loop)
  struct Cursor { int s, h, i0, k, tp; long hb, lb, lo; };
  constexpr bool RUNNING = !GENERAL && !STEPS;
  auto step_needed = [&](const Cursor& c) __attribute__((always_inline)) -> bool {
    if (!GENERAL || !mk.allow) return true;
    return mask_rect_tall(mk, b, c.i0, min(d.Sq, c.i0 + KM) - 1, j_wg0, j_wg1) != 0;
  };
  auto advance = [&](Cursor& c) __attribute__((always_inline)) {      // to the next needed step (or the end)
    if (STEPS) {
      int k = c.k + 1, h = c.h;
      if (k == per_head) { k = 0; ++h; }
      c.i0 = __builtin_amdgcn_readfirstlane(c.tp) * KM;
      c.k = k;
      c.h = h;
      ++c.s;
      int kn = k + 1;
      if (kn == per_head) kn = 0;
      c.tp = tl[kn];
      return;
    }
    if (GENERAL && have_bits) {
      int t = next_bit(bits, c.i0 / KM + 1, spH);
      if (t >= spH) { ++c.h; t = next_bit(bits, 0, spH); }
      c.i0 = t * KM;
      c.s = (c.h < G && t < spH) ? c.h * spH + t : n_all;
      return;
    }
    if (RUNNING) {
      ++c.s;
      c.i0 += KM;
      c.lb += 256;
      const bool wrap = c.i0 >= d.Sq;
      c.i0 = wrap ? 0 : c.i0;
      c.h += wrap ? 1 : 0;
      c.hb += wrap ? d.q_sh * 2 : 0;
      c.lo += wrap ? 256 : 0;
      return;
    }
    do {
      ++c.s;
      c.i0 += KM;
      if (c.i0 >= d.Sq) { c.i0 = 0; ++c.h; }
    } while (c.s < n_all && !step_needed(c));
    if (GENERAL) {                                 // wave-uniform (the bitmap is read through the vector path)
      c.s = __builtin_amdgcn_readfirstlane(c.s);
      c.h = __builtin_amdgcn_readfirstlane(c.h);
      c.i0 = __builtin_amdgcn_readfirstlane(c.i0);
    }
  };
  Cursor cursor = {0, 0, 0, 0, 0, 0, 0, 0};
  if (STEPS) {
    if (per_head > 0) {
      cursor.i0 = __builtin_amdgcn_readfirstlane(tl[0]) * KM;
      cursor.tp = tl[per_head > 1 ? 1 : 0];
    }
  } else if (GENERAL && have_bits) {
    const int t = next_bit(bits, 0, spH);
    cursor.i0 = t * KM;
    cursor.s = t < spH ? t : n_all;
  } else if (!step_needed(cursor)) {
    advance(cursor);
  }
  int n = n_all;                                   // number of steps this workgroup performs
  if (STEPS) n = G * per_head;
  if (GENERAL && mk.allow) {
    n = G * per_head;
    if (!have_bits) {
      n = 0;
      for (Cursor c = cursor; c.s < n_all; advance(c)) ++n;
    }
  }
  if ((GENERAL || STEPS) && n == 0) {              // keys that no query sees: dK = dV = 0, nothing to read
    const u32x4 z = {0, 0, 0, 0};
    for (int c = tid; c < KN * CPR; c += 256) {
      const int j = j_wg0 + c / CPR, col = (c % CPR) * 8;
      if (j >= d.Skv) continue;
      const long off = b * d.kv_sb + hk * d.kv_sh + (long)j * d.kv_ss + col;
      *(u32x4*)((uint16_t*)a.dk + off) = z;
      *(u32x4*)((uint16_t*)a.dv + off) = z;
    }
    return;
  }

  // ---- K operands of this wave's keys: lane holds key j_wave0 + 32 kb + kl, columns 16 ks + 8 g ..
  // They are held as bf16(K * scale * log2 e), so that the accumulation Q K'^T started at -L log2 e
  // is already the exponent of P (Section 3.2's recomputation, P = exp(S - L)) and needs no
  // multiply-add per element; dK uses Q and dS only, so nothing else sees the scaled copy.
  // Both loads are issued AFTER the first tile copies (load_kv is called there): the three
  // transfers a workgroup starts with then share one round trip to memory instead of taking one
  // each.
  const float c2 = d.scale * LOG2E;
  bf16x8 kf[KVB][KS];
  char* const vres = smem + NSTG * SM::STAGE;
  auto load_kv = [&]() __attribute__((always_inline)) {
    // A lane needs ITS key row (16 bytes of it per k-step): fetched directly, every load
    // instruction would touch 32 rows with 32 bytes each, half a memory line per request.  Each
    // wave fetches its rows whole instead (16 lanes per 256-byte row), parks them in the part of
    // the V area that its own rows will occupy, and reads its operands back from there; the V
    // rows, fetched meanwhile, are stored once every wave has its K operands.
    // All of these loads are issued before the first of them is waited for (rows past the last
    // key re-read it and are zeroed afterwards: a branch around a load would make every load
    // wait for the one before it).
    constexpr int WR = 32 * KVB;                   // key rows of a wave
    constexpr int KIT = WR * CPR / 64;
    char* const kst = vres + wave * WR * SM::P;
    const uint16_t* const k_head = (const uint16_t*)a.k + b * d.kv_sb + hk * d.kv_sh;
    const uint16_t* const v_head = (const uint16_t*)a.v + b * d.kv_sb + hk * d.kv_sh;
    u32x4 xk[KIT];
#pragma unroll
    for (int it = 0; it < KIT; ++it) {
      const int c = it * 64 + lane, r = c / CPR, col = (c % CPR) * 8, j = min(j_wave0 + r, d.Skv - 1);
      xk[it] = *(const u32x4*)(k_head + (long)j * d.kv_ss + col);
    }
    // ---- V rows of the workgroup -> LDS (plain row-major: only read as whole rows)
    constexpr int VIT = KN * CPR / 256;
    u32x4 vy[VIT];
#pragma unroll
    for (int it = 0; it < VIT; ++it) {
      const int c = it * 256 + tid, r = c / CPR, col = (c % CPR) * 8, j = min(j_wg0 + r, d.Skv - 1);
      vy[it] = *(const u32x4*)(v_head + (long)j * d.kv_ss + col);
    }
    const u32x4 zero4 = {0, 0, 0, 0};
#pragma unroll
    for (int it = 0; it < KIT; ++it) {
      const int c = it * 64 + lane, r = c / CPR, col = (c % CPR) * 8;
      *(u32x4*)(kst + r * SM::P + col * 2) = j_wave0 + r < d.Skv ? xk[it] : zero4;
    }
#pragma unroll
    for (int it = 0; it < VIT; ++it) {
      const int c = it * 256 + tid, r = c / CPR;
      if (j_wg0 + r >= d.Skv) vy[it] = zero4;
    }
#pragma unroll
    for (int kb = 0; kb < KVB; ++kb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        u32x4 x = *(const u32x4*)(kst + (32 * kb + kl) * SM::P + (16 * ks + 8 * g) * 2);
#pragma unroll
        for (int w = 0; w < 4; ++w)
          x[w] = pack2_bf16(__uint_as_float(x[w] << 16) * c2, __uint_as_float(x[w] & 0xffff0000u) * c2);
        kf[kb][ks] = __builtin_bit_cast(bf16x8, x);
      }
    __syncthreads();                               // every wave has read its K rows back
#pragma unroll
    for (int it = 0; it < VIT; ++it) {
      const int c = it * 256 + tid, r = c / CPR, col = (c % CPR) * 8;
      *(u32x4*)(vres + r * SM::P + col * 2) = vy[it];
    }
  // Finish these loads here: otherwise their first use inside the loop would make the compiler
  // drain every copy in flight.
#pragma unroll
  for (int kb = 0; kb < KVB; ++kb)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(kf[kb][ks]));
  };

  // ---- tile copies.  In the interleaved tile the logical rows 4 j + w (j = 0..7) of Q occupy the
  // 8 consecutive physical rows 20 w .. 20 w + 7, and those of dO the next 8: a "run" of 8 SPR
  // 16-byte slots.  Wave w copies the two runs of group w, each with NCR wave-level copies of 64
  // slots (the last one re-covers the tail of the previous so that no copy crosses a run); lane l
  // of a copy starting at slot a fills slot a + l = (row (a + l) / SPR of the run, chunk
  // (a + l) % SPR; the pad chunk re-reads the last one).  Every copy therefore has a wave-uniform
  // base and the per-lane offsets are the same for all runs.  The 64 statistics of the step are
  // one more copy of 4 bytes per lane, issued by every wave.
  const char* const q0 = (const char*)a.q + (b * d.q_sb) * 2;
  const char* const g0 = (const char*)a.d_o + (b * d.q_sb) * 2;
  const char* const l0 = (const char*)a.stats + ((long)b * d.Hq * a.sq_pad) * 8;
  const unsigned row_bytes = (unsigned)(d.q_ss * 2);
  auto run_start = [&](int c) __attribute__((always_inline)) -> int { return c + 1 < NCR ? 64 * c : SM::RUN - 64; };
  unsigned cp_off[NCR];
#pragma unroll
  for (int c = 0; c < NCR; ++c) {
    const int sl = run_start(c) + lane;
    cp_off[c] = (unsigned)(4 * (sl / SM::SPR)) * row_bytes + (unsigned)min(sl % SM::SPR, CPR - 1) * 16;
  }
  // One step's copies: the scalar part (tile addresses) and the copies themselves, numbered
  // 0 .. NDMA - 1 so that the dense loop can spread them over the matrix instructions of a phase.
  constexpr int NDMA = 2 * NCR + 1;                // copies per wave and step
  struct Tile { const char *qb, *gb, *lb; char* dst; int rows; long tile; };
  if (RUNNING) {                                   // (the dense cursor still stands at step 0)
    cursor.hb = (long)(hk * G) * d.q_sh * 2 + (long)wave * row_bytes;
    cursor.lb = (long)(uintptr_t)l0 + (long)(hk * G) * a.sq_pad * 8;
    cursor.lo = (long)(uintptr_t)a.stats_ovl + ((long)b * d.Hq + hk * G) * 256;
  }
  auto tile_of = [&](const Cursor& c, char* st) __attribute__((always_inline)) -> Tile {
    if constexpr (RUNNING) {
      // the short last step of a head takes rows Sq-32 .. Sq-1 and their own statistics (selected
      // without a branch: one would cut the steady-state loop into pieces)
      const int i0_eff = min(c.i0, d.Sq - KM);
      const long tile = c.hb + (long)((unsigned long long)(unsigned)i0_eff * row_bytes);
      Tile t;
      t.rows = KM;
      t.tile = tile;
      t.qb = q0 + tile;
      t.gb = g0 + tile;
      t.lb = (const char*)(uintptr_t)(c.i0 != i0_eff ? c.lo : c.lb);
      t.dst = st;
      return t;
    }
    // (wave-uniform by construction; said explicitly because with a media mask the cursor derives
    // from bitmap words read through the vector path)
    const int hq = __builtin_amdgcn_readfirstlane(hk * G + c.h), i0 = __builtin_amdgcn_readfirstlane(c.i0);
    Tile t;
    t.rows = min(KM, d.Sq - i0);
    // the dense kernel's short last step takes rows Sq-32 .. Sq-1 and their own statistics
    // (selected by arithmetic: a branch here would cut the steady-state loop into pieces)
    const int i0_eff = GENERAL ? i0 : min(i0, d.Sq - KM);
    t.tile = ((long)hq * d.q_sh + (long)i0_eff * d.q_ss) * 2;
    t.qb = q0 + t.tile + (long)wave * row_bytes;   // this wave's first row: tile row w
    t.gb = g0 + t.tile + (long)wave * row_bytes;
    const long lb_std = (long)(uintptr_t)l0 + ((long)hq * a.sq_pad + i0) * 8;
    if (GENERAL) {
      t.lb = (const char*)(uintptr_t)lb_std;
    } else {
      const long lb_ovl = (long)(uintptr_t)a.stats_ovl + ((long)b * d.Hq + hq) * 256;
      const long pick = -(long)(i0 != i0_eff);     // all ones for the short step
      t.lb = (const char*)(uintptr_t)(lb_std + ((lb_ovl - lb_std) & pick));
    }
    t.dst = st;
    return t;
  };
  const unsigned smem_u = lds_base(smem);
  auto issue_part = [&](const Tile& t, int k) __attribute__((always_inline)) {   // full tiles only
    const unsigned dst = smem_u + (unsigned)(t.dst - smem), qdst = dst + 20 * wave * SM::P;
    if (k == NDMA - 1) dma4u(t.lb, lane * 4, dst + SM::STAT_OFF);
    else if (k % 2 == 0) dma16u(t.qb, cp_off[k / 2], qdst + run_start(k / 2) * 16);
    else dma16u(t.gb, cp_off[k / 2], qdst + 8 * SM::P + run_start(k / 2) * 16);
  };
  auto issue_tile = [&](const Cursor& c, char* st) __attribute__((always_inline)) {
    const Tile t = tile_of(c, st);
    if (!GENERAL || t.rows == KM) {
#pragma unroll
      for (int k = 0; k < NDMA; ++k) issue_part(t, k);
      return;
    }
    char* const qdst = st + 20 * wave * SM::P;     // ragged last tile of a head: clamp the rows
    char* const gdst = qdst + 8 * SM::P;
#pragma unroll
    for (int c = 0; c < NCR; ++c) {
      const int sl = run_start(c) + lane;
      const unsigned r = (unsigned)min(4 * (sl / SM::SPR) + wave, t.rows - 1);     // row of the tile
      const unsigned off = r * row_bytes + (unsigned)min(sl % SM::SPR, CPR - 1) * 16;
      dma16s(q0 + t.tile, off, qdst + run_start(c) * 16);
      dma16s(g0 + t.tile, off, gdst + run_start(c) * 16);
    }
    dma4s(t.lb, lane * 4, st + SM::STAT_OFF);
  };

  f32x16 dk[KVB][DB], dv[KVB][DB];
#pragma unroll
  for (int kb = 0; kb < KVB; ++kb)
#pragma unroll
    for (int i = 0; i < DB; ++i) { dk[kb][i] = zero16(); dv[kb][i] = zero16(); }

  // ---- building blocks ------------------------------------------------------------------------
  // S = Q K^T and dP = dO V^T of one step: lane = key column, registers = query rows.  The four
  // LDS operands of a k-step are fetched while the matrix instructions of the previous one run.
  // What a score phase needs before its first matrix instruction: the operands of k-step 0 and the
  // starting values of the accumulations, which are the statistics of the query rows -- S starts
  // at -L log2 e and dP at -delta, so that neither difference needs a vector instruction.  The
  // dense loop fetches them while the previous phase still computes.
  struct FirstY { bf16x8 qa, ga, va[KVB]; f32x16 nl, nd; };
  auto first_y = [&](const char* __restrict__ t, const char* __restrict__ vw) __attribute__((always_inline)) -> FirstY {
    FirstY f;
    f.qa = *(const bf16x8*)(t + ilv_off<D>(kl, 0, 8 * g));
    f.ga = *(const bf16x8*)(t + ilv_off<D>(kl, KM, 8 * g));
#pragma unroll
    for (int kb = 0; kb < KVB; ++kb) f.va[kb] = *(const bf16x8*)(vw + kb * 32 * SM::P);
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const f32x4 nl = *(const f32x4*)(t + SM::STAT_OFF + (8 * q4 + 4 * g) * 4);
      const f32x4 nd = *(const f32x4*)(t + SM::STAT_OFF + 128 + (8 * q4 + 4 * g) * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) { f.nl[4 * q4 + e] = nl[e]; f.nd[4 * q4 + e] = nd[e]; }
    }
    return f;
  };
  // S = Q K^T and dP = dO V^T of one step: lane = key column, registers = query rows.  The four
  // LDS operands of a k-step are fetched while the matrix instructions of the previous one run;
  // per_unit(m) is issued right after matrix instruction m, tail() three instructions before the end.
  auto score = [&](const char* __restrict__ t, const char* __restrict__ vw, f32x16 (&s)[KVB],
                   f32x16 (&p)[KVB], auto&& per_unit, const FirstY& f, auto&& tail) __attribute__((always_inline)) {
    const char* qrow = t + ilv_off<D>(kl, 0, 8 * g);
    const char* grow = t + ilv_off<D>(kl, KM, 8 * g);
    bf16x8 qa[2], ga[2], va[2][KVB];               // two operand sets, used alternately
    qa[0] = f.qa;
    ga[0] = f.ga;
#pragma unroll
    for (int kb = 0; kb < KVB; ++kb) va[0][kb] = f.va[kb];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int cu = ks & 1, nx = cu ^ 1;
      if (ks + 1 < KS) {
        qa[nx] = *(const bf16x8*)(qrow + (ks + 1) * 32);
        ga[nx] = *(const bf16x8*)(grow + (ks + 1) * 32);
#pragma unroll
        for (int kb = 0; kb < KVB; ++kb) va[nx][kb] = *(const bf16x8*)(vw + kb * 32 * SM::P + (ks + 1) * 32);
      }
#pragma unroll
      for (int j = 0; j < 2 * KVB; ++j) {          // S of both key blocks, then dP
        const int kb = j % KVB;
        if (j < KVB) s[kb] = mfma32(qa[cu], kf[kb][ks], ks == 0 ? f.nl : s[kb]);
        else p[kb] = mfma32(ga[cu], va[cu][kb], ks == 0 ? f.nd : p[kb]);
        per_unit(ks * 2 * KVB + j);                // vector work in the shadow of this instruction
        if (ks * 2 * KVB + j == 2 * KVB * KS - 3) tail();
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  auto nothing = [](int) __attribute__((always_inline)) {};
  auto no_tail = []() __attribute__((always_inline)) {};
  // masked elements of a step's scores -> -inf (wave-uniform decision, rarely taken)
  auto mask_scores = [&](int st, f32x16 (&s)[KVB]) __attribute__((always_inline)) {
    if (!GENERAL || !mk.allow) return;
    const int i0 = (st % spH) * KM;
    const int cls = mask_rect_tall(mk, b, i0, min(d.Sq, i0 + KM) - 1, min(j_wave0, d.Skv - 1),
                              min(d.Skv - 1, j_wave0 + 32 * KVB - 1));
    if (cls == 1) return;
    asm volatile("" ::: "memory");
    // all rows of the step in one chunk of the bitmap (the usual case): one probe per key
    // instead of one per element
    const bool one_chunk = cls == 2 && i0 / mk.q_chunk == (min(d.Sq, i0 + KM) - 1) / mk.q_chunk;
#pragma unroll
    for (int kb = 0; kb < KVB; ++kb) {
      const int j = j_wave0 + 32 * kb + kl;
      const bool key_ok = one_chunk && j < d.Skv && mask_elem(mk, b, i0, j);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = i0 + 8 * (v / 4) + 4 * g + (v % 4);
        bool ok = cls != 0 && j < d.Skv && i < d.Sq;
        if (ok) ok = one_chunk ? key_ok : mask_elem(mk, b, i, j);
        if (!ok) s[kb][v] = -INFINITY;
      }
    }
  };
  // Conversion of scores into operands, element x of a step (x = 0 .. 16 KVB - 1: four query rows
  // q4 = x / (4 KVB) of key block kb = (x / 4) % KVB, row e = x % 4 of the four): p = exp2(s), dS = p dP,
  // both differences already formed by the accumulation, packed in pairs as bf16 into word
  // 2 (q4 % 2) + e / 2 of operand q4 / 2 of the key block.
  // In two halves -- the exponential, then everything that uses it -- so that the pipelined loop
  // can start an element under one matrix instruction and finish it under the next: a
  // transcendental result read by the very next instruction costs an idle issue slot.
  struct Carry { float pr, ds, ex; };
  auto conv_start = [&](int x, const f32x16 (&s)[KVB]) __attribute__((always_inline)) -> float {
    const int q4 = x / (4 * KVB), kb = (x / 4) % KVB, e = x % 4, v = 4 * q4 + e;
    return __builtin_amdgcn_exp2f(s[kb][v]);
  };
  auto conv_finish = [&](int x, Carry& cy, const f32x16 (&p)[KVB],
                         u32x4 (&pwo)[KVB][2], u32x4 (&swo)[KVB][2]) __attribute__((always_inline)) {
    const int q4 = x / (4 * KVB), kb = (x / 4) % KVB, e = x % 4, v = 4 * q4 + e;
    const float pr = cy.ex;
    const float ds = pr * p[kb][v];
    if (e % 2 == 0) { cy.pr = pr; cy.ds = ds; return; }
    pwo[kb][q4 >> 1][2 * (q4 & 1) + e / 2] = pack2_bf16(cy.pr, pr);
    swo[kb][q4 >> 1][2 * (q4 & 1) + e / 2] = pack2_bf16(cy.ds, ds);
  };
  auto conv_elem = [&](int x, Carry& cy, const f32x16 (&s)[KVB], const f32x16 (&p)[KVB],
                       u32x4 (&pwo)[KVB][2], u32x4 (&swo)[KVB][2]) __attribute__((always_inline)) {
    cy.ex = conv_start(x, s);
    conv_finish(x, cy, p, pwo, swo);
  };
  auto convert = [&](const f32x16 (&s)[KVB], const f32x16 (&p)[KVB],
                     u32x4 (&pwo)[KVB][2], u32x4 (&swo)[KVB][2]) __attribute__((always_inline)) {
    Carry cy;
#pragma unroll
    for (int x = 0; x < 16 * KVB; ++x) conv_elem(x, cy, s, p, pwo, swo);
  };
  // dV^T += dO^T P and dK^T += Q^T dS of one step (two k-steps of 16 query rows)
  auto contract = [&](const char* __restrict__ t, const u32x4 (&pwi)[KVB][2], const u32x4 (&swi)[KVB][2]) __attribute__((always_inline)) {
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 gt = load_tr_operand_ilv<D>(t, KM + 16 * t2, 32 * db, lane);
        const bf16x8 qt = load_tr_operand_ilv<D>(t, 16 * t2, 32 * db, lane);
#pragma unroll
        for (int kb = 0; kb < KVB; ++kb) {
          mfma32_acc<GENERAL>(dv[kb][db], gt, __builtin_bit_cast(bf16x8, pwi[kb][t2]));
          mfma32_acc<GENERAL>(dk[kb][db], qt, __builtin_bit_cast(bf16x8, swi[kb][t2]));
        }
      }
  };
  // contract(step i) on the matrix core together with convert(step i+1) on the vector ALU: every
  // matrix instruction is followed by the conversion of 32 / (8 DB) elements, and nothing is
  // scheduled across these units, so the two pipes stay busy together.  The transposed operands of
  // a group of four matrix instructions are fetched one group ahead.
  struct FirstX { bf16x8 gt, qt; };                // the first transposed operands of a contraction
  auto first_x = [&](const char* __restrict__ t0) __attribute__((always_inline)) -> FirstX {
    return {load_tr_operand_ilv<D>(t0, KM, 0, lane), load_tr_operand_ilv<D>(t0, 0, 0, lane)};
  };
  // hook(m) is issued right after matrix instruction m.  From instruction NM - 4 on, every LDS
  // read of step i has returned (its last operands are consumed there).
  auto contract_convert = [&](const char* __restrict__ t0,
                              const u32x4 (&pwi)[KVB][2], const u32x4 (&swi)[KVB][2],
                              const f32x16 (&s)[KVB], const f32x16 (&p)[KVB],
                              u32x4 (&pwo)[KVB][2], u32x4 (&swo)[KVB][2], const FirstX& f, auto&& hook) __attribute__((always_inline)) {
    constexpr int NM = 4 * KVB * DB, EPM = (XE + NM - 1) / NM;   // matrix instructions, elements per instruction
    bf16x8 gt[2], qt[2];                           // two operand sets, used alternately
    gt[0] = f.gt;
    qt[0] = f.qt;
    Carry cy;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      const int c = m / (2 * KVB), t2 = c / DB, db = c % DB, j = m % (2 * KVB), cu = c & 1;
      if (j == 0 && c + 1 < 2 * DB) {
        gt[cu ^ 1] = load_tr_operand_ilv<D>(t0, KM + 16 * ((c + 1) / DB), 32 * ((c + 1) % DB), lane);
        qt[cu ^ 1] = load_tr_operand_ilv<D>(t0, 16 * ((c + 1) / DB), 32 * ((c + 1) % DB), lane);
      }
      if (j % 2 == 0) mfma32_acc<GENERAL>(dv[j / 2][db], gt[cu], __builtin_bit_cast(bf16x8, pwi[j / 2][t2]));
      else mfma32_acc<GENERAL>(dk[j / 2][db], qt[cu], __builtin_bit_cast(bf16x8, swi[j / 2][t2]));
#pragma unroll
      for (int x = m * EPM; x < (m + 1) * EPM && x < XE; ++x) {
        const float ex = conv_start(x, s);         // (first: the instruction after it must not read it)
        if (x > 0) conv_finish(x - 1, cy, p, pwo, swo);
        cy.ex = ex;
        if (x == XE - 1) conv_finish(x, cy, p, pwo, swo);
      }
      hook(m);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  constexpr int NM_X = 4 * KVB * DB;               // matrix instructions of a contraction

  // ---- pipeline over the needed steps.  Step number q of the sequence lives in ring stage q % 4.
  // Iteration i contracts step i while converting step i + 1 (already scored); then, at the one
  // barrier of the iteration, every wave is done with step i, whose stage takes step i + 4, and
  // step i + 2 -- issued two iterations ago -- has landed; then step i + 2 is scored.
  DKDV_STAMP(stamp_a);
  int e[NSTG + 1];                                 // step ids of steps i .. i + 4 (static indexing only)
#pragma unroll
  for (int q = 0; q <= NSTG; ++q) e[q] = n_all;
#pragma unroll
  for (int q = 0; q < NSTG; ++q) {
    if (q < n) {
      e[q] = cursor.s;
      issue_tile(cursor, smem + q * SM::STAGE);
      advance(cursor);
    }
  }
  DKDV_STAMP(stamp_b);
  load_kv();
  DKDV_STAMP(stamp_c);
  wait_vmcnt<0>();
  __syncthreads();                                 // V rows and the first tiles are in LDS
  DKDV_STAMP(stamp1);
  const char* const vw = vres + (wave * 32 * KVB + kl) * SM::P + g * 16;

  f32x16 s[KVB], p[KVB];
  u32x4 pf0[KVB][2] = {}, sf0[KVB][2] = {}, pf1[KVB][2] = {}, sf1[KVB][2] = {};   // packed P and dS operands
  if (n > 0) {
    score(smem, vw, s, p, nothing, first_y(smem, vw), no_tail);
    mask_scores(e[0], s);
    convert(s, p, pf0, sf0);
    if (n > 1) { score(smem + SM::STAGE, vw, s, p, nothing, first_y(smem + SM::STAGE, vw), no_tail); mask_scores(e[1], s); }
  }
  auto mid = [&](auto all_in_flight, bool issue, char* st_copy) __attribute__((always_inline)) {
    // (The general variant may spill registers inside the loop; its spill stores are counted with
    // the copies but complete out of order with them, so it always waits for everything.)
    // all_in_flight: steps i + 2 and i + 3 were both issued, so leaving one step's copies
    // outstanding still guarantees that step i + 2 has landed
    if constexpr (decltype(all_in_flight)::value) wait_vmcnt<NDMA>();
    else wait_vmcnt<0>();
    wg_barrier();
    if (issue) {
      e[4] = cursor.s;
      issue_tile(cursor, st_copy);
      advance(cursor);
    }
  };
  // One full iteration.  Dense variant: the barrier sits inside the contraction, right after the
  // matrix instruction that consumes the last LDS operands of step i; behind it the first operands
  // of the score phase (step i + 2, landed by then) are fetched while the contraction finishes, and
  // the score phase in turn fetches the first operands of the next contraction (step i + 1) and
  // sends out the copies of step i + 4 one at a time between its matrix instructions.
  FirstX fx = first_x(smem);
  FirstY fy;
  auto full_iter = [&](char* st_copy, const char* __restrict__ t0, const char* __restrict__ t1,
                       const char* __restrict__ t2, const char* __restrict__ vw_, const u32x4 (&pfi)[KVB][2],
                       const u32x4 (&sfi)[KVB][2], u32x4 (&pfo)[KVB][2], u32x4 (&sfo)[KVB][2]) __attribute__((always_inline)) {
    auto next_x = [&]() __attribute__((always_inline)) { fx = first_x(t1); };
    if constexpr (GENERAL) {
      contract_convert(t0, pfi, sfi, s, p, pfo, sfo, fx, nothing);
      mid(std::false_type{}, true, st_copy);
      score(t2, vw_, s, p, nothing, first_y(t2, vw_), next_x);
    } else {
      contract_convert(t0, pfi, sfi, s, p, pfo, sfo, fx, [&](int m) __attribute__((always_inline)) {
        if (m == NM_X - 4) {
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // (nothing is in flight here any more)
          mid(std::true_type{}, false, st_copy);
          asm volatile("" ::: "memory");
        }
        if (m == NM_X - 3) fy = first_y(t2, vw_);
      });
      e[4] = cursor.s;
      const Tile tl = tile_of(cursor, st_copy);
      advance(cursor);
      constexpr int NU = 2 * KVB * KS, EVERY = NU / NDMA;
      static_assert(EVERY >= 1, "more copies than matrix instructions in the score phase");
      score(t2, vw_, s, p, [&](int m) __attribute__((always_inline)) {
        if (m % EVERY == EVERY - 1 && m / EVERY < NDMA) issue_part(tl, m / EVERY);
      }, fy, next_x);
    }
    mask_scores(e[2], s);
    e[0] = e[1]; e[1] = e[2]; e[2] = e[3]; e[3] = e[4];
  };
  auto stage = [&](int q) __attribute__((always_inline)) -> char* { return smem + (q % NSTG) * SM::STAGE; };
  int i = 0;
  while (i + 5 < n) {                              // two full iterations per trip, each issuing a step
    full_iter(stage(i), stage(i), stage(i + 1), stage(i + 2), vw, pf0, sf0, pf1, sf1);
    full_iter(stage(i + 1), stage(i + 1), stage(i + 2), stage(i + 3), vw, pf1, sf1, pf0, sf0);
    i += 2;
  }
  for (; i < n; ++i) {                             // the last (at most five) iterations
    contract(stage(i), pf0, sf0);
    mid(std::false_type{}, i + 4 < n, stage(i));
    if (i + 1 < n) convert(s, p, pf0, sf0);
    if (i + 2 < n) { score(stage(i + 2), vw, s, p, nothing, first_y(stage(i + 2), vw), no_tail); mask_scores(e[2], s); }
    e[0] = e[1]; e[1] = e[2]; e[2] = e[3]; e[3] = e[4];
  }

  DKDV_STAMP(stamp2);
  // ---- write dK = scale * acc, dV = acc (transposed accumulators: lane = key row).  The last
  // matrix instructions must have retired before their registers are read.
  // (the accumulators are operands of the statement, so that the compiler cannot read them before it)
#pragma unroll
  for (int kb = 0; kb < KVB; ++kb) {
    if constexpr (DB == 4)
      asm volatile("s_nop 15\n\ts_nop 15" : "+a"(dk[kb][0]), "+a"(dk[kb][1]), "+a"(dk[kb][2]), "+a"(dk[kb][3]),
                   "+a"(dv[kb][0]), "+a"(dv[kb][1]), "+a"(dv[kb][2]), "+a"(dv[kb][3]));
    else if constexpr (DB == 3)
      asm volatile("s_nop 15\n\ts_nop 15" : "+a"(dk[kb][0]), "+a"(dk[kb][1]), "+a"(dk[kb][2]),
                   "+a"(dv[kb][0]), "+a"(dv[kb][1]), "+a"(dv[kb][2]));
    else
      asm volatile("s_nop 15\n\ts_nop 15" : "+a"(dk[kb][0]), "+a"(dk[kb][1]), "+a"(dv[kb][0]), "+a"(dv[kb][1]));
  }
  // A lane holds one key row, four columns at a time: stored as they are, every instruction
  // would touch 32 rows with 16 bytes each.  Each wave turns its rows around through LDS instead
  // (the ring and the V rows are free once every wave has left the loop) and writes whole
  // 256-byte rows, 16 bytes per lane.
  __syncthreads();
  constexpr int RP = D * 2 + 16;                   // row pitch of the turn-around buffer (padded against bank conflicts)
  static_assert(NWV * 2 * 32 * KVB * RP <= SM::RING, "the turn-around buffers fit the ring and V area");
  char* const tk = smem + wave * (2 * 32 * KVB * RP);
  char* const tv = tk + 32 * KVB * RP;
#pragma unroll
  for (int kb = 0; kb < KVB; ++kb)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int col = 32 * db + 8 * q4 + 4 * g;
        u32x2 yk = {pack2_bf16(dk[kb][db][4 * q4] * d.scale, dk[kb][db][4 * q4 + 1] * d.scale),
                    pack2_bf16(dk[kb][db][4 * q4 + 2] * d.scale, dk[kb][db][4 * q4 + 3] * d.scale)};
        u32x2 yv = {pack2_bf16(dv[kb][db][4 * q4], dv[kb][db][4 * q4 + 1]),
                    pack2_bf16(dv[kb][db][4 * q4 + 2], dv[kb][db][4 * q4 + 3])};
        *(u32x2*)(tk + (32 * kb + kl) * RP + col * 2) = yk;
        *(u32x2*)(tv + (32 * kb + kl) * RP + col * 2) = yv;
      }
  // (each wave reads back only what it wrote itself: no barrier, the LDS queue keeps the order)
  constexpr int LPR = D / 8;                       // lanes per row, eight bf16 each
  constexpr int RPI = 64 / LPR;                    // rows per instruction
  constexpr bool EVEN = 64 % LPR == 0 && (32 * KVB) % RPI == 0;   // else: idle lanes, and a last instruction with fewer rows
  const int rsub = lane / LPR, cb = (lane % LPR) * 16;
#pragma unroll 4
  for (int r0 = 0; r0 < 32 * KVB; r0 += RPI) {
    const int r = r0 + rsub, j = j_wave0 + r;
    if (!EVEN && (rsub >= RPI || r >= 32 * KVB)) continue;
    const u32x4 yk = *(const u32x4*)(tk + r * RP + cb);
    const u32x4 yv = *(const u32x4*)(tv + r * RP + cb);
    if (j >= d.Skv) continue;
    const long off = (b * d.kv_sb + hk * d.kv_sh + (long)j * d.kv_ss) * 2 + cb;
    *(u32x4*)((char*)a.dk + off) = yk;
    *(u32x4*)((char*)a.dv + off) = yv;
  }
#ifdef LVX_DKDV_PROBE
  wait_vmcnt<0>();
  const unsigned long long stamp3 = __builtin_readcyclecounter();
  if (tid == 0) {
    atomicAdd(&dkdv_probe[0], stamp1 - stamp0);
    atomicAdd(&dkdv_probe[1], stamp2 - stamp1);
    atomicAdd(&dkdv_probe[2], stamp3 - stamp2);
    atomicAdd(&dkdv_probe[3], 1ull);
    atomicAdd(&dkdv_probe[4], (unsigned long long)n);
    atomicAdd(&dkdv_probe[5], stamp_a - stamp0);     // of the set-up: until the first tile copy goes out,
    atomicAdd(&dkdv_probe[6], stamp_b - stamp_a);    // issuing the first four steps' copies,
    atomicAdd(&dkdv_probe[7], stamp_c - stamp_b);    // K and V from memory into registers and LDS (the rest: the last wait)
  }
#endif
}

template <int D, bool GENERAL, bool STEPS = false>
hipError_t launch(const BwdArgs& a, hipStream_t s) {
  const long grid = xcd_grid(a.d.B * a.d.Hkv, (a.d.Skv + DkvSmem<D, kvb_of(GENERAL)>::KN - 1) / DkvSmem<D, kvb_of(GENERAL)>::KN);
  static SmemOnce once;
  using SM = DkvSmem<D, kvb_of(GENERAL)>;
  hipError_t e = ensure_dynamic_lds((const void*)bwd_dkdv_bf16_kernel<D, GENERAL, STEPS>, SM::TOTAL, &once);
  if (e != hipSuccess) return e;
  bwd_dkdv_bf16_kernel<D, GENERAL, STEPS><<<(unsigned)grid, 256, SM::TOTAL, s>>>(a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_bwd_dkdv_bf16(const BwdArgs& a, hipStream_t s) {
  const Dims& d = a.d;
  // a mask that only selects whole steps for whole workgroups runs on the dense kernel
  const bool rows_ok = d.Sq % KM == 0 || d.Sq >= KM;           // (a ragged Sq needs 32 rows to overlap)
  const bool steps = a.mask.allow != nullptr && rows_ok && a.mask.q_chunk % KM == 0 &&
                     a.mask.kv_block % DkvSmem<128, 2>::KN == 0 && (d.Sq + KM - 1) / KM <= dkdv_step_list_cap<128>();
  static_assert(DkvSmem<64, 2>::KN == DkvSmem<128, 2>::KN && dkdv_step_list_cap<64>() == dkdv_step_list_cap<128>() &&
                DkvSmem<96, 2>::KN == DkvSmem<128, 2>::KN && dkdv_step_list_cap<96>() == dkdv_step_list_cap<128>(),
                "the test above is the same for both head dims");
  if (steps) return d.D == 64 ? launch<64, false, true>(a, s) : d.D == 96 ? launch<96, false, true>(a, s) : launch<128, false, true>(a, s);
  const bool general = a.mask.allow != nullptr || !rows_ok;
  if (d.D == 64) return general ? launch<64, true>(a, s) : launch<64, false>(a, s);
  if (d.D == 96) return general ? launch<96, true>(a, s) : launch<96, false>(a, s);
  return general ? launch<128, true>(a, s) : launch<128, false>(a, s);
}

}  // namespace lvx

#ifdef LVX_DKDV_PROBE
extern "C" int lvx_debug_dkdv_probe(unsigned long long* out8) {
  if (hipDeviceSynchronize() != hipSuccess) return 1;
  if (hipMemcpyFromSymbol(out8, HIP_SYMBOL(lvx::dkdv_probe), 8 * sizeof(unsigned long long)) != hipSuccess) return 1;
  const unsigned long long z[8] = {};
  return hipMemcpyToSymbol(HIP_SYMBOL(lvx::dkdv_probe), z, sizeof(z)) == hipSuccess ? 0 : 1;
}
#endif
