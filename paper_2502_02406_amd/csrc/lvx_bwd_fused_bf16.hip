// bf16 backward, all five matrix products of Table 1 in one key-stationary kernel: S and dP are
// formed once and feed dV, dK AND dQ (the two-kernel backward forms them twice: 14 units of work
// for the 10 that Table 1 counts).  Probabilities are recomputed from the saved statistic L
// (Section 3.2 saves only x, O and L):
//   p_ij = exp(scale <Q_i, K_j> - L_i),   dS_ij = p_ij (<dO_i, V_j> - delta_i).
//
// Workgroup = 4 wavefronts = 256 keys of one (batch, K/V head), one wave per SIMD with the whole
// register file.  A wave owns 64 keys (two 32-key blocks): their dK^T / dV^T accumulators fill the
// accumulation registers, their V operands sit in ordinary registers, and K' = bf16(K scale log2 e)
// of all 256 keys stays in LDS, where it serves two products: S = Q K'^T (plain reads, one key
// per lane) and dQ += dS K' (transposing reads, keys along the contraction).
// The query rows of all heads that share the K/V head are streamed 32 at a time ("steps"): [Q; dO]
// tiles and their 64 row statistics travel HBM -> LDS by direct copies into a ring of three stages.
// S and dP put one KEY per lane and 16 query rows in a lane's registers, so P and dS, rounded to
// bf16, are already the B operands of dV^T += dO^T P and dK^T += Q^T dS.  For dQ the keys must lie
// along the contraction instead: every wave leaves its dS (64 keys x 32 rows, bf16) in LDS, and
// after the step's barrier each wave forms ONE 32 x 32 block of dQ^T -- its quarter of the head
// dimension -- over all 256 keys, with K'^T and dS^T both fetched by transposing reads.
//
// dQ across workgroups.  Every workgroup of a K/V head adds a 32 x D tile per step to the same
// float32 array.  Float atomics are far too slow for that (about 8e10 elements/s on this chip
// against the 5e11 needed), so a wave takes a lock on its quarter of the tile, loads the old values
// straight into the accumulator of its dQ product, and stores the result back.  All of this
// traffic bypasses the caches that are not coherent between XCDs (agent-scope accesses), so it is
// correct wherever the hardware places the workgroups.  Locks are taken two steps ahead and
// released two steps late, so that no round trip is waited for; a wave never spins on a lock while
// it holds a later one in step order, and the walk over the steps is cut where it wraps around, so
// no cycle of waiting waves can form.  Spins are bounded: a wave that gives up sets the error word
// of the workspace and goes on, so the kernel always ends.
// The tiles are kept in the register order of the matrix instruction ("fragment order": one
// kilobyte per load or store instruction) in a workspace; dq_tiles_add_kernel adds them to dq_accum.
#include "lvx_internal.h"
#include "lvx_mfma.h"

#include <type_traits>

// Measurement builds only (python -m paper_2502_02406_amd.build --define LVX_PROBE=<bits>): parts of
// the kernel switched off to see what each costs.  RESULTS ARE WRONG with any bit set.
//   1  no dQ product (its matrix instructions and operand reads)
//   2  no loads of old dQ tiles (the accumulation starts from zero)
//   4  no stores of dQ tiles inside the loop (one store at the very end keeps the product alive)
//   8  no locks
//  16  cycle counters per wave, added up in the words after the error word: cycles waited for
//      memory before a step's barrier, cycles inside the barrier, cycles of the whole kernel, waves
#ifndef LVX_PROBE
#define LVX_PROBE 0
#endif

namespace lvx {

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr int NWV = 4;                 // waves per workgroup
constexpr int KVB = 2;                 // 32-key blocks per wave
constexpr int KM = 32;                 // query rows per step
constexpr int NSTG = 3;                // ring stages
constexpr int KN = NWV * 32 * KVB;     // keys per workgroup
constexpr int SPIN_LIMIT = 1 << 18;    // tries for a lock before a wave gives up (each with a short sleep)

// dK^T / dV^T accumulation, written out so that the accumulators stay in the accumulation file by
// construction (the compiler does not know this is a matrix instruction; nothing else touches
// the accumulators until the epilogue).
__device__ __forceinline__ void mfma32_acc(f32x16& acc, bf16x8 a, bf16x8 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

template <int D> struct FusedSmem {
  static constexpr int CPR = D / 8;                 // 16-byte chunks of data per row
  static constexpr int P = (D + 8) * 2;             // row pitch in bytes
  static constexpr int SPR = P / 16;                // 16-byte slots per row
  // [Q; dO] tile: 64 logical rows (Q 0..31, dO 32..63); logical row r lives in group r % 4 at row
  // r / 4; a group is 16 rows plus 64 bytes, which puts the groups 64 bytes apart modulo 256: b128
  // reads of one column chunk by 16 consecutive logical rows and transposing reads of 4
  // consecutive logical rows x 64 bytes are then both free of bank conflicts.
  static constexpr int GS = 16 * P + 64;
  static constexpr int TILE = 4 * GS;
  static constexpr int STAT_OFF = TILE;             // 32 x -L log2(e), then 32 x -delta
  static constexpr int STAGE = TILE + 256;
  static constexpr int RUN = 8 * SPR;               // slots of one run: 8 consecutive rows of a group
  static constexpr int NCR = (RUN + 63) / 64;       // wave-level copies (64 slots) per run
  // K' of the workgroup's 256 keys, the same interleaving with groups of 64 rows
  static constexpr int KGS = 64 * P + 64;
  static constexpr int K_BYTES = 4 * KGS;
  // dS of one step: 64 bytes per key, as four chunks of 16.  Query row r = 8 q4 + 4 gw + e (the
  // registers of a score block: q4 = 0..3, gw the half-wave, e = 0..3) lives in chunk 2 gw + q4 / 2,
  // at byte 8 (q4 % 2) + 2 e: a lane's eight values of one half of the rows (its B operand of dK)
  // are one chunk, written and read back whole.  Chunk h of key j is stored at slot h ^ (j / 4 % 4):
  // b128 accesses of 16 consecutive keys and transposing reads of 4 keys x 64 bytes then touch
  // every bank once.
  static constexpr int DS_BYTES = KN * 64;
  // the two dS buffers come first, so that one address bit tells them apart
  static constexpr int OFF_DS = 0;
  static constexpr int OFF_RING = 2 * DS_BYTES;
  static constexpr int OFF_K = OFF_RING + NSTG * STAGE;
  static constexpr int TOTAL = OFF_K + K_BYTES;
  static_assert((DS_BYTES & (DS_BYTES - 1)) == 0, "the buffers are told apart by one address bit");
  static_assert(GS % 256 == 64 && KGS % 256 == 64, "groups must sit 64 bytes apart modulo 256");
  static_assert(TOTAL <= 160 * 1024, "LDS of one compute unit");
};

// byte offset of logical row rl + rc (rc a compile-time multiple of 4) of a [Q; dO] tile
template <int D> __device__ __forceinline__ int qg_off(int rl, int rc, int colb) {
  return (rl & 3) * FusedSmem<D>::GS + ((rl >> 2) + (rc >> 2)) * FusedSmem<D>::P + colb;
}
template <int D> __device__ __forceinline__ int kres_off(int rl, int rc, int colb) {
  return (rl & 3) * FusedSmem<D>::KGS + ((rl >> 2) + (rc >> 2)) * FusedSmem<D>::P + colb;
}
__device__ __forceinline__ bf16x8 join8(s16x4 lo, s16x4 hi) {
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  s16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// One lock word per dQ tile.  Agent scope, relaxed: the data path carries its own cache
// policy, and the order of data accesses against lock accesses is kept with explicit waits.
typedef int __attribute__((address_space(1))) gint;
__device__ __forceinline__ int lock_try(int* lk) {          // 0 = taken by this call
  if (LVX_PROBE & 8) return 0;
  return __hip_atomic_exchange((gint*)lk, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void lock_release(int* lk) {
  if (LVX_PROBE & 8) return;
  __hip_atomic_store((gint*)lk, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
bwd_fused_bf16_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  using SM = FusedSmem<D>;
  constexpr int KS = D / 16, DB = D / 32, CPR = SM::CPR, NCR = SM::NCR;
  static_assert(DB == NWV, "each wave forms one 32-column block of dQ");

  const Dims& d = a.d;
  const int G = d.Hq / d.Hkv;
  const int n_kt = d.Skv / KN;                     // (the host passes whole tiles only)
  HeadWork hw;
  if (!xcd_decode(blockIdx.x, d.B * d.Hkv, n_kt, &hw)) return;
  const int b = hw.head / d.Hkv, hk = hw.head % d.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, kl = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j_wg0 = hw.item * KN;
  const int j_wave0 = j_wg0 + wave * 32 * KVB;

  // ---- steps: the G heads of the group, KM rows at a time; step id s = head * spH + row tile.
  // When Sq is no multiple of 32 the last step of a head takes rows Sq-32 .. Sq-1 with the
  // statistics of BwdArgs::stats_ovl, in which the rows seen before contribute nothing.
  const int spH = (d.Sq + KM - 1) / KM;
  const int n_all = G * spH;
  // the walk starts at a step that differs from one key tile to the next, so that the workgroups
  // of a head do not queue up for the same dQ tile, and is cut in two where it wraps around
  const int s_start = (int)(((long)hw.item * a.dq_stagger) % n_all);

  char* const kres = smem + SM::OFF_K;

  // ---- tile copies (the layout of the copies follows the interleaved tile: the logical rows
  // 4 j + w, j = 0..7, of Q occupy 8 consecutive rows of group w and those of dO the next 8: a
  // "run"; wave w copies the two runs of group w, each with NCR wave-level copies of 64 slots)
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
  constexpr int NDMA = 2 * NCR + 1;                // copies per wave and step
  struct Tile { const char *qb, *gb, *lb; char* dst; };
  auto tile_of = [&](int h, int t, char* st) __attribute__((always_inline)) -> Tile {   // row tile t of head h of the group
    const int hq = hk * G + h, i0 = t * KM;
    const int i0_eff = min(i0, d.Sq - KM);
    Tile tl;
    const long off = ((long)hq * d.q_sh + (long)i0_eff * d.q_ss) * 2 + (long)wave * row_bytes;
    tl.qb = q0 + off;
    tl.gb = g0 + off;
    const long lb_std = (long)(uintptr_t)l0 + ((long)hq * a.sq_pad + i0) * 8;
    const long lb_ovl = (long)(uintptr_t)a.stats_ovl + ((long)b * d.Hq + hq) * 256;
    const long pick = -(long)(i0 != i0_eff);       // all ones for the short step
    tl.lb = (const char*)(uintptr_t)(lb_std + ((lb_ovl - lb_std) & pick));
    tl.dst = st;
    return tl;
  };
  const unsigned smem_u = lds_base(smem);
  auto issue_part = [&](const Tile& t, int k) __attribute__((always_inline)) {
    const unsigned dst = smem_u + (unsigned)(t.dst - smem), qdst = dst + wave * SM::GS;
    if (k == NDMA - 1) dma4u(t.lb, lane * 4, dst + SM::STAT_OFF);
    else if (k % 2 == 0) dma16u(t.qb, cp_off[k / 2], qdst + run_start(k / 2) * 16);
    else dma16u(t.gb, cp_off[k / 2], qdst + 8 * SM::P + run_start(k / 2) * 16);
  };
  auto issue_tile = [&](int s, char* st) __attribute__((always_inline)) {     // (divides: not for the steady state)
    const Tile t = tile_of(s / spH, s % spH, st);
#pragma unroll
    for (int k = 0; k < NDMA; ++k) issue_part(t, k);
  };

  // ---- dQ tiles of this wave: its quarter (32 columns) of tile s is one kilobyte per q4 at
  // dq_tiles + (tile * 4 + wave) * 4 KB, lane l's four floats at l * 16
  const long tile0 = ((long)b * d.Hq + (long)hk * G) * spH;         // first tile of this head group
  const __amdgpu_buffer_rsrc_t dq_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (char*)a.dq_tiles + (tile0 * 4 + wave) * 4096, 0, (int)((long)n_all * 16384), 0x00020000);
  int* const lock0 = a.dq_locks + tile0;            // one lock per tile, handled by wave 0 for the workgroup
  auto lock_of = [&](int s) __attribute__((always_inline)) -> int* { return lock0 + s; };
  constexpr int AGENT = 16;                        // cache policy of the buffer accesses: sc1
  // This wave's block of dQ^T (lane = query row, registers = columns): `dq` is the accumulator of
  // the step being contracted and what is stored afterwards; `dq_old` receives the old values of
  // the NEXT step's tile, which that step's first dQ instruction takes as its starting value.  Two
  // sets, because the loads must be issued BEFORE the stores: vector-memory operations retire in
  // issue order, so whatever is waited for after a store waits for the store, and an agent-scope
  // store takes far longer than a load.
  f32x16 dq, dq_old;
  unsigned long long pr_wait = 0, pr_bar = 0;
  const unsigned long long pr_t0 = (LVX_PROBE & 16) ? __builtin_readcyclecounter() : 0;
  bool probe_final = false;
  if (LVX_PROBE & 2) dq_old = zero16();
  const int dq_voff = lane * 16;
  auto dq_load_part = [&](int s, int q4) __attribute__((always_inline)) {
    if (LVX_PROBE & 2) return;
    const u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(dq_rsrc, dq_voff, s * 16384 + q4 * 1024, AGENT);
#pragma unroll
    for (int e = 0; e < 4; ++e) dq_old[4 * q4 + e] = __uint_as_float(x[e]);
  };
  auto dq_store_part = [&](int s, int q4) __attribute__((always_inline)) {
    if ((LVX_PROBE & 4) && !probe_final) return;
    const u32x4 x = {__float_as_uint(dq[4 * q4]), __float_as_uint(dq[4 * q4 + 1]), __float_as_uint(dq[4 * q4 + 2]),
                     __float_as_uint(dq[4 * q4 + 3])};
    __builtin_amdgcn_raw_buffer_store_b128(x, dq_rsrc, dq_voff, s * 16384 + q4 * 1024, AGENT);
  };
  auto dq_load = [&](int s) __attribute__((always_inline)) {
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) dq_load_part(s, q4);
  };
  auto dq_store = [&](int s) __attribute__((always_inline)) {
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) dq_store_part(s, q4);
  };
  // lane 0 tries until it has the lock; a wave that gives up reports it and goes on
  auto lock_spin = [&](int* lk) __attribute__((always_inline)) {
    if (LVX_PROBE & 8) return;
    if (lane == 0) {
      int tries = 0;
      while (lock_try(lk) != 0) {
        if (++tries > SPIN_LIMIT) { __hip_atomic_store((gint*)a.dq_err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break; }
        __builtin_amdgcn_s_sleep(4);
      }
    }
  };

  f32x16 dk[KVB][DB], dv[KVB][DB];
#pragma unroll
  for (int kb = 0; kb < KVB; ++kb)
#pragma unroll
    for (int i = 0; i < DB; ++i) { dk[kb][i] = zero16(); dv[kb][i] = zero16(); }

  // ---- first tiles of the first segment, then K' -> LDS and V -> registers
  const int n_seg0 = n_all - s_start;              // steps of the first segment (>= 1)
#pragma unroll
  for (int q = 0; q < NSTG; ++q)
    if (q < n_seg0) issue_tile(s_start + q, smem + SM::OFF_RING + q * SM::STAGE);

  const float c2 = d.scale * LOG2E;
  bf16x8 vf[KVB][KS];
  {
    // Rows are fetched whole (16 lanes per 256-byte row).  Each wave parks its 64 V rows in its
    // own slice of the K' area, reads its operands back, and only then K' is stored there.
    constexpr int WR = 32 * KVB;
    constexpr int VIT = WR * CPR / 64, KIT = KN * CPR / 256;
    u32x4 vy[VIT], ky[KIT];
    const uint16_t* const kg = (const uint16_t*)a.k + b * d.kv_sb + hk * d.kv_sh;
    const uint16_t* const vg = (const uint16_t*)a.v + b * d.kv_sb + hk * d.kv_sh;
#pragma unroll
    for (int it = 0; it < VIT; ++it) {
      const int c = it * 64 + lane, r = c / CPR, col = (c % CPR) * 8;
      vy[it] = *(const u32x4*)(vg + (long)(j_wave0 + r) * d.kv_ss + col);
    }
#pragma unroll
    for (int it = 0; it < KIT; ++it) {
      const int c = it * 256 + tid, r = c / CPR, col = (c % CPR) * 8;
      ky[it] = *(const u32x4*)(kg + (long)(j_wg0 + r) * d.kv_ss + col);
    }
    char* const vst = kres + wave * WR * SM::P;
#pragma unroll
    for (int it = 0; it < VIT; ++it) {
      const int c = it * 64 + lane, r = c / CPR, col = (c % CPR) * 8;
      *(u32x4*)(vst + r * SM::P + col * 2) = vy[it];
    }
#pragma unroll
    for (int kb = 0; kb < KVB; ++kb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        vf[kb][ks] = *(const bf16x8*)(vst + (32 * kb + kl) * SM::P + (16 * ks + 8 * g) * 2);
#pragma unroll
    for (int kb = 0; kb < KVB; ++kb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(vf[kb][ks]));
    __syncthreads();                               // every wave has its V operands
#pragma unroll
    for (int it = 0; it < KIT; ++it) {
      const int c = it * 256 + tid, r = c / CPR, col = (c % CPR) * 8;
      u32x4 x = ky[it];
#pragma unroll
      for (int w = 0; w < 4; ++w)
        x[w] = pack2_bf16(__uint_as_float(x[w] << 16) * c2, __uint_as_float(x[w] & 0xffff0000u) * c2);
      *(u32x4*)(kres + kres_off<D>(r, 0, col * 2)) = x;
    }
  }

  // ---- lane constants of the LDS accesses
  // K' rows of this lane's keys (B operand of S): key 64 wave + 32 kb + kl, columns 16 ks + 8 g
  const int krow_off = SM::OFF_K + kres_off<D>(kl, 64 * wave, 16 * g);
  // K'^T (A operand of dQ): rows = this wave's 32 columns, k = keys
  const int jj = lane & 15, half = (lane >> 4) & 1;
  const int ktb_off = SM::OFF_K + kres_off<D>(4 * g + (jj >> 2), 0, (32 * wave + 16 * half + 4 * (jj & 3)) * 2);
  // dS chunks this lane writes (and reads back for dK): key 64 wave + 32 kb + kl, chunk 2 g + t2, at
  // ds_w0 ^ (16 t2) (+ 2048 kb).  ds_w0 addresses the buffer being written, ds_o the same chunks in
  // the buffer being read; both (and ds_r) change buffers every iteration by flipping one address bit.
  static_assert(SM::OFF_DS == 0, "the offsets below are LDS addresses");
  int ds_w0 = (64 * wave + kl) * 64 + (((2 * g) ^ (kl >> 2)) & 3) * 16;
  int ds_o = ds_w0;
  // dS^T (B operand of dQ): lane = query row 16 half + i of the transposing read's group, k = keys
  // 16 kk + 8 h + 4 g + (jj >> 2); the lane supplies rows 16 half + 4 (jj & 3) .. + 3 of its key:
  // chunk 2 (jj & 1) + half, byte 8 ((jj >> 1) & 1); key / 4 % 4 = (2 h + g) % 4, so h flips bit 5
  int ds_r[2];
  ds_r[0] = (4 * g + (jj >> 2)) * 64 + (((2 * (jj & 1) + half) ^ g) & 3) * 16 + ((jj >> 1) & 1) * 8;
  ds_r[1] = ds_r[0] ^ 32;
  auto ds_flip = [&]() __attribute__((always_inline)) {
    ds_w0 ^= SM::DS_BYTES;
    ds_o ^= SM::DS_BYTES;
#pragma unroll
    for (int v = 0; v < 2; ++v) ds_r[v] ^= SM::DS_BYTES;
  };

  // ---- building blocks ------------------------------------------------------------------------
  f32x16 s[KVB], p[KVB];                           // S and dP of the step being scored / converted
  u32x4 pf[KVB][2] = {};                           // packed P of the step being contracted

  // S = Q K'^T and dP = dO V^T of the step in stage t (lane = key, registers = query rows); both
  // accumulations start from the rows' statistics, -L log2 e and -delta, so that S is already the
  // exponent of P and dP - delta needs no instruction.  hook(m) runs after matrix instruction m.
  auto score = [&](const char* __restrict__ t, auto&& hook) __attribute__((always_inline)) {
    const char* qrow = t + qg_off<D>(kl, 0, 16 * g);
    const char* grow = t + qg_off<D>(kl, KM, 16 * g);
    int krow_v = krow_off;
    asm volatile("" : "+v"(krow_v));                // (see the contraction phase)
    const char* const krow = smem + krow_v;
    // (the statistics are read once per accumulator, straight into its registers: a separate copy
    // would be 32 more registers alive at the point where the kernel has the fewest to spare)
#pragma unroll
    for (int kb = 0; kb < KVB; ++kb) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4 x = *(const f32x4*)(t + SM::STAT_OFF + (8 * q4 + 4 * g) * 4);
        const f32x4 y = *(const f32x4*)(t + SM::STAT_OFF + 128 + (8 * q4 + 4 * g) * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { s[kb][4 * q4 + e] = x[e]; p[kb][4 * q4 + e] = y[e]; }
      }
      asm volatile("" ::: "memory");               // (keeps the two reads apart: merged, they would need the copy)
    }
    // One set of operand registers: an operand of the next k-step is fetched as soon as the last
    // matrix instruction that reads the current one has been issued (three instructions ahead of
    // its first use).
    bf16x8 qa, ga, ka[KVB];
    qa = *(const bf16x8*)qrow;
#pragma unroll
    for (int kb = 0; kb < KVB; ++kb) ka[kb] = *(const bf16x8*)(krow + kb * 8 * SM::P);
    ga = *(const bf16x8*)grow;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int j = 0; j < 2 * KVB; ++j) {
        const int kb = j % KVB;
        if (j < KVB) s[kb] = mfma32(qa, ka[kb], s[kb]);
        else p[kb] = mfma32(ga, vf[kb][ks], p[kb]);
        if (ks + 1 < KS) {
          if (j == KVB - 1) {
            qa = *(const bf16x8*)(qrow + (ks + 1) * 32);
#pragma unroll
            for (int k2 = 0; k2 < KVB; ++k2) ka[k2] = *(const bf16x8*)(krow + k2 * 8 * SM::P + (ks + 1) * 32);
          }
          if (j == 2 * KVB - 1) ga = *(const bf16x8*)(grow + (ks + 1) * 32);
        }
        hook(ks * 2 * KVB + j);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  auto nothing = [](int) __attribute__((always_inline)) {};

  // Conversion of element x of a step (x = 0 .. 31: query rows q4 = x / 8 of key block kb =
  // (x / 4) % 2, row e = x % 4 of the four): p = exp2(s), dS = p dP, packed in pairs as bf16.  P goes
  // into the operand registers; dS of four rows goes to LDS (the buffer ds_w0 addresses) as one unit.
  struct Carry { float pr, ds; unsigned w0; unsigned u[KVB][2]; };
  auto conv_elem = [&](int x, Carry& cy) __attribute__((always_inline)) {
    const int q4 = x / (4 * KVB), kb = (x / 4) % KVB, e = x % 4, v = 4 * q4 + e;
    const float pr = __builtin_amdgcn_exp2f(s[kb][v]);
    const float ds = pr * p[kb][v];
    if (e % 2 == 0) { cy.pr = pr; cy.ds = ds; return; }
    pf[kb][q4 >> 1][2 * (q4 & 1) + e / 2] = pack2_bf16(cy.pr, pr);
    const unsigned w = pack2_bf16(cy.ds, ds);
    if (e == 1) { cy.w0 = w; return; }
    if (q4 % 2 == 0) { cy.u[kb][0] = cy.w0; cy.u[kb][1] = w; return; }
    const u32x4 u = {cy.u[kb][0], cy.u[kb][1], cy.w0, w};      // rows 16 t2 + 4 g .., then 16 t2 + 8 + 4 g ..
    const int t2 = q4 >> 1;
    *(u32x4*)(smem + (t2 == 0 ? ds_w0 : ds_w0 ^ 16) + kb * 32 * 64) = u;
  };

  // The contraction phase of step i (stage t, dS in the buffer ds_o and ds_r address) with the
  // conversion of step i + 1 (dS into the buffer ds_w0 addresses) in its shadow: dV^T += dO^T P (16 matrix instructions), dK^T += Q^T dS (16), then
  // this wave's block of dQ^T += K'^T dS^T over the 256 keys (16).  P of step i + 1 replaces P of
  // step i in the same registers, which is why dV goes first and the conversion starts at the
  // ninth instruction.  (After the last step of a segment the conversion works on stale scores;
  // nothing reads what it leaves.)
  auto contract = [&](const char* __restrict__ t) __attribute__((always_inline)) {
    constexpr int NV = 2 * DB * KVB;               // matrix instructions of dV (and of dK)
    constexpr int NQ = KN / 16;                    // of dQ
    constexpr int NM = 2 * NV + NQ, C0 = NV / 2, XE = 16 * KVB;
    const char* const trb = t + qg_off<D>(4 * g + (jj >> 2), 0, (16 * half + 4 * (jj & 3)) * 2);
    // (Lane constants pass through an empty statement inside the loop: otherwise every address
    // "constant + offset" is itself loop-invariant, gets hoisted, and comes back as an addition in
    // front of each access instead of the instruction's own offset field.)
    int ktb_v = ktb_off, dsr0 = ds_r[0], dsr1 = ds_r[1], dso = ds_o;
    asm volatile("" : "+v"(ktb_v), "+v"(dsr0), "+v"(dsr1), "+v"(dso));
    const char* const ktb_ = smem + ktb_v;
    auto tr_op = [&](int rbase, int n0) __attribute__((always_inline)) -> bf16x8 {
      return join8(lds_read_tr(trb + qg_off<D>(0, rbase, n0 * 2)), lds_read_tr(trb + qg_off<D>(0, rbase + 8, n0 * 2)));
    };
    auto ds_own = [&](int kb, int t2) __attribute__((always_inline)) -> bf16x8 {   // B operand of dK: this lane's key, rows 16 t2 ..
      return *(const bf16x8*)(smem + (t2 == 0 ? dso : dso ^ 16) + kb * 32 * 64);
    };
    auto kt_op = [&](int kk) __attribute__((always_inline)) -> bf16x8 {
      return join8(lds_read_tr(ktb_ + kres_off<D>(0, 16 * kk, 0)), lds_read_tr(ktb_ + kres_off<D>(0, 16 * kk + 8, 0)));
    };
    auto dst_op = [&](int kk) __attribute__((always_inline)) -> bf16x8 {
      return join8(lds_read_tr(smem + dsr0 + (16 * kk) * 64), lds_read_tr(smem + dsr1 + (16 * kk + 8) * 64));
    };
    // Instruction m of the phase: 0 .. NV - 1 are dV; from NV on dK (even) and dQ (odd) alternate.
    // The sixteen dQ instructions accumulate into one block, each waiting for the one before it:
    // with an independent instruction between two of them the matrix pipe never idles.
    bf16x8 at[2];                                  // transposed operands of dV / dK, used alternately
    bf16x8 sb[KVB];                                // dS operands of dK for the current half of the rows
    bf16x8 kt[2], dt[2];                           // operands of dQ, used alternately
    at[0] = tr_op(KM, 0);
    Carry cy;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      const bool is_dq = m >= NV && ((m - NV) & 1) != 0;
      if (is_dq && (LVX_PROBE & 1)) {
      } else if (!is_dq) {
        // u: number of this instruction among the 2 NV of dV and dK
        const int u = m < NV ? m : NV + (m - NV) / 2;
        const bool is_dk = u >= NV;
        const int c = (u % NV) / KVB, t2 = c / DB, db = c % DB, kb = u % KVB, cu = (u / KVB) & 1;
        if (kb == 0 && u + KVB < 2 * NV) {         // the operand of the next pair of these instructions
          const int un = u + KVB, cn = (un % NV) / KVB;
          at[cu ^ 1] = tr_op((un >= NV ? 0 : KM) + 16 * (cn / DB), 32 * (cn % DB));
        }
        if (u == NV - 2) {                         // ... and of the first dQ instruction
          kt[0] = kt_op(0);
          dt[0] = dst_op(0);
        }
        if (is_dk && kb == 0 && db == 0) {
#pragma unroll
          for (int k2 = 0; k2 < KVB; ++k2) sb[k2] = ds_own(k2, t2);
        }
        if (!is_dk) mfma32_acc(dv[kb][db], at[cu], __builtin_bit_cast(bf16x8, pf[kb][t2]));
        else mfma32_acc(dk[kb][db], at[cu], sb[kb]);
      } else {
        const int kk = (m - NV) / 2, cu = kk & 1;
        if (kk + 1 < NQ) {
          kt[cu ^ 1] = kt_op(kk + 1);
          dt[cu ^ 1] = dst_op(kk + 1);
        }
        dq = mfma32(kt[cu], dt[cu], kk == 0 ? dq_old : dq);
      }
      if (m >= C0) {
#pragma unroll
        for (int x = (m - C0) * XE / (NM - C0); x < (m - C0 + 1) * XE / (NM - C0); ++x) conv_elem(x, cy);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto convert_all = [&]() __attribute__((always_inline)) {
    Carry cy;
#pragma unroll
    for (int x = 0; x < 16 * KVB; ++x) conv_elem(x, cy);
  };

  // ---- the two segments of the walk --------------------------------------------------------
  // Within a segment of n steps, step q (q = 0 .. n - 1, step id s0 + q) lives in ring stage q % 3
  // and its dS in buffer q % 2.  Per step i: contraction of step i with the conversion of step
  // i + 1; the one barrier; then the locks (the try of step i + 2 goes out, that of step i + 1 is
  // looked at, that of step i - 2 is released), the old values of step i + 1's dQ block are loaded,
  // the copies of step i + 3 go out, the dQ block of step i is stored, and step i + 2 is scored.
#pragma nounroll
  for (int seg = 0; seg < 2; ++seg) {
    const int s0 = seg == 0 ? s_start : 0;
    const int n = seg == 0 ? n_seg0 : s_start;
    if (n == 0) break;
    if (seg == 1) {
#pragma unroll
      for (int q = 0; q < NSTG; ++q)
        if (q < n) issue_tile(s0 + q, smem + SM::OFF_RING + q * SM::STAGE);
    }
    // lock of the first step (wave 0 takes the locks for the workgroup: per-wave locks would let
    // two workgroups wait for each other through their barriers); the try for the second step
    // goes out as well
    int got_next = 0;                              // result of the try for step i + 1 (wave 0, lane 0)
    if (wave == 0) {
      lock_spin(lock_of(s0));
      if (n > 1 && lane == 0) got_next = lock_try(lock_of(s0 + 1));
    }
    wait_vmcnt<0>();
    __syncthreads();                               // tiles, K', everything in LDS; the first lock is held
    asm volatile("" ::: "memory");
    dq_load(s0);
    char* st_a = smem + SM::OFF_RING;              // stages of steps i, i + 1, i + 2
    char* st_b = st_a + SM::STAGE;
    char* st_c = st_a + 2 * SM::STAGE;
    // dS of the first step goes into buffer 0 and is read from there
    ds_w0 &= SM::DS_BYTES - 1;
    ds_o &= SM::DS_BYTES - 1;
#pragma unroll
    for (int v = 0; v < 2; ++v) ds_r[v] &= SM::DS_BYTES - 1;
    score(st_a, nothing);
    convert_all();
    ds_w0 ^= SM::DS_BYTES;                         // from here on: read from one buffer, write the other
    if (n > 1) score(st_b, nothing);
    __syncthreads();                               // dS of the first step is in LDS

    // The contraction phase of step j, then the workgroup makes sure it owns the lock of step
    // j + 1 (the try went out an iteration ago) and meets at the step's one barrier.  A workgroup
    // waits for a lock only while the locks it holds are of earlier steps, and the try for step
    // j + 2 goes out only after step j + 1 is owned.
    // Vector-memory operations retire in issue order, and the steady state issues the stores of a
    // step's dQ block last: leaving four operations outstanding (stores_last) waits for the tile
    // copies and the loads, not for the stores.
    auto contract_and_meet = [&](int j, bool stores_last) __attribute__((always_inline)) {
      contract(st_a);
      if (wave == 0 && j + 1 < n) {
        if (__builtin_expect(__builtin_amdgcn_readfirstlane(got_next) != 0, 0)) lock_spin(lock_of(s0 + j + 1));
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      unsigned long long t0 = 0, t1 = 0;
      if (LVX_PROBE & 16) t0 = __builtin_readcyclecounter();
      if (stores_last) wait_vmcnt<4>();
      else wait_vmcnt<0>();
      if (LVX_PROBE & 16) t1 = __builtin_readcyclecounter();
      wg_barrier();
      if (LVX_PROBE & 16) { const unsigned long long t2 = __builtin_readcyclecounter(); pr_wait += t1 - t0; pr_bar += t2 - t1; }
      asm volatile("" ::: "memory");
    };
    // What follows the barrier of step i, and then the contraction of step i + 1.  full: steps
    // i + 1 .. i + 3 all exist (the steady state: nothing is conditional, the memory operations go
    // out one at a time between the matrix instructions of the scoring, and the loads of the old dQ
    // values sit in the same basic block as their first use, so that the wait the compiler puts
    // before it counts the stores behind them instead of waiting for everything).
    int h3 = (s0 + 3) / spH, t3 = (s0 + 3) % spH;   // head and row tile of step i + 3
    auto iteration = [&](auto full_t, int i) __attribute__((always_inline)) {
      constexpr bool FULL = decltype(full_t)::value;
      const bool more1 = FULL || i + 1 < n, more2 = FULL || i + 2 < n, more3 = FULL || i + 3 < n;
      // The stores of step i - 2 were issued two iterations ago, before everything the wait before
      // the barrier covered: they have completed in every wave, and its lock can go.
      // (Iterations 0 and 1 have nothing to release and write a spare word instead.)
      if (wave == 0 && lane == 0) {
        lock_release(i > 1 ? lock_of(s0 + i - 2) : a.dq_err + 1);
        if (more2) got_next = lock_try(lock_of(s0 + i + 2));
      }
      asm volatile("" ::: "memory");
      const int sc = __builtin_amdgcn_readfirstlane(s0 + i);   // (wave-uniform; said explicitly for the buffer accesses)
      if (FULL) {
        const Tile tl = tile_of(h3, t3, st_a);
        score(st_c, [&](int m) __attribute__((always_inline)) {
          if (m < NDMA) issue_part(tl, m);
          else if (m < 4 + NDMA) dq_load_part(sc + 1, m - NDMA);
          else if (m < 8 + NDMA) dq_store_part(sc, m - 4 - NDMA);
        });
      } else {
        if (more1) dq_load(sc + 1);
        if (more3) {
          const Tile tl = tile_of(h3, t3, st_a);
#pragma unroll
          for (int k = 0; k < NDMA; ++k) issue_part(tl, k);
        }
        dq_store(sc);
        if (more2) score(st_c, nothing);
      }
      if (++t3 == spH) { t3 = 0; ++h3; }
      char* const t_ = st_a; st_a = st_b; st_b = st_c; st_c = t_;
      ds_flip();
      if (more1) contract_and_meet(i + 1, FULL);
    };
    contract_and_meet(0, false);
    int i = 0;
    for (; i + 3 < n; ++i) iteration(std::true_type{}, i);
    for (; i < n; ++i) iteration(std::false_type{}, i);
    // every wave's stores of the last block must have completed before its lock is released
    wait_vmcnt<0>();
    __syncthreads();                               // (also: the next segment's copies overwrite the stages)
    asm volatile("" ::: "memory");
    if (wave == 0 && lane == 0) {
      if (n > 1) lock_release(lock_of(s0 + n - 2));
      lock_release(lock_of(s0 + n - 1));
    }
  }

  if (LVX_PROBE & 4) { probe_final = true; dq_store(0); }
  if ((LVX_PROBE & 16) && lane == 0) {
    atomicAdd((unsigned long long*)(a.dq_err + 2), pr_wait);
    atomicAdd((unsigned long long*)(a.dq_err + 4), pr_bar);
    atomicAdd((unsigned long long*)(a.dq_err + 6), __builtin_readcyclecounter() - pr_t0);
    atomicAdd((unsigned long long*)(a.dq_err + 8), 1ull);
  }
  // ---- write dK = scale * acc, dV = acc (transposed accumulators: lane = key row).  The last matrix instructions must have retired before their registers are read.
#pragma unroll
  for (int kb = 0; kb < KVB; ++kb) {
    static_assert(DB == 4, "accumulator operands below are written out for four blocks");
    asm volatile("s_nop 15\n\ts_nop 15" : "+a"(dk[kb][0]), "+a"(dk[kb][1]), "+a"(dk[kb][2]), "+a"(dk[kb][3]),
                 "+a"(dv[kb][0]), "+a"(dv[kb][1]), "+a"(dv[kb][2]), "+a"(dv[kb][3]));
  }
  // Each wave turns its rows around through LDS and writes whole 256-byte rows, 16 bytes per lane.
  __syncthreads();
  constexpr int RP = D * 2 + 16;                   // row pitch of the turn-around buffer
  static_assert(NWV * 2 * 32 * KVB * RP <= SM::TOTAL, "the turn-around buffers fit");
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
  constexpr int LPR = D / 8, RPI = 64 / LPR;
  const int rsub = lane / LPR, cb = (lane % LPR) * 16;
#pragma unroll 4
  for (int r0 = 0; r0 < 32 * KVB; r0 += RPI) {
    const int r = r0 + rsub, j = j_wave0 + r;
    const u32x4 yk = *(const u32x4*)(tk + r * RP + cb);
    const u32x4 yv = *(const u32x4*)(tv + r * RP + cb);
    const long off = (b * d.kv_sb + hk * d.kv_sh + (long)j * d.kv_ss) * 2 + cb;
    *(u32x4*)((char*)a.dk + off) = yk;
    *(u32x4*)((char*)a.dv + off) = yv;
  }
}

// dq_accum[b,h,i,:] += ln 2 * (the tiles' values for row i): the tiles hold sum dS K' with
// K' = K scale log2 e.  Row i is row i % 32 of tile i / 32, and -- when Sq is no multiple of 32 --
// the last tile of a head holds rows Sq-32 .. Sq-1 instead, so that a row of the last 32 may
// appear in two tiles (it contributes to one of them only: the other saw zero probabilities).
// One thread per 4 columns.
__global__ void __launch_bounds__(256) dq_tiles_add_kernel(Dims d, const float* tiles, float* dq_accum) {
  const int D = d.D, spH = (d.Sq + KM - 1) / KM;
  const long t = (long)blockIdx.x * 256 + threadIdx.x;
  const int c4 = (int)(t % (D / 4));
  const long row = t / (D / 4);
  if (row >= (long)d.B * d.Hq * d.Sq) return;
  const int i = (int)(row % d.Sq);
  const long bh = row / d.Sq;
  const int col = c4 * 4, w = col / 32, q4 = (col % 32) / 8, gg = (col % 8) / 4;
  auto frag = [&](int tile, int r) -> f32x4 {       // row r of tile `tile`
    return *(const f32x4*)(tiles + (((bh * spH + tile) * 4 + w) * 4 + q4) * 256 + (r + 32 * gg) * 4);
  };
  f32x4 x = {0.f, 0.f, 0.f, 0.f};
  const int last0 = d.Sq - KM;                      // first row of a ragged last tile
  const bool ragged = d.Sq % KM != 0;
  if (!(ragged && i / KM == spH - 1)) x += frag(i / KM, i % KM);
  if (ragged && i >= last0) x += frag(spH - 1, i - last0);
  const float f = 1.0f / LOG2E;
  f32x4* const out = (f32x4*)(dq_accum + row * D + col);
  f32x4 y = *out;
  y[0] += f * x[0]; y[1] += f * x[1]; y[2] += f * x[2]; y[3] += f * x[3];
  *out = y;
}

// zero fill of n 16-byte words (no memset call: callers may capture the stream in a graph)
__global__ void __launch_bounds__(256) fill_zero_kernel(u32x4* p, long n) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = u32x4{0, 0, 0, 0};
}

}  // namespace

bool bwd_fused_bf16_supported(const Dims& d, bool masked) {
  return !masked && d.D == 128 && d.Skv >= KN && d.Sq >= KM;
}

size_t bwd_fused_ws_bytes(const Dims& d) {          // tiles, then lock words and the error word
  const size_t tiles = (size_t)d.B * d.Hq * ((d.Sq + KM - 1) / KM);
  return tiles * 16384 + (tiles * sizeof(int) + 255) / 256 * 256 + 256;
}

hipError_t launch_bwd_fused_bf16(const BwdArgs& a_in, hipStream_t s) {
  BwdArgs a = a_in;
  const Dims& d = a.d;
  const size_t tiles = (size_t)d.B * d.Hq * ((d.Sq + KM - 1) / KM);
  const size_t lock_bytes = (tiles * sizeof(int) + 255) / 256 * 256;
  a.dq_locks = (int*)((char*)a.dq_tiles + tiles * 16384);
  a.dq_err = (int*)((char*)a.dq_locks + lock_bytes);
  const long n16 = (long)((tiles * 16384 + lock_bytes + 256) / 16);
  fill_zero_kernel<<<(unsigned)((n16 + 255) / 256), 256, 0, s>>>((u32x4*)a.dq_tiles, n16);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  a.d.Skv = d.Skv / KN * KN;                        // whole tiles of 256 keys; the caller handles the rest
  a.dq_stagger = 5;
  using SM = FusedSmem<128>;
  static SmemOnce once;
  e = ensure_dynamic_lds((const void*)bwd_fused_bf16_kernel<128>, SM::TOTAL, &once);
  if (e != hipSuccess) return e;
  const long grid = xcd_grid(d.B * d.Hkv, a.d.Skv / KN);
  bwd_fused_bf16_kernel<128><<<(unsigned)grid, 256, SM::TOTAL, s>>>(a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  const long threads = (long)d.B * d.Hq * d.Sq * (d.D / 4);
  dq_tiles_add_kernel<<<(unsigned)((threads + 255) / 256), 256, 0, s>>>(d, a.dq_tiles, a.dq_accum);
  return hipGetLastError();
}

}  // namespace lvx
