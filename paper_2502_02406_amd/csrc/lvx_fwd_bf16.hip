// bf16 forward kernel: the FlashAttention call of Algorithm 1 for a short query block against a
// long local K/V block, on the gfx950 matrix cores.
//
// Workgroup = 4 wavefronts = 256 query rows of one (batch, K/V head) -- the rows of its group of
// query heads, one after the other -- one wave per SIMD with
// the whole register file.  A wave owns 64 query rows (two 32-row blocks): their Q operands and
// the O^T accumulators live in the accumulation registers for the whole kernel, so every K or V
// operand fetched from LDS feeds two matrix instructions.
// K/V tiles of 64 keys travel HBM -> LDS by direct global-to-LDS copies into a ring of four
// stages, issued two tiles ahead, one barrier per tile.
// Transposed tiles S^T = K Q^T put one QUERY per lane (the softmax statistics are per-lane
// scalars; the two half-waves exchange one value per half) and 16 keys in a lane's registers, so
// P^T, rounded to bf16, is already the B operand of O^T += V^T P^T, with V^T fetched by
// transposing LDS reads.
// Online softmax with a lazy reference r per row, in units of log2: p = exp2(s scale log2 e - r).
// r starts as the maximum of the row's first 32 scores.  Later halves are converted against the
// current r without looking at their maximum first; the sum of the 16 probabilities a lane
// produced tells afterwards whether one of them can have topped 2^LAZY, and only then (rarely) r
// is raised to the new maximum, O^T and the sums shrink, and the half is converted again.  The
// result is still exact, since any reference cancels between numerator and denominator.  (Q is not pre-multiplied by the
// scale: rounding the product to bf16 would cost about 1e-3 of L on rows with large scores.)
// The loop runs over 32-key halves and is software pipelined inside each wave: while the matrix
// core contracts half h (O) and scores half h+2 (S), the vector ALU turns the scores of half h+1
// into probabilities; two sets of score registers alternate.
// The grid is cut along the KV axis (split-KV) when the query block alone cannot fill the chip;
// partial (O, L) pairs are combined by the merge kernel.
#include "lvx_internal.h"
#include "lvx_mfma.h"
#include "lvx_kv_ring.h"

#include <type_traits>

namespace lvx {

namespace {

using namespace kvring;
constexpr float LAZY_SUM = 64.0f;      // a lane's 16 probabilities of a half may add up to this (2^LAZY, LAZY = 6)
                                       // before the reference is raised: no probability in use exceeds it
#ifndef LVX_FWD_XE
#define LVX_FWD_XE 8
#endif
#ifndef LVX_MASKED_WG_FACTOR
#define LVX_MASKED_WG_FACTOR 4L
#endif
constexpr int XE = LVX_FWD_XE;                  // elements of a half converted during the contraction (of 32)

// Dense attention with Skv a multiple of 64 only: no mask code and no ragged tile, so that nothing
// stands between the phases of the pipeline (masked and ragged problems: lvx_fwd_general_bf16.hip).
// LIST = 1: the same kernel over a list of key tiles -- those that EVERY row of the workgroup sees
// under a media mask (FwdArgs::pass == 1).  Nothing is masked inside such a tile; only the tile
// numbers come from the list, which the KV splits share evenly.  The other visible tiles are left
// to a launch of the general kernel (pass == 2), and the partial results of both are combined.
// LIST = 2: a mask whose text chunks are multiples of 32 rows and whose key blocks are multiples
// of 64 keys never cuts through a (32-row block, key tile) pair: the list then holds the tiles
// that ANY row of the workgroup sees, each with one bit per 32-row block of the workgroup, and a
// row block that does not see a tile converts its scores against a reference of +infinity --
// every probability is exp2(-inf) = 0 -- so that the whole mask costs two selects per half tile
// and one launch does it all.  (A workgroup moves at the pace of its busiest wave anyway: a wave
// that skipped the tile would wait at the barrier.)
template <int D, int LIST = 0>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
fwd_bf16_kernel(FwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  using SM = KvSmem<D>;
  constexpr int KS = D / 16, DB = D / 32, CPR = SM::CPR, NCR = SM::NCR;

  const Dims& d = a.d;
  const int G = d.Hq / d.Hkv;
  // The query rows of the G heads that share a K/V head are one list of G * Sq rows (row r = head
  // r / Sq of the group, its row r % Sq), cut into tiles of 256: short query blocks -- one
  // worker's share of the text, or a single token -- then fill tiles instead of leaving one
  // mostly empty tile per head, and every K/V tile fetched serves all heads of the group.
  // (LIST tiles the rows of each head by itself: a mask works on the rows of one head)
  constexpr bool PACK = !LIST;
  const int rows_kv = PACK ? G * d.Sq : d.Sq;
  const int n_qt = (rows_kv + QM - 1) / QM;
  const int per_split = PACK ? n_qt : G * n_qt;
  int b, hk, split, hq0, qt;
  if constexpr (LIST == 2) {
    // Under a mask the query tiles of a head differ in how many key tiles they see (under a causal
    // one, the later the tile the more).  Workgroups start in the order of their numbers: the later
    // query tiles go first, so that the short ones fill the gaps the long ones leave at the end;
    // the head varies fastest, which keeps a head's workgroups on one XCD (number mod 8) whenever
    // the head count is a multiple of 8.
    const int n_hq = d.B * d.Hq;
    const int head = (int)(blockIdx.x % n_hq), rest = (int)(blockIdx.x / n_hq);
    split = rest % a.n_split;
    qt = n_qt - 1 - rest / a.n_split;
    if (qt < 0) return;
    b = head / d.Hq;
    hq0 = head % d.Hq;
    hk = hq0 / G;
  } else {
    HeadWork hw;
    if (!xcd_decode(blockIdx.x, d.B * d.Hkv, a.n_split * per_split, &hw)) return;
    b = hw.head / d.Hkv;
    hk = hw.head % d.Hkv;
    split = hw.item / per_split;
    hq0 = hk * G + (PACK ? 0 : (hw.item % per_split) / n_qt);   // PACK: the first head of the group
    qt = hw.item % n_qt;
  }

  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, ql = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r_wave0 = qt * QM + wave * 32 * QB;     // first row (of the group's list) of this wave

  // KV range of this split, in tiles
  const int n_tiles = (d.Skv + TN - 1) / TN;
  const int tps = (n_tiles + a.n_split - 1) / a.n_split;
  int t_begin = split * tps;                        // (LIST: re-cut below over the list)
  int t_end = min(n_tiles, t_begin + tps);

  // ---- stationary operands: Q of this lane's rows r_wave0 + 32 qb + ql of the list
  const float c2 = d.scale * LOG2E;
  bf16x8 qf[QB][KS];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    // (rows past the last one re-read it and become zero: a branch around the loads would make
    // each of them wait for the one before)
    const int r = r_wave0 + 32 * qb + ql, rc = min(r, rows_kv - 1);
    const int hq = PACK ? hq0 + rc / d.Sq : hq0, i = PACK ? rc % d.Sq : rc;
    const long off = b * d.q_sb + hq * d.q_sh + (long)i * d.q_ss;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const u32x4 x = *(const u32x4*)((const uint16_t*)a.q + off + 16 * ks + 8 * g);
      qf[qb][ks] = __builtin_bit_cast(bf16x8, r < rows_kv ? x : u32x4{0, 0, 0, 0});
    }
  }
  // These loads are finished (and the operands moved into the accumulation registers) below, once
  // the tile list has been built -- its probes of the bitmap travel with them -- and before the
  // tile copies start: the copies are not counted by the compiler, so nothing may wait on memory later.

  // LIST: the tiles every row of the workgroup sees, compacted into a list (in the area of the
  // mask window; its length in the last word), shared evenly by the splits.  From here on
  // t_begin, t_end and the cursor are POSITIONS in the list; tile_at turns one into a tile.
  int* const tlist = (int*)(smem + SM::RING + SM::BITS_BYTES);
  constexpr int LIST_CAP = SM::WIN_BYTES / 4 - 1;
  constexpr int VIS_SHIFT = 24;                     // LIST = 2: a list entry is tile | row-block bits << 24
  if (LIST) {
    const int i_wg0 = qt * QM, i_wg1 = min(d.Sq, i_wg0 + QM) - 1;
    const int c0 = i_wg0 / a.mask.q_chunk, h = i_wg1 / a.mask.q_chunk - c0 + 1;     // chunks of this workgroup's rows
    const int w = (d.Skv - 1) / a.mask.kv_block + 1;
    // full[f]: all h chunks see key block f (LIST = 2: bit k = the k-th 32-row block of the
    // workgroup, which lies in one chunk, sees it); then the tile plane
    unsigned* const full = (unsigned*)(smem + SM::RING);
    unsigned* const plane = full + ((w + 1) & ~1);
    for (int f = tid; f < w; f += 256) {
      unsigned ok;
      if (LIST == 2) {
        ok = 0;
#pragma unroll
        for (int k = 0; k < QM / 32; ++k) {          // (all probes on their way at once: rows past the last re-read it)
          const int i = i_wg0 + 32 * k, ic = min(i, d.Sq - 1);
          const uint8_t on = a.mask.allow[b * a.mask.stride_b + (long)(ic / a.mask.q_chunk) * a.mask.stride_q + f];
          ok |= (i < d.Sq && on != 0 ? 1u : 0u) << k;
        }
      } else {
        ok = 1;
        for (int c = 0; c < h; ++c) ok &= a.mask.allow[b * a.mask.stride_b + (long)(c0 + c) * a.mask.stride_q + f] != 0;
      }
      full[f] = ok;
    }
    __syncthreads();
    for (int base = 0; base < n_tiles; base += 256) {          // workgroup-uniform trip count
      const int t = base + tid;
      bool on = t < n_tiles;
      if (on) {
        const int fa = (t * TN) / a.mask.kv_block, fb = (t * TN + TN - 1) / a.mask.kv_block;
        for (int f = fa; f <= fb; ++f) on = on && full[f] != 0;
      }
      const unsigned long long m = __ballot(on);
      if ((tid & 63) == 0 && t < n_tiles) *(unsigned long long*)(plane + t / 32) = m;
    }
    __syncthreads();
    if (wave == 0) {
      // (the words of 64 tiles each are fetched 64 at a time, one per lane, and handed round from
      // the registers: read one by one from LDS, each would wait for the one before it; words
      // without a visible tile -- most of them under a sparse mask -- cost nothing more)
      int count = 0;
      const int n_words = (n_tiles + 63) / 64;
      for (int w0 = 0; w0 < n_words; w0 += 64) {               // wave-uniform trip counts
        const int nw = min(64, n_words - w0);
        const unsigned long long mine = lane < nw ? *(const unsigned long long*)(plane + 2 * (w0 + lane)) : 0ull;
        for (int k = 0; k < nw; ++k) {
          const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)mine, k);
          const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(mine >> 32), k);
          const unsigned long long m = ((unsigned long long)hi << 32) | lo;
          if (m == 0ull) continue;
          const int base = (w0 + k) * 64;
          if ((m >> lane) & 1ull) {
            int entry = base + lane;
            if (LIST == 2) entry |= (int)(full[((base + lane) * TN) / a.mask.kv_block] << VIS_SHIFT);
            tlist[count + __popcll(m & ((1ull << lane) - 1ull))] = entry;
          }
          count += (int)__popcll(m);
        }
      }
      if (lane == 0) tlist[LIST_CAP] = count;
    }
    __syncthreads();
    const int nn = __builtin_amdgcn_readfirstlane(tlist[LIST_CAP]);
    t_begin = (int)((long)split * nn / a.n_split);
    t_end = (int)((long)(split + 1) * nn / a.n_split);
  }
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+a"(qf[qb][ks]));
  auto tile_of = [&](int entry) __attribute__((always_inline)) -> int {
    return LIST == 2 ? entry & ((1 << VIS_SHIFT) - 1) : entry;
  };
  auto tile_at = [&](int pos) __attribute__((always_inline)) -> int {
    return LIST ? tile_of(__builtin_amdgcn_readfirstlane(tlist[pos])) : pos;
  };
  // LIST = 2: which of this wave's QB row blocks see tile number T_ of this workgroup's share of
  // the list (bit qb); everything otherwise
  auto vis_at = [&](int T_) __attribute__((always_inline)) -> int {
    if constexpr (LIST == 2)
      return (__builtin_amdgcn_readfirstlane(tlist[t_begin + T_]) >> (VIS_SHIFT + QB * wave)) & ((1 << QB) - 1);
    else
      return (1 << QB) - 1;
  };
  const int nt = max(t_end - t_begin, 0);          // number of tiles this workgroup performs
  auto next_tile = [&](int t) __attribute__((always_inline)) -> int { return min(t, t_end); };
  int cursor = t_begin;                            // next tile to issue

  // ---- tile copies.  Group w of a tile (logical rows 4 j + w, j = 0..15) is contiguous in LDS:
  // RUN slots of 16 bytes.  Wave w copies group w of the K tile and of the V tile, each with NCR
  // wave-level copies of 64 slots (the last one re-covers the tail of the previous so that no copy
  // crosses the group); lane l of a copy starting at slot a fills slot a + l = (row (a + l) / SPR
  // of the group, chunk (a + l) % SPR; the pad chunk re-reads the last one).
  const char* const k0 = (const char*)a.k + (b * d.kv_sb + hk * d.kv_sh) * 2;
  const char* const v0 = (const char*)a.v + (b * d.kv_sb + hk * d.kv_sh) * 2;
  const unsigned row_bytes = (unsigned)(d.kv_ss * 2);
  auto run_start = [&](int c) __attribute__((always_inline)) -> int { return c + 1 < NCR ? 64 * c : SM::RUN - 64; };
  unsigned cp_off[NCR];
#pragma unroll
  for (int c = 0; c < NCR; ++c) {
    const int sl = run_start(c) + lane;
    cp_off[c] = (unsigned)(4 * (sl / SM::SPR)) * row_bytes + (unsigned)min(sl % SM::SPR, CPR - 1) * 16;
  }
  // A tile's copies are numbered 0 .. NDMA - 1, so that the dense loop can spread them over the
  // matrix instructions of a phase: issued back to back, each waits for the one before it to be
  // accepted by the memory pipeline, and the wave would stand still for hundreds of cycles.
  const unsigned smem_u = lds_base(smem);
  auto issue_part = [&](int t, char* st, int k) __attribute__((always_inline)) {   // full tiles only
    const long tile = (long)t * TN * row_bytes + (long)wave * row_bytes;           // this wave's first row: tile row w
    const unsigned kdst = smem_u + (unsigned)(st - smem) + wave * SM::GS;
    if (k % 2 == 0) dma16u(k0 + tile, cp_off[k / 2], kdst + run_start(k / 2) * 16);
    else dma16u(v0 + tile, cp_off[k / 2], kdst + SM::TILE + run_start(k / 2) * 16);
  };
  auto issue_tile = [&](int t, char* st) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < 2 * NCR; ++k) issue_part(t, st, k);
  };
  constexpr int NDMA = 2 * NCR;                    // copies per wave and tile

  // ---- softmax state of this lane's two query rows (both half-waves keep identical copies)
  f32x16 oacc[QB][DB];                 // O^T, relative to the reference
  float r[QB], l_run[QB], l_half[QB];  // reference, this lane's share of the sum of p over the halves
                                       // accepted so far, and over the half being converted
  // the reference that conversions subtract: r itself, or (LIST = 2) +infinity for a row block
  // that does not see the tile whose scores are being converted
  float rq_own[QB];
  float (&rq)[QB] = *(LIST == 2 ? &rq_own : &r);
  auto set_rq = [&](int vb) __attribute__((always_inline)) {
    if constexpr (LIST == 2) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) rq[qb] = ((vb >> qb) & 1) ? r[qb] : INFINITY;
    }
  };
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
    for (int i = 0; i < DB; ++i) { oacc[qb][i] = zero16(); asm volatile("" : "+a"(oacc[qb][i])); }
    r[qb] = 0.f;
    l_run[qb] = 0.f;
    l_half[qb] = 0.f;
  }

  // ---- building blocks, all on one 32-key half hb of the tile at st ---------------------------
  struct FirstK { bf16x8 k; };
  auto first_k = [&](const char* __restrict__ st, int hb) __attribute__((always_inline)) -> bf16x8 {
    return *(const bf16x8*)(st + tile_off<D>(ql, 32 * hb, 16 * g));
  };
  auto first_vt = [&](const char* __restrict__ st, int hb) __attribute__((always_inline)) -> bf16x8 {
    return tile_tr_operand<D>(st + SM::TILE, 32 * hb, 0, lane);
  };
  // S^T = K Q^T: lane = query column, registers = keys.  first: the K operand of k-step 0,
  // fetched by the caller (during the previous phase in the steady state); per_unit(m) is vector
  // work issued right after matrix instruction m (0 .. 2 KS - 1), to run in its shadow; tail(),
  // issued three instructions before the end, fetches the first operand of the next phase.
  auto score = [&](const char* __restrict__ st, int hb, f32x16 (&s)[QB], auto&& per_unit, bf16x8 first,
                   auto&& tail) __attribute__((always_inline)) {
    const char* krow = st + tile_off<D>(ql, 32 * hb, 16 * g);
    bf16x8 ka[2];
    ka[0] = first;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int cu = ks & 1;
      if (ks + 1 < KS) ka[cu ^ 1] = *(const bf16x8*)(krow + (ks + 1) * 32);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        if (ks == 0) mfma_first(s[qb], ka[cu], qf[qb][ks]);
        else mfma_next(s[qb], ka[cu], qf[qb][ks]);
        per_unit(ks * QB + qb);
        if (ks * QB + qb == QB * KS - 3) tail();
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    asm volatile("s_nop 7" ::: "memory");          // the last results settle before anything reads them
  };
  auto nothing = [](int) __attribute__((always_inline)) {};
  auto no_tail = []() __attribute__((always_inline)) {};
  // The matrix instructions are opaque to the compiler, so nothing makes a reader (or writer) of
  // fresh scores wait for them.  In the pipelined loop a half's scores are first touched two
  // matrix instructions into the next phase; everywhere else this wait comes first.
  auto settle_scores = [&](f32x16 (&s)[QB]) __attribute__((always_inline)) {
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" : "+v"(s[0]), "+v"(s[1]));
  };
  // Waits until every matrix instruction issued so far has written its result.  The accumulators
  // are operands of the statement, so that the compiler cannot read them before it.
  auto drain_oacc = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      if constexpr (DB == 4)
        asm volatile("s_nop 15\n\ts_nop 15" : "+a"(oacc[qb][0]), "+a"(oacc[qb][1]), "+a"(oacc[qb][2]), "+a"(oacc[qb][3]));
      else if constexpr (DB == 3)
        asm volatile("s_nop 15\n\ts_nop 15" : "+a"(oacc[qb][0]), "+a"(oacc[qb][1]), "+a"(oacc[qb][2]));
      else
        asm volatile("s_nop 15\n\ts_nop 15" : "+a"(oacc[qb][0]), "+a"(oacc[qb][1]));
    }
  };
  // Conversion of scores into the P^T operands, element x of a half (x = 0..31: query block
  // qb = x / 16, register v = x % 16): p = exp2(s c2 - r), added to the half's sum and packed in pairs as
  // bf16 into word (v % 8) / 2 of operand v / 8 of the query block.
  struct Carry { float p; };
  auto conv_elem = [&](int x, Carry& cy, const f32x16 (&s)[QB], u32x4 (&pw)[QB][2]) __attribute__((always_inline)) {
    const int qb = x / 16, v = x % 16;
    const float pr = __builtin_amdgcn_exp2f(fmaf(s[qb][v], c2, -rq[qb]));
    if (v == 0) l_half[qb] = pr;
    else l_half[qb] += pr;
    if (v % 2 == 0) { cy.p = pr; return; }
    pw[qb][v / 8][(v % 8) / 2] = pack2_bf16(cy.p, pr);
  };
  auto convert = [&](const f32x16 (&s)[QB], u32x4 (&pw)[QB][2]) __attribute__((always_inline)) {
    Carry cy;
#pragma unroll
    for (int x = 0; x < 32; ++x) conv_elem(x, cy, s, pw);
  };
  // a row's largest score of a half, in units of log2 (c2 > 0)
  auto row_max = [&](const f32x16& sv) __attribute__((always_inline)) -> float {
    float m = fmaxf(fmaxf(sv[0], sv[1]), sv[2]);
#pragma unroll
    for (int v = 3; v < 15; v += 2) m = fmaxf(fmaxf(m, sv[v]), sv[v + 1]);
    return xhalf_max(fmaxf(m, sv[15])) * c2;
  };
  // After a half has been converted, before its probabilities are used: accept it, or (rarely)
  // redo it.  A lane's sum of 16 probabilities bounds each of them, so a sum within LAZY_SUM
  // proves that none overflowed or is too large for the accumulation; a larger one (infinity
  // included) sends the whole wave through the raise: r goes up to the row's maximum where that
  // is larger, O^T -- no matrix instruction on it is in flight between two phases once drained
  // -- and the accepted sums shrink by alpha = 2^(old - new), and the half is converted again
  // from its scores, which are still in their registers.  Rows that keep their reference get
  // identical values again.
  auto commit = [&](const f32x16 (&s)[QB], u32x4 (&pw)[QB][2], int vb) __attribute__((always_inline)) {
    bool need = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) need |= !(l_half[qb] <= LAZY_SUM);
    if (__builtin_expect(__any(need), 0)) {
      asm volatile("" ::: "memory");               // keep this a real, rarely taken branch
      drain_oacc();
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        if (LIST == 2 && !((vb >> qb) & 1)) continue;          // (scores the rows do not see raise nothing)
        const float r_new = fmaxf(r[qb], row_max(s[qb]));
        const float alpha = __builtin_amdgcn_exp2f(r[qb] - r_new);
        r[qb] = r_new;
        l_run[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
          for (int v = 0; v < 16; ++v) oacc[qb][db][v] *= alpha;
        }
      }
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {            // the new values settle before a matrix instruction reads them
        if constexpr (DB == 4)
          asm volatile("s_nop 7" : "+a"(oacc[qb][0]), "+a"(oacc[qb][1]), "+a"(oacc[qb][2]), "+a"(oacc[qb][3]));
        else if constexpr (DB == 3)
          asm volatile("s_nop 7" : "+a"(oacc[qb][0]), "+a"(oacc[qb][1]), "+a"(oacc[qb][2]));
        else
          asm volatile("s_nop 7" : "+a"(oacc[qb][0]), "+a"(oacc[qb][1]));
      }
      set_rq(vb);
      convert(s, pw);
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) l_run[qb] += l_half[qb];
  };
  // O^T += V^T P^T over the 32 keys of a half (two k-steps of 16 keys)
  auto contract = [&](const char* __restrict__ st, int hb, const u32x4 (&pw)[QB][2]) __attribute__((always_inline)) {
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 vt = tile_tr_operand<D>(st + SM::TILE, 32 * hb + 16 * t2, 32 * db, lane);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) mfma_acc(oacc[qb][db], vt, __builtin_bit_cast(bf16x8, pw[qb][t2]));
      }
  };
  // contract(half h) on the matrix core; on the vector ALU, after two matrix instructions (the
  // scores of half h+1 have settled by then), the first XE conversions of half h+1.
  // The transposed operand of a pair of matrix instructions is fetched one pair ahead, and nothing
  // is scheduled across the units.
  auto contract_convert = [&](const char* __restrict__ st, int hb, const u32x4 (&pi)[QB][2],
                              f32x16 (&s)[QB], u32x4 (&po)[QB][2], Carry& cy, bf16x8 first,
                              auto&& tail) __attribute__((always_inline)) {
    constexpr int NM = 2 * DB * QB;                // matrix instructions
    constexpr int M0 = 2;                          // first unit with conversions
    static_assert(NM > M0 + 1, "no room for the conversions");
    bf16x8 vt[2];
    vt[0] = first;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      const int c = m / QB, t2 = c / DB, db = c % DB, qb = m % QB, cu = c & 1;
      if (qb == 0 && c + 1 < 2 * DB)
        vt[cu ^ 1] = tile_tr_operand<D>(st + SM::TILE, 32 * hb + 16 * ((c + 1) / DB), 32 * ((c + 1) % DB), lane);
      mfma_acc(oacc[qb][db], vt[cu], __builtin_bit_cast(bf16x8, pi[qb][t2]));
      if (m >= M0) {
#pragma unroll
        for (int x = (m - M0) * XE / (NM - M0); x < (m - M0 + 1) * XE / (NM - M0); ++x) conv_elem(x, cy, s, po);
      }
      if (m == NM - 3) tail();
      __builtin_amdgcn_sched_barrier(0);
    }
    // the conversions stay in this phase (their results are only used two phases later, and
    // would otherwise sink towards the branch that follows the next phase)
    static_assert(XE % 8 == 0 && XE <= 16, "the words pinned here are those of elements 0 .. XE - 1");
    float& lh0 = l_half[0];
    asm volatile("" : "+v"(po[0][0]), "+v"(lh0));
    if constexpr (XE == 16) asm volatile("" : "+v"(po[0][1]));
  };
  // score(half h+2) together with the remaining conversions of half h+1
  auto score_convert = [&](const char* __restrict__ st, int hb, f32x16 (&s_new)[QB], const f32x16 (&s)[QB],
                           u32x4 (&po)[QB][2], Carry& cy, bf16x8 first, auto&& tail,
                           auto&& extra) __attribute__((always_inline)) {
    constexpr int NU = QB * KS;                    // matrix instructions of a score phase
    score(st, hb, s_new, [&](int m) __attribute__((always_inline)) {
#pragma unroll
      for (int x = XE + m * (32 - XE) / NU; x < XE + (m + 1) * (32 - XE) / NU; ++x) conv_elem(x, cy, s, po);
      extra(m);
    }, first, tail);
  };

  // ---- pipeline.  Tile number q of the sequence lives in ring stage q % 4.  Per tile T (halves
  // 2T and 2T+1): contract 2T | convert 2T+1 | score 2T+2, then contract 2T+1 | convert 2T+2, the
  // one barrier of the tile -- every wave is done with tile T, whose stage takes tile T + 4, and
  // tile T + 2, issued two tiles ago, has landed -- and score 2T+3.
#pragma unroll
  for (int q = 0; q < NSTG; ++q) {
    if (q < nt) {
      issue_tile(tile_at(cursor), smem + q * SM::STAGE);
      cursor = next_tile(cursor + 1);
    }
  }
  wait_vmcnt<0>();
  __syncthreads();
  auto stage = [&](int q) __attribute__((always_inline)) -> char* { return smem + (q % NSTG) * SM::STAGE; };
  auto mid = [&](auto all_in_flight, bool issue, char* st_copy) __attribute__((always_inline)) {
    // all_in_flight: tiles T + 2 and T + 3 were both issued, so leaving one tile's copies
    // outstanding still guarantees that tile T + 2 has landed
    if constexpr (decltype(all_in_flight)::value) wait_vmcnt<NDMA>();
    else wait_vmcnt<0>();
    wg_barrier();
    if (issue) {
      issue_tile(tile_at(cursor), st_copy);
      cursor = next_tile(cursor + 1);
    }
  };

  f32x16 s0[QB], s1[QB];                           // scores of even / odd halves
  u32x4 p0[QB][2] = {}, p1[QB][2] = {};            // packed P^T operands of even / odd halves
  Carry cy;
  if (nt > 0) {
    score(smem, 0, s0, nothing, first_k(smem, 0), no_tail);
    settle_scores(s0);
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) r[qb] = row_max(s0[qb]);     // no probability of the first half exceeds 1
    // (LIST = 2: rows that do not see the first tile start from a reference that means nothing
    // yet; any finite one will do, their first visible tile raises it if it has to)
    set_rq(vis_at(0));
    convert(s0, p0);
    commit(s0, p0, vis_at(0));
    score(smem, 1, s1, nothing, first_k(smem, 1), no_tail);
  }
  int T = 0;
  int id_next = LIST && cursor < t_end ? tlist[cursor] : 0;     // LIST: number of the next tile to copy
  bf16x8 fk;
  bf16x8 fvt = first_vt(smem, 0);                  // handed from phase to phase
  asm volatile("" : "+v"(fvt));                    // (in hand before the loop: both ways into it then agree on what is in flight)
  for (; T + 4 < nt; ++T) {                        // full tiles: tile T + 1 is scored, tile T + 4 issued
    char* const sa = stage(T);
    char* const sb = stage(T + 1);
    const int vb_t = vis_at(T), vb_n = vis_at(T + 1);          // (the conversions under way are tile T's)
    contract_convert(sa, 0, p0, s1, p1, cy, fvt, [&]() __attribute__((always_inline)) { fk = first_k(sb, 0); });
    asm volatile("" : "+v"(fk));                   // (waited for here, where the compiler still knows what is in flight)
    score_convert(sb, 0, s0, s1, p1, cy, fk, [&]() __attribute__((always_inline)) { fvt = first_vt(sa, 1); }, nothing);
    asm volatile("" : "+v"(fvt));
    commit(s1, p1, vb_t);
    set_rq(vb_n);                                  // from here on: scores of tile T + 1
    contract_convert(sa, 1, p1, s0, p0, cy, fvt, [&]() __attribute__((always_inline)) { fk = first_k(sb, 1); });
    asm volatile("" : "+v"(fk));
    mid(std::true_type{}, false, sa);
    // the copies of tile T + 4 go out during the phase (LIST: its number was fetched a tile ago)
    const int t_new = LIST ? tile_of(__builtin_amdgcn_readfirstlane(id_next)) : cursor;
    cursor = next_tile(cursor + 1);
    if (LIST) id_next = tlist[cursor < t_end ? cursor : t_begin];
    constexpr int EVERY = QB * KS / NDMA;
    static_assert(EVERY >= 1, "more copies than matrix instructions in the score phase");
    score_convert(sb, 1, s1, s0, p0, cy, fk, [&]() __attribute__((always_inline)) { fvt = first_vt(sb, 0); },
                  [&](int m) __attribute__((always_inline)) {
                    if (m % EVERY == EVERY - 1 && m / EVERY < NDMA) issue_part(t_new, sa, m / EVERY);
                  });
    asm volatile("" : "+v"(fvt));
    commit(s0, p0, vb_n);
  }
  for (; T < nt; ++T) {                            // the last (at most four) tiles, phase after phase
    const bool more = T + 1 < nt;
    const int vb_t = vis_at(T), vb_n = more ? vis_at(T + 1) : 0;
    contract(stage(T), 0, p0);
    settle_scores(s1);                             // (outside the pipelined loop the wait comes first, as a real dependence)
    convert(s1, p1);
    commit(s1, p1, vb_t);                          // (a raise comes before anything relative to the new reference is added)
    if (more) { score(stage(T + 1), 0, s0, nothing, first_k(stage(T + 1), 0), no_tail); }
    contract(stage(T), 1, p1);
    if (more) { settle_scores(s0); set_rq(vb_n); convert(s0, p0); commit(s0, p0, vb_n); }
    mid(std::false_type{}, T + 4 < nt, stage(T));
    if (more) { score(stage(T + 1), 1, s1, nothing, first_k(stage(T + 1), 1), no_tail); }
  }

  // ---- epilogue: O = acc / l, L = r ln 2 + ln l (the reference is in units of log2).  The last
  // matrix instructions must have retired before their registers are read.
  drain_oacc();
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float l_tot = xhalf_sum(l_run[qb]);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    const float lse = l_tot > 0.f ? r[qb] * (1.f / LOG2E) + logf(l_tot) : -INFINITY;
    const int r = r_wave0 + 32 * qb + ql;
    if (r >= rows_kv) continue;
    const int hq = PACK ? hq0 + r / d.Sq : hq0, i = PACK ? r % d.Sq : r;
    const long row = ((long)b * d.Hq + hq) * d.Sq + i;
    if (a.n_split > 1 || a.partial) {
      const long slice = (long)(a.part0 + split) * d.B * d.Hq * d.Sq;
      float* o = a.o_part + (slice + row) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          f32x4 y = {oacc[qb][db][4 * q4] * inv, oacc[qb][db][4 * q4 + 1] * inv, oacc[qb][db][4 * q4 + 2] * inv,
                     oacc[qb][db][4 * q4 + 3] * inv};
          *(f32x4*)(o + 32 * db + 8 * q4 + 4 * g) = y;
        }
      if (g == 0) a.lse_part[slice + row] = lse;
      continue;
    }
    if (a.merge_into) {
      // Rescale of Algorithm 1 with the running (O, L) of this row: L' = ln(e^L + e^dL),
      // O' = e^(L - L') O + e^(dL - L') dO, where dO = acc / l is this visit's result
      const float L0 = a.lse[row];
      const float M = fmaxf(L0, lse);
      float w0 = 0.f, w1 = 0.f, L1 = -INFINITY;
      if (M != -INFINITY) {
        const float e0 = expf(L0 - M), e1 = expf(lse - M);
        L1 = M + logf(e0 + e1);
        w0 = expf(L0 - L1);
        w1 = expf(lse - L1) * inv;
      }
      float* o = (float*)a.o + row * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          float* dst = o + 32 * db + 8 * q4 + 4 * g;
          const f32x4 x = *(const f32x4*)dst;
          f32x4 y = {w0 * x[0] + w1 * oacc[qb][db][4 * q4], w0 * x[1] + w1 * oacc[qb][db][4 * q4 + 1],
                     w0 * x[2] + w1 * oacc[qb][db][4 * q4 + 2], w0 * x[3] + w1 * oacc[qb][db][4 * q4 + 3]};
          *(f32x4*)dst = y;
        }
      // (both half-waves of the row have read L0 above: the loads precede this store in program order)
      if (g == 0) a.lse[row] = L1;
      continue;
    }
    const long off = b * d.q_sb + hq * d.q_sh + (long)i * d.q_ss;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const float y0 = oacc[qb][db][4 * q4] * inv, y1 = oacc[qb][db][4 * q4 + 1] * inv,
                    y2 = oacc[qb][db][4 * q4 + 2] * inv, y3 = oacc[qb][db][4 * q4 + 3] * inv;
        const int col = 32 * db + 8 * q4 + 4 * g;
        if (a.o_is_f32) {
          f32x4 y = {y0, y1, y2, y3};
          *(f32x4*)((float*)a.o + off + col) = y;
        } else {
          u32x2 y = {pack2_bf16(y0, y1), pack2_bf16(y2, y3)};
          *(u32x2*)((uint16_t*)a.o + off + col) = y;
        }
      }
    if (g == 0) a.lse[row] = lse;
  }
}

template <int D, int LIST = 0>
hipError_t launch(const FwdArgs& a, long grid, hipStream_t s) {
  static SmemOnce once;
  const hipError_t e = ensure_dynamic_lds((const void*)fwd_bf16_kernel<D, LIST>, KvSmem<D>::TOTAL, &once);
  if (e != hipSuccess) return e;
  fwd_bf16_kernel<D, LIST><<<(unsigned)grid, 256, KvSmem<D>::TOTAL, s>>>(a);
  return hipGetLastError();
}

}  // namespace

int fwd_bf16_pick_split(const Dims& d, int n_cu, bool masked) {
  // one workgroup per CU; split the KV axis until the grid covers the chip.  With a media mask the
  // visible work differs from one query tile to the next (the splits of a tile share its visible
  // key tiles evenly), so four times as many workgroups are made to even the load out.
  // (the dense kernel tiles the rows of a whole group of query heads, the general one each head's)
  const bool dense = !masked && (d.Skv % TN == 0 || d.Skv >= 2 * TN);   // (a ragged key count: whole tiles on the dense kernel)
  const long base = dense ? (long)d.B * d.Hkv * (((long)(d.Hq / d.Hkv) * d.Sq + QM - 1) / QM)
                          : (long)d.B * d.Hq * ((d.Sq + QM - 1) / QM);
  const int n_tiles = (d.Skv + TN - 1) / TN;
  long cap = n_tiles / 16;                // keep at least 16 tiles (1024 keys) per split
  if (cap < 1) cap = 1;
  if (!masked) {
    // about 4.5 TFLOP/s per compute unit in this kernel; partial results are float32 rows written
    // once and read once at about 3 TB/s
    const double t_full = 4.0 * QM * (double)d.Skv * d.D / 4.5e12;
    const double t_part = 2.0 * (double)d.B * d.Hq * d.Sq * d.D * 4.0 / 3e12;
    return pick_split_balanced(base, n_cu, cap, t_full, t_part);
  }
  long want = (LVX_MASKED_WG_FACTOR * n_cu + base - 1) / base;
  if (want < 1) want = 1;
  if (want > cap) want = cap;
  if (want > 64) want = 64;
  return (int)want;
}

namespace {
bool list_fits(const Dims& d, const MaskDev& m) {
  // the list and its scratch fit the mask areas of the dense kernel's LDS layout, tiles are whole
  const int n_tiles = (d.Skv + TN - 1) / TN, w = (d.Skv - 1) / m.kv_block + 1;
  return m.allow != nullptr && d.Skv % TN == 0 && n_tiles <= KvSmem<128>::WIN_BYTES / 4 - 1 &&
         ((w + 1) & ~1) + (n_tiles + 63) / 64 * 2 <= KvSmem<128>::BITS_BYTES / 4;
}
}  // namespace
// one launch of the dense kernel over the tiles any row of a workgroup sees: the mask never cuts
// through a 32-row block or a key tile
bool fwd_bf16_one_pass_fits(const Dims& d, const MaskDev& m) {
  return list_fits(d, m) && m.q_chunk % 32 == 0 && m.kv_block % TN == 0;
}
bool fwd_bf16_two_pass_fits(const Dims& d, const MaskDev& m) {
  return list_fits(d, m) && m.q_chunk >= 8 && !fwd_bf16_one_pass_fits(d, m);
}

hipError_t launch_fwd_bf16(const FwdArgs& a, hipStream_t s) {
  const Dims& d = a.d;
  if (a.pass == 1) {                               // the dense kernel over the tiles every row of a workgroup sees
    const long grid = xcd_grid(d.B * d.Hkv, a.n_split * (d.Hq / d.Hkv) * ((d.Sq + QM - 1) / QM));
    return d.D == 64 ? launch<64, 1>(a, grid, s) : d.D == 96 ? launch<96, 1>(a, grid, s) : launch<128, 1>(a, grid, s);
  }
  if (a.pass == 0 && fwd_bf16_one_pass_fits(d, a.mask)) {
    const long grid = (long)d.B * d.Hq * a.n_split * ((d.Sq + QM - 1) / QM);
    return d.D == 64 ? launch<64, 2>(a, grid, s) : d.D == 96 ? launch<96, 2>(a, grid, s) : launch<128, 2>(a, grid, s);
  }
#ifdef LVX_FWD_TWO_WAVES
  // Measurement builds only (python -m paper_2502_02406_amd.build --define LVX_FWD_TWO_WAVES=1): dense
  // problems too run the general kernel, whose eight waves of 32 rows put two waves on every SIMD.
  return launch_fwd_general_bf16(a, s);
#endif
  if (a.mask.allow != nullptr || d.Skv % TN != 0) return launch_fwd_general_bf16(a, s);
  const int n_qt = (int)(((long)(d.Hq / d.Hkv) * d.Sq + QM - 1) / QM);
  const long grid = xcd_grid(d.B * d.Hkv, a.n_split * n_qt);
  return d.D == 64 ? launch<64>(a, grid, s) : d.D == 96 ? launch<96>(a, grid, s) : launch<128>(a, grid, s);
}

}  // namespace lvx
