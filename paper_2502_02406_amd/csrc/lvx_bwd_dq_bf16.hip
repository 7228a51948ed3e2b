// bf16 backward, query-stationary kernel: dQ of one K/V block.  Table 1 of the paper counts the
// backward as five matrix products; this kernel performs three of them (S, dP, dQ) with the
// probabilities recomputed from the saved statistic L (Section 3.2 saves only x, O and L):
//   p_ij = exp(scale <Q_i, K_j> - L_i),   dS_ij = p_ij (<dO_i, V_j> - delta_i),   dQ_i += scale dS_ij K_j.
// S and dP are also formed by the key-stationary kernel (7 products for the 5 that Table 1
// counts); the alternative, one kernel that scatters dQ with float atomics, is bounded by the L2
// atomic rate (about one float per channel per clock), far below the matrix cores.
//
// Workgroup = 4 wavefronts = 256 query rows of one (batch, query head), one wave per SIMD with
// the whole register file.  A wave owns 64 query rows (two 32-row blocks): their Q and dO operands
// and the dQ^T accumulators live in the accumulation registers for the whole kernel, so every K
// or V operand fetched from LDS feeds two matrix instructions.  K/V tiles of 64 keys travel
// HBM -> LDS by direct global-to-LDS copies into a ring of four stages, issued two tiles ahead,
// one barrier per tile.
// Transposed tiles S^T = K Q^T and dP^T = V dO^T put one QUERY per lane (its statistics are
// per-lane scalars) and 16 keys in a lane's registers, so dS^T, rounded to bf16, is already the
// B operand of dQ^T += K^T dS^T, with K^T fetched by transposing LDS reads.
// The loop runs over 32-key halves and is software pipelined inside each wave: while the matrix
// core contracts half h (dQ) and scores half h+2 (S, dP), the vector ALU turns the scores of half
// h+1 into dS; two sets of score registers alternate.
#include "lvx_internal.h"
#include "lvx_mfma.h"
#include "lvx_kv_ring.h"

#include <type_traits>

namespace lvx {

namespace {

using namespace kvring;
constexpr int PF = 1;                  // LDS operand prefetch distance, in k-steps (operand sets = PF + 1)
constexpr int XE = 8;                  // elements of a half converted during the contraction (of 32)
template <int D> using DqSmem = KvSmem<D>;

// Measurement builds only (python -m paper_2502_02406_amd.build --define LVX_DQ_PROBE=1): every
// workgroup adds the clocks of its three phases (set-up until the first tiles are in place; the
// loop; the epilogue until its stores have been acknowledged), a count and its number of tiles to
// dq_probe, which lvx_debug_dq_probe copies out and clears.
#ifdef LVX_DQ_PROBE
__device__ unsigned long long dq_probe[8];
#define DQ_STAMP(x) const unsigned long long x = __builtin_readcyclecounter()
#else
#define DQ_STAMP(x)
#endif

// GENERAL = false: dense attention and Skv a multiple of 64 (no mask code, no ragged tile, so that
// the steady-state loop is one basic block); GENERAL = true: everything else.
// LIST (with GENERAL = false): the dense kernel over a list of key tiles -- those that EVERY row
// of the workgroup sees under a media mask (BwdArgs::dq_pass == 1).  Inside such a tile nothing is
// masked, so the loop is the dense one; only the tile numbers come from the list.  The other
// visible tiles are left to a launch of the general kernel (dq_pass == 2).
// LIST = 2: a mask whose text chunks are multiples of 32 rows and whose key blocks are multiples
// of 64 keys never cuts through a (32-row block, key tile) pair: the list then holds the tiles
// that ANY row of the workgroup sees, each with one bit per 32-row block of the workgroup; the
// dS operands of a row block that does not see a tile are replaced by zeros as they are packed
// (whatever its scores gave, nothing of it reaches a matrix instruction).  One launch does it all.
template <int D, bool GENERAL, int LIST = 0>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
bwd_dq_bf16_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  using SM = DqSmem<D>;
  constexpr int KS = D / 16, DB = D / 32, CPR = SM::CPR, NCR = SM::NCR;

  const Dims& d = a.d;
  const int G = d.Hq / d.Hkv;
  // Dense variant (PACK): the query rows of the G heads that share a K/V head are one list of
  // G * Sq rows (row r = head r / Sq of the group, its row r % Sq), cut into tiles of 256, so that
  // short query blocks fill tiles instead of leaving one mostly empty tile per head.  The general
  // variant tiles each head's rows (its mask code works on rows of one head).
  static_assert(!(GENERAL && LIST), "the tile list is a variant of the dense kernel");
  constexpr bool PACK = !GENERAL && !LIST;         // (a mask works on the rows of one head)
  const int rows_lim = PACK ? G * d.Sq : d.Sq;      // rows of the list this workgroup's tiles are cut from
  const int n_qt = (rows_lim + QM - 1) / QM;
  const int per_split = PACK ? n_qt : G * n_qt;
  int b, hk, split, hq, qt;
  if constexpr (LIST == 2) {
    // (as in the forward: the later query tiles, which under a causal mask see the most key tiles,
    // start first; the head varies fastest)
    const int n_hq = d.B * d.Hq;
    const int head = (int)(blockIdx.x % n_hq), rest = (int)(blockIdx.x / n_hq);
    split = rest % a.n_split_dq;
    qt = n_qt - 1 - rest / a.n_split_dq;
    if (qt < 0) return;
    b = head / d.Hq;
    hq = head % d.Hq;
    hk = hq / G;
  } else {
    HeadWork hw;
    if (!xcd_decode(blockIdx.x, d.B * d.Hkv, a.n_split_dq * per_split, &hw)) return;
    b = hw.head / d.Hkv;
    hk = hw.head % d.Hkv;
    split = hw.item / per_split;
    hq = hk * G + (PACK ? 0 : (hw.item % per_split) / n_qt);   // PACK: the first head of the group
    qt = hw.item % n_qt;
  }

  DQ_STAMP(stamp0);
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, ql = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i_wave0 = qt * QM + wave * 32 * QB;     // first row (of the head, or of the group's list) of this wave

  // KV range of this split, in tiles
  const int n_tiles = (d.Skv + TN - 1) / TN;
  const int tps = (n_tiles + a.n_split_dq - 1) / a.n_split_dq;
  int t_begin = split * tps;                        // (with a media mask: re-cut below over the visible tiles)
  int t_end = min(n_tiles, t_begin + tps);

  // ---- stationary operands and statistics of this lane's query rows i_wave0 + 32 qb + ql
  // The dense variant folds the statistics into the matrix products (FOLD): Q is held as
  // bf16(Q * scale * log2 e) and the accumulations start from 16 copies of -L log2 e and of -delta
  // (a lane's registers all belong to one query row), so that S^T comes out as the exponent of P
  // and dP^T as dP - delta without a vector instruction.
  constexpr bool FOLD = !GENERAL;
  const float c2 = d.scale * LOG2E;
  bf16x8 qf[QB][KS], gf[QB][KS];
  float nl2[QB], nd[QB];               // -L log2(e) (-inf: no probability mass) and -delta
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    // (rows past the last one re-read it and become zero: no branch stands between the loads, so
    // all of them are on their way before the first is waited for)
    const int r = i_wave0 + 32 * qb + ql, rc = min(r, rows_lim - 1);
    const bool ok = r < rows_lim;
    const int hq_l = PACK ? hq + rc / d.Sq : hq, i = PACK ? rc % d.Sq : rc;
    const long off = b * d.q_sb + hq_l * d.q_sh + (long)i * d.q_ss;
    const u32x4 zero4 = {0, 0, 0, 0};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 x = *(const u32x4*)((const uint16_t*)a.q + off + 16 * ks + 8 * g);
      u32x4 y = *(const u32x4*)((const uint16_t*)a.d_o + off + 16 * ks + 8 * g);
      x = ok ? x : zero4;
      y = ok ? y : zero4;
      if (FOLD) {
#pragma unroll
        for (int w = 0; w < 4; ++w)
          x[w] = pack2_bf16(__uint_as_float(x[w] << 16) * c2, __uint_as_float(x[w] & 0xffff0000u) * c2);
      }
      qf[qb][ks] = __builtin_bit_cast(bf16x8, x);
      gf[qb][ks] = __builtin_bit_cast(bf16x8, y);
    }
    const long slot = (((long)b * d.Hq + hq_l) * a.sq_pad + (i & ~31)) * 2 + (i & 31);
    const float st_l = a.stats[slot], st_d = a.stats[slot + 32];
    nl2[qb] = ok ? st_l : -INFINITY;
    nd[qb] = ok ? st_d : 0.f;
  }
  // Finish these loads (and move the operands into the accumulation registers) before the tile
  // copies start: the copies are not counted by the compiler, so nothing may wait on memory later.
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      asm volatile("" : "+a"(qf[qb][ks]));
      asm volatile("" : "+a"(gf[qb][ks]));
    }
    asm volatile("" : "+v"(nl2[qb]), "+v"(nd[qb]));
  }
  f32x16 nl2x[FOLD ? QB : 1], ndx[FOLD ? QB : 1];  // the starting values of the accumulations
  if (FOLD) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) { nl2x[qb][v] = nl2[qb]; ndx[qb][v] = nd[qb]; }
      asm volatile("" : "+v"(nl2x[qb]), "+v"(ndx[qb]));
    }
  }

  // ---- tiles this workgroup needs (media mask: tiles visible to none of its rows are skipped).
  // The window of the bitmap that its rows and key range can touch is copied to LDS, and the
  // visibility of every tile is worked out by all threads at once into a bit array, so that the
  // loop never waits on the bitmap.
  const int i_wg0 = qt * QM, i_wg1 = min(d.Sq, i_wg0 + QM) - 1;
  MaskDev mk = a.mask;
  unsigned* const bits = (unsigned*)(smem + SM::RING);
  bool have_bits = false, have_cls = false;
  const unsigned *cls_any = bits, *cls_all = bits; // this wave's class planes (valid with have_cls)
  const unsigned* seen = bits;                     // per key block: which chunks of the workgroup see it (valid with have_cls)
  int nt = max(t_end - t_begin, 0);                // number of tiles this workgroup performs
  if (GENERAL && mk.allow) {
    auto share = [&](int nn) __attribute__((always_inline)) {   // the splits share the visible tiles evenly
      const int k0 = (int)((long)split * nn / a.n_split_dq), k1 = (int)((long)(split + 1) * nn / a.n_split_dq);
      t_begin = nth_bit(bits, k0, n_tiles);
      t_end = k1 > k0 ? nth_bit(bits, k1 - 1, n_tiles) + 1 : t_begin;
      nt = k1 - k0;
    };
    uint8_t* const win = (uint8_t*)smem + SM::RING + SM::BITS_BYTES;
    if (plan_masked_tiles<D>(a.mask, b, i_wg0, i_wg1, d.Sq, d.Skv, n_tiles, bits, SM::BITS_BYTES, win,
                             SM::WIN_BYTES, tid, &mk, &seen, a.dq_pass == 2)) {
      // visibility of every tile, and its class (nothing / everything / mixed) for every wave's
      // rows: the loop then reads the bitmap for mixed tiles only
      have_bits = have_cls = true;
      const int pw = bit_plane_words(n_tiles);
      cls_any = bits + (1 + 2 * wave) * pw;
      cls_all = bits + (2 + 2 * wave) * pw;
      share(__builtin_amdgcn_readfirstlane((int)bits[0]));
    } else if (n_tiles <= (SM::BITS_BYTES - 16) * 8) {
      // (shapes the planner does not take) bits over ALL tiles of the key range, probe by probe
      mk = mask_to_lds(a.mask, b, i_wg0 / mk.q_chunk, i_wg1 / mk.q_chunk, 0, (d.Skv - 1) / mk.kv_block, win,
                       SM::WIN_BYTES, tid, 256);
      have_bits = true;
      share(build_bits(bits, n_tiles, tid, 256, [&](int t) {
        return mask_rect_tall(mk, b, i_wg0, i_wg1, t * TN, min(d.Skv, t * TN + TN) - 1) != 0;
      }));
    } else if (t_begin < t_end) {
      mk = mask_to_lds(a.mask, b, i_wg0 / mk.q_chunk, i_wg1 / mk.q_chunk, (t_begin * TN) / mk.kv_block,
                       (min(d.Skv, t_end * TN) - 1) / mk.kv_block, win, SM::WIN_BYTES, tid, 256);
    }
  }
  // LIST: the tiles every row of the workgroup sees, compacted into a list (in the area of the
  // mask window; its length in the last word), shared evenly by the splits.  From here on
  // t_begin, t_end and the cursor are POSITIONS in the list; tile_at turns one into a tile.
  int* const tlist = (int*)(smem + SM::RING + SM::BITS_BYTES);
  constexpr int LIST_CAP = SM::WIN_BYTES / 4 - 1;
  constexpr int VIS_SHIFT = 24;                    // LIST = 2: a list entry is tile | row-block bits << 24
  if (LIST) {
    const int c0 = i_wg0 / a.mask.q_chunk, h = i_wg1 / a.mask.q_chunk - c0 + 1;     // chunks of this workgroup's rows
    const int w = (d.Skv - 1) / a.mask.kv_block + 1;
    // full[f]: 1 if all h chunks see key block f (LIST = 2: bit k = the k-th 32-row block of the
    // workgroup, which lies in one chunk, sees it); then the tile plane
    unsigned* const full = bits;
    unsigned* const plane = bits + ((w + 1) & ~1);
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
            if (LIST == 2) entry |= (int)(bits[((base + lane) * TN) / a.mask.kv_block] << VIS_SHIFT);
            tlist[count + __popcll(m & ((1ull << lane) - 1ull))] = entry;
          }
          count += (int)__popcll(m);
        }
      }
      if (lane == 0) tlist[LIST_CAP] = count;
    }
    __syncthreads();
    const int nn = __builtin_amdgcn_readfirstlane(tlist[LIST_CAP]);
    t_begin = (int)((long)split * nn / a.n_split_dq);
    t_end = (int)((long)(split + 1) * nn / a.n_split_dq);
    nt = t_end - t_begin;
  }
  auto tile_of = [&](int entry) __attribute__((always_inline)) -> int {
    return LIST == 2 ? entry & ((1 << VIS_SHIFT) - 1) : entry;
  };
  auto tile_at = [&](int pos) __attribute__((always_inline)) -> int {
    return LIST ? tile_of(__builtin_amdgcn_readfirstlane(tlist[pos])) : pos;
  };
  // LIST = 2: which of this wave's QB row blocks see tile number T_ of this workgroup's share of
  // the list (bit qb); vcur holds that for the tile whose scores are being converted
  auto vis_at = [&](int T_) __attribute__((always_inline)) -> int {
    if constexpr (LIST == 2)
      return (__builtin_amdgcn_readfirstlane(tlist[t_begin + T_]) >> (VIS_SHIFT + QB * wave)) & ((1 << QB) - 1);
    else
      return (1 << QB) - 1;
  };
  int vcur = (1 << QB) - 1;
  int crow[QB] = {};                               // this lane's rows' chunks, relative to the window
  if (GENERAL && have_cls) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
      crow[qb] = min(i_wave0 + 32 * qb + ql, d.Sq - 1) / mk.q_chunk - i_wg0 / mk.q_chunk;
  }
  // does row (qb, this lane) see key j?  From the per-block words in LDS when the planner ran,
  // else from the bitmap itself.
  auto sees = [&](int qb, int i, int j) __attribute__((always_inline)) -> bool {
    if (have_cls) return (seen[j / mk.kv_block] >> crow[qb]) & 1u;
    return mask_elem(mk, b, i, j);
  };
  auto tile_needed = [&](int t) __attribute__((always_inline)) -> bool {
    if (!GENERAL || !mk.allow) return true;
    return mask_rect(mk, b, i_wg0, i_wg1, t * TN, min(d.Skv, t * TN + TN) - 1) != 0;
  };
  auto next_tile = [&](int t) __attribute__((always_inline)) -> int {
    if (GENERAL && have_bits) return next_bit(bits, t, t_end);
    while (t < t_end && !tile_needed(t)) ++t;
    return __builtin_amdgcn_readfirstlane(min(t, t_end));      // wave-uniform (the bitmap is read through the vector path)
  };
  int cursor = next_tile(t_begin);                 // next tile to issue
  if (GENERAL && mk.allow && !have_bits) {
    nt = 0;
    for (int t = cursor; t < t_end; t = next_tile(t + 1)) ++nt;
  }

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
    const int rows = min(TN, d.Skv - t * TN);
    if (!GENERAL || rows == TN) {
#pragma unroll
      for (int k = 0; k < 2 * NCR; ++k) issue_part(t, st, k);
      return;
    }
    const long tile = (long)t * TN * row_bytes;    // ragged last tile: clamp the rows
    char* const kdst = st + wave * SM::GS;
    char* const vdst = kdst + SM::TILE;
#pragma unroll
    for (int c = 0; c < NCR; ++c) {
      const int sl = run_start(c) + lane;
      const unsigned r = (unsigned)min(4 * (sl / SM::SPR) + wave, rows - 1);
      const unsigned off = r * row_bytes + (unsigned)min(sl % SM::SPR, CPR - 1) * 16;
      dma16s(k0 + tile, off, kdst + run_start(c) * 16);
      dma16s(v0 + tile, off, vdst + run_start(c) * 16);
    }
  };
  constexpr int NDMA = 2 * NCR;                    // copies per wave and tile

  f32x16 dq[QB][DB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int i = 0; i < DB; ++i) { dq[qb][i] = zero16(); asm volatile("" : "+a"(dq[qb][i])); }

  // ---- building blocks, all on one 32-key half hb of the tile at st ---------------------------
  // S^T = K Q^T and dP^T = V dO^T: lane = query column, registers = keys.  The LDS operands of a
  // k-step are fetched while the matrix instructions of the previous one run; per_unit(m) is
  // vector work issued right after matrix instruction m (0 .. 4 KS - 1), to run in its shadow.
  static_assert(PF == 1, "the hand-over of first operands between phases assumes one set in flight");
  struct FirstKV { bf16x8 k, v; };                 // first operands of a score phase
  auto first_kv = [&](const char* __restrict__ st, int hb) __attribute__((always_inline)) -> FirstKV {
    const char* krow = st + tile_off<D>(ql, 32 * hb, 16 * g);
    return {*(const bf16x8*)krow, *(const bf16x8*)(krow + SM::TILE)};
  };
  auto first_kt = [&](const char* __restrict__ st, int hb) __attribute__((always_inline)) -> bf16x8 {
    return tile_tr_operand<D>(st, 32 * hb, 0, lane);
  };
  // first: the operands of k-step 0, fetched by the caller (during the previous phase in the
  // steady state); tail(): issued three matrix instructions before the end, fetches the first
  // operands of the next phase, so that no phase starts by waiting for LDS.
  auto score = [&](const char* __restrict__ st, int hb, f32x16 (&s)[QB], f32x16 (&p)[QB],
                   auto&& per_unit, const FirstKV& first, auto&& tail) __attribute__((always_inline)) {
    const char* krow = st + tile_off<D>(ql, 32 * hb, 16 * g);
    const char* vrow = krow + SM::TILE;
    bf16x8 ka[PF + 1], va[PF + 1];                 // operand sets, used in rotation
    ka[0] = first.k;
    va[0] = first.v;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int cu = ks % (PF + 1), nx = (ks + PF) % (PF + 1);
      if (ks + PF < KS) {
        ka[nx] = *(const bf16x8*)(krow + (ks + PF) * 32);
        va[nx] = *(const bf16x8*)(vrow + (ks + PF) * 32);
      }
#pragma unroll
      for (int j = 0; j < 2 * QB; ++j) {           // S^T of both query blocks, then dP^T
        const int qb = j % QB;
        if (j < QB) {
          if (ks == 0 && FOLD) mfma_from(s[qb], ka[cu], qf[qb][ks], nl2x[qb]);
          else if (ks == 0) mfma_first(s[qb], ka[cu], qf[qb][ks]);
          else mfma_next(s[qb], ka[cu], qf[qb][ks]);
        } else {
          if (ks == 0 && FOLD) mfma_from(p[qb], va[cu], gf[qb][ks], ndx[qb]);
          else if (ks == 0) mfma_first(p[qb], va[cu], gf[qb][ks]);
          else mfma_next(p[qb], va[cu], gf[qb][ks]);
        }
        per_unit(ks * 2 * QB + j);                 // vector work in the shadow of this instruction
        if (ks * 2 * QB + j == 2 * QB * KS - 3) tail();
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
  // key tail and masked elements of a half's scores -> -inf (wave-uniform decision, rarely taken)
  auto mask_scores = [&](int t, int hb, f32x16 (&s)[QB]) __attribute__((always_inline)) {
    if (!GENERAL) return;
    const int j0 = t * TN + 32 * hb;
    int cls = 1;
    if (mk.allow && i_wave0 < d.Sq)
      cls = have_cls ? class_of(cls_any, cls_all, t)      // (of the whole tile: fine for either half)
                     : mask_rect_tall(mk, b, i_wave0, min(d.Sq, i_wave0 + 32 * QB) - 1, min(j0, d.Skv - 1),
                                 min(d.Skv, j0 + 32) - 1);
    if (cls == 1 && j0 + 32 <= d.Skv) return;
    asm volatile("" ::: "memory");
    settle_scores(s);
    // mixed, but all keys of the half in one block of the bitmap (the usual case: blocks are
    // frames): one probe per query row instead of one per element
    const bool one_block = cls == 2 && j0 / mk.kv_block == (min(d.Skv, j0 + 32) - 1) / mk.kv_block;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int i = i_wave0 + 32 * qb + ql;
      const bool row_ok = one_block && i < d.Sq && sees(qb, i, j0);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int j = j0 + 8 * (v / 4) + 4 * g + (v % 4);
        bool ok = j < d.Skv && cls != 0;
        if (ok && cls == 2) ok = one_block ? row_ok : (i < d.Sq && sees(qb, i, j));
        if (!ok) s[qb][v] = -INFINITY;
      }
    }
  };
  // Conversion of scores into the dS operands, element x of a half (x = 0..31: query block
  // qb = x / 16, register v = x % 16): p = exp2(s c2 - L2), dS = p (dP - delta) -- with FOLD both
  // differences were formed by the accumulation already -- packed in pairs as bf16 into word
  // (v % 8) / 2 of operand v / 8 of the query block.
  // An element is started (its exp2) in one place and finished (multiply, packing) in the next, so
  // that between the matrix instructions of the pipelined loop the exponential's result is never
  // read by the very next instruction, which costs an idle issue slot: conv_elem(x) finishes
  // element x - 1 and starts element x; conv_last finishes element 31 of the half.
  struct Carry { float ds, ex; };
  auto conv_start = [&](int x, const f32x16 (&s)[QB]) __attribute__((always_inline)) -> float {
    const int qb = x / 16, v = x % 16;
    return __builtin_amdgcn_exp2f(FOLD ? s[qb][v] : fmaf(s[qb][v], c2, nl2[qb]));
  };
  auto conv_finish = [&](int x, Carry& cy, const f32x16 (&p)[QB], u32x4 (&dsw)[QB][2]) __attribute__((always_inline)) {
    const int qb = x / 16, v = x % 16;
    const float ds = cy.ex * (FOLD ? p[qb][v] : p[qb][v] + nd[qb]);
    if (v % 2 == 0) { cy.ds = ds; return; }
    const unsigned w2 = pack2_bf16(cy.ds, ds);
    dsw[qb][v / 8][(v % 8) / 2] = (LIST != 2 || ((vcur >> qb) & 1)) ? w2 : 0u;
  };
  auto conv_elem = [&](int x, Carry& cy, const f32x16 (&s)[QB], const f32x16 (&p)[QB],
                       u32x4 (&dsw)[QB][2]) __attribute__((always_inline)) {
    if (x > 0) conv_finish(x - 1, cy, p, dsw);
    cy.ex = conv_start(x, s);
  };
  auto conv_last = [&](Carry& cy, const f32x16 (&p)[QB], u32x4 (&dsw)[QB][2]) __attribute__((always_inline)) {
    conv_finish(31, cy, p, dsw);
  };
  auto convert = [&](const f32x16 (&s)[QB], const f32x16 (&p)[QB], u32x4 (&dsw)[QB][2]) __attribute__((always_inline)) {
    Carry cy;
#pragma unroll
    for (int x = 0; x < 32; ++x) conv_elem(x, cy, s, p, dsw);
    conv_last(cy, p, dsw);
  };
  // dQ^T += K^T dS^T over the 32 keys of a half (two k-steps of 16 keys)
  auto contract = [&](const char* __restrict__ st, int hb, const u32x4 (&dsw)[QB][2]) __attribute__((always_inline)) {
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 kt = tile_tr_operand<D>(st, 32 * hb + 16 * t2, 32 * db, lane);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) mfma_acc(dq[qb][db], kt, __builtin_bit_cast(bf16x8, dsw[qb][t2]));
      }
  };
  // contract(half h) on the matrix core together with the first XE conversions of half h+1 on
  // the vector ALU; the transposed operand of a pair of matrix instructions is fetched one pair
  // ahead, and nothing is scheduled across the units.
  auto contract_convert = [&](const char* __restrict__ st, int hb, const u32x4 (&dsi)[QB][2],
                              const f32x16 (&s)[QB], const f32x16 (&p)[QB], u32x4 (&dso)[QB][2],
                              Carry& cy, bf16x8 first, auto&& tail) __attribute__((always_inline)) {
    constexpr int NM = 2 * DB * QB;                // matrix instructions
    bf16x8 kt[PF + 1];
    kt[0] = first;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      const int c = m / QB, t2 = c / DB, db = c % DB, qb = m % QB, cu = c % (PF + 1);
      if (qb == 0 && c + PF < 2 * DB)
        kt[(c + PF) % (PF + 1)] = tile_tr_operand<D>(st, 32 * hb + 16 * ((c + PF) / DB), 32 * ((c + PF) % DB), lane);
      mfma_acc(dq[qb][db], kt[cu], __builtin_bit_cast(bf16x8, dsi[qb][t2]));
#pragma unroll
      for (int x = m * XE / NM; x < (m + 1) * XE / NM; ++x) conv_elem(x, cy, s, p, dso);
      if (m == NM - 3) tail();
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // score(half h+2) together with the remaining conversions of half h+1
  auto score_convert = [&](const char* __restrict__ st, int hb, f32x16 (&s_new)[QB], f32x16 (&p_new)[QB],
                           const f32x16 (&s)[QB], const f32x16 (&p)[QB], u32x4 (&dso)[QB][2],
                           Carry& cy, const FirstKV& first, auto&& tail, auto&& extra) __attribute__((always_inline)) {
    constexpr int NU = 2 * QB * KS;                // matrix instructions of a score phase
    score(st, hb, s_new, p_new, [&](int m) __attribute__((always_inline)) {
#pragma unroll
      for (int x = XE + m * (32 - XE) / NU; x < XE + (m + 1) * (32 - XE) / NU; ++x) conv_elem(x, cy, s, p, dso);
      extra(m);
    }, first, tail);
    conv_last(cy, p, dso);
  };

  // ---- pipeline.  Tile number q of the sequence lives in ring stage q % 4.  Per tile T (halves
  // 2T and 2T+1): contract 2T | convert 2T+1 | score 2T+2, then contract 2T+1 | convert 2T+2, the
  // one barrier of the tile -- every wave is done with tile T, whose stage takes tile T + 4, and
  // tile T + 2, issued two tiles ago, has landed -- and score 2T+3.
  int e[NSTG + 1];                                 // tile ids of tiles T .. T + 4 (static indexing only)
#pragma unroll
  for (int q = 0; q <= NSTG; ++q) e[q] = t_end;
#pragma unroll
  for (int q = 0; q < NSTG; ++q) {
    if (q < nt) {
      e[q] = cursor;
      issue_tile(tile_at(cursor), smem + q * SM::STAGE);
      cursor = next_tile(cursor + 1);
    }
  }
  wait_vmcnt<0>();
  __syncthreads();
  DQ_STAMP(stamp1);
  auto stage = [&](int q) __attribute__((always_inline)) -> char* { return smem + (q % NSTG) * SM::STAGE; };
  auto mid = [&](auto all_in_flight, bool issue, char* st_copy) __attribute__((always_inline)) {
    // (The general variant may spill registers inside the loop; its spill stores are counted with
    // the copies but complete out of order with them, so it always waits for everything.)
    // all_in_flight: tiles T + 2 and T + 3 were both issued, so leaving one tile's copies
    // outstanding still guarantees that tile T + 2 has landed
    if constexpr (decltype(all_in_flight)::value) wait_vmcnt<NDMA>();
    else wait_vmcnt<0>();
    wg_barrier();
    if (issue) {
      e[4] = cursor;
      issue_tile(tile_at(cursor), st_copy);
      cursor = next_tile(cursor + 1);
    }
  };

  f32x16 s0[QB], p0[QB], s1[QB], p1[QB];           // scores of even / odd halves
  u32x4 ds0[QB][2] = {}, ds1[QB][2] = {};          // packed dS operands of even / odd halves
  Carry cy;
  if (nt > 0) {
    vcur = vis_at(0);
    score(smem, 0, s0, p0, nothing, first_kv(smem, 0), no_tail);
    mask_scores(e[0], 0, s0);
    settle_scores(s0);
    settle_scores(p0);
    convert(s0, p0, ds0);
    score(smem, 1, s1, p1, nothing, first_kv(smem, 1), no_tail);
    mask_scores(e[0], 1, s1);
  }
  int T = 0;
  int id_next = LIST && cursor < t_end ? tlist[cursor] : 0;     // LIST: number of the next tile to copy
  FirstKV fkv;
  bf16x8 fkt = first_kt(smem, 0);                  // handed from phase to phase
  for (; T + 4 < nt; ++T) {                        // full tiles: tile T + 1 is scored, tile T + 4 issued
    char* const sa = stage(T);
    char* const sb = stage(T + 1);
    const int vnext = vis_at(T + 1);               // (the conversions under way are tile T's)
    contract_convert(sa, 0, ds0, s1, p1, ds1, cy, fkt, [&]() __attribute__((always_inline)) { fkv = first_kv(sb, 0); });
    score_convert(sb, 0, s0, p0, s1, p1, ds1, cy, fkv, [&]() __attribute__((always_inline)) { fkt = first_kt(sa, 1); }, nothing);
    mask_scores(e[1], 0, s0);
    vcur = vnext;                                  // from here on: scores of tile T + 1
    contract_convert(sa, 1, ds1, s0, p0, ds0, cy, fkt, [&]() __attribute__((always_inline)) { fkv = first_kv(sb, 1); });
    if constexpr (GENERAL) {
      mid(std::false_type{}, true, sa);
      score_convert(sb, 1, s1, p1, s0, p0, ds0, cy, fkv, [&]() __attribute__((always_inline)) { fkt = first_kt(sb, 0); }, nothing);
    } else {
      mid(std::true_type{}, false, sa);
      // the copies of tile T + 4 go out during the phase (LIST: its number was fetched a tile ago,
      // and the operands waited for here were fetched after it)
      const int t_new = LIST ? tile_of(__builtin_amdgcn_readfirstlane(id_next)) : cursor;
      e[4] = t_new;
      cursor = next_tile(cursor + 1);
      if (LIST) id_next = tlist[cursor < t_end ? cursor : t_begin];
      constexpr int EVERY = 2 * QB * KS / NDMA;
      static_assert(EVERY >= 1, "more copies than matrix instructions in the score phase");
      score_convert(sb, 1, s1, p1, s0, p0, ds0, cy, fkv, [&]() __attribute__((always_inline)) { fkt = first_kt(sb, 0); },
                    [&](int m) __attribute__((always_inline)) {
                      if (m % EVERY == EVERY - 1 && m / EVERY < NDMA) issue_part(t_new, sa, m / EVERY);
                    });
    }
    mask_scores(e[1], 1, s1);
    e[0] = e[1]; e[1] = e[2]; e[2] = e[3]; e[3] = e[4];
  }
  for (; T < nt; ++T) {                            // the last (at most four) tiles
    const bool more = T + 1 < nt;
    contract(stage(T), 0, ds0);
    settle_scores(s1);                             // (outside the pipelined loop the wait comes first, as a real dependence)
    settle_scores(p1);
    convert(s1, p1, ds1);
    if (more) vcur = vis_at(T + 1);
    if (more) { score(stage(T + 1), 0, s0, p0, nothing, first_kv(stage(T + 1), 0), no_tail); mask_scores(e[1], 0, s0); }
    contract(stage(T), 1, ds1);
    if (more) { settle_scores(s0); settle_scores(p0); convert(s0, p0, ds0); }
    mid(std::false_type{}, T + 4 < nt, stage(T));
    if (more) { score(stage(T + 1), 1, s1, p1, nothing, first_kv(stage(T + 1), 1), no_tail); mask_scores(e[1], 1, s1); }
    e[0] = e[1]; e[1] = e[2]; e[2] = e[3]; e[3] = e[4];
  }

  // ---- dQ += scale * acc.  The accumulators are transposed (lane = query row, registers =
  // columns), which would make every store instruction touch 64 rows; each wave therefore turns
  // its 64 rows around through LDS (the ring is free by now) and adds them to dq_accum a row
  // pair at a time, 64 lanes on 1 KB of consecutive addresses: read-add-write when this workgroup
  // is the only one on its rows in this launch (launches follow each other in stream order);
  // when the key range is split over several workgroups, each stores its sums in its own slice
  // of the workspace and a reduction follows the kernel (float atomics from every split would
  // be bounded by the L2 atomic rate, about 80 G elements per second).
  // The last matrix instructions must have retired before their registers are read.
  DQ_STAMP(stamp2);
  if constexpr (DB == 4) {
    asm volatile("s_nop 15\n\ts_nop 15" : "+a"(dq[0][0]), "+a"(dq[0][1]), "+a"(dq[0][2]), "+a"(dq[0][3]),
                 "+a"(dq[1][0]), "+a"(dq[1][1]), "+a"(dq[1][2]), "+a"(dq[1][3]));
  } else if constexpr (DB == 3) {
    asm volatile("s_nop 15\n\ts_nop 15" : "+a"(dq[0][0]), "+a"(dq[0][1]), "+a"(dq[0][2]),
                 "+a"(dq[1][0]), "+a"(dq[1][1]), "+a"(dq[1][2]));
  } else {
    asm volatile("s_nop 15\n\ts_nop 15" : "+a"(dq[0][0]), "+a"(dq[0][1]), "+a"(dq[1][0]), "+a"(dq[1][1]));
  }
  __syncthreads();                                 // every wave is done reading the ring
  constexpr int RP = (D + 4) * 4;                  // row pitch in bytes (+16: the b128 writes of 16 rows tile the banks)
  static_assert(NWV * 32 * QB * RP <= SM::RING, "the turn-around buffer must fit the ring");
  char* const tbuf = smem + wave * (32 * QB * RP);
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4 y = {dq[qb][db][4 * q4] * d.scale, dq[qb][db][4 * q4 + 1] * d.scale,
                         dq[qb][db][4 * q4 + 2] * d.scale, dq[qb][db][4 * q4 + 3] * d.scale};
        *(f32x4*)(tbuf + (32 * qb + ql) * RP + (32 * db + 8 * q4 + 4 * g) * 4) = y;
      }
  // (each wave reads back only what it wrote itself: no barrier, the LDS queue keeps the order)
  constexpr int LPR = D / 4;                       // lanes per row, four floats each
  constexpr int RPI = 64 / LPR;                    // rows per instruction
  constexpr bool EVEN = 64 % LPR == 0 && (32 * QB) % RPI == 0;    // else: idle lanes, and a last instruction with fewer rows
  const int rsub = lane / LPR, col = (lane % LPR) * 4;
  const bool whole = a.n_split_dq == 1;            // else: this split's own slice of the partial sums
  float* const out0 = (whole ? a.dq_accum : a.dq_part + (long)split * d.B * d.Hq * d.Sq * D) +
                      (((long)b * d.Hq + hq) * d.Sq) * D;
  // (dq_accum and the partial sums are contiguous [B,Hq,Sq,D]: row i of the group's list is row i
  // past the first row of the group's first head)
  // Eight instructions' worth of rows at a time: their old values are all requested before the
  // first sum is stored (a store, or a branch, between two loads would make the second wait for
  // the first: one round trip per instruction instead of one per eight).  Rows past the last one
  // re-read it and store nothing.
  constexpr int NB = 8;
  for (int r00 = 0; r00 < 32 * QB; r00 += NB * RPI) {
    f32x4 old[NB];
    if (whole) {
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int i = min(i_wave0 + r00 + u * RPI + rsub, rows_lim - 1);
        old[u] = *(const f32x4*)(out0 + (long)i * D + col);
      }
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int r = r00 + u * RPI + rsub, i = i_wave0 + r;
      const bool ok = i < rows_lim && r < 32 * QB && (EVEN || rsub < RPI);
      if (!ok) continue;
      f32x4 y = *(const f32x4*)(tbuf + r * RP + col * 4);
      if (whole) y += old[u];
      *(f32x4*)(out0 + (long)i * D + col) = y;
    }
  }
#ifdef LVX_DQ_PROBE
  wait_vmcnt<0>();
  const unsigned long long stamp3 = __builtin_readcyclecounter();
  if (tid == 0) {
    atomicAdd(&dq_probe[0], stamp1 - stamp0);
    atomicAdd(&dq_probe[1], stamp2 - stamp1);
    atomicAdd(&dq_probe[2], stamp3 - stamp2);
    atomicAdd(&dq_probe[3], 1ull);
    atomicAdd(&dq_probe[4], (unsigned long long)nt);
  }
#endif
}

template <int D, bool GENERAL, int LIST = 0>
hipError_t launch(const BwdArgs& a, long grid, hipStream_t s) {
  static SmemOnce once;
  hipError_t e = ensure_dynamic_lds((const void*)bwd_dq_bf16_kernel<D, GENERAL, LIST>, DqSmem<D>::TOTAL, &once);
  if (e != hipSuccess) return e;
  bwd_dq_bf16_kernel<D, GENERAL, LIST><<<(unsigned)grid, 256, DqSmem<D>::TOTAL, s>>>(a);
  return hipGetLastError();
}

}  // namespace

int bwd_bf16_pick_split(const Dims& d, int n_cu, bool masked) {
  // one workgroup per CU; split the KV axis until the grid covers the chip (four times as many
  // workgroups with a media mask, whose visible work differs from one query tile to the next)
  // (the dense kernel tiles the rows of a whole group of query heads, the general one each head's)
  const bool dense = !masked && (d.Skv % TN == 0 || d.Skv >= 2 * TN);
  const long base = dense ? (long)d.B * d.Hkv * (((long)(d.Hq / d.Hkv) * d.Sq + QM - 1) / QM)
                          : (long)d.B * d.Hq * ((d.Sq + QM - 1) / QM);
  const int n_tiles = (d.Skv + TN - 1) / TN;
  long cap = n_tiles / 16;                // keep at least 16 tiles (1024 keys) per split
  if (cap < 1) cap = 1;
  if (!masked) {
    // about 5.5 TFLOP/s per compute unit in this kernel; a split's sums are float32 rows written
    // once and read once by the reduction at about 3 TB/s
    const double t_full = 6.0 * QM * (double)d.Skv * d.D / 5.5e12;
    const double t_part = 2.0 * (double)d.B * d.Hq * d.Sq * d.D * 4.0 / 3e12;
    return pick_split_balanced(base, n_cu, cap, t_full, t_part);
  }
  long want = (4L * n_cu + base - 1) / base;
  if (want < 1) want = 1;
  if (want > cap) want = cap;
  if (want > 64) want = 64;
  return (int)want;
}

namespace {

hipError_t launch_one(const BwdArgs& a, bool general, hipStream_t s) {
  const Dims& d = a.d;
  const int G = d.Hq / d.Hkv;
  const bool list = a.dq_pass == 1 || a.dq_pass == 3;   // the dense kernel over a list of tiles: rows tiled per head
  const long per_split = general || list ? (long)G * ((d.Sq + QM - 1) / QM) : ((long)G * d.Sq + QM - 1) / QM;
  const long grid = a.dq_pass == 3 ? (long)d.B * d.Hq * a.n_split_dq * ((d.Sq + QM - 1) / QM)
                                   : xcd_grid(d.B * d.Hkv, (int)(a.n_split_dq * per_split));
  hipError_t e;
  if (a.dq_pass == 3) e = d.D == 64 ? launch<64, false, 2>(a, grid, s) : d.D == 96 ? launch<96, false, 2>(a, grid, s) : launch<128, false, 2>(a, grid, s);
  else if (list) e = d.D == 64 ? launch<64, false, 1>(a, grid, s) : d.D == 96 ? launch<96, false, 1>(a, grid, s) : launch<128, false, 1>(a, grid, s);
  else if (d.D == 64) e = general ? launch<64, true>(a, grid, s) : launch<64, false>(a, grid, s);
  else if (d.D == 96) e = general ? launch<96, true>(a, grid, s) : launch<96, false>(a, grid, s);
  else e = general ? launch<128, true>(a, grid, s) : launch<128, false>(a, grid, s);
  if (e == hipSuccess && a.n_split_dq > 1)
    e = launch_dq_reduce(a.dq_part, a.n_split_dq, (long)d.B * d.Hq * d.Sq * d.D, a.dq_accum, s);
  return e;
}

}  // namespace

hipError_t launch_bwd_dq_bf16(const BwdArgs& a, hipStream_t s) {
  const Dims& d = a.d;
  if (a.mask.allow != nullptr) {
    // Two launches when the general kernel's planner is sure to take the mask (it must leave out
    // exactly the tiles of the first launch) and the tile list fits: the dense kernel on the key
    // tiles every row of a workgroup sees, then the general kernel on the other visible tiles.
    // Both add into dq_accum, one after the other on the stream.
    const int n_tiles = (d.Skv + TN - 1) / TN;
    const int h_max = (QM - 1) / a.mask.q_chunk + 2, w = (d.Skv - 1) / a.mask.kv_block + 1;
    // One launch of the dense kernel over the tiles any row of a workgroup sees, when the mask
    // never cuts through a 32-row block or a key tile and the list fits.
    const bool fits = d.Skv % TN == 0 && n_tiles <= DqSmem<128>::WIN_BYTES / 4 - 1 &&
                      ((w + 1) & ~1) + (n_tiles + 63) / 64 * 2 <= DqSmem<128>::BITS_BYTES / 4;
    if (fits && a.mask.q_chunk % 32 == 0 && a.mask.kv_block % TN == 0) {
      BwdArgs p3 = a;
      p3.dq_pass = 3;
      if (p3.n_split_dq > 1) p3.n_split_dq /= 2;    // (its workgroups start longest first: half the splits even the load out)
      return launch_one(p3, false, s);
    }
    const bool two = d.Skv % TN == 0 && plan_fits(h_max, w, n_tiles, DqSmem<128>::BITS_BYTES, DqSmem<128>::WIN_BYTES) &&
                     n_tiles <= DqSmem<128>::WIN_BYTES / 4 - 1 && ((w + 1) & ~1) + (n_tiles + 63) / 64 * 2 <= DqSmem<128>::BITS_BYTES / 4;
    if (!two) return launch_one(a, true, s);
    BwdArgs p1 = a, p2 = a;
    p1.dq_pass = 1;
    p2.dq_pass = 2;
    const hipError_t e = launch_one(p1, false, s);
    return e != hipSuccess ? e : launch_one(p2, true, s);
  }
  const int tail = d.Skv % TN;
  if (tail == 0) return launch_one(a, false, s);
  if (d.Skv < 2 * TN) return launch_one(a, true, s);
  // A key count that is no multiple of the tile: the dense kernel takes the whole tiles, the
  // general one the few keys that are left; dQ is a sum over keys, and both add into dq_accum
  // one after the other on the stream.
  BwdArgs head = a;
  head.d.Skv = d.Skv - tail;
  hipError_t e = launch_one(head, false, s);
  if (e != hipSuccess) return e;
  BwdArgs rest = a;
  rest.k = (const uint16_t*)a.k + (long)head.d.Skv * d.kv_ss;
  rest.v = (const uint16_t*)a.v + (long)head.d.Skv * d.kv_ss;
  rest.d.Skv = tail;
  rest.n_split_dq = 1;
  rest.dq_part = nullptr;
  return launch_one(rest, true, s);
}

hipError_t launch_bwd_bf16(const BwdArgs& a, unsigned stages, hipStream_t s) {
  hipError_t e = hipSuccess;
  if ((stages & 6) == 6 && a.dq_tiles != nullptr) {
    // One pass over the whole tiles of 256 keys with the fused kernel; the keys that are left go
    // through the two kernels below (dQ is a sum over keys, dK and dV rows are independent).
    e = launch_bwd_fused_bf16(a, s);
    const int done = a.d.Skv / 256 * 256;
    if (e != hipSuccess || done == a.d.Skv) return e;
    BwdArgs rest = a;
    rest.k = (const uint16_t*)a.k + (long)done * a.d.kv_ss;
    rest.v = (const uint16_t*)a.v + (long)done * a.d.kv_ss;
    rest.dk = (uint16_t*)a.dk + (long)done * a.d.kv_ss;
    rest.dv = (uint16_t*)a.dv + (long)done * a.d.kv_ss;
    rest.d.Skv = a.d.Skv - done;
    rest.n_split_dq = 1;
    rest.dq_part = nullptr;
    rest.dq_tiles = nullptr;
    return launch_bwd_bf16(rest, stages, s);
  }
  if (stages & 2) e = launch_bwd_dkdv_bf16(a, s);
  if (e == hipSuccess && (stages & 4)) e = launch_bwd_dq_bf16(a, s);
  return e;
}

}  // namespace lvx

#ifdef LVX_DQ_PROBE
extern "C" int lvx_debug_dq_probe(unsigned long long* out8) {
  if (hipDeviceSynchronize() != hipSuccess) return 1;
  if (hipMemcpyFromSymbol(out8, HIP_SYMBOL(lvx::dq_probe), 8 * sizeof(unsigned long long)) != hipSuccess) return 1;
  const unsigned long long z[8] = {};
  return hipMemcpyToSymbol(HIP_SYMBOL(lvx::dq_probe), z, sizeof(z)) == hipSuccess ? 0 : 1;
}
#endif
