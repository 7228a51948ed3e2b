// bf16 forward kernel for masked or ragged problems (media mask present, or Skv not a multiple of
// the key tile): the FlashAttention call of Algorithm 1 with every matrix instruction left to the
// compiler.  The dense kernel (lvx_fwd_bf16.hip) pins registers and hand-schedules its pipeline
// around matrix instructions the compiler cannot see; mask code between its phases -- branches,
// lane-masked regions, probes of the bitmap -- proved fragile there, so everything that needs it
// runs here instead.
//
// Workgroup = 8 wavefronts = 256 query rows of one (batch, query head), one workgroup per CU; each
// wave owns 32 rows whose Q operands stay in registers for the whole kernel.  K/V tiles of 64 keys
// travel HBM -> LDS by direct global-to-LDS copies into a ring of four stages, issued three tiles
// ahead, one barrier per tile.  Per tile a wave computes S^T = K Q^T (keys in registers, one query
// column per lane), the online softmax in that layout (row statistics are per-lane scalars; the
// two half-waves exchange one value per tile), and O^T += V^T P^T with P^T taken straight from the
// score registers and V^T fetched by transposing LDS reads.  The running maximum is only raised
// when a tile exceeds it by more than 2^6 (any reference value cancels between numerator and
// denominator).  With a media mask the window of the bitmap the workgroup can touch is copied to
// LDS and the visibility of every tile is worked out by all threads at once; KV splits share the
// visible tiles evenly; waves skip tiles none of their rows see.  Unmasked ragged problems run a
// half-tile software pipeline (score product of the next half under the softmax of the current).
// The grid is cut along the KV axis (split-KV) when the query block alone cannot fill the chip;
// partial (O, L) pairs are combined by the merge kernel.
#include "lvx_internal.h"
#include "lvx_mfma.h"

#include <type_traits>


namespace lvx {

namespace {

constexpr int BM = 256;       // query rows per workgroup
constexpr int BN = 64;        // keys per tile
constexpr int NW = 8;         // waves per workgroup
constexpr int NS = 4;         // LDS ring stages
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LAZY = 6.0f;  // raise the running max only when a tile tops it by 2^LAZY

template <int D> struct FwdSmem {
  static constexpr int CPR = D / 8;            // 16-byte chunks of real data per row
  static constexpr int KCH = CPR + 1;          // K row: + 16 B pad  (conflict-free b128 reads)
  static constexpr int VCH = CPR + 4;          // V row: + 64 B pad  (conflict-free transposing reads)
  static constexpr int KP = KCH * 16, VP = VCH * 16;
  static constexpr int K_BYTES = BN * KP;      // = KCH wave-copies of 1 KB
  static constexpr int V_BYTES = BN * VP;      // = VCH wave-copies of 1 KB
  static constexpr int STAGE = K_BYTES + V_BYTES;
  static constexpr int NCOPY = KCH + VCH;      // wave-level copies per tile
  static constexpr int L = (NCOPY + NW - 1) / NW;   // copies issued by every wave per tile
  static constexpr int RING = NS * STAGE;
  static constexpr int BITS_BYTES = 4096;      // visibility bits of up to 32704 tiles (media mask only)
  static constexpr int WIN_BYTES = 8192;       // window of the mask bitmap (media mask only)
  static constexpr int TOTAL = RING + BITS_BYTES + WIN_BYTES;
};

template <int D>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
fwd_general_bf16_kernel(FwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  using SM = FwdSmem<D>;
  constexpr int KS = D / 16;            // k-steps of the QK^T product
  constexpr int DB = D / 32;            // 32-row blocks of O^T
  constexpr int L = SM::L;

  const Dims& d = a.d;
  const int G = d.Hq / d.Hkv;
  const int n_qt = (d.Sq + BM - 1) / BM;
  HeadWork hw;
  if (!xcd_decode(blockIdx.x, d.B * d.Hkv, a.n_split * G * n_qt, &hw)) return;
  const int b = hw.head / d.Hkv, hk = hw.head % d.Hkv;
  const int split = hw.item / (G * n_qt);
  const int hq = hk * G + (hw.item % (G * n_qt)) / n_qt;
  const int qt = hw.item % n_qt;

  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, ql = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i_wave0 = qt * BM + wave * 32;          // first query row of this wave
  const int i_lane = i_wave0 + ql;                  // this lane's query row (column of S^T)

  // KV range of this split, in tiles
  const int n_tiles = (d.Skv + BN - 1) / BN;
  const int tps = (n_tiles + a.n_split - 1) / a.n_split;
  int t_begin = split * tps;                        // (with a media mask: re-cut below over the visible tiles)
  int t_end = min(n_tiles, t_begin + tps);

  // Q operands (B of S^T = K Q^T): lane holds row i_lane, columns 16 ks + 8 g + 0..7
  bf16x8 qf[KS];
  {
    const uint16_t* qrow = (const uint16_t*)a.q + b * d.q_sb + hq * d.q_sh + (long)i_lane * d.q_ss;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 x = {0, 0, 0, 0};
      if (i_lane < d.Sq) x = *(const u32x4*)(qrow + 16 * ks + 8 * g);
      qf[ks] = __builtin_bit_cast(bf16x8, x);
    }
    // Touch the registers now, so that these loads are complete before the tile copies start:
    // otherwise the first use inside the loop would make the compiler drain every copy in flight.
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[ks]));
  }

  // ---- tile copies: wave w issues copies n = w, w + 8, ... (mod NCOPY; the few surplus copies
  // repeat an earlier one).  Copy n < KCH fills 1 KB of the K stage, the others of the V stage;
  // lane l of copy n fills 16-byte slot 64 n + l = (row, chunk) of the padded tile; pad slots
  // re-read the row's last chunk.
  const char* kbase = (const char*)((const uint16_t*)a.k + b * d.kv_sb + hk * d.kv_sh);
  const char* vbase = (const char*)((const uint16_t*)a.v + b * d.kv_sb + hk * d.kv_sh);
  const long row_bytes = d.kv_ss * 2;
  auto copy_slot = [&](int i, int& row, int& col, int& lds, bool& is_k) {
    const int n = (wave + NW * i) % SM::NCOPY;
    is_k = n < SM::KCH;
    const int slot = 64 * (is_k ? n : n - SM::KCH) + lane;
    const int ch = is_k ? SM::KCH : SM::VCH;
    row = slot / ch;
    col = min(slot % ch, SM::CPR - 1) * 16;
    lds = is_k ? n * 1024 : SM::K_BYTES + (n - SM::KCH) * 1024;
  };
  unsigned cp_off[L];
#pragma unroll
  for (int i = 0; i < L; ++i) {
    int row, col, lds; bool is_k;
    copy_slot(i, row, col, lds, is_k);
    cp_off[i] = (unsigned)(row * row_bytes + col);
  }
  auto issue_tile = [&](int t, char* st) {
    const int j0 = t * BN;
    const int rows = min(BN, d.Skv - j0);
    const char* kt = kbase + (long)j0 * row_bytes;
    const char* vt = vbase + (long)j0 * row_bytes;
    if (rows == BN) {
#pragma unroll
      for (int i = 0; i < L; ++i) {
        int row, col, lds; bool is_k;
        copy_slot(i, row, col, lds, is_k);           // lds, is_k: wave-uniform
        dma16s(is_k ? kt : vt, cp_off[i], st + lds);
      }
    } else {                                          // ragged last tile: re-read its last row
      asm volatile("" ::: "memory");
#pragma unroll
      for (int i = 0; i < L; ++i) {
        int row, col, lds; bool is_k;
        copy_slot(i, row, col, lds, is_k);
        dma16s(is_k ? kt : vt, (unsigned)(min(row, rows - 1) * row_bytes + col), st + lds);
      }
    }
  };

  // which tiles does this workgroup need at all (media mask)?  The window of the bitmap that its
  // rows and key range can touch is copied to LDS, and the visibility of every tile is worked out
  // by all threads at once into a bit array, so that the loop never waits on the bitmap.
  const int i_wg0 = qt * BM, i_wg1 = min(d.Sq, i_wg0 + BM) - 1;
  MaskDev mk = a.mask;
  unsigned* const bits = (unsigned*)(smem + SM::RING);
  bool have_bits = false;
  if (mk.allow) {
    if (n_tiles <= (SM::BITS_BYTES - 16) * 8) {
      // bits over ALL tiles of the key range; the splits then share the visible tiles evenly
      mk = mask_to_lds(a.mask, b, i_wg0 / mk.q_chunk, i_wg1 / mk.q_chunk, 0, (d.Skv - 1) / mk.kv_block,
                       (uint8_t*)smem + SM::RING + SM::BITS_BYTES, SM::WIN_BYTES, tid, 64 * NW);
      have_bits = true;
      const int nn = build_bits(bits, n_tiles, tid, 64 * NW, [&](int t) {
        // (pass 2 leaves the tiles that every row of the workgroup sees to the other launch)
        const int c = mask_rect_tall(mk, b, i_wg0, i_wg1, t * BN, min(d.Skv, t * BN + BN) - 1);
        return c != 0 && !(a.pass == 2 && c == 1);
      });
      const int k0 = (int)((long)split * nn / a.n_split), k1 = (int)((long)(split + 1) * nn / a.n_split);
      t_begin = nth_bit(bits, k0, n_tiles);
      t_end = k1 > k0 ? nth_bit(bits, k1 - 1, n_tiles) + 1 : t_begin;
    } else if (t_begin < t_end) {
      mk = mask_to_lds(a.mask, b, i_wg0 / mk.q_chunk, i_wg1 / mk.q_chunk, (t_begin * BN) / mk.kv_block,
                       (min(d.Skv, t_end * BN) - 1) / mk.kv_block, (uint8_t*)smem + SM::RING + SM::BITS_BYTES,
                       SM::WIN_BYTES, tid, 64 * NW);
    }
  }
  auto next_tile = [&](int t) -> int {
    if (mk.allow) {
      if (have_bits) return next_bit(bits, t, t_end);
      for (; t < t_end; ++t) {
        const int c = mask_rect(mk, b, i_wg0, i_wg1, t * BN, min(d.Skv, t * BN + BN) - 1);
        if (c != 0 && !(a.pass == 2 && c == 1)) break;
      }
    }
    return __builtin_amdgcn_readfirstlane(min(t, t_end));      // wave-uniform (the bitmap is read through the vector path)
  };
  auto wave_class = [&](int t) -> int {               // 0 skip, 1 dense, 2 per-element mask
    if (t >= t_end || i_wave0 >= d.Sq) return 0;
    if (!mk.allow) return 1;
    return mask_rect_tall(mk, b, i_wave0, min(d.Sq - 1, i_wave0 + 31), t * BN, min(d.Skv, t * BN + BN) - 1);
  };

  f32x16 oacc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i) oacc[i] = zero16();
  float m_ref = -INFINITY;     // reference maximum of raw scores baked into l_run and oacc
  float l_run = 0.f;           // this lane's share of the running sum of exp
  const float c2 = d.scale * LOG2E;

  // ---- building blocks, all on one 32-key HALF of a tile (kb = 0 or 1) -----------------------
  // S^T half: 32 keys x 32 queries
  auto scores_half = [&](const char* ks_, int kb, f32x16& s) {
    s = zero16();
    const char* krow = ks_ + (kb * 32 + ql) * SM::KP + g * 16;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) s = mfma32(*(const bf16x8*)(krow + ks * 32), qf[ks], s);
  };
  // key tail and mixed-mask elements -> -inf
  auto mask_half = [&](int t, int kb, int cls, f32x16& s) {
    const int j0 = t * BN + kb * 32;
    if (j0 + 32 > d.Skv || cls == 2) {
      asm volatile("" ::: "memory");            // a real branch: never speculate this into the hot path
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int j = j0 + 8 * (v / 4) + 4 * g + (v % 4);
        bool ok = j < d.Skv;
        if (ok && cls == 2) ok = (i_lane < d.Sq) && mask_elem(mk, b, i_lane, j);
        if (!ok) s[v] = -INFINITY;
      }
    }
  };
  auto half_max = [&](const f32x16& s) -> float {
    float m = s[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) m = fmaxf(m, s[v]);
    return m;
  };
  // the (rare) raise of the reference maximum, given this lane's maximum of a new score half
  auto raise_ref = [&](float tmax) {
    tmax = xhalf_max(tmax);
    // (tmax - m_ref) * c2 > LAZY: NaN (both -inf) compares false, m_ref = -inf with a finite tmax true
    if (__any((tmax - m_ref) * c2 > LAZY)) {
      asm volatile("" ::: "memory");            // keep this a real, rarely taken branch
      const float m_new = fmaxf(m_ref, tmax);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f((m_ref - m_safe) * c2);   // m_ref = -inf -> 0
      m_ref = m_new;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;
    }
  };
  // P half = exp2((s - m_ref) c2), row sums, and O^T += V^T P^T for these 32 keys (no overlap)
  auto probs_pv_half = [&](const char* vs_, int kb, f32x16& s) {
    const float mc = (m_ref == -INFINITY) ? 0.f : m_ref * c2;
    float psum = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float pr = __builtin_amdgcn_exp2f(fmaf(s[v], c2, -mc));
      s[v] = pr;
      psum += pr;
    }
    l_run += psum;
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
      const bf16x8 pf = cvt_operand(s, 8 * t2);
#pragma unroll
      for (int db = 0; db < DB; ++db)
        oacc[db] = mfma32(load_tr_operand(vs_, SM::VP, 32 * kb + 16 * t2, 32 * db, lane), pf, oacc[db]);
    }
  };
  // Hand-interleaved half step of the dense pipeline.  The score product of the NEXT half (nxt)
  // runs on the matrix core while the vector ALU turns the CURRENT half's scores (cur, keys kb of
  // the tile at vs_) into probabilities; then P V of the current half runs while the vector ALU
  // takes the maximum of the next half.  LDS operands are fetched one phase ahead, so that no
  // matrix instruction waits for an LDS round trip: kop holds the K operands of the half being
  // scored and is refilled, during the P V phase, with those of half kb_pre of the tile at k_pre;
  // the V operands are fetched during the score phase.  Scheduling barriers keep the chunks (and
  // with them the register pressure) as written.  Returns this lane's maximum of nxt.
  auto fused_half = [&](const char* k_pre, int kb_pre, const char* vs_, int kb, f32x16& cur,
                        f32x16& nxt, bf16x8 (&kop)[KS]) -> float {
    // (the 16 probabilities of a lane are produced KS-th by KS-th under the score k-steps:
    // elements [16 c / KS, 16 (c + 1) / KS) under step c, which is 2 or 3 of them when KS = 6)
    const float mc = (m_ref == -INFINITY) ? 0.f : m_ref * c2;
    float psum = 0.f;
    bf16x8 pfrag[2], vop[KS];                     // KS == 2 * DB V operands per half
    nxt = zero16();
#pragma unroll
    for (int c = 0; c < KS; ++c) {
      vop[c] = load_tr_operand(vs_, SM::VP, 32 * kb + 16 * (c / DB), 32 * (c % DB), lane);
      nxt = mfma32(kop[c], qf[c], nxt);
#pragma unroll
      for (int e = 16 * c / KS; e < 16 * (c + 1) / KS; ++e) {
        const float pr = __builtin_amdgcn_exp2f(fmaf(cur[e], c2, -mc));
        cur[e] = pr;
        psum += pr;
      }
      if (16 * c / KS < 8 && 16 * (c + 1) / KS >= 8) pfrag[0] = cvt_operand(cur, 0);
      if (c == KS - 1) pfrag[1] = cvt_operand(cur, 8);
      __builtin_amdgcn_sched_barrier(0);
    }
    l_run += psum;
    const char* krow = k_pre + (kb_pre * 32 + ql) * SM::KP + g * 16;
    float tmax = -INFINITY;
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
#pragma unroll
      for (int db = 0; db < DB; ++db) oacc[db] = mfma32(vop[t2 * DB + db], pfrag[t2], oacc[db]);
#pragma unroll
      for (int i = 0; i < KS / 2; ++i) kop[t2 * (KS / 2) + i] = *(const bf16x8*)(krow + (t2 * (KS / 2) + i) * 32);
#pragma unroll
      for (int i = 0; i < 8; ++i) tmax = fmaxf(tmax, nxt[8 * t2 + i]);
      __builtin_amdgcn_sched_barrier(0);
    }
    return tmax;
  };

  // ---- pipeline over the needed tiles: id0 is being finished, id1 gets its scores, id2 is in
  // flight, id3 is issued.  Tile number q of the sequence lives in ring stage q % NS.
  int id0 = next_tile(t_begin);
  int id1 = id0 < t_end ? next_tile(id0 + 1) : t_end;
  int id2 = id1 < t_end ? next_tile(id1 + 1) : t_end;
  if (id0 < t_end) issue_tile(id0, smem);
  if (id1 < t_end) issue_tile(id1, smem + SM::STAGE);
  if (id2 < t_end) issue_tile(id2, smem + 2 * SM::STAGE);
  if (id0 < t_end) {
    if (id2 < t_end) wait_vmcnt<2 * L>();
    else if (id1 < t_end) wait_vmcnt<L>();
    else wait_vmcnt<0>();
    wg_barrier();
  }
  int seq = 0;                                   // sequence number of id0
  // Per tile, in both loops: wait until tile id1 has landed (tile id0 already has), cross the
  // barrier (every wave is then done with tile seq - 1, whose stage is free), issue tile id3.
  auto advance = [&](char* st_copy) {
    if (id1 < t_end && id2 < t_end) wait_vmcnt<L>();
    else wait_vmcnt<0>();
    wg_barrier();
    int id3 = t_end;
    if (id2 < t_end) id3 = next_tile(id2 + 1);
    if (id3 < t_end) issue_tile(id3, st_copy);
    return id3;
  };
  const bool slow = mk.allow != nullptr || i_wave0 >= d.Sq;   // wave-uniform
  if (!slow) {
    // dense pipeline, one 32-key half ahead.  The three LDS stages a tile step touches are
    // distinct, and saying so (__restrict__) keeps the compiler from draining the copies in
    // flight before the LDS reads of the step.
    const int ragged_tile = (d.Skv % BN) ? n_tiles - 1 : -1;
    f32x16 s0, s1;
    bf16x8 kop[KS];
    if (id0 < t_end) {
      scores_half(smem, 0, s0);
      if (id0 == ragged_tile) { asm volatile("" ::: "memory"); mask_half(id0, 0, 1, s0); }
      raise_ref(half_max(s0));
#pragma unroll
      for (int c = 0; c < KS; ++c) kop[c] = *(const bf16x8*)(smem + (32 + ql) * SM::KP + g * 16 + c * 32);
    }
    auto tile_step = [&](auto last_t, char* __restrict__ st_copy, const char* __restrict__ st_next,
                         const char* __restrict__ st_cur) {
      constexpr bool LAST = decltype(last_t)::value;
      const int id3 = advance(st_copy);            // tile id1 (if any) has landed from here on
      const char* vs_ = st_cur + SM::K_BYTES;
      // first half -> probabilities, second half of the same tile -> scores
      float tm = fused_half(st_next, 0, vs_, 0, s0, s1, kop);
      if (id0 == ragged_tile) { asm volatile("" ::: "memory"); mask_half(id0, 1, 1, s1); tm = half_max(s1); }
      raise_ref(tm);
      if constexpr (!LAST) {
        // second half -> probabilities, first half of the next tile -> scores
        tm = fused_half(st_next, 1, vs_, 1, s1, s0, kop);
        if (id1 == ragged_tile) { asm volatile("" ::: "memory"); mask_half(id1, 0, 1, s0); tm = half_max(s0); }
        raise_ref(tm);
      } else {
        probs_pv_half(vs_, 1, s1);
      }
      id0 = id1; id1 = id2; id2 = id3;
      ++seq;
    };
    while (id1 < t_end)
      tile_step(std::false_type{}, smem + ((seq + 3) % NS) * SM::STAGE, smem + ((seq + 1) % NS) * SM::STAGE,
                smem + (seq % NS) * SM::STAGE);
    if (id0 < t_end)
      tile_step(std::true_type{}, smem + ((seq + 3) % NS) * SM::STAGE, smem + ((seq + 1) % NS) * SM::STAGE,
                smem + (seq % NS) * SM::STAGE);
  } else {
    // general path (media mask, or a wave without query rows): tile by tile, no software pipeline
    auto tile_step = [&](char* __restrict__ st_copy, const char* __restrict__ st_cur) {
      const int cls = wave_class(id0);
      if (cls != 0) {
        f32x16 s0, s1;
        scores_half(st_cur, 0, s0);
        scores_half(st_cur, 1, s1);
        mask_half(id0, 0, cls, s0);
        mask_half(id0, 1, cls, s1);
        raise_ref(fmaxf(half_max(s0), half_max(s1)));
        probs_pv_half(st_cur + SM::K_BYTES, 0, s0);
        probs_pv_half(st_cur + SM::K_BYTES, 1, s1);
      }
      const int id3 = advance(st_copy);
      id0 = id1; id1 = id2; id2 = id3;
      ++seq;
    };
    while (id0 < t_end)
      tile_step(smem + ((seq + 3) % NS) * SM::STAGE, smem + (seq % NS) * SM::STAGE);
  }

  // ---- epilogue: O = acc / l, L = m * scale + ln l
  const float l_tot = xhalf_sum(l_run);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  const float lse = l_tot > 0.f ? m_ref * d.scale + logf(l_tot) : -INFINITY;
  if (i_lane >= d.Sq) return;
  const long row = ((long)b * d.Hq + hq) * d.Sq + i_lane;
  if (a.n_split > 1 || a.partial) {
    const long slice = (long)(a.part0 + split) * d.B * d.Hq * d.Sq;
    float* o = a.o_part + (slice + row) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 y = {oacc[db][4 * q4] * inv, oacc[db][4 * q4 + 1] * inv, oacc[db][4 * q4 + 2] * inv,
                   oacc[db][4 * q4 + 3] * inv};
        *(f32x4*)(o + 32 * db + 8 * q4 + 4 * g) = y;
      }
    if (g == 0) a.lse_part[slice + row] = lse;
    return;
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
        f32x4 y = {w0 * x[0] + w1 * oacc[db][4 * q4], w0 * x[1] + w1 * oacc[db][4 * q4 + 1],
                   w0 * x[2] + w1 * oacc[db][4 * q4 + 2], w0 * x[3] + w1 * oacc[db][4 * q4 + 3]};
        *(f32x4*)dst = y;
      }
    // (both half-waves of the row have read L0 above: the loads precede this store in program order)
    if (g == 0) a.lse[row] = L1;
    return;
  }
  const long off = b * d.q_sb + hq * d.q_sh + (long)i_lane * d.q_ss;
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const float y0 = oacc[db][4 * q4] * inv, y1 = oacc[db][4 * q4 + 1] * inv,
                  y2 = oacc[db][4 * q4 + 2] * inv, y3 = oacc[db][4 * q4 + 3] * inv;
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

template <int D>
hipError_t launch(const FwdArgs& a, long grid, hipStream_t s) {
  static SmemOnce once;
  const hipError_t e = ensure_dynamic_lds((const void*)fwd_general_bf16_kernel<D>, FwdSmem<D>::TOTAL, &once);
  if (e != hipSuccess) return e;
  fwd_general_bf16_kernel<D><<<(unsigned)grid, 512, FwdSmem<D>::TOTAL, s>>>(a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd_general_bf16(const FwdArgs& a, hipStream_t s) {
  const Dims& d = a.d;
  const int G = d.Hq / d.Hkv;
  const int n_qt = (d.Sq + BM - 1) / BM;
  const long grid = xcd_grid(d.B * d.Hkv, a.n_split * G * n_qt);
  return d.D == 64 ? launch<64>(a, grid, s) : d.D == 96 ? launch<96>(a, grid, s) : launch<128>(a, grid, s);
}

}  // namespace lvx
