// C ABI of the library (see include/lvx.h): argument validation on the host, workspace carving,
// KV-split choice, and kernel launches on the caller's stream.  Nothing here allocates or
// synchronises.
#include "../../include/lvx.h"
#include "lvx_internal.h"

#include <math.h>

using namespace lvx;

namespace {

constexpr size_t ALIGN = 256;
constexpr bool FUSED_BY_DEFAULT = false;   // lvx_xattn_bwd: one fused kernel where it applies, else dK/dV + dQ kernels
inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

int device_cu_count() {
  static int n = 0;
  if (n == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      n = v;
    else
      return 256;
  }
  return n;
}

lvx_status check_problem(const lvx_problem* p, lvx_dtype dtype) {
  if (!p) return LVX_ERR_NULL;
  if (dtype != LVX_F32 && dtype != LVX_BF16) return LVX_ERR_DTYPE;
  if (p->B < 1 || p->Hq < 1 || p->Hkv < 1 || p->Sq < 1 || p->Skv < 1 || p->D < 1) return LVX_ERR_SHAPE;
  if (p->Hq % p->Hkv != 0) return LVX_ERR_SHAPE;
  if (p->B > 65535 || p->Hq > 65535) return LVX_ERR_SHAPE;
  if (p->D != 64 && p->D != 96 && p->D != 128) return LVX_ERR_UNSUPPORTED;
  // rows are read with 16-byte vector accesses: strides must keep that alignment
  const int64_t vec = dtype == LVX_F32 ? 4 : 8;
  const int64_t qs[3] = {p->q_sb, p->q_sh, p->q_ss}, ks[3] = {p->kv_sb, p->kv_sh, p->kv_ss};
  for (int i = 0; i < 3; ++i)
    if (qs[i] % vec != 0 || ks[i] % vec != 0) return LVX_ERR_STRIDE;
  if (p->q_ss < p->D || p->kv_ss < p->D) return LVX_ERR_STRIDE;
  if (p->Sq > 1 && p->q_sh < 0) return LVX_ERR_STRIDE;
  if (p->q_sh < 0 || p->q_sb < 0 || p->kv_sh < 0 || p->kv_sb < 0) return LVX_ERR_STRIDE;
  if (p->Hq > 1 && p->q_sh < (int64_t)p->D) return LVX_ERR_STRIDE;
  if (p->Hkv > 1 && p->kv_sh < (int64_t)p->D) return LVX_ERR_STRIDE;
  if (p->B > 1 && (p->q_sb < (int64_t)p->D || p->kv_sb < (int64_t)p->D)) return LVX_ERR_STRIDE;
  return LVX_OK;
}

lvx_status check_mask(const lvx_problem* p, const lvx_mask* m) {
  if (!m) return LVX_OK;
  if (!m->allow) return LVX_ERR_NULL;
  if (m->q_chunk < 1 || m->kv_block < 1 || m->n_q_chunks < 1 || m->n_kv_blocks < 1) return LVX_ERR_MASK;
  if ((int64_t)m->n_q_chunks * m->q_chunk < p->Sq) return LVX_ERR_MASK;
  if ((int64_t)m->n_kv_blocks * m->kv_block < p->Skv) return LVX_ERR_MASK;
  if (m->stride_q < m->n_kv_blocks || m->stride_b < 0) return LVX_ERR_MASK;
  return LVX_OK;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

Dims make_dims(const lvx_problem* p) {
  Dims d;
  d.B = p->B; d.Hq = p->Hq; d.Hkv = p->Hkv; d.Sq = p->Sq; d.Skv = p->Skv; d.D = p->D;
  d.q_sb = p->q_sb; d.q_sh = p->q_sh; d.q_ss = p->q_ss;
  d.kv_sb = p->kv_sb; d.kv_sh = p->kv_sh; d.kv_ss = p->kv_ss;
  d.scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->D);
  return d;
}

MaskDev make_mask(const lvx_mask* m) {
  MaskDev r;
  if (!m) { r.allow = nullptr; r.q_chunk = r.kv_block = 1; r.n_q_chunks = r.n_kv_blocks = 0; r.stride_b = r.stride_q = 0; return r; }
  r.allow = m->allow; r.q_chunk = m->q_chunk; r.kv_block = m->kv_block;
  r.n_q_chunks = m->n_q_chunks; r.n_kv_blocks = m->n_kv_blocks;
  r.stride_b = (long)m->stride_b; r.stride_q = (long)m->stride_q;
  return r;
}

int fwd_split(const Dims& d, lvx_dtype dtype, bool masked) {
  return dtype == LVX_BF16 ? fwd_bf16_pick_split(d, device_cu_count(), masked) : 1;
}
int bwd_split(const Dims& d, lvx_dtype dtype, bool masked) {
  return dtype == LVX_BF16 ? bwd_bf16_pick_split(d, device_cu_count(), masked) : 1;
}

// bf16, no mask, a key count that is no multiple of the 64-key tile (and at least two tiles): the
// dense kernel takes the whole tiles, the general kernel the keys that are left, as one more
// partial result of the combine.
constexpr int FWD_TILE = 64;
bool fwd_has_tail(const Dims& d, lvx_dtype dtype, bool masked) {
  return dtype == LVX_BF16 && !masked && d.Skv % FWD_TILE != 0 && d.Skv >= 2 * FWD_TILE;
}
// launches of the bf16 forward that leave partial results in slices [0, n_split (+ 1)) of
// o_part / lse_part: every split of the whole tiles, then the tail
hipError_t launch_fwd_bf16_parts(FwdArgs a, hipStream_t s) {
  const int tail = a.d.Skv % FWD_TILE;
  FwdArgs head = a;
  head.partial = 1;
  head.part0 = 0;
  head.d.Skv = a.d.Skv - tail;
  hipError_t e = launch_fwd_bf16(head, s);
  if (e != hipSuccess) return e;
  FwdArgs rest = a;
  rest.partial = 1;
  rest.part0 = a.n_split;
  rest.n_split = 1;
  rest.k = (const uint16_t*)a.k + (long)head.d.Skv * a.d.kv_ss;
  rest.v = (const uint16_t*)a.v + (long)head.d.Skv * a.d.kv_ss;
  rest.d.Skv = tail;
  return launch_fwd_bf16(rest, s);
}

// bf16 under a media mask that fits (fwd_bf16_two_pass_fits): the dense kernel over the key tiles
// that every row of a workgroup sees, then the general kernel on the other visible tiles; each
// launch leaves n_split partial results (slices [0, n_split) and [n_split, 2 n_split)).
int fwd_two_pass_split(int n_split, int reserve) {   // each launch's split count: both launches' parts (and
  const int cap = (LVX_MAX_PARTS - reserve) / 2;      // `reserve` others) go into one combine
  return n_split < cap ? n_split : cap;
}
bool fwd_two_pass(const Dims& d, lvx_dtype dtype, const MaskDev& m) {
  return dtype == LVX_BF16 && fwd_bf16_two_pass_fits(d, m);
}
hipError_t launch_fwd_bf16_two_pass(FwdArgs a, hipStream_t s) {
  a.partial = 1;
  a.pass = 1;
  a.part0 = 0;
  const hipError_t e = launch_fwd_bf16(a, s);
  if (e != hipSuccess) return e;
  a.pass = 2;
  a.part0 = a.n_split;
  return launch_fwd_bf16(a, s);
}

// How lvx_xattn_fwd runs a problem: the KV splits of each launch, whether a ragged tail or a media
// mask makes it two launches, and the partial results the combine then reads.
struct FwdPlan { int n_split; bool tail, two; int n_parts; };
FwdPlan fwd_plan(const Dims& d, lvx_dtype dtype, const MaskDev& m) {
  const bool masked = m.allow != nullptr;
  FwdPlan f;
  f.n_split = fwd_split(d, dtype, masked);
  f.tail = fwd_has_tail(d, dtype, masked);
  f.two = masked && fwd_two_pass(d, dtype, m);
  if (f.tail && f.n_split > LVX_MAX_PARTS - 1) f.n_split = LVX_MAX_PARTS - 1;
  if (f.two) f.n_split = fwd_two_pass_split(f.n_split, 0);
  // (one launch over tile lists: its workgroups start longest first, which evens the load out
  // with half the splits the other masked forms want)
  if (masked && dtype == LVX_BF16 && fwd_bf16_one_pass_fits(d, m) && f.n_split > 1) f.n_split /= 2;
  f.n_parts = f.two ? 2 * f.n_split : f.n_split + (f.tail ? 1 : 0);
  return f;
}

size_t fwd_ws(const Dims& d, int n_split) {
  if (n_split <= 1) return ALIGN;   // never zero, so that a valid workspace pointer is always passed
  const size_t rows = (size_t)d.B * d.Hq * d.Sq;
  return align_up(rows * d.D * sizeof(float) * n_split) + align_up(rows * sizeof(float) * n_split);
}
// lvx_xattn_fwd_merge: the splits' partial results (bf16 kernels that split the key range), or one
// float32 partial result (float32 kernels, which have no fused epilogue)
int fwd_merge_split(const Dims& d, lvx_dtype dtype, bool masked) {
  const int n = fwd_split(d, dtype, masked);
  return n < LVX_MAX_PARTS ? n : LVX_MAX_PARTS - 1;     // the running state is one more part of the combine
}
size_t fwd_merge_ws(const Dims& d, lvx_dtype dtype, int n_split) {
  return fwd_ws(d, dtype == LVX_F32 ? 2 : n_split);      // (fwd_ws(d, 2) holds more than one partial result)
}
int sq_padded(const Dims& d) { return (d.Sq + 31) / 32 * 32; }
bool has_stats_ovl(const Dims& d) { return d.Sq % 32 != 0 && d.Sq >= 32; }
size_t stats_floats(const Dims& d) { return 2 * (size_t)d.B * d.Hq * sq_padded(d); }
size_t bwd_ws_fixed(const Dims& d) {   // delta [B,Hq,Sq] + padded statistics [B,Hq,sq_pad/32][2][32]
                                       // (+ those of the last 32 rows, [B,Hq][2][32], when Sq is ragged)
  return align_up((size_t)d.B * d.Hq * d.Sq * sizeof(float)) +
         align_up((stats_floats(d) + (has_stats_ovl(d) ? (size_t)d.B * d.Hq * 64 : 0)) * sizeof(float));
}
size_t bwd_ws_part(const Dims& d, int n_split) {   // the dQ kernel's partial sums [n_split, B,Hq,Sq,D] when it splits
  return n_split > 1 ? align_up((size_t)n_split * d.B * d.Hq * d.Sq * d.D * sizeof(float)) : 0;
}
size_t bwd_ws(const Dims& d, int n_split, bool fused) {   // ... + the fused kernel's dQ tiles and locks
  return bwd_ws_fixed(d) + bwd_ws_part(d, n_split) + (fused ? align_up(bwd_fused_ws_bytes(d)) : 0);
}

}  // namespace

namespace lvx {
size_t fwd_workspace_need(const lvx_problem* p, lvx_dtype dtype, const lvx_mask* mask) {
  if (check_problem(p, dtype) != LVX_OK || check_mask(p, mask) != LVX_OK) return 0;
  const Dims d = make_dims(p);
  return fwd_ws(d, fwd_plan(d, dtype, make_mask(mask)).n_parts);
}
}  // namespace lvx

extern "C" {

const char* lvx_strerror(lvx_status s) {
  switch (s) {
    case LVX_OK: return "ok";
    case LVX_ERR_NULL: return "required pointer is NULL";
    case LVX_ERR_SHAPE: return "invalid shape";
    case LVX_ERR_DTYPE: return "unsupported dtype";
    case LVX_ERR_STRIDE: return "invalid or misaligned stride / pointer";
    case LVX_ERR_MASK: return "mask geometry does not cover the problem";
    case LVX_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case LVX_ERR_UNSUPPORTED: return "unsupported head dimension or projection shape";
    case LVX_ERR_HIP: return "HIP launch failed";
  }
  return "unknown status";
}

size_t lvx_xattn_workspace_bytes(const lvx_problem* p, lvx_dtype dtype, int which) {
  if (check_problem(p, dtype) != LVX_OK) return 0;
  const Dims d = make_dims(p);
  // (the size does not depend on whether the call will carry a mask: the larger of the two split counts)
  const auto larger = [](int x, int y) { return x > y ? x : y; };
  const int tail_part = fwd_has_tail(d, dtype, false) ? 1 : 0;        // (one more partial result: the tail's)
  // (a masked bf16 call may run as two launches that leave their splits' partial results side by side)
  const int masked_parts = dtype == LVX_BF16 ? 2 * fwd_two_pass_split(fwd_split(d, dtype, true), 0) : fwd_split(d, dtype, true);
  if (which == LVX_WS_FWD)
    return fwd_ws(d, larger(larger(masked_parts, fwd_split(d, dtype, true)), fwd_split(d, dtype, false) + tail_part));
  if (which == LVX_WS_BWD)
    return bwd_ws(d, larger(bwd_split(d, dtype, true), bwd_split(d, dtype, false)),
                  dtype == LVX_BF16 && bwd_fused_bf16_supported(d, false));
  if (which == LVX_WS_FWD_MERGE)
  {
    const int masked_merge = dtype == LVX_BF16 ? 2 * fwd_two_pass_split(fwd_merge_split(d, dtype, true), 1) : 1;
    return fwd_merge_ws(d, dtype, larger(larger(masked_merge, fwd_merge_split(d, dtype, true)),
                                         fwd_merge_split(d, dtype, false) + tail_part));
  }
  return 0;
}

lvx_status lvx_xattn_fwd(const lvx_problem* p, lvx_dtype dtype, const void* q, const void* k,
                         const void* v, const lvx_mask* mask, void* o, lvx_dtype o_dtype,
                         float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
  lvx_status st = check_problem(p, dtype);
  if (st != LVX_OK) return st;
  if (!q || !k || !v || !o || !lse) return LVX_ERR_NULL;
  if (o_dtype != dtype && o_dtype != LVX_F32) return LVX_ERR_DTYPE;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return LVX_ERR_STRIDE;
  if ((st = check_mask(p, mask)) != LVX_OK) return st;
  FwdArgs a;
  a.d = make_dims(p);
  a.mask = make_mask(mask);
  a.q = q; a.k = k; a.v = v; a.o = o; a.o_is_f32 = o_dtype == LVX_F32; a.lse = lse;
  a.merge_into = 0;
  a.partial = 0; a.part0 = 0; a.pass = 0;
  const FwdPlan plan = fwd_plan(a.d, dtype, a.mask);
  a.n_split = plan.n_split;
  const bool tail = plan.tail, two = plan.two;
  const int n_parts = plan.n_parts;
  a.o_part = nullptr; a.lse_part = nullptr;
  const size_t need = fwd_ws(a.d, n_parts);
  if (!workspace || ((uintptr_t)workspace % ALIGN) != 0 || workspace_bytes < need) return LVX_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)hip_stream;
  const size_t rows = (size_t)a.d.B * a.d.Hq * a.d.Sq;
  if (n_parts > 1) {
    a.o_part = (float*)workspace;
    a.lse_part = (float*)((char*)workspace + align_up(rows * a.d.D * sizeof(float) * n_parts));
  }
  hipError_t e = two    ? launch_fwd_bf16_two_pass(a, s)
                 : tail ? launch_fwd_bf16_parts(a, s)
                        : dtype == LVX_BF16 ? launch_fwd_bf16(a, s) : launch_fwd_f32(a, s);
  if (e != hipSuccess) return LVX_ERR_HIP;
  if (n_parts > 1) {
    MergeArgs m;
    m.n_parts = n_parts;
    for (int i = 0; i < n_parts; ++i) {
      m.o_parts[i] = a.o_part + (size_t)i * rows * a.d.D;
      m.lse_parts[i] = a.lse_part + (size_t)i * rows;
    }
    m.rows = (long)rows; m.D = a.d.D; m.o_out = o; m.lse_out = lse;
    m.Hq = a.d.Hq; m.Sq = a.d.Sq; m.o_sb = a.d.q_sb; m.o_sh = a.d.q_sh; m.o_ss = a.d.q_ss;
    e = launch_merge(m, 1, a.o_is_f32, s);
    if (e != hipSuccess) return LVX_ERR_HIP;
  }
  return LVX_OK;
}

lvx_status lvx_xattn_fwd_merge(const lvx_problem* p, lvx_dtype dtype, const void* q, const void* k,
                               const void* v, const lvx_mask* mask, float* o_acc, float* lse_acc,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
  lvx_status st = check_problem(p, dtype);
  if (st != LVX_OK) return st;
  if (!q || !k || !v || !o_acc || !lse_acc) return LVX_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o_acc)) return LVX_ERR_STRIDE;
  if ((st = check_mask(p, mask)) != LVX_OK) return st;
  FwdArgs a;
  a.d = make_dims(p);
  if (dtype == LVX_F32 && (a.d.q_ss != a.d.D || a.d.q_sh != (long)a.d.Sq * a.d.D ||
                           a.d.q_sb != (long)a.d.Hq * a.d.Sq * a.d.D))
    return LVX_ERR_STRIDE;      // the float32 kernels write their result with Q's strides
  a.mask = make_mask(mask);
  a.q = q; a.k = k; a.v = v; a.o_is_f32 = 1;
  a.partial = 0; a.part0 = 0; a.pass = 0;
  a.n_split = fwd_merge_split(a.d, dtype, mask != nullptr);
  const bool tail = fwd_has_tail(a.d, dtype, mask != nullptr);
  const bool two = mask != nullptr && fwd_two_pass(a.d, dtype, a.mask);
  if (tail && a.n_split > LVX_MAX_PARTS - 2) a.n_split = LVX_MAX_PARTS - 2;    // (the running state and the tail are parts too)
  if (two) a.n_split = fwd_two_pass_split(a.n_split, 1);
  if (mask != nullptr && dtype == LVX_BF16 && fwd_bf16_one_pass_fits(a.d, a.mask) && a.n_split > 1) a.n_split /= 2;
  const int n_launch_parts = two ? 2 * a.n_split : a.n_split + (tail ? 1 : 0);
  a.o_part = nullptr; a.lse_part = nullptr;
  const size_t need = fwd_merge_ws(a.d, dtype, n_launch_parts);
  if (!workspace || ((uintptr_t)workspace % ALIGN) != 0 || workspace_bytes < need) return LVX_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)hip_stream;
  const size_t rows = (size_t)a.d.B * a.d.Hq * a.d.Sq;
  if (dtype == LVX_BF16 && a.n_split == 1 && !tail && !two) {   // Rescale in the kernel's epilogue
    a.o = o_acc; a.lse = lse_acc; a.merge_into = 1;
    return launch_fwd_bf16(a, s) == hipSuccess ? LVX_OK : LVX_ERR_HIP;
  }
  // partial result(s) in the workspace, then one combine over the running state and them
  a.merge_into = 0;
  const int n_parts = dtype == LVX_BF16 ? n_launch_parts : 1;
  float* const o_part = (float*)workspace;
  float* const l_part = (float*)((char*)workspace + align_up(rows * a.d.D * sizeof(float) * n_parts));
  hipError_t e;
  if (dtype == LVX_BF16) {
    a.o = nullptr; a.lse = nullptr; a.o_part = o_part; a.lse_part = l_part;
    e = two ? launch_fwd_bf16_two_pass(a, s) : tail ? launch_fwd_bf16_parts(a, s) : launch_fwd_bf16(a, s);
  } else {
    a.o = o_part; a.lse = l_part; a.n_split = 1;
    e = launch_fwd_f32(a, s);
  }
  if (e != hipSuccess) return LVX_ERR_HIP;
  MergeArgs m;
  m.n_parts = n_parts + 1;
  m.o_parts[0] = o_acc; m.lse_parts[0] = lse_acc;
  for (int i = 0; i < n_parts; ++i) {
    m.o_parts[i + 1] = o_part + (size_t)i * rows * a.d.D;
    m.lse_parts[i + 1] = l_part + (size_t)i * rows;
  }
  m.rows = (long)rows; m.D = a.d.D; m.o_out = o_acc; m.lse_out = lse_acc;
  m.Hq = a.d.Hq; m.Sq = a.d.Sq; m.o_ss = a.d.D; m.o_sh = (long)a.d.Sq * a.d.D; m.o_sb = (long)a.d.Hq * a.d.Sq * a.d.D;
  e = launch_merge(m, 1, 1, s);
  return e == hipSuccess ? LVX_OK : LVX_ERR_HIP;
}

lvx_status lvx_xattn_merge(int32_t B, int32_t Hq, int32_t Sq, int32_t D, int32_t n_parts,
                           const void* const* o_parts, const float* const* lse_parts,
                           lvx_dtype part_dtype, void* o_out, lvx_dtype out_dtype, float* lse_out,
                           void* hip_stream) {
  if (!o_parts || !lse_parts || !o_out || !lse_out) return LVX_ERR_NULL;
  if (B < 1 || Hq < 1 || Sq < 1 || n_parts < 1 || n_parts > LVX_MAX_PARTS) return LVX_ERR_SHAPE;
  if (D != 64 && D != 96 && D != 128) return LVX_ERR_UNSUPPORTED;
  if ((part_dtype != LVX_F32 && part_dtype != LVX_BF16) || (out_dtype != LVX_F32 && out_dtype != LVX_BF16))
    return LVX_ERR_DTYPE;
  if (!aligned16(o_out)) return LVX_ERR_STRIDE;
  MergeArgs m;
  for (int i = 0; i < n_parts; ++i) {
    if (!o_parts[i] || !lse_parts[i]) return LVX_ERR_NULL;
    if (!aligned16(o_parts[i])) return LVX_ERR_STRIDE;
    m.o_parts[i] = o_parts[i];
    m.lse_parts[i] = lse_parts[i];
  }
  m.n_parts = n_parts;
  m.rows = (long)B * Hq * Sq; m.D = D; m.o_out = o_out; m.lse_out = lse_out;
  m.Hq = Hq; m.Sq = Sq; m.o_ss = D; m.o_sh = (long)Sq * D; m.o_sb = (long)Hq * Sq * D;
  hipError_t e = launch_merge(m, part_dtype == LVX_F32, out_dtype == LVX_F32, (hipStream_t)hip_stream);
  return e == hipSuccess ? LVX_OK : LVX_ERR_HIP;
}

lvx_status lvx_xattn_bwd(const lvx_problem* p, lvx_dtype dtype, const void* q, const void* k,
                         const void* v, const void* o, const float* lse, const void* d_o,
                         const lvx_mask* mask, float* dq_accum, void* dk, void* dv,
                         void* workspace, size_t workspace_bytes, void* hip_stream) {
  return lvx_xattn_bwd_stages(p, dtype, q, k, v, o, lse, d_o, mask, dq_accum, dk, dv, workspace,
                              workspace_bytes, hip_stream, LVX_BWD_ALL);
}

lvx_status lvx_xattn_bwd_stages(const lvx_problem* p, lvx_dtype dtype, const void* q, const void* k,
                                const void* v, const void* o, const float* lse, const void* d_o,
                                const lvx_mask* mask, float* dq_accum, void* dk, void* dv,
                                void* workspace, size_t workspace_bytes, void* hip_stream,
                                unsigned stages) {
  lvx_status st = check_problem(p, dtype);
  if (st != LVX_OK) return st;
  if ((stages & LVX_BWD_ALL) == 0 || (stages & ~(unsigned)(LVX_BWD_ALL | LVX_BWD_FUSED | LVX_BWD_SPLIT))) return LVX_ERR_SHAPE;
  if ((stages & LVX_BWD_FUSED) && (stages & LVX_BWD_SPLIT)) return LVX_ERR_SHAPE;
  if (!q || !k || !v || !o || !lse || !d_o || !dq_accum || !dk || !dv) return LVX_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o) ||
      !aligned16(dq_accum) || !aligned16(dk) || !aligned16(dv))
    return LVX_ERR_STRIDE;
  if ((st = check_mask(p, mask)) != LVX_OK) return st;
  BwdArgs a;
  a.d = make_dims(p);
  a.mask = make_mask(mask);
  a.n_split_dq = bwd_split(a.d, dtype, mask != nullptr);
  a.dq_pass = 0;
  // the kernel that forms all five products at once: where it applies, unless the caller asks for
  // the two-kernel form (or only for one of the two kernels)
  const bool can_fuse = dtype == LVX_BF16 && bwd_fused_bf16_supported(a.d, mask != nullptr);
  const bool want_fuse = (stages & LVX_BWD_FUSED) || (FUSED_BY_DEFAULT && !(stages & LVX_BWD_SPLIT));
  const bool fused = can_fuse && want_fuse && (stages & (LVX_BWD_DKDV | LVX_BWD_DQ)) == (LVX_BWD_DKDV | LVX_BWD_DQ);
  const size_t need = bwd_ws(a.d, a.n_split_dq, can_fuse);
  if (!workspace || ((uintptr_t)workspace % ALIGN) != 0 || workspace_bytes < need) return LVX_ERR_WORKSPACE;
  a.q = q; a.k = k; a.v = v; a.o = o; a.d_o = d_o; a.lse = lse;
  a.delta = (float*)workspace;
  a.sq_pad = sq_padded(a.d);
  a.stats = (float*)((char*)workspace + align_up((size_t)a.d.B * a.d.Hq * a.d.Sq * sizeof(float)));
  a.stats_ovl = has_stats_ovl(a.d) ? a.stats + stats_floats(a.d) : nullptr;
  a.dq_accum = dq_accum; a.dk = dk; a.dv = dv;
  a.dq_part = a.n_split_dq > 1 ? (float*)((char*)workspace + bwd_ws_fixed(a.d)) : nullptr;
  a.dq_tiles = fused ? (float*)((char*)workspace + bwd_ws_fixed(a.d) + bwd_ws_part(a.d, a.n_split_dq)) : nullptr;
  a.dq_locks = nullptr; a.dq_err = nullptr; a.dq_stagger = 0;
  hipStream_t s = (hipStream_t)hip_stream;
  hipError_t e = hipSuccess;
  if (stages & LVX_BWD_DELTA) e = launch_delta(a.d, o, d_o, dtype == LVX_F32, lse, a.delta, a.stats, a.sq_pad, a.stats_ovl, s);
  if (e != hipSuccess) return LVX_ERR_HIP;
  if (stages & (LVX_BWD_DKDV | LVX_BWD_DQ))
    e = dtype == LVX_BF16 ? launch_bwd_bf16(a, stages & LVX_BWD_ALL, s) : launch_bwd_f32(a, stages & LVX_BWD_ALL, s);
  return e == hipSuccess ? LVX_OK : LVX_ERR_HIP;
}

lvx_status lvx_xattn_bwd_error_word(const lvx_problem* p, lvx_dtype dtype, const lvx_mask* mask,
                                    void* workspace, size_t workspace_bytes, const int** word) {
  lvx_status st = check_problem(p, dtype);
  if (st != LVX_OK) return st;
  if (!word) return LVX_ERR_NULL;
  if ((st = check_mask(p, mask)) != LVX_OK) return st;
  const Dims d = make_dims(p);
  const int n_split = bwd_split(d, dtype, mask != nullptr);
  const bool fused = dtype == LVX_BF16 && bwd_fused_bf16_supported(d, mask != nullptr);
  if (!workspace || ((uintptr_t)workspace % ALIGN) != 0 || workspace_bytes < bwd_ws(d, n_split, fused)) return LVX_ERR_WORKSPACE;
  *word = fused ? (const int*)((char*)workspace + bwd_ws_fixed(d) + bwd_ws_part(d, n_split) + bwd_fused_ws_bytes(d) - 256)
                : nullptr;
  return LVX_OK;
}

lvx_status lvx_xattn_dq_finalize(const lvx_problem* p, const float* dq_accum, void* dq,
                                 lvx_dtype dtype, void* hip_stream) {
  lvx_status st = check_problem(p, dtype);
  if (st != LVX_OK) return st;
  if (!dq_accum || !dq) return LVX_ERR_NULL;
  if (!aligned16(dq_accum) || !aligned16(dq)) return LVX_ERR_STRIDE;
  hipError_t e = launch_dq_finalize(make_dims(p), dq_accum, dq, dtype == LVX_F32, (hipStream_t)hip_stream);
  return e == hipSuccess ? LVX_OK : LVX_ERR_HIP;
}

lvx_status lvx_xattn_project(const lvx_projection* p, lvx_dtype dtype, const void* x, const void* w,
                             int n_out, void* const* out, void* hip_stream) {
  if (!p || !x || !w || !out) return LVX_ERR_NULL;
  if (n_out < 1 || n_out > 2) return LVX_ERR_SHAPE;
  for (int o = 0; o < n_out; ++o)
    if (!out[o]) return LVX_ERR_NULL;
  if (p->B <= 0 || p->S <= 0 || p->E <= 0 || p->H <= 0 || p->D <= 0) return LVX_ERR_SHAPE;
  if ((long)n_out * p->H * p->D > INT32_MAX) return LVX_ERR_SHAPE;
  if (dtype != LVX_F32 && dtype != LVX_BF16) return LVX_ERR_DTYPE;
  const int esz = dtype == LVX_F32 ? 4 : 2;
  if (p->x_ss < p->E || p->x_sb != (int64_t)p->S * p->x_ss) return LVX_ERR_STRIDE;
  if (dtype == LVX_BF16) {                           // 16-byte copies and stores
    if ((p->x_ss * esz) % 16 != 0 || !aligned16(x) || !aligned16(w)) return LVX_ERR_STRIDE;
    for (int o = 0; o < n_out; ++o)
      if (!aligned16(out[o])) return LVX_ERR_STRIDE;
  }
  ProjArgs a{};
  a.x = x;
  a.w = w;
  for (int o = 0; o < n_out; ++o) a.out[o] = out[o];
  a.M = (long)p->B * p->S;
  a.ldx = p->x_ss;
  a.S = p->S;
  a.E = p->E;
  a.N = n_out * p->H * p->D;
  a.H = p->H;
  a.D = p->D;
  if (dtype == LVX_BF16 && !project_bf16_supported(a)) return LVX_ERR_UNSUPPORTED;
  // (a tile's copies address its rows with 32-bit byte offsets from the tile's first row)
  if (dtype == LVX_BF16 && 256 * p->x_ss * esz > (int64_t)UINT32_MAX) return LVX_ERR_STRIDE;
  const hipError_t e = launch_project(a, dtype == LVX_F32, (hipStream_t)hip_stream);
  return e == hipSuccess ? LVX_OK : LVX_ERR_HIP;
}

lvx_status lvx_xattn_project_bwd(const lvx_projection* p, lvx_dtype dtype, const void* x, const void* w,
                                 int n_out, const void* const* d_out, void* dx, float* dw,
                                 void* hip_stream) {
  if (!p || !x || !w || !d_out) return LVX_ERR_NULL;
  if (n_out < 1 || n_out > 2) return LVX_ERR_SHAPE;
  for (int o = 0; o < n_out; ++o)
    if (!d_out[o]) return LVX_ERR_NULL;
  if (!dx && !dw) return LVX_ERR_NULL;
  if (p->B <= 0 || p->S <= 0 || p->E <= 0 || p->H <= 0 || p->D <= 0) return LVX_ERR_SHAPE;
  if ((long)n_out * p->H * p->D > INT32_MAX) return LVX_ERR_SHAPE;
  if (dtype != LVX_F32 && dtype != LVX_BF16) return LVX_ERR_DTYPE;
  const int esz = dtype == LVX_F32 ? 4 : 2;
  if (p->x_ss < p->E || p->x_sb != (int64_t)p->S * p->x_ss) return LVX_ERR_STRIDE;
  if (dtype == LVX_BF16) {                           // 16-byte copies and stores
    if ((p->x_ss * esz) % 16 != 0 || !aligned16(x) || !aligned16(w)) return LVX_ERR_STRIDE;
    if ((dx && !aligned16(dx)) || (dw && !aligned16(dw))) return LVX_ERR_STRIDE;
    for (int o = 0; o < n_out; ++o)
      if (!aligned16(d_out[o])) return LVX_ERR_STRIDE;
  }
  ProjBwdArgs a{};
  a.x = x;
  a.w = w;
  for (int o = 0; o < n_out; ++o) a.g[o] = d_out[o];
  a.dx = dx;
  a.dw = dw;
  a.M = (long)p->B * p->S;
  a.ldx = p->x_ss;
  a.S = p->S;
  a.E = p->E;
  a.N = n_out * p->H * p->D;
  a.H = p->H;
  a.D = p->D;
  a.n_cu = device_cu_count();
  const hipError_t e = launch_project_bwd(a, dtype == LVX_F32, (hipStream_t)hip_stream);
  return e == hipSuccess ? LVX_OK : LVX_ERR_HIP;
}

}  // extern "C"
