// Internal launch interface between the C-ABI host layer (lvx_api.hip) and the kernels.
// Everything here is private to the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/lvx.h"

namespace lvx {

// Media mask as the kernels see it (allow == nullptr means dense attention).
struct MaskDev {
  const uint8_t* allow;
  int q_chunk, kv_block, n_q_chunks, n_kv_blocks;
  long stride_b, stride_q;
};

// Shape, strides (in elements) and scale shared by every kernel.
struct Dims {
  int B, Hq, Hkv, Sq, Skv, D;
  long q_sb, q_sh, q_ss;
  long kv_sb, kv_sh, kv_ss;
  float scale;          // multiplies Q K^T (natural-log domain)
};

struct FwdArgs {
  Dims d;
  MaskDev mask;
  const void *q, *k, *v;
  void* o;              // final output (Q's strides) when n_split == 1
  int o_is_f32;         // 1: o is float32, 0: o has the input dtype
  int merge_into;       // 1 (n_split == 1 only): o (float32, CONTIGUOUS [B,Hq,Sq,D]) and lse hold a running
                        // result; the kernel leaves in them the Rescale of it with this visit's result
  float* lse;           // [B,Hq,Sq]
  int n_split;          // number of KV splits handled by separate workgroups
  int partial;          // 1: write partial results even with n_split == 1 (this launch is one of several
                        // whose results are combined)
  int part0;            // index of the partial slice that split 0 of this launch writes
  int pass;             // media mask, bf16: 0 = one launch over every visible tile; 1 = this launch takes the key
                        // tiles that EVERY row of a workgroup sees (dense kernel over a list of them), 2 = this
                        // launch takes the other visible tiles (general kernel)
  float* o_part;        // [n_split, B,Hq,Sq,D] float32, contiguous (n_split > 1)
  float* lse_part;      // [n_split, B,Hq,Sq]
};

struct BwdArgs {
  Dims d;
  MaskDev mask;
  const void *q, *k, *v, *o, *d_o;
  const float* lse;     // final statistic, [B,Hq,Sq]
  float* delta;         // workspace, [B,Hq,Sq]: rowsum(dO * O)
  float* stats;         // workspace, [B,Hq,sq_pad/32][2][32]: per group of 32 query rows, 32 values of
                        // -L * log2(e) (-inf for rows without keys and pad rows), then 32 of -delta
  int sq_pad;           // Sq rounded up to a multiple of 32
  float* stats_ovl;     // workspace, [B,Hq][2][32], only when Sq % 32 != 0 and Sq >= 32 (else nullptr): the
                        // same two rows of 32 values for the query rows Sq-32 .. Sq-1, with -inf in place of
                        // -L * log2(e) for the rows that the last full group already covers.  A kernel that
                        // walks the rows 32 at a time takes rows Sq-32 .. Sq-1 as its last step instead of a
                        // short one: the rows it has seen before then contribute nothing.
  float* dq_accum;      // [B,Hq,Sq,D] float32, accumulated into
  void *dk, *dv;        // K's strides, input dtype, overwritten
  int n_split_dq;       // KV splits of the dQ kernel
  int dq_pass;          // media mask, dQ kernel: 0 = one launch over every visible tile; 1 = this launch takes the
                        // key tiles that EVERY row of a workgroup sees (dense kernel over a list of them),
                        // 2 = this launch takes the other visible tiles (general kernel)
  float* dq_part;       // workspace, [n_split_dq, B,Hq,Sq,D] float32: the splits' sums (n_split_dq > 1),
                        // added to dq_accum by a reduction that follows the kernel
  // fused kernel (all five products in one pass): workspace of bwd_fused_ws_bytes, zeroed by the launch
  float* dq_tiles;      // [B,Hq,ceil(Sq/32)] tiles of 32 rows x 128 columns in matrix-register order
  int* dq_locks;        // one word per (tile, wave): 0 = free          (set by the launch)
  int* dq_err;          // nonzero after the kernel: a wave gave up on a lock, dQ is invalid   (set by the launch)
  int dq_stagger;       // steps by which consecutive key tiles start apart   (set by the launch)
};

struct MergeArgs {
  const void* o_parts[64];
  const float* lse_parts[64];
  int n_parts;
  long rows;            // B*Hq*Sq
  int D;
  void* o_out;
  float* lse_out;
  // output addressing: row r = ((b*Hq + h)*Sq + i) -> o_out + b*o_sb + h*o_sh + i*o_ss
  int Hq, Sq;
  long o_sb, o_sh, o_ss;
};

// Projection out[o][b, h, s, c] = sum_e x[b, s, e] w[(o H + h) D + c, e], tokens flattened to M = B S rows.
struct ProjArgs {
  const void* x;        // [M, E], row stride ldx elements
  const void* w;        // [N, E] contiguous, N = n_out * H * D
  void* out[2];         // each [B, H, S, D] contiguous, x's dtype
  long M, ldx;
  int S, E, N, H, D;
};
bool project_bf16_supported(const ProjArgs& a);   // shapes the matrix-core kernel takes
hipError_t launch_project(const ProjArgs& a, int is_f32, hipStream_t s);

// Gradients of the projection: dx[m, e] = sum_n g[m, n] w[n, e] (rounded to the tensors' type),
// dw[n, e] += sum_m g[m, n] x[m, e] (float32), g given head-major per output like ProjArgs::out.
struct ProjBwdArgs {
  const void* x;        // [M, E], row stride ldx elements
  const void* w;        // [N, E] contiguous
  const void* g[2];     // each [B, H, S, D] contiguous
  void* dx;             // [M, E], row stride ldx, or null
  float* dw;            // [N, E] contiguous, or null
  long M, ldx;
  int S, E, N, H, D;
  int n_cu;             // compute units of the device (picks dw's tile height and token split)
  int dw_parts;         // set by launch_project_bwd: parts the token range of dw is cut into, and the
  unsigned dw_tiles_grid;   // workgroups of one part
};
bool project_bwd_bf16_supported(const ProjBwdArgs& a);   // shapes the matrix-core kernels take
hipError_t launch_project_bwd(const ProjBwdArgs& a, int is_f32, hipStream_t s);

// Bytes of workspace that lvx_xattn_fwd needs for exactly this call (with this mask or without
// one; lvx_xattn_workspace_bytes returns the larger of the two cases); 0 for invalid arguments.
size_t fwd_workspace_need(const lvx_problem* p, lvx_dtype dtype, const lvx_mask* mask);

// kernels for float32 tensors (plain FMA, correctness-grade)
hipError_t launch_fwd_f32(const FwdArgs& a, hipStream_t s);
hipError_t launch_bwd_f32(const BwdArgs& a, unsigned stages, hipStream_t s);   // stages: 2 = dK/dV, 4 = dQ
// kernels for bfloat16 tensors (MFMA)
hipError_t launch_fwd_bf16(const FwdArgs& a, hipStream_t s);
hipError_t launch_bwd_bf16(const BwdArgs& a, unsigned stages, hipStream_t s);
hipError_t launch_bwd_dkdv_bf16(const BwdArgs& a, hipStream_t s);
hipError_t launch_bwd_dq_bf16(const BwdArgs& a, hipStream_t s);
// all five products in one kernel (dense, head dim 128, at least 256 keys and 32 query rows):
// handles the first Skv / 256 * 256 keys; needs BwdArgs::dq_tiles
bool bwd_fused_bf16_supported(const Dims& d, bool masked);
size_t bwd_fused_ws_bytes(const Dims& d);
hipError_t launch_bwd_fused_bf16(const BwdArgs& a, hipStream_t s);
// Raises a kernel's dynamic LDS limit once per device (the attribute belongs to the device's copy
// of the kernel).  `done` is the caller's per-kernel table; a race between host threads only
// repeats a harmless call.
constexpr int LVX_MAX_DEVICES = 64;
struct SmemOnce { bool done[LVX_MAX_DEVICES] = {}; };
inline hipError_t ensure_dynamic_lds(const void* kernel, int bytes, SmemOnce* once) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < LVX_MAX_DEVICES;
  if (tracked && once->done[dev]) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && tracked) once->done[dev] = true;
  return e;
}

// Number of KV splits for `base` workgroups that each walk the whole key range on n_cu compute
// units: the count (at most cap) that minimises rounds * t_full / splits + splits * t_part, where
// rounds = ceil(base * splits / n_cu), t_full is one workgroup's time over the whole range and
// t_part what one more set of partial results costs (written, read again and summed).  Covers
// both a grid smaller than the chip and one slightly larger than a multiple of it (288
// workgroups on 256 units would take two rounds for the work of 1.125).
inline int pick_split_balanced(long base, int n_cu, long cap, double t_full, double t_part) {
  int best = 1;
  double best_t = 1e300;
  for (long s = 1; s <= cap && s <= 64; ++s) {
    const long rounds = (base * s + n_cu - 1) / n_cu;
    const double t = (double)rounds * t_full / (double)s + (s > 1 ? (double)s * t_part + 10e-6 : 0.0);
    if (t < best_t * 0.97) {                       // more splits only for a gain of 3 %
      best_t = t;
      best = (int)s;
    }
  }
  return best;
}
int fwd_bf16_pick_split(const Dims& d, int n_cu, bool masked);
bool fwd_bf16_two_pass_fits(const Dims& d, const MaskDev& m);   // a masked forward may run as passes 1 and 2
bool fwd_bf16_one_pass_fits(const Dims& d, const MaskDev& m);   // ... or as one launch of the dense kernel over tile lists
hipError_t launch_fwd_general_bf16(const FwdArgs& a, hipStream_t s);   // masked or ragged problems
int bwd_bf16_pick_split(const Dims& d, int n_cu, bool masked);
// memory-bound helpers
hipError_t launch_merge(const MergeArgs& a, int part_is_f32, int out_is_f32, hipStream_t s);
hipError_t launch_delta(const Dims& d, const void* o, const void* d_o, int is_f32, const float* lse,
                        float* delta, float* stats, int sq_pad, float* stats_ovl, hipStream_t s);
// dq_accum[i] += sum over the n_parts slices of `parts` (each n floats, n a multiple of 4)
hipError_t launch_dq_reduce(const float* parts, int n_parts, long n, float* dq_accum, hipStream_t s);
hipError_t launch_dq_finalize(const Dims& d, const float* dq_accum, void* dq, int is_f32,
                              hipStream_t s);

}  // namespace lvx
