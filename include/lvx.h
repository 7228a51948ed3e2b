/*
 * lvx.h -- C ABI of the MI355X (gfx950) cross-attention path of LV-XAttn.
 *
 * One worker of LV-XAttn keeps its large key/value block in local HBM and is
 * visited by small query blocks (Algorithm 1 of the paper).  Per visit it runs
 *   FlashAttention(Q_j, K_i, V_i) -> (dO partial, dL partial)   lvx_xattn_fwd
 *   Rescale(O_j, L_j, dO, dL)                                    lvx_xattn_merge
 * and, in the backward pass, recomputes the attention probabilities from the
 * saved statistic L instead of storing them (Section 3.2)       lvx_xattn_bwd,
 * after recomputing Q, K and V from the token features          lvx_xattn_project.
 *
 * General rules for every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The library
 *     never allocates, frees or synchronises; all work is enqueued on the HIP
 *     stream the caller passes (a hipStream_t cast to void*, NULL = default).
 *   - Scratch memory is a caller-provided workspace whose size comes from
 *     lvx_xattn_workspace_bytes; it must be 256-byte aligned.
 *   - lvx_problem / lvx_mask structs and the pointer arrays of lvx_xattn_merge
 *     live in HOST memory and are read before the call returns.
 *   - Errors are returned as negative lvx_status values; argument errors are
 *     detected on the host before anything is launched.  No exceptions, no aborts.
 *   - The library keeps no state between calls that a result depends on (it only
 *     caches, per device, the number of compute units and which kernels have had
 *     their LDS limit raised; lvx_xattn_fwd_static is the one exception and says
 *     so).  Calls on different streams may run concurrently as long as their
 *     buffers do not overlap.
 *
 * Tensor layout (all strides in ELEMENTS, innermost dimension D contiguous)
 *   Q, O, dO, dQ : [B, Hq,  Sq,  D]   strides q_sb, q_sh, q_ss
 *   K, V, dK, dV : [B, Hkv, Skv, D]   strides kv_sb, kv_sh, kv_ss
 *     (strides let a K/V *block* be a view into a larger tensor)
 *   L (LSE), delta : [B, Hq, Sq] float32, contiguous, natural logarithm,
 *     -inf for a query row that sees no key.
 *   Grouped-query attention: query head hq reads K/V head hq / (Hq / Hkv)
 *     (contiguous groups); dK/dV sum over the heads of a group.
 *   Supported head dims D: 64, 96, 128.  Sq, Skv >= 1, no multiple-of-tile rule.
 */
#ifndef LVX_H
#define LVX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LVX_OK = 0,
  LVX_ERR_NULL = -1,        /* a required pointer is NULL */
  LVX_ERR_SHAPE = -2,       /* non-positive size, Hq % Hkv != 0, too many parts/splits */
  LVX_ERR_DTYPE = -3,       /* unknown or unsupported dtype combination */
  LVX_ERR_STRIDE = -4,      /* stride too small for the shape, or misaligned for vector access */
  LVX_ERR_MASK = -5,        /* mask geometry does not cover Sq x Skv */
  LVX_ERR_WORKSPACE = -6,   /* workspace NULL, misaligned or smaller than required */
  LVX_ERR_UNSUPPORTED = -7, /* head dim other than 64 / 96 / 128; projection shape the bf16 kernel does not take */
  LVX_ERR_HIP = -8          /* a kernel launch failed (hipGetLastError) */
} lvx_status;

typedef enum { LVX_F32 = 0, LVX_BF16 = 1 } lvx_dtype;

/* The attention problem of Section 2: O = softmax(Q K^T * softmax_scale) V per (batch, head). */
typedef struct {
  int32_t B, Hq, Hkv, Sq, Skv, D;
  int64_t q_sb, q_sh, q_ss;      /* batch / head / row strides of Q, O, dO, dQ */
  int64_t kv_sb, kv_sh, kv_ss;   /* batch / head / row strides of K, V, dK, dV */
  float softmax_scale;           /* <= 0 selects the paper's 1/sqrt(D) */
} lvx_problem;

/* Optional media mask (not in the paper; part of this library's problem statement):
 * query row i may attend key row j iff
 *   allow[b * stride_b + (i / q_chunk) * stride_q + (j / kv_block)] != 0.
 * A masked score is -infinity.  Pass NULL for dense attention.  To mask a K/V block that is a
 * window [j0, j0+Skv) of a longer sequence (j0 a multiple of kv_block), offset `allow` by
 * j0 / kv_block columns. */
typedef struct {
  const uint8_t* allow;          /* device pointer */
  int32_t q_chunk, kv_block;     /* text tokens per chunk, visual tokens per block (>= 1) */
  int32_t n_q_chunks, n_kv_blocks; /* must satisfy n_q_chunks*q_chunk >= Sq, n_kv_blocks*kv_block >= Skv */
  int64_t stride_b, stride_q;    /* element strides; stride_b = 0 shares the bitmap across batch */
} lvx_mask;

enum { LVX_WS_FWD = 0, LVX_WS_BWD = 1, LVX_WS_FWD_MERGE = 2 };
enum { LVX_MAX_PARTS = 64 };

/* Bytes of workspace lvx_xattn_fwd (which = LVX_WS_FWD), lvx_xattn_bwd (LVX_WS_BWD) or
 * lvx_xattn_fwd_merge (LVX_WS_FWD_MERGE) needs for this problem and dtype.  Returns 0 on invalid
 * arguments. */
size_t lvx_xattn_workspace_bytes(const lvx_problem* p, lvx_dtype dtype, int which);

/* Forward pass of one visit (Algorithm 1, the FlashAttention call; Section 2 defines the result):
 *   O[b,h,i,:] = sum_j softmax_j(scale * <Q_i, K_j>) V_j,   L[b,h,i] = ln sum_j exp(scale * <Q_i, K_j>)
 * over the Skv keys passed.  q/k/v have type `dtype`; o has type `o_dtype`, which is either `dtype`
 * or LVX_F32 (use LVX_F32 for partial results that will be merged).  o uses Q's strides.
 * A row with no visible key gets O = 0, L = -inf.  Overwrites o and lse. */
lvx_status lvx_xattn_fwd(const lvx_problem* p, lvx_dtype dtype, const void* q, const void* k,
                         const void* v, const lvx_mask* mask, void* o, lvx_dtype o_dtype,
                         float* lse, void* workspace, size_t workspace_bytes, void* hip_stream);

/* lvx_xattn_fwd for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, result and kernels as
 * lvx_xattn_fwd, but no workspace: the KV splits' partial results go into a device array of
 * LVX_STATIC_SCRATCH_BYTES that the library holds on every GPU it runs on until the process ends.
 * Problems whose lvx_xattn_workspace_bytes(p, dtype, LVX_WS_FWD) exceeds that size are refused with
 * LVX_ERR_WORKSPACE before anything is launched.  Allocates nothing.  The stream must belong to
 * the current device.  Every call on a GPU shares that GPU's array: two calls that overlap in
 * time on one GPU (different streams, or different host threads) race; calls on one stream do not. */
enum { LVX_STATIC_SCRATCH_BYTES = 64 << 20 };
lvx_status lvx_xattn_fwd_static(const lvx_problem* p, lvx_dtype dtype, const void* q, const void* k,
                                const void* v, const lvx_mask* mask, void* o, lvx_dtype o_dtype,
                                float* lse, void* hip_stream);

/* Rescale of Algorithm 1, for n_parts >= 1 partial results of the same query block:
 *   L' = ln sum_k exp(L_k),   O' = sum_k exp(L_k - L') O_k        (all L_k = -inf -> O' = 0, L' = -inf)
 * o_parts[k] is a contiguous [B,Hq,Sq,D] device tensor of type part_dtype, lse_parts[k] a contiguous
 * [B,Hq,Sq] float32 device tensor; the two pointer arrays themselves are host arrays of n_parts
 * entries (n_parts <= LVX_MAX_PARTS).  o_out (contiguous, out_dtype) may alias o_parts[0] when the
 * two dtypes have the same size, and lse_out may alias lse_parts[0]: the running (O_j, L_j) of
 * Algorithm 1 is updated in place with n_parts = 2.  The identity element is (O, L) = (0, -inf). */
lvx_status lvx_xattn_merge(int32_t B, int32_t Hq, int32_t Sq, int32_t D, int32_t n_parts,
                           const void* const* o_parts, const float* const* lse_parts,
                           lvx_dtype part_dtype, void* o_out, lvx_dtype out_dtype, float* lse_out,
                           void* hip_stream);

/* One visit of Algorithm 1 in a single call: the FlashAttention call on the K/V block passed,
 * followed by Rescale into the running result of the query block.  On entry (o_acc, lse_acc) hold
 * the result over the keys visited so far -- float32, contiguous [B,Hq,Sq,D] and [B,Hq,Sq];
 * (0, -inf) before the first visit -- and on return the result over those keys and the Skv keys
 * passed, exactly as lvx_xattn_fwd into a float32 partial result followed by lvx_xattn_merge of
 * the two would leave it (the partial result never goes through memory when the kernel does not
 * split the key range).  Both are updated in place.  With dtype LVX_F32, Q must be contiguous
 * (LVX_ERR_STRIDE otherwise). */
lvx_status lvx_xattn_fwd_merge(const lvx_problem* p, lvx_dtype dtype, const void* q, const void* k,
                               const void* v, const lvx_mask* mask, float* o_acc, float* lse_acc,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* Backward pass of one visit: gradients of loss = sum(O * dO) for the K/V block passed, with the
 * attention probabilities recomputed as p_ij = exp(scale * <Q_i, K_j> - L_i) from the saved L
 * (Section 3.2 saves only x, O and L; Table 1 counts the five matrix products).
 *   o, lse : the FINAL output and statistic of the whole key range (after all merges), even when
 *            k/v are only one block of it.  o and d_o have type `dtype` and use Q's strides.
 *   dk, dv : type `dtype`, K's strides, OVERWRITTEN with this block's gradients (they are final:
 *            no other block contributes to them).
 *   dq_accum : float32, contiguous [B,Hq,Sq,D], ACCUMULATED into (+=).  The caller zeroes it before
 *            the first block and converts with lvx_xattn_dq_finalize after the last.
 * No gradient flows through L.  Rows with L = -inf get zero gradients. */
lvx_status lvx_xattn_bwd(const lvx_problem* p, lvx_dtype dtype, const void* q, const void* k,
                         const void* v, const void* o, const float* lse, const void* d_o,
                         const lvx_mask* mask, float* dq_accum, void* dk, void* dv,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* MEASUREMENT ONLY (not part of the method's interface; bench.py times single kernels with it):
 * the same call restricted to some of its kernels.  `stages` is a bit set of
 * LVX_BWD_DELTA (delta = rowsum(dO * O) into the workspace), LVX_BWD_DKDV (dK and dV) and
 * LVX_BWD_DQ (dQ accumulation).  DKDV and DQ read the delta a previous DELTA stage left in the
 * same workspace.  lvx_xattn_bwd is this call with LVX_BWD_ALL. */
enum { LVX_BWD_DELTA = 1, LVX_BWD_DKDV = 2, LVX_BWD_DQ = 4, LVX_BWD_ALL = 7,
       /* with DKDV and DQ both set: form all five products in ONE kernel where the problem allows it
        * (dense bf16, D = 128, at least 256 keys and 32 query rows), or never; neither = the library's choice */
       LVX_BWD_FUSED = 8, LVX_BWD_SPLIT = 16 };
lvx_status lvx_xattn_bwd_stages(const lvx_problem* p, lvx_dtype dtype, const void* q, const void* k,
                                const void* v, const void* o, const float* lse, const void* d_o,
                                const lvx_mask* mask, float* dq_accum, void* dk, void* dv,
                                void* workspace, size_t workspace_bytes, void* hip_stream,
                                unsigned stages);

/* Where lvx_xattn_bwd reports that it could not finish dQ.  For dense bf16 problems with D = 128 the
 * backward forms all five products of Table 1 in one kernel whose workgroups add their dQ tiles
 * into one array under per-tile locks; a wave that cannot get a lock within a bounded number of
 * tries (which takes another wave that never releases one: a fault, not load) gives up, so that
 * the kernel always ends, and sets a word in the workspace.  *word receives the DEVICE address of
 * that word for a call with these arguments and this workspace (NULL when the call uses no such
 * kernel); it is 0 after a call whose dQ is complete.  Read it after synchronising the stream. */
lvx_status lvx_xattn_bwd_error_word(const lvx_problem* p, lvx_dtype dtype, const lvx_mask* mask,
                                    void* workspace, size_t workspace_bytes, const int** word);

/* dq (type `dtype`, Q's strides) = dq_accum (float32, contiguous) rounded to `dtype`. */
lvx_status lvx_xattn_dq_finalize(const lvx_problem* p, const float* dq_accum, void* dq,
                                 lvx_dtype dtype, void* hip_stream);

/* The projections of Section 2 that make the attention operands, Q = x W_Q and K, V = y W_K,
 * y W_V, which Section 3.2 has the backward pass compute again from the saved token features
 * instead of keeping Q, K and V:
 *     out[o][b, h, s, c] = sum_e x[b, s, e] * w[(o * H + h) * D + c, e],   o = 0 .. n_out - 1.
 * x      device, [B, S, E] of `dtype`, strides x_sb, x_ss in elements (features contiguous);
 *        the batches must follow each other, x_sb == S * x_ss (LVX_ERR_STRIDE otherwise).
 * w      device, [n_out * H * D, E] of `dtype`, contiguous: the projection matrices TRANSPOSED
 *        (one row of E weights per output column, the layout of a linear layer's weight) and
 *        stacked, e.g. W_K^T on top of W_V^T with n_out = 2, so that y is read once for both.
 * out    host array of n_out (1 or 2) device pointers, each [B, H, S, D] of `dtype`, contiguous
 *        -- the layout lvx_xattn_fwd / lvx_xattn_bwd read -- overwritten.
 * LVX_BF16 runs on the matrix cores (float32 accumulation, one rounding of the result) and needs
 * E % 64 == 0, (n_out * H * D) % 256 == 0 and (H * D) % 128 == 0 (LVX_ERR_UNSUPPORTED
 * otherwise); B * S is arbitrary.  LVX_F32 takes any shape (plain FMA, correctness-grade).
 * LVX_BF16: pointers and x's row stride must be 16-byte aligned.  No workspace. */
typedef struct {
  int32_t B, S, E;          /* batches, tokens per batch, embedding width */
  int32_t H, D;             /* heads and head dim of ONE output */
  int64_t x_sb, x_ss;       /* strides of x in elements */
} lvx_projection;
lvx_status lvx_xattn_project(const lvx_projection* p, lvx_dtype dtype, const void* x, const void* w,
                             int n_out, void* const* out, void* hip_stream);

/* The chain rule through those projections (Section 2's linear maps; Section 3.2 evaluates them
 * again in the backward pass precisely so that dK and dV can be carried back to the visual tokens
 * and to W_K, W_V without K and V having been kept).  With d_out[o] = d loss / d out[o]:
 *     dx[b, s, e]              = sum_{o, h, c} d_out[o][b, h, s, c] * w[(o * H + h) * D + c, e]
 *     dw[(o * H + h) * D + c, e] += sum_{b, s} d_out[o][b, h, s, c] * x[b, s, e].
 * p, x, w, n_out as for lvx_xattn_project (same layouts, same stride rules).
 * d_out  host array of n_out (1 or 2) device pointers, each [B, H, S, D] of `dtype`, contiguous
 *        (what lvx_xattn_bwd writes as dK, dV, and lvx_xattn_dq_finalize as dQ).
 * dx     device, [B, S, E] of `dtype` with x's strides, OVERWRITTEN (one rounding of a float32
 *        sum); NULL = not wanted.
 * dw     device, [n_out * H * D, E] float32, contiguous, ACCUMULATED INTO: the caller zeroes it
 *        before the first K/V block of a step, and each block's call adds its tokens' part
 *        (the order of the additions is the order of the calls: results repeat bit for bit);
 *        NULL = not wanted.  At least one of dx, dw must be given.
 * LVX_BF16 runs on the matrix cores when E % 256 == 0, (H * D) % 256 == 0, D % 8 == 0,
 * B * S < 2^24 and B * S * H * D < 2^30; other shapes, and LVX_F32, take a plain kernel (one
 * float32 sum per element in the order of the definition: correctness-grade, slow).
 * LVX_BF16: pointers and x's row stride must be 16-byte aligned.  No workspace.
 * When dw has fewer tiles of 256 x 256 than the GPU has compute units, the tokens are divided
 * among several workgroups per tile, which add their sums to dw one after the other in a fixed
 * order (so results still repeat bit for bit); whose turn it is stands in a small table inside the
 * library, one per GPU, that every call leaves as it found it.  Two such calls running at the same
 * time on one GPU (different streams) would share that table: do not overlap them.  Waits are
 * bounded; a workgroup whose turn never came writes NaN over its part of dw instead of a sum. */
lvx_status lvx_xattn_project_bwd(const lvx_projection* p, lvx_dtype dtype, const void* x, const void* w,
                                 int n_out, const void* const* d_out, void* dx, float* dw,
                                 void* hip_stream);

/* Human-readable name of a status code (static storage). */
const char* lvx_strerror(lvx_status s);

#ifdef __cplusplus
}
#endif
#endif /* LVX_H */
