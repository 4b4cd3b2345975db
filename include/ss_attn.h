/* ss_attn.h -- C ABI of the co-sharded attention library for MI355X (gfx950).
 *
 * One call runs one GPU's share of a multi-head attention operator, forward or
 * backward, as k sub-operators executed one after another on one HIP stream.
 * This is the SuperScaler "co-shard" plan (Section 2 of the paper): the
 * operator is partitioned along one axis by op-trans (Section 3.1) into
 * functionally equivalent sub-operators, every sub-operator is assigned to the
 * same device by op-assign and ordered by op-order (Section 3.2), and peak
 * memory falls because only one sub-operator's scratch is alive at a time while
 * its forward is recomputed inside the backward (Sections 2 and 6.3).
 *
 * The operator itself (the paper names it, it does not print it):
 *   S[i,j] = scale * <Q[i,:],K[j,:]> + Bias[h,i,j];  masked pairs get -inf
 *   P      = softmax over j of S ;  O = P V ;  Y = sigmoid(G)*O if gated else O
 * and the backward produces dQ, dK, dV, dG and the bias gradient for dY.
 *
 * All pointers are DEVICE pointers unless said otherwise; the descriptor and
 * the size outputs are HOST memory.  The library allocates no device memory and
 * never synchronises: all work is enqueued on the caller's stream and the call
 * returns while it may still be running.  It keeps no state between calls, except
 * the opt-in timing instrumentation at the end of this file.
 */
#ifndef SS_ATTN_H
#define SS_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SS_F32 = 0, SS_BF16 = 1 } ss_dtype;
typedef enum { SS_AXIS_HEAD = 0, SS_AXIS_ROW = 1 } ss_axis; /* ROW = the batch-like axis b */
typedef enum { SS_MASK_NONE = 0, SS_MASK_CAUSAL = 1, SS_MASK_REGION = 2 } ss_mask_kind;
typedef enum { SS_BIAS_NONE = 0, SS_BIAS_DENSE = 1, SS_BIAS_RELPOS = 2 } ss_bias_kind;

enum {
  SS_OK = 0,
  SS_ERR_NULL = -1,        /* a required pointer is NULL                               */
  SS_ERR_BAD_SHAPE = -2,   /* B,H,S,D < 1, bad strides, bad window or mask period      */
  SS_ERR_BAD_RANGE = -3,   /* lo < 0, lo >= hi, or hi beyond the axis extent           */
  SS_ERR_BAD_K = -4,       /* k < 1 or k > hi-lo                                       */
  SS_ERR_UNSUPPORTED = -5, /* no kernel for this dtype / D / S / bias / mask / flags   */
  SS_ERR_WORKSPACE = -6,   /* workspace NULL, too small, or not 256-byte aligned       */
  SS_ERR_HIP = -7,         /* a kernel launch failed (hipGetLastError text on stderr)  */
  SS_ERR_STATIC_SCRATCH = -8 /* ss_attn_bwd_static: the share needs more than its buffer */
};

/* desc.flags */
enum {
  SS_FLAG_GENERIC_KERNELS = 1 /* force the plain (non-MFMA) kernels; any D <= 256, any dtype */
};

/* Describes the WHOLE operator and this GPU's share of it.
 *
 * Activations Q,K,V,G,Y,dY,dQ,dK,dV,dG all share one layout: element (b,s,h,d)
 * is at  b*stride_b + s*stride_s + h*stride_h + d  (strides in elements, d
 * contiguous).  A packed [B,S,H,D] tensor has stride_h=D, stride_s=H*D,
 * stride_b=S*H*D.  For SS_BF16 every stride must be a multiple of 8 elements
 * and every base pointer 16-byte aligned.
 *
 * Bias (additive, shared by all rows b):
 *   SS_BIAS_DENSE : bias[h][i][j], packed [H,S,S], dtype bias_dtype.
 *   SS_BIAS_RELPOS: table[h][r],   packed [H,(2*win_h-1)*(2*win_w-1)], S must equal
 *                   win_h*win_w; token i sits at (i / win_w, i % win_w) and the
 *                   pair (i,j) uses r = (yi-yj+win_h-1)*(2*win_w-1) + (xi-xj+win_w-1).
 * Mask:
 *   SS_MASK_CAUSAL: pair (i,j) is masked iff j > i.
 *   SS_MASK_REGION: region_ids is int32 [mask_period,S]; row b uses line b % mask_period;
 *                   pair (i,j) is masked iff the two ids differ.
 *   Precondition (not checked on the device): every query keeps at least one key.
 *   Both mask kinds guarantee it (the diagonal is never masked).
 *
 * The share: indices [lo,hi) of shard_axis (heads, or rows b).  It is cut into k
 * consecutive chunks, chunk c = [lo + floor(c*n/k), lo + floor((c+1)*n/k)), n = hi-lo
 * (the uniform partition of Section 4's RVD notation, balanced when k does not
 * divide n), executed in order c = 0..k-1.
 */
typedef struct {
  int32_t B, H, S, D;
  int32_t dtype;       /* ss_dtype of the activations                              */
  float scale;         /* multiplies <Q,K>                                         */
  int64_t stride_b, stride_s, stride_h;
  int32_t bias_kind;   /* ss_bias_kind                                             */
  int32_t bias_dtype;  /* ss_dtype of bias / table                                 */
  int32_t win_h, win_w;
  int32_t mask_kind;   /* ss_mask_kind                                             */
  int32_t mask_period;
  int32_t gated;       /* 1: G holds gate logits, sigmoid applied inside           */
  int32_t shard_axis;  /* ss_axis                                                  */
  int32_t lo, hi;
  int32_t k;           /* co-shard factor, 1 <= k <= hi-lo                         */
  uint32_t flags;
} ss_attn_desc;

/* Validates the descriptor and reports the device workspace each call needs, in
 * bytes (host outputs, either may be NULL).  The backward workspace holds one
 * chunk's recomputed softmax statistics and pre-gated output gradient and is
 * reused by every chunk, so it shrinks as k grows; this is what makes
 * peak memory = caller tensors + workspace fall with k (Section 6.3).  Parts that
 * do not depend on k (a transposed copy of a dense bias, group partial sums of the
 * bias gradient) are included in the figure.
 * Needs no GPU.  Returns SS_OK or a negative error. */
int ss_attn_workspace_bytes(const ss_attn_desc* desc, size_t* fwd_bytes, size_t* bwd_bytes);

/* Host-only helper: the sub-range of chunk c (0 <= c < k) under the rule above. */
int ss_attn_chunk_range(const ss_attn_desc* desc, int32_t c, int32_t* chunk_lo, int32_t* chunk_hi);

/* Forward (Section 2, co-shard; operator as defined at the top of this file).
 *   Q,K,V   in : activations, whole-operator tensors.
 *   bias    in : per bias_kind, NULL iff SS_BIAS_NONE.
 *   region_ids in : per mask_kind, NULL unless SS_MASK_REGION.
 *   G       in : gate logits, NULL iff !gated.
 *   Y       out: activations layout; only slices inside [lo,hi) are written.
 *   lse     out: optional float [B,H,S] (log of the softmax normaliser, natural log);
 *                only entries inside the share are written.  May be NULL.
 *   workspace  : device scratch of at least fwd_bytes (may be NULL when that is 0).
 *   hip_stream : a hipStream_t (NULL = the default stream).
 * Nothing is enqueued when an error is returned by validation. */
int ss_attn_fwd(const ss_attn_desc* desc, const void* Q, const void* K, const void* V,
                const void* bias, const int32_t* region_ids, const void* G,
                void* Y, float* lse,
                void* workspace, size_t workspace_bytes, void* hip_stream);

/* Backward (Section 2: each sub-operator's forward is recomputed; Section 5:
 * the bias is read by every sub-operator, so its gradient is value-split and
 * the chunks' parts are summed, here in a fixed order so that the result does
 * not depend on k bit for bit).
 *   dY      in : gradient of the loss w.r.t. Y.
 *   lse     in : optional, as written by ss_attn_fwd; NULL = recompute per chunk.
 *   dQ,dK,dV out: activations layout, slices inside the share only.
 *   dBias   out: optional float; DENSE: [H,S,S], RELPOS: [H,R].  OVERWRITTEN with the
 *                sum over the rows of this share (HEAD axis: only heads in [lo,hi)
 *                are written).  NULL = not wanted.  Ignored for SS_BIAS_NONE.
 *   dG      out: gradient w.r.t. the gate logits; required iff gated.
 *   workspace  : at least bwd_bytes, 256-byte aligned. */
int ss_attn_bwd(const ss_attn_desc* desc, const void* Q, const void* K, const void* V,
                const void* bias, const int32_t* region_ids, const void* G,
                const void* dY, const float* lse,
                void* dQ, void* dK, void* dV, float* dBias, void* dG,
                void* workspace, size_t workspace_bytes, void* hip_stream);

/* The backward for callers that cannot allocate device memory and have no workspace to hand
 * over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and kernels as ss_attn_bwd, but the scratch is a buffer built into
 * the library (SS_ATTN_STATIC_SCRATCH_BYTES of device memory per GPU the library is used on,
 * held until the process ends) instead of a caller workspace.  The call allocates and frees
 * nothing.  A share whose ss_attn_workspace_bytes backward figure exceeds the buffer is
 * rejected with SS_ERR_STATIC_SCRATCH before anything is enqueued (raise k, or use
 * ss_attn_bwd).  Every call on one GPU shares that GPU's buffer: two calls that may run at
 * the same time on one GPU (different streams or threads) race; calls on one stream are safe.
 * The buffer keeps the previous call's contents; no part of it needs to start at zero. */
#define SS_ATTN_STATIC_SCRATCH_BYTES (32u << 20)
int ss_attn_bwd_static(const ss_attn_desc* desc, const void* Q, const void* K, const void* V,
                       const void* bias, const int32_t* region_ids, const void* G,
                       const void* dY, const float* lse,
                       void* dQ, void* dK, void* dV, float* dBias, void* dG, void* hip_stream);

/* Static text for an error code (never NULL). */
const char* ss_strerror(int code);

/* Host-only: which kernel family a descriptor is served by: "mfma_bf16" (bf16
 * activations, D in {32,64,128}), "mfma_bf16_short" (bf16, D = 32, S <= 64, not
 * gated: one wavefront holds a whole score matrix) or "plain_fp32" (everything
 * else, and whenever SS_FLAG_GENERIC_KERNELS is set).  NULL for an invalid
 * descriptor. */
const char* ss_attn_kernel_family(const ss_attn_desc* desc);

/* Benchmark instrumentation, not part of the method.  While enabled, every kernel
 * the scheduler launches is bracketed by two HIP events recorded on the launch
 * stream (this is the only state the library keeps, and the only time it creates
 * HIP objects).  ss_attn_profile_read waits for the recorded events, returns the
 * summed duration in milliseconds and the number of launches of one kernel since
 * the last read, and resets both.  Not thread-safe. */
typedef enum {
  SS_K_FWD = 0, SS_K_RECOMPUTE = 1, SS_K_DQ = 2, SS_K_DKDV = 3, SS_K_DBIAS = 4, SS_K_TABLE_REDUCE = 5,
  SS_K_DQ_DKDV = 6,   /* dQ and dK/dV in one launch (small shares with long rows) */
  SS_K_DBIAS_FOLD = 7, /* fold of completed bias-gradient group partials into the result */
  SS_K_RECOMPUTE_DQ = 8, /* recompute pass and dQ in one launch (head size 32, large shares) */
  SS_K_COUNT = 9
} ss_kernel_id;
int ss_attn_profile_enable(int on);
int ss_attn_profile_read(int kernel, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* SS_ATTN_H */
