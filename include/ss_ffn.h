/* ss_ffn.h -- C ABI of the co-sharded feed-forward operator for MI355X (gfx950).
 *
 * The other half of the co-shard plan (Section 6.1, "parallelization plans": attention heads and
 * feed-forward hidden dimensions are partitioned; Section 6.3: co-shard is applied to the
 * attention and feed-forward operators, with recompute).  One call runs one GPU's share of the
 * position-wise feed-forward operator the paper cites,
 *
 *     Z = X W1 + b1 ;  H = act(Z) ;  Y = H W2 (+ b2)        X [T,dm], W1 [dm,dh], W2 [dh,dm]
 *
 * as k sub-operators executed one after another on one HIP stream (op-trans along the hidden
 * dimension, Section 3.1; op-assign to one device and op-order, Section 3.2).  The share is the
 * hidden range [lo,hi).  Unlike the head split of attention every sub-operator contributes to the
 * whole output: Y and dX are value-split partial sums (Section 4; Section 5 for the gradient of
 * the shared input).  By default the partial sum between chunks lives in the output tensor itself
 * (bf16: every chunk's product is accumulated in fp32 on top of the widened partial sum and rounded
 * once per chunk), so the workspace holds one chunk's hidden activations and nothing else, and
 * shrinks as 1/k: the point of the plan (Sections 2 and 6.3).  Y and dX then carry one bf16
 * rounding per chunk and differ between k in the last bits.  With SS_FFN_FLAG_EXACT_SUM the partial
 * sum is kept in fp32 in the workspace instead (4 T dm more bytes for k > 1, more than the hidden
 * activations the split frees when hi-lo < 2 dm) and Y and dX are the same bits for every k.
 * dW1, db1, dW2 and db2 are disjoint slices or whole-operator sums and never depend on k.  Only one
 * chunk's hidden activations [T, (hi-lo)/k] are alive at a time, and the backward recomputes them.
 *
 * All pointers are DEVICE pointers unless said otherwise; the descriptor and size outputs are HOST
 * memory.  The library allocates no device memory and never synchronises the host; the work is
 * enqueued on the caller's stream, except that ss_ffn_bwd forks dW2 and the bias gradients onto a
 * helper stream of the library's own (one per device, default priority, created on first use) and
 * joins it back into the caller's stream with events before the call returns: to the caller the
 * call is ordered on its stream like any other.  That stream is the only state the library keeps;
 * the fork / join events are created and released per call, so calls from several host threads or
 * on several caller streams of one device are independent (their helper work is merely queued on
 * the same helper stream).  Error codes are those of ss_attn.h.
 */
#ifndef SS_FFN_H
#define SS_FFN_H

#include <stddef.h>
#include <stdint.h>

#include "ss_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SS_ACT_RELU = 0, SS_ACT_GELU_TANH = 1 } ss_act;

/* Describes the operator and this GPU's share.  All matrices are row-major bf16 (dtype must be
 * SS_BF16), leading dimensions in elements and multiples of 8, base pointers 16-byte aligned:
 *   X, Y, dY, dX : [T, dm], row stride ld_x
 *   W1, dW1      : [dm, dh], row stride ld_w1        b1, db1 : [dh]
 *   W2, dW2      : [dh, dm], row stride ld_w2        b2, db2 : [dm]
 * dm and dh multiples of 8; every operand smaller than 2 GiB and every leading dimension below
 * 2^22 elements (SS_ERR_UNSUPPORTED otherwise).  lo and hi multiples of 8; chunk boundaries fall on
 * multiples of 16 hidden columns counted from lo (ss_ffn_chunk_range). */
typedef struct {
  int32_t T, dm, dh;
  int32_t dtype; /* SS_BF16 */
  int32_t act;   /* ss_act */
  int64_t ld_x, ld_w1, ld_w2;
  int32_t lo, hi; /* this GPU's hidden range */
  int32_t k;      /* co-shard factor, 1 <= k <= ceil((hi-lo)/16) */
  int32_t flags;  /* 0 or SS_FFN_FLAG_EXACT_SUM */
} ss_ffn_desc;

enum {
  SS_FFN_FLAG_EXACT_SUM = 1 /* fp32 partial sums of Y / dX in the workspace: identical bits for every k */
};

/* Workspace bytes ss_ffn_fwd / ss_ffn_bwd need (host outputs).  Forward: one chunk's H.  Backward:
 * one chunk's H and act'(Z) (overwritten by dZ).  Both shrink as 1/k.  With SS_FFN_FLAG_EXACT_SUM
 * and k > 1 the fp32 accumulator of Y (forward) or dX (backward) is added. */
int ss_ffn_workspace_bytes(const ss_ffn_desc* desc, size_t* fwd_bytes, size_t* bwd_bytes);

/* Hidden range of chunk c (0 <= c < k): balanced in units of 16 columns counted from lo. */
int ss_ffn_chunk_range(const ss_ffn_desc* desc, int32_t c, int32_t* lo, int32_t* hi);

/* Y = sum over the share's chunks of act(X W1[:,c] + b1[c]) W2[c,:], plus b2 if b2 != NULL.
 * Y holds the partial sum between chunks (written once, by the last chunk, with
 * SS_FFN_FLAG_EXACT_SUM).  workspace: 256-byte aligned, >= fwd_bytes. */
int ss_ffn_fwd(const ss_ffn_desc* desc, const void* X, const void* W1, const void* b1, const void* W2, const void* b2,
               void* Y, void* workspace, size_t workspace_bytes, void* stream);

/* Gradients for dY.  dX [T,dm]: partial sum over the share.  dW1 / db1 / dW2: only columns / entries
 * / rows [lo,hi) are written (the rest of these full-size tensors is left untouched).  db2 [dm] may
 * be NULL (skipped); it is the full gradient of b2, independent of the share. */
int ss_ffn_bwd(const ss_ffn_desc* desc, const void* X, const void* W1, const void* b1, const void* W2, const void* dY,
               void* dX, void* dW1, void* db1, void* dW2, void* db2, void* workspace, size_t workspace_bytes,
               void* stream);

/* Benchmark instrumentation as in ss_attn.h: kernels of the feed-forward path.  While it is enabled
 * the helper stream is not used, so that every kernel is timed running alone. */
typedef enum {
  SS_FK_UP = 0,      /* H = act(X W1 + b1) (forward and recompute)   */
  SS_FK_DOWN = 1,    /* Y += H W2                                    */
  SS_FK_DH = 2,      /* dZ = (dY W2^T) * act'(Z)                     */
  SS_FK_DW2 = 3,     /* dW2 = H^T dY                                 */
  SS_FK_DW1 = 4,     /* dW1 = X^T dZ                                 */
  SS_FK_DX = 5,      /* dX += dZ W1^T                                */
  SS_FK_COLSUM = 6,  /* db1, db2                                     */
  SS_FK_COUNT = 7
} ss_ffn_kernel_id;
int ss_ffn_profile_enable(int on);
int ss_ffn_profile_read(int kernel, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* SS_FFN_H */
