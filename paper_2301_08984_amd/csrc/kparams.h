// Kernel-side view of one co-shard sub-task (one chunk of the share).
// Filled by the host scheduler, passed by value to every kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssa {

struct KP {
  // whole-operator activations, element (b,s,h,d) at b*sb + s*ss + h*sh + d
  const void *Q, *K, *V, *G, *dY;
  void *Y, *dQ, *dK, *dV, *dG;
  int64_t sb, ss, sh;
  // gradient w.r.t. the un-gated output: dY itself, or the chunk's pre-gated copy in the
  // workspace; element (b,s,h,d) at (b - do_b0)*do_sb + s*do_ss + (h - do_h0)*do_sh + d, where
  // (do_b0, do_h0) is the first (row, head) the buffer holds: (0,0) for a whole-operator tensor,
  // the chunk's origin for chunk-sized scratch
  const void* dO;
  int64_t do_sb, do_ss, do_sh;
  int do_b0, do_h0;
  void* dO_out;  // recompute pass writes here when gated (same indexing as dO)
  // softmax statistics, (b,h,s) at (b - lse_b0)*lse_sb + (h - lse_h0)*lse_sh + s, origins as above
  float* lse_out;       // forward: optional caller tensor; recompute: workspace
  const float* lse;     // backward kernels read this
  int64_t lse_sb, lse_sh;
  int lse_b0, lse_h0;
  float* delta;         // rowsum(dO*O), workspace; (b,h,s) at (b - dl_b0)*dl_sb + (h - dl_h0)*dl_sh + s
  int64_t dl_sb, dl_sh;
  int dl_b0, dl_h0;
  // bias / mask
  const void* bias;     // dense [H,S,S] or table [H,R]
  const void* biasT;    // workspace copy of a dense bf16 bias with the last two axes swapped (or nullptr)
  const int32_t* region;
  float* dbias_acc;     // dense fp32 [H,S,S] accumulator (caller's dBias, or workspace for RELPOS)
  int dbias_accumulate; // 0: this chunk starts the sum, 1: continue from the stored value
  // shapes and the chunk
  int B, H, S, D;
  int b0, b1, h0, h1;
  // grouped bias-gradient sums: partial sums per group of sm_gw consecutive global rows, fp32 in the
  // workspace (nullptr: not grouped / bias gradient not wanted).  Group g, head h sits at
  // [((g - sm_g0) % sm_ring) * sm_hs + (h - sm_h0)][S*S]: a ring of sm_ring group slots (complete groups
  // are folded into the result after every chunk and their slots reused), sm_hs heads per slot from
  // head sm_h0 on
  float* sm_partial;
  int sm_gw, sm_g0, sm_ring, sm_hs, sm_h0;
  int share_b0;     // first row of the whole share
  int share_units;  // (row, head) pairs in the whole share [lo,hi): kernel-shape choices use this, never the chunk
  float scale;
  int bias_kind, bias_bf16, mask_kind, mask_period, win_h, win_w, gated;
};

// launchers (each returns the hipError_t of the launch)
hipError_t launch_generic_fwd(const KP& p, bool bf16, bool recompute, hipStream_t st);
hipError_t launch_generic_dq(const KP& p, bool bf16, hipStream_t st);
hipError_t launch_generic_dkdv(const KP& p, bool bf16, hipStream_t st);
hipError_t launch_generic_dbias(const KP& p, bool bf16, hipStream_t st);
// dTable[h][r] = sum of dense[h][i][j] over idx(i,j)=r, heads [h0,h1), fixed order
hipError_t launch_relpos_reduce(const float* dense, float* table, int h0, int h1, int S, int win_h,
                                int win_w, hipStream_t st);
hipError_t launch_fill_zero(float* p, size_t n, hipStream_t st);

bool small_supported(const KP& p, bool bf16);
hipError_t launch_small_fwd(const KP& p, hipStream_t st);
hipError_t launch_small_bwd(const KP& p, hipStream_t st);
// Folds the complete slices [s0, s1) of `slice` consecutive groups each (the last may be shorter:
// `ngroups` groups exist) into dense[h][i][j], heads h = hd0 .. hd0 + nh - 1 (slot heads 0 .. nh-1):
// every slice is summed in ascending group order into its first group's slot, then the slice sums
// are added in ascending order to dense (which starts from zero when `first`).  The additions are
// the same whatever the chunking, so the result does not depend on k.
hipError_t launch_group_fold(float* partial, float* dense, int ring, int hs, int hd0, int nh, int S, int slice,
                             int s0, int s1, int ngroups, bool first, hipStream_t st);

bool mfma_supported(const KP& p, bool bf16);
hipError_t launch_mfma_fwd(const KP& p, bool recompute, hipStream_t st);
hipError_t launch_mfma_dq(const KP& p, hipStream_t st);
hipError_t launch_mfma_dkdv(const KP& p, hipStream_t st);
hipError_t launch_mfma_dbias(const KP& p, hipStream_t st);
bool mfma_fuses_dq_dkdv(const KP& p);
hipError_t launch_mfma_dq_dkdv(const KP& p, hipStream_t st);
bool mfma_fuses_recompute_dq(const KP& p);
hipError_t launch_mfma_recompute_dq(const KP& p, hipStream_t st);
bool mfma_wants_bias_transpose(const KP& p);
int mfma_dbias_group_rows(const KP& p);        // 0, or rows per group of the grouped bias-gradient sum  // the backward kernels read a transposed bias copy
hipError_t launch_bias_transpose(const void* bias, void* biasT, int S, int h0, int h1, hipStream_t st);

}  // namespace ssa
