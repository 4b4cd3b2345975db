// C ABI, descriptor validation and the chunk scheduler: the share [lo,hi) is cut
// into k chunks which are enqueued one after another on the caller's stream
// (op-order), all on the current device (op-assign), every chunk reusing the same
// workspace (co-shard, Section 2 of the paper).
#include "../../include/ss_attn.h"
#include "kparams.h"

#include <cstdio>
#include <mutex>
#include <vector>

// Built-in scratch of ss_attn_bwd_static: one copy per GPU the library runs on, held until the
// process ends.  Host code never uses this name as an address: it asks the runtime for the
// device address once per device (static_scratch below) and passes that pointer on.
static __device__ __align__(256) unsigned char scratch[SS_ATTN_STATIC_SCRATCH_BYTES];

namespace {

using ssa::KP;

constexpr size_t ALIGN = 256;
inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }
inline size_t esize(int dtype) { return dtype == SS_BF16 ? 2 : 4; }

int validate(const ss_attn_desc* d) {
  if (!d) return SS_ERR_NULL;
  if (d->B < 1 || d->H < 1 || d->S < 1 || d->D < 1) return SS_ERR_BAD_SHAPE;
  if (d->dtype != SS_F32 && d->dtype != SS_BF16) return SS_ERR_UNSUPPORTED;
  if (d->stride_h < d->D || d->stride_s < d->D || d->stride_b < d->D) return SS_ERR_BAD_SHAPE;
  if (d->dtype == SS_BF16 && (d->stride_h % 8 || d->stride_s % 8 || d->stride_b % 8 || d->D % 8))
    return SS_ERR_BAD_SHAPE;
  if (d->bias_kind < SS_BIAS_NONE || d->bias_kind > SS_BIAS_RELPOS) return SS_ERR_UNSUPPORTED;
  if (d->bias_kind != SS_BIAS_NONE && d->bias_dtype != SS_F32 && d->bias_dtype != SS_BF16)
    return SS_ERR_UNSUPPORTED;
  if (d->bias_kind == SS_BIAS_RELPOS &&
      (d->win_h < 1 || d->win_w < 1 || (int64_t)d->win_h * d->win_w != d->S))
    return SS_ERR_BAD_SHAPE;
  if (d->mask_kind < SS_MASK_NONE || d->mask_kind > SS_MASK_REGION) return SS_ERR_UNSUPPORTED;
  if (d->mask_kind == SS_MASK_REGION && d->mask_period < 1) return SS_ERR_BAD_SHAPE;
  if (d->gated != 0 && d->gated != 1) return SS_ERR_BAD_SHAPE;
  if (d->shard_axis != SS_AXIS_HEAD && d->shard_axis != SS_AXIS_ROW) return SS_ERR_UNSUPPORTED;
  const int extent = d->shard_axis == SS_AXIS_HEAD ? d->H : d->B;
  if (d->lo < 0 || d->lo >= d->hi || d->hi > extent) return SS_ERR_BAD_RANGE;
  if (d->k < 1 || d->k > d->hi - d->lo) return SS_ERR_BAD_K;
  if (d->flags & ~(uint32_t)SS_FLAG_GENERIC_KERNELS) return SS_ERR_UNSUPPORTED;
  if (d->D > 256) return SS_ERR_UNSUPPORTED;
  // grid dimensions y,z carry heads and rows
  if (d->H > 65535 || d->B > 65535) return SS_ERR_UNSUPPORTED;
  return SS_OK;
}

inline void chunk(const ss_attn_desc* d, int c, int* a, int* b) {
  const int64_t n = d->hi - d->lo;
  *a = d->lo + (int)((c * n) / d->k);
  *b = d->lo + (int)(((c + 1) * n) / d->k);
}

struct WsLayout {
  size_t lse, delta, dO, dense, partial, biasT, total;
  // grouped bias-gradient sums: rows per group (0: none), first group and group count of the share,
  // groups per slice of the two-level sum, ring of group slots kept in the workspace, heads per slot
  int gw, g0, ngroups, slice, ring, hs;
};

constexpr int SMALL_GW = 8;  // rows per bias-gradient group of the short-sequence kernels

enum Family { FAM_PLAIN = 0, FAM_MFMA = 1, FAM_SMALL = 2 };

KP base_params(const ss_attn_desc* d);

WsLayout bwd_layout(const ss_attn_desc* d, Family fam) {
  const int64_t n = d->hi - d->lo;
  const int64_t nmax = (n + d->k - 1) / d->k;  // largest chunk of the balanced split
  const int64_t Bc = d->shard_axis == SS_AXIS_ROW ? nmax : d->B;
  const int64_t Hc = d->shard_axis == SS_AXIS_HEAD ? nmax : d->H;
  WsLayout w{};
  size_t off = 0;
  w.lse = off;   off += align_up((size_t)(Bc * Hc * d->S) * 4);
  w.delta = off; off += align_up((size_t)(Bc * Hc * d->S) * 4);
  w.dO = off;
  if (d->gated) off += align_up((size_t)(Bc * d->S * Hc * d->D) * esize(d->dtype));
  w.dense = off;
  if (d->bias_kind == SS_BIAS_RELPOS) off += align_up((size_t)d->H * d->S * d->S * 4);
  w.partial = off;
  const int row_lo = d->shard_axis == SS_AXIS_ROW ? d->lo : 0;
  const int row_hi = d->shard_axis == SS_AXIS_ROW ? d->hi : d->B;
  // rows per group: fixed for the short-sequence kernels, shape-dependent for the tiled kernel
  w.gw = 0;
  if (d->bias_kind != SS_BIAS_NONE) {
    if (fam == FAM_SMALL) w.gw = SMALL_GW;
    else if (fam == FAM_MFMA) w.gw = ssa::mfma_dbias_group_rows(base_params(d));
  }
  if (w.gw > 0) {
    w.g0 = row_lo / w.gw;
    w.ngroups = (row_hi - 1) / w.gw - w.g0 + 1;
    // slices depend on the share only, so that the order of additions does not depend on k
    w.slice = w.ngroups / 16 < 1 ? 1 : (w.ngroups / 16 > 32 ? 32 : w.ngroups / 16);
    if (d->shard_axis == SS_AXIS_ROW) {
      // complete slices are folded into the result after every chunk: what stays alive is the slice
      // under way plus the groups the next chunk touches
      const int64_t per_chunk = (nmax + w.gw - 1) / w.gw + 1;
      w.ring = (int)(w.slice + per_chunk < w.ngroups ? w.slice + per_chunk : w.ngroups);
      w.hs = d->H;
    } else {
      w.ring = w.ngroups;   // a chunk of heads walks every row: all groups, but only the chunk's heads
      w.hs = (int)nmax;
    }
    off += align_up((size_t)w.ring * w.hs * d->S * d->S * 4);
  }
  w.biasT = off;
  if (d->bias_kind == SS_BIAS_DENSE && d->bias_dtype == SS_BF16) off += align_up((size_t)d->H * d->S * d->S * 2);
  w.total = off;
  return w;
}

KP base_params(const ss_attn_desc* d) {
  KP p{};
  p.sb = d->stride_b; p.ss = d->stride_s; p.sh = d->stride_h;
  p.B = d->B; p.H = d->H; p.S = d->S; p.D = d->D;
  p.scale = d->scale;
  p.bias_kind = d->bias_kind; p.bias_bf16 = d->bias_dtype == SS_BF16;
  p.mask_kind = d->mask_kind; p.mask_period = d->mask_period > 0 ? d->mask_period : 1;
  p.win_h = d->win_h; p.win_w = d->win_w; p.gated = d->gated;
  p.share_units = (d->hi - d->lo) * (d->shard_axis == SS_AXIS_HEAD ? d->B : d->H);
  p.share_b0 = d->shard_axis == SS_AXIS_ROW ? d->lo : 0;
  p.sm_gw = SMALL_GW;
  return p;
}

Family family_of(const ss_attn_desc* d) {
  if (d->flags & SS_FLAG_GENERIC_KERNELS) return FAM_PLAIN;
  const KP p = base_params(d);
  const bool bf16 = d->dtype == SS_BF16;
  if (ssa::small_supported(p, bf16)) return FAM_SMALL;
  if (ssa::mfma_supported(p, bf16)) return FAM_MFMA;
  return FAM_PLAIN;
}

inline void set_chunk(KP& p, const ss_attn_desc* d, int c) {
  int a, b;
  chunk(d, c, &a, &b);
  if (d->shard_axis == SS_AXIS_HEAD) { p.b0 = 0; p.b1 = d->B; p.h0 = a; p.h1 = b; }
  else { p.b0 = a; p.b1 = b; p.h0 = 0; p.h1 = d->H; }
}

// Device address of this GPU's copy of `scratch`, looked up on the first call per device.
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[MAX_DEVICES] = {nullptr};

int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
    fprintf(stderr, "ss_attn: hipGetDevice: %s (device %d)\n", hipGetErrorString(e), dev);
    return SS_ERR_HIP;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      fprintf(stderr, "ss_attn: hipGetSymbolAddress(scratch): %s\n", hipGetErrorString(e));
      return SS_ERR_HIP;
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return SS_OK;
}

int hip_fail(hipError_t e, const char* what) {
  fprintf(stderr, "ss_attn: %s: %s\n", what, hipGetErrorString(e));
  return SS_ERR_HIP;
}
// optional per-kernel timing with HIP events (benchmark instrumentation)
struct ProfRec { hipEvent_t a, b; int kind; };
bool g_prof_on = false;
std::vector<ProfRec> g_prof_pending;
double g_prof_ms[SS_K_COUNT] = {0};
int64_t g_prof_n[SS_K_COUNT] = {0};

struct ProfScope {
  hipStream_t st; int kind; hipEvent_t a = nullptr, b = nullptr; bool on;
  ProfScope(hipStream_t s, int k) : st(s), kind(k), on(g_prof_on) {
    if (on) {
      on = hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess &&
           hipEventRecord(a, st) == hipSuccess;
    }
  }
  ~ProfScope() {
    if (on && hipEventRecord(b, st) == hipSuccess) g_prof_pending.push_back({a, b, kind});
  }
};

#define SS_LAUNCH(kind, expr, what)                   \
  do {                                                \
    hipError_t e_;                                    \
    {                                                 \
      ProfScope ps_(st, kind);                        \
      e_ = (expr);                                    \
    }                                                 \
    if (e_ != hipSuccess) return hip_fail(e_, what);  \
  } while (0)

}  // namespace

extern "C" {

const char* ss_strerror(int code) {
  switch (code) {
    case SS_OK: return "ok";
    case SS_ERR_NULL: return "a required pointer is NULL";
    case SS_ERR_BAD_SHAPE: return "bad shape, stride, window or mask period";
    case SS_ERR_BAD_RANGE: return "bad [lo,hi) for the shard axis";
    case SS_ERR_BAD_K: return "co-shard factor k must satisfy 1 <= k <= hi-lo";
    case SS_ERR_UNSUPPORTED: return "unsupported dtype / head size / bias / mask / flags";
    case SS_ERR_WORKSPACE: return "workspace missing, too small or not 256-byte aligned";
    case SS_ERR_HIP: return "HIP kernel launch failed";
    case SS_ERR_STATIC_SCRATCH: return "the backward needs more scratch than the built-in buffer of ss_attn_bwd_static holds";
    default: return "unknown error code";
  }
}

const char* ss_attn_kernel_family(const ss_attn_desc* d) {
  if (validate(d) != SS_OK) return nullptr;
  switch (family_of(d)) {
    case FAM_SMALL: return "mfma_bf16_short";
    case FAM_MFMA: return "mfma_bf16";
    default: return "plain_fp32";
  }
}

int ss_attn_profile_enable(int on) {
  g_prof_on = on != 0;
  return SS_OK;
}

int ss_attn_profile_read(int kernel, double* total_ms, int64_t* launches) {
  if (kernel < 0 || kernel >= SS_K_COUNT) return SS_ERR_BAD_RANGE;
  for (ProfRec& r : g_prof_pending) {
    float ms = 0.f;
    if (hipEventSynchronize(r.b) == hipSuccess && hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
      g_prof_ms[r.kind] += ms;
      g_prof_n[r.kind] += 1;
    }
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
  }
  g_prof_pending.clear();
  if (total_ms) *total_ms = g_prof_ms[kernel];
  if (launches) *launches = g_prof_n[kernel];
  g_prof_ms[kernel] = 0;
  g_prof_n[kernel] = 0;
  return SS_OK;
}

int ss_attn_workspace_bytes(const ss_attn_desc* d, size_t* fwd_bytes, size_t* bwd_bytes) {
  const int rc = validate(d);
  if (rc != SS_OK) return rc;
  if (fwd_bytes) *fwd_bytes = 0;
  if (bwd_bytes) *bwd_bytes = bwd_layout(d, family_of(d)).total;
  return SS_OK;
}

int ss_attn_chunk_range(const ss_attn_desc* d, int32_t c, int32_t* lo, int32_t* hi) {
  const int rc = validate(d);
  if (rc != SS_OK) return rc;
  if (!lo || !hi) return SS_ERR_NULL;
  if (c < 0 || c >= d->k) return SS_ERR_BAD_K;
  int a, b;
  chunk(d, c, &a, &b);
  *lo = a; *hi = b;
  return SS_OK;
}

int ss_attn_fwd(const ss_attn_desc* d, const void* Q, const void* K, const void* V, const void* bias,
                const int32_t* region_ids, const void* G, void* Y, float* lse, void* workspace,
                size_t workspace_bytes, void* hip_stream) {
  (void)workspace; (void)workspace_bytes;
  const int rc = validate(d);
  if (rc != SS_OK) return rc;
  if (!Q || !K || !V || !Y) return SS_ERR_NULL;
  if (d->bias_kind != SS_BIAS_NONE && !bias) return SS_ERR_NULL;
  if (d->mask_kind == SS_MASK_REGION && !region_ids) return SS_ERR_NULL;
  if (d->gated && !G) return SS_ERR_NULL;
  hipStream_t st = (hipStream_t)hip_stream;
  const bool bf16 = d->dtype == SS_BF16;
  KP p = base_params(d);
  p.Q = Q; p.K = K; p.V = V; p.G = G; p.Y = Y; p.bias = bias; p.region = region_ids;
  p.lse_out = lse; p.lse_sb = (int64_t)d->H * d->S; p.lse_sh = d->S;
  const Family fam = family_of(d);
  for (int c = 0; c < d->k; ++c) {
    set_chunk(p, d, c);
    if (fam == FAM_SMALL) SS_LAUNCH(SS_K_FWD, ssa::launch_small_fwd(p, st), "forward (short)");
    else if (fam == FAM_MFMA) SS_LAUNCH(SS_K_FWD, ssa::launch_mfma_fwd(p, false, st), "forward");
    else SS_LAUNCH(SS_K_FWD, ssa::launch_generic_fwd(p, bf16, false, st), "forward (generic)");
  }
  return SS_OK;
}

int ss_attn_bwd_static(const ss_attn_desc* d, const void* Q, const void* K, const void* V, const void* bias,
                       const int32_t* region_ids, const void* G, const void* dY, const float* lse, void* dQ,
                       void* dK, void* dV, float* dBias, void* dG, void* hip_stream) {
  const int rc = validate(d);
  if (rc != SS_OK) return rc;
  if (bwd_layout(d, family_of(d)).total > (size_t)SS_ATTN_STATIC_SCRATCH_BYTES) return SS_ERR_STATIC_SCRATCH;
  void* ptr = nullptr;
  const int rs = static_scratch(&ptr);
  if (rs != SS_OK) return rs;
  // nothing in the backward relies on scratch that starts at zero: every region is written by
  // the call before it is read, so the previous call's contents need no clearing
  return ss_attn_bwd(d, Q, K, V, bias, region_ids, G, dY, lse, dQ, dK, dV, dBias, dG, ptr,
                     (size_t)SS_ATTN_STATIC_SCRATCH_BYTES, hip_stream);
}

int ss_attn_bwd(const ss_attn_desc* d, const void* Q, const void* K, const void* V, const void* bias,
                const int32_t* region_ids, const void* G, const void* dY, const float* lse, void* dQ,
                void* dK, void* dV, float* dBias, void* dG, void* workspace, size_t workspace_bytes,
                void* hip_stream) {
  const int rc = validate(d);
  if (rc != SS_OK) return rc;
  if (!Q || !K || !V || !dY || !dQ || !dK || !dV) return SS_ERR_NULL;
  if (d->bias_kind != SS_BIAS_NONE && !bias) return SS_ERR_NULL;
  if (d->mask_kind == SS_MASK_REGION && !region_ids) return SS_ERR_NULL;
  if (d->gated && (!G || !dG)) return SS_ERR_NULL;
  const Family fam = family_of(d);
  const WsLayout w = bwd_layout(d, fam);
  if (!workspace || workspace_bytes < w.total || ((uintptr_t)workspace % ALIGN)) return SS_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  const bool bf16 = d->dtype == SS_BF16;
  char* ws = (char*)workspace;
  const bool want_dbias = d->bias_kind != SS_BIAS_NONE && dBias != nullptr;

  KP p = base_params(d);
  p.Q = Q; p.K = K; p.V = V; p.G = G; p.dY = dY; p.bias = bias; p.region = region_ids;
  p.dQ = dQ; p.dK = dK; p.dV = dV; p.dG = dG;
  const bool mfma = fam == FAM_MFMA;
  if (mfma && ssa::mfma_wants_bias_transpose(p)) {
    // the K-stationary kernels read bias[h][i][j] along i: give them a transposed copy, once per call
    const int h0 = d->shard_axis == SS_AXIS_HEAD ? d->lo : 0, h1 = d->shard_axis == SS_AXIS_HEAD ? d->hi : d->H;
    SS_LAUNCH(SS_K_TABLE_REDUCE, ssa::launch_bias_transpose(bias, ws + w.biasT, d->S, h0, h1, st), "bias transpose");
    p.biasT = ws + w.biasT;
  }
  float* dense = nullptr;
  if (want_dbias) {
    dense = d->bias_kind == SS_BIAS_DENSE ? dBias : (float*)(ws + w.dense);
    p.dbias_acc = dense;
  }
  // grouped bias-gradient sums: slot addressing for the chunk, and the fold of the slices that the
  // chunk just completed (ROW split: groups complete as the rows go by; HEAD split: a chunk walks
  // every row of its heads, so all of its groups complete at once)
  int slices_done = 0;
  auto set_groups = [&](KP& q) {
    q.sm_g0 = w.g0; q.sm_ring = w.ring; q.sm_hs = w.hs;
    q.sm_h0 = d->shard_axis == SS_AXIS_HEAD ? q.h0 : 0;
  };
  auto fold_groups = [&](const KP& q, int c) -> int {
    const int nslices = (w.ngroups + w.slice - 1) / w.slice;
    int s0, s1, hd0, nh;
    if (d->shard_axis == SS_AXIS_HEAD) {
      s0 = 0; s1 = nslices; hd0 = q.h0; nh = q.h1 - q.h0;
    } else {
      const int done = c == d->k - 1 ? nslices : (q.b1 / w.gw - w.g0) / w.slice;
      s0 = slices_done; s1 = done > slices_done ? done : slices_done; hd0 = 0; nh = d->H;
      slices_done = s1;
    }
    if (s1 <= s0) return SS_OK;
    SS_LAUNCH(SS_K_DBIAS_FOLD,
              ssa::launch_group_fold(q.sm_partial, dense, w.ring, w.hs, hd0, nh, d->S, w.slice, s0, s1, w.ngroups,
                                     s0 == 0, st),
              "bias gradient group fold");
    return SS_OK;
  };
  for (int c = 0; c < d->k; ++c) {
    set_chunk(p, d, c);
    const int64_t Bc = p.b1 - p.b0, Hc = p.h1 - p.h0;
    (void)Bc;
    // chunk-sized scratch holds the chunk's (row, head) pairs from its origin (b0, h0) on
    const int64_t st_sb = Hc * d->S, st_sh = d->S;
    p.delta = (float*)(ws + w.delta); p.dl_sb = st_sb; p.dl_sh = st_sh; p.dl_b0 = p.b0; p.dl_h0 = p.h0;
    if (lse) {
      p.lse = lse; p.lse_out = nullptr; p.lse_sb = (int64_t)d->H * d->S; p.lse_sh = d->S; p.lse_b0 = 0; p.lse_h0 = 0;
    } else {
      p.lse_out = (float*)(ws + w.lse); p.lse = p.lse_out; p.lse_sb = st_sb; p.lse_sh = st_sh;
      p.lse_b0 = p.b0; p.lse_h0 = p.h0;
    }
    if (d->gated) {
      p.do_sh = d->D; p.do_ss = Hc * d->D; p.do_sb = (int64_t)d->S * p.do_ss;
      p.dO_out = (void*)(ws + w.dO); p.dO = p.dO_out; p.do_b0 = p.b0; p.do_h0 = p.h0;
    } else {
      p.dO = dY; p.dO_out = nullptr; p.do_sb = p.sb; p.do_ss = p.ss; p.do_sh = p.sh; p.do_b0 = 0; p.do_h0 = 0;
    }
    // the first chunk that touches a bias-gradient entry starts its sum: for a HEAD split every
    // chunk owns its heads; for a ROW split chunk 0 starts and later chunks continue in row order
    p.dbias_accumulate = (d->shard_axis == SS_AXIS_ROW && c > 0) ? 1 : 0;
    if (fam == FAM_SMALL) {
      // one fused kernel per chunk; group partial sums of the bias gradient live in the workspace
      // across chunks and are reduced once the last chunk that touches them is enqueued
      p.sm_partial = want_dbias ? (float*)(ws + w.partial) : nullptr;
      set_groups(p);
      SS_LAUNCH(SS_K_DKDV, ssa::launch_small_bwd(p, st), "backward (short)");
      if (want_dbias) {
        const int rf = fold_groups(p, c);
        if (rf != SS_OK) return rf;
        if (d->bias_kind == SS_BIAS_RELPOS && (d->shard_axis == SS_AXIS_HEAD || c == d->k - 1)) {
          const int h0 = d->shard_axis == SS_AXIS_HEAD ? p.h0 : 0;
          const int h1 = d->shard_axis == SS_AXIS_HEAD ? p.h1 : d->H;
          SS_LAUNCH(SS_K_TABLE_REDUCE,
                    ssa::launch_relpos_reduce(dense, dBias, h0, h1, d->S, d->win_h, d->win_w, st),
                    "relative-position table reduce");
        }
      }
      continue;
    }
    if (mfma) {
      if (ssa::mfma_fuses_recompute_dq(p)) {
        SS_LAUNCH(SS_K_RECOMPUTE_DQ, ssa::launch_mfma_recompute_dq(p, st), "recompute + dQ");
        SS_LAUNCH(SS_K_DKDV, ssa::launch_mfma_dkdv(p, st), "dK/dV");
      } else {
        SS_LAUNCH(SS_K_RECOMPUTE, ssa::launch_mfma_fwd(p, true, st), "recompute");
        if (ssa::mfma_fuses_dq_dkdv(p)) {
          SS_LAUNCH(SS_K_DQ_DKDV, ssa::launch_mfma_dq_dkdv(p, st), "dQ + dK/dV");
        } else {
          SS_LAUNCH(SS_K_DQ, ssa::launch_mfma_dq(p, st), "dQ");
          SS_LAUNCH(SS_K_DKDV, ssa::launch_mfma_dkdv(p, st), "dK/dV");
        }
      }
      if (want_dbias) {
        if (w.gw > 0) {  // grouped sum: partials in the workspace, folded into the result as the groups complete
          p.sm_partial = (float*)(ws + w.partial);
          p.sm_gw = w.gw;
          set_groups(p);
        }
        SS_LAUNCH(SS_K_DBIAS, ssa::launch_mfma_dbias(p, st), "dBias");
        if (w.gw > 0) {
          const int rf = fold_groups(p, c);
          if (rf != SS_OK) return rf;
        }
      }
    } else {
      SS_LAUNCH(SS_K_RECOMPUTE, ssa::launch_generic_fwd(p, bf16, true, st), "recompute (generic)");
      SS_LAUNCH(SS_K_DQ, ssa::launch_generic_dq(p, bf16, st), "dQ (generic)");
      SS_LAUNCH(SS_K_DKDV, ssa::launch_generic_dkdv(p, bf16, st), "dK/dV (generic)");
      if (want_dbias) SS_LAUNCH(SS_K_DBIAS, ssa::launch_generic_dbias(p, bf16, st), "dBias (generic)");
    }
    if (want_dbias && d->bias_kind == SS_BIAS_RELPOS &&
        (d->shard_axis == SS_AXIS_HEAD || c == d->k - 1)) {
      const int h0 = d->shard_axis == SS_AXIS_HEAD ? p.h0 : 0;
      const int h1 = d->shard_axis == SS_AXIS_HEAD ? p.h1 : d->H;
      SS_LAUNCH(SS_K_TABLE_REDUCE, ssa::launch_relpos_reduce(dense, dBias, h0, h1, d->S, d->win_h, d->win_w, st),
                "relative-position table reduce");
    }
  }
  return SS_OK;
}

}  // extern "C"
