// C ABI of the co-sharded feed-forward operator: validation, chunk plan, workspace layout and the
// sequence of kernel launches per chunk (include/ss_ffn.h).
#include "../../include/ss_ffn.h"

#include <cstdio>
#include <mutex>

#include "ffn_kernels.h"

namespace {

constexpr int UNIT = 16;  // chunk boundaries fall on multiples of 16 hidden columns counted from lo

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

int validate(const ss_ffn_desc* d) {
  if (!d) return SS_ERR_NULL;
  if (d->T < 1 || d->dm < 8 || d->dh < 8 || (d->dm & 7) || (d->dh & 7)) return SS_ERR_BAD_SHAPE;
  if (d->ld_x < d->dm || d->ld_w1 < d->dh || d->ld_w2 < d->dm || (d->ld_x & 7) || (d->ld_w1 & 7) || (d->ld_w2 & 7))
    return SS_ERR_BAD_SHAPE;
  if (d->dtype != SS_BF16 || (d->act != SS_ACT_RELU && d->act != SS_ACT_GELU_TANH) ||
      (d->flags & ~(int32_t)SS_FFN_FLAG_EXACT_SUM))
    return SS_ERR_UNSUPPORTED;
  if (d->lo < 0 || d->lo >= d->hi || d->hi > d->dh || (d->lo & 7) || (d->hi & 7)) return SS_ERR_BAD_RANGE;
  const int units = (d->hi - d->lo + UNIT - 1) / UNIT;
  if (d->k < 1 || d->k > units) return SS_ERR_BAD_K;
  // 32-bit byte offsets inside one operand, also for the rows of a ragged tile that lie past the
  // end of the matrix (up to 255 of them): their offsets must not wrap back into the matrix
  if (d->ld_x >= (1 << 22) || d->ld_w1 >= (1 << 22) || d->ld_w2 >= (1 << 22)) return SS_ERR_UNSUPPORTED;
  const int64_t lim = (int64_t)1 << 31;
  if ((int64_t)d->T * d->ld_x * 2 >= lim || (int64_t)d->dm * d->ld_w1 * 2 >= lim || (int64_t)d->dh * d->ld_w2 * 2 >= lim)
    return SS_ERR_UNSUPPORTED;
  return SS_OK;
}

void chunk(const ss_ffn_desc* d, int c, int* a, int* b) {
  const int n = d->hi - d->lo, units = (n + UNIT - 1) / UNIT;
  const int64_t ua = (int64_t)c * units / d->k, ub = (int64_t)(c + 1) * units / d->k;
  *a = d->lo + (int)(ua * UNIT < n ? ua * UNIT : n);
  *b = d->lo + (int)(ub * UNIT < n ? ub * UNIT : n);
}

struct Ws {
  size_t H, D, acc, total;
  int64_t ldh;
};
Ws layout(const ss_ffn_desc* d, bool backward) {
  int wmax = 0;
  for (int c = 0; c < d->k; ++c) {
    int a, b;
    chunk(d, c, &a, &b);
    if (b - a > wmax) wmax = b - a;
  }
  Ws w;
  w.ldh = (wmax + 7) & ~7;
  const size_t hb = align256((size_t)d->T * w.ldh * 2);
  size_t off = 0;
  w.H = off; off += hb;
  w.D = off; if (backward) off += hb;
  // the fp32 partial sum between chunks exists only when the caller asks for sums that do not depend
  // on k bit for bit; otherwise the partial sum lives in the output tensor itself
  w.acc = off; if (d->k > 1 && (d->flags & SS_FFN_FLAG_EXACT_SUM)) off += align256(ssa::gemm_acc_bytes(d->T, d->dm));
  w.total = off;
  return w;
}

int hip_fail(hipError_t e, const char* what) {
  std::fprintf(stderr, "ss_ffn: %s: %s\n", what, hipGetErrorString(e));
  return SS_ERR_HIP;
}

bool g_on = false;
double g_ms[SS_FK_COUNT] = {0};
int64_t g_n[SS_FK_COUNT] = {0};
struct Pending { hipEvent_t a, b; int kind; };
Pending g_pending[4096];
int g_npending = 0;
struct Prof {
  hipStream_t st; int kind; bool on; hipEvent_t a, b;
  Prof(hipStream_t s, int k) : st(s), kind(k), on(g_on && g_npending < 4096) {
    if (on) { (void)hipEventCreate(&a); (void)hipEventCreate(&b); (void)hipEventRecord(a, st); }
  }
  ~Prof() {
    if (on) { (void)hipEventRecord(b, st); g_pending[g_npending++] = Pending{a, b, kind}; }
  }
};
void drain() {
  for (int i = 0; i < g_npending; ++i) {
    float ms = 0.f;
    (void)hipEventSynchronize(g_pending[i].b);
    (void)hipEventElapsedTime(&ms, g_pending[i].a, g_pending[i].b);
    g_ms[g_pending[i].kind] += ms;
    g_n[g_pending[i].kind] += 1;
    (void)hipEventDestroy(g_pending[i].a);
    (void)hipEventDestroy(g_pending[i].b);
  }
  g_npending = 0;
}

#define FF_LAUNCH_ON(stream_, kind, expr, what)      \
  do {                                               \
    hipError_t e_;                                   \
    {                                                \
      Prof ps_(stream_, kind);                       \
      e_ = (expr);                                   \
    }                                                \
    if (e_ != hipSuccess) {                          \
      FF_ON_ERROR;                                   \
      return hip_fail(e_, what);                     \
    }                                                \
  } while (0)
#define FF_ON_ERROR ((void)0)
#define FF_LAUNCH(kind, expr, what) FF_LAUNCH_ON(st, kind, expr, what)

// A helper stream per device (default priority, created on first use under a lock, kept until the
// process ends): dW2 = H^T dY needs only H, and the bias gradients only dY or dZ, so they are forked
// onto the helper stream, run beside the products of the caller's stream -- dZ = (dY W2^T) act'(Z)
// has too few tiles to fill the chip -- and are joined back before the next chunk overwrites H and
// dZ, and before the call returns.  The fork and join events belong to ONE call (created when it
// starts, released when it returns; the runtime keeps a released event alive until the work that
// waits on it has passed), so calls from several host threads or on several caller streams share
// nothing but the helper stream, on which each call's launches are ordered after its own fork.
std::mutex g_side_mu;
hipStream_t g_side_stream[64] = {nullptr};
int g_side_state[64] = {0};  // 0 not tried, 1 ready, -1 unavailable
hipStream_t side_stream() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(g_side_mu);
  if (g_side_state[dev] == 0) {
    g_side_state[dev] = hipStreamCreateWithFlags(&g_side_stream[dev], hipStreamNonBlocking) == hipSuccess ? 1 : -1;
    (void)hipGetLastError();
  }
  return g_side_state[dev] == 1 ? g_side_stream[dev] : nullptr;
}
// the fork / join events of one ss_ffn_bwd call
struct Side {
  hipStream_t s = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
  bool ok = false;
  explicit Side(bool want) {
    if (!want) return;
    s = side_stream();
    ok = s && hipEventCreateWithFlags(&fork, hipEventDisableTiming) == hipSuccess &&
         hipEventCreateWithFlags(&join, hipEventDisableTiming) == hipSuccess;
    if (!ok) (void)hipGetLastError();
  }
  ~Side() {
    if (fork) (void)hipEventDestroy(fork);
    if (join) (void)hipEventDestroy(join);
  }
};

ssa::GemmArgs gemm(const void* A, int64_t lda, const void* B, int64_t ldb, int M, int N, int K) {
  ssa::GemmArgs g{};
  g.A = (const uint16_t*)A; g.B = (const uint16_t*)B; g.lda = lda; g.ldb = ldb; g.M = M; g.N = N; g.K = K;
  return g;
}

}  // namespace

extern "C" {

int ss_ffn_workspace_bytes(const ss_ffn_desc* d, size_t* fwd_bytes, size_t* bwd_bytes) {
  const int rc = validate(d);
  if (rc != SS_OK) return rc;
  if (fwd_bytes) *fwd_bytes = layout(d, false).total;
  if (bwd_bytes) *bwd_bytes = layout(d, true).total;
  return SS_OK;
}

int ss_ffn_chunk_range(const ss_ffn_desc* d, int32_t c, int32_t* lo, int32_t* hi) {
  const int rc = validate(d);
  if (rc != SS_OK) return rc;
  if (c < 0 || c >= d->k) return SS_ERR_BAD_RANGE;
  int a, b;
  chunk(d, c, &a, &b);
  if (lo) *lo = a;
  if (hi) *hi = b;
  return SS_OK;
}

int ss_ffn_fwd(const ss_ffn_desc* d, const void* X, const void* W1, const void* b1, const void* W2, const void* b2,
               void* Y, void* workspace, size_t workspace_bytes, void* stream) {
  const int rc = validate(d);
  if (rc != SS_OK) return rc;
  if (!X || !W1 || !b1 || !W2 || !Y) return SS_ERR_NULL;
  const Ws w = layout(d, false);
  if (!workspace || workspace_bytes < w.total || ((uintptr_t)workspace & 255)) return SS_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  const uint16_t* W1p = (const uint16_t*)W1;
  const uint16_t* W2p = (const uint16_t*)W2;
  const bool exact = (d->flags & SS_FFN_FLAG_EXACT_SUM) != 0 || d->k == 1;
  for (int c = 0; c < d->k; ++c) {
    int a, b;
    chunk(d, c, &a, &b);
    const int nc = b - a;
    if (nc <= 0) continue;
    // H_c = act(X W1[:, a:b] + b1[a:b])
    ssa::GemmArgs up = gemm(X, d->ld_x, W1p + a, d->ld_w1, d->T, nc, d->dm);
    up.bias = (const uint16_t*)b1 + a; up.out = (uint16_t*)(ws + w.H); up.ldo = w.ldh; up.act = d->act;
    FF_LAUNCH(SS_FK_UP, ssa::launch_gemm(up, false, false, ssa::EPI_ACT, st), "H = act(X W1 + b1)");
    // Y += H_c W2[a:b, :]; the last chunk adds b2 and writes Y
    ssa::GemmArgs dn = gemm(ws + w.H, w.ldh, W2p + (int64_t)a * d->ld_w2, d->ld_w2, d->T, d->dm, nc);
    dn.acc32 = (float*)(ws + w.acc); dn.accumulate = c > 0; dn.last = c == d->k - 1;
    dn.bias = dn.last ? (const uint16_t*)b2 : nullptr; dn.out = (uint16_t*)Y; dn.ldo = d->ld_x;
    FF_LAUNCH(SS_FK_DOWN, ssa::launch_gemm(dn, false, false, exact ? ssa::EPI_ACC : ssa::EPI_ACC16, st), "Y += H W2");
  }
  return SS_OK;
}

int ss_ffn_bwd(const ss_ffn_desc* d, const void* X, const void* W1, const void* b1, const void* W2, const void* dY,
               void* dX, void* dW1, void* db1, void* dW2, void* db2, void* workspace, size_t workspace_bytes,
               void* stream) {
  const int rc = validate(d);
  if (rc != SS_OK) return rc;
  if (!X || !W1 || !b1 || !W2 || !dY || !dX || !dW1 || !db1 || !dW2) return SS_ERR_NULL;
  const Ws w = layout(d, true);
  if (!workspace || workspace_bytes < w.total || ((uintptr_t)workspace & 255)) return SS_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  const uint16_t* W1p = (const uint16_t*)W1;
  const uint16_t* W2p = (const uint16_t*)W2;
  uint16_t* Hc = (uint16_t*)(ws + w.H);
  uint16_t* Dc = (uint16_t*)(ws + w.D);
  const bool exact = (d->flags & SS_FFN_FLAG_EXACT_SUM) != 0 || d->k == 1;
  Side side_obj(!g_on);  // per-kernel timing wants the kernels one at a time
  Side* side = side_obj.ok ? &side_obj : nullptr;
  bool pending = false;  // work on the helper stream that the caller's stream has not waited for yet
  // run `launch` on the helper stream after everything enqueued on the caller's stream so far
  auto fork = [&]() {
    return side && hipEventRecord(side->fork, st) == hipSuccess && hipStreamWaitEvent(side->s, side->fork, 0) == hipSuccess;
  };
  auto join = [&]() {
    if (!pending) return hipSuccess;
    pending = false;
    const hipError_t e = hipEventRecord(side->join, side->s);
    return e != hipSuccess ? e : hipStreamWaitEvent(st, side->join, 0);
  };
  // a failed launch still leaves the caller's stream ordered after whatever runs on the helper stream
#undef FF_ON_ERROR
#define FF_ON_ERROR ((void)join())
  if (db2) {
    if (fork()) {
      pending = true;
      FF_LAUNCH_ON(side->s, SS_FK_COLSUM, ssa::launch_colsum(dY, d->ld_x, d->T, d->dm, db2, side->s), "db2");
    } else {
      FF_LAUNCH(SS_FK_COLSUM, ssa::launch_colsum(dY, d->ld_x, d->T, d->dm, db2, st), "db2");
    }
  }
  for (int c = 0; c < d->k; ++c) {
    int a, b;
    chunk(d, c, &a, &b);
    const int nc = b - a;
    if (nc <= 0) continue;
    // the helper stream still reads H and dZ of the previous chunk
    if (join() != hipSuccess) return hip_fail(hipGetLastError(), "join");
    // recompute: H_c = act(Z_c), D_c = act'(Z_c)
    ssa::GemmArgs up = gemm(X, d->ld_x, W1p + a, d->ld_w1, d->T, nc, d->dm);
    up.bias = (const uint16_t*)b1 + a; up.out = Hc; up.out2 = Dc; up.ldo = w.ldh; up.act = d->act;
    FF_LAUNCH(SS_FK_UP, ssa::launch_gemm(up, false, false, ssa::EPI_ACT, st), "recompute H, act'(Z)");
    // dW2[a:b, :] = H_c^T dY, beside the products that follow when the helper stream is there
    ssa::GemmArgs gw2 = gemm(Hc, w.ldh, dY, d->ld_x, nc, d->dm, d->T);
    gw2.out = (uint16_t*)dW2 + (int64_t)a * d->ld_w2; gw2.ldo = d->ld_w2;
    if (fork()) {
      pending = true;
      FF_LAUNCH_ON(side->s, SS_FK_DW2, ssa::launch_gemm(gw2, true, false, ssa::EPI_STORE, side->s), "dW2 = H^T dY");
    } else {
      FF_LAUNCH(SS_FK_DW2, ssa::launch_gemm(gw2, true, false, ssa::EPI_STORE, st), "dW2 = H^T dY");
    }
    // dZ_c = (dY W2[a:b,:]^T) * D_c, in place over D_c
    ssa::GemmArgs dh = gemm(dY, d->ld_x, W2p + (int64_t)a * d->ld_w2, d->ld_w2, d->T, nc, d->dm);
    dh.mul = Dc; dh.ldm = w.ldh; dh.out = Dc; dh.ldo = w.ldh;
    FF_LAUNCH(SS_FK_DH, ssa::launch_gemm(dh, false, true, ssa::EPI_MUL, st), "dZ = (dY W2^T) act'(Z)");
    // db1[a:b] = column sums of dZ_c
    if (fork()) {
      pending = true;
      FF_LAUNCH_ON(side->s, SS_FK_COLSUM, ssa::launch_colsum(Dc, w.ldh, d->T, nc, (uint16_t*)db1 + a, side->s), "db1");
    } else {
      FF_LAUNCH(SS_FK_COLSUM, ssa::launch_colsum(Dc, w.ldh, d->T, nc, (uint16_t*)db1 + a, st), "db1");
    }
    // dW1[:, a:b] = X^T dZ_c
    ssa::GemmArgs gw1 = gemm(X, d->ld_x, Dc, w.ldh, d->dm, nc, d->T);
    gw1.out = (uint16_t*)dW1 + a; gw1.ldo = d->ld_w1;
    FF_LAUNCH(SS_FK_DW1, ssa::launch_gemm(gw1, true, false, ssa::EPI_STORE, st), "dW1 = X^T dZ");
    // dX += dZ_c W1[:, a:b]^T; the last chunk writes dX
    ssa::GemmArgs gx = gemm(Dc, w.ldh, W1p + a, d->ld_w1, d->T, d->dm, nc);
    gx.acc32 = (float*)(ws + w.acc); gx.accumulate = c > 0; gx.last = c == d->k - 1;
    gx.out = (uint16_t*)dX; gx.ldo = d->ld_x;
    FF_LAUNCH(SS_FK_DX, ssa::launch_gemm(gx, false, true, exact ? ssa::EPI_ACC : ssa::EPI_ACC16, st), "dX += dZ W1^T");
  }
  if (join() != hipSuccess) return hip_fail(hipGetLastError(), "join");
  return SS_OK;
#undef FF_ON_ERROR
#define FF_ON_ERROR ((void)0)
}

int ss_ffn_profile_enable(int on) {
  if (!on) drain();
  g_on = on != 0;
  return SS_OK;
}

int ss_ffn_profile_read(int kernel, double* total_ms, int64_t* launches) {
  if (kernel < 0 || kernel >= SS_FK_COUNT) return SS_ERR_BAD_RANGE;
  drain();
  if (total_ms) *total_ms = g_ms[kernel];
  if (launches) *launches = g_n[kernel];
  g_ms[kernel] = 0;
  g_n[kernel] = 0;
  return SS_OK;
}

}  // extern "C"
