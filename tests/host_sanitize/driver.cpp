// Host-only driver for an AddressSanitizer + UndefinedBehaviorSanitizer build of the library's host
// code (descriptor validation, chunk plan, workspace layout, the planner): calls every entry point
// that runs without a GPU on seeded random and boundary inputs.  The kernel launchers that the
// scheduler would call are stubbed out below: no call in this driver gets past validation.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ss_attn.h"
#include "ss_ffn.h"
#include "ss_plan.h"
#include "../../paper_2301_08984_amd/csrc/kparams.h"
#include "../../paper_2301_08984_amd/csrc/ffn_kernels.h"

namespace ssa {
// stubs: host-side shape predicates answer as for an unsupported shape, launchers must never run
#define SS_STUB_LAUNCH(name, ...) \
  hipError_t name(__VA_ARGS__) { std::fprintf(stderr, "unexpected launch: " #name "\n"); std::abort(); }
SS_STUB_LAUNCH(launch_generic_fwd, const KP&, bool, bool, hipStream_t)
SS_STUB_LAUNCH(launch_generic_dq, const KP&, bool, hipStream_t)
SS_STUB_LAUNCH(launch_generic_dkdv, const KP&, bool, hipStream_t)
SS_STUB_LAUNCH(launch_generic_dbias, const KP&, bool, hipStream_t)
SS_STUB_LAUNCH(launch_relpos_reduce, const float*, float*, int, int, int, int, int, hipStream_t)
SS_STUB_LAUNCH(launch_fill_zero, float*, size_t, hipStream_t)
SS_STUB_LAUNCH(launch_small_fwd, const KP&, hipStream_t)
SS_STUB_LAUNCH(launch_small_bwd, const KP&, hipStream_t)
SS_STUB_LAUNCH(launch_group_fold, float*, float*, int, int, int, int, int, int, int, int, int, bool, hipStream_t)
SS_STUB_LAUNCH(launch_mfma_fwd, const KP&, bool, hipStream_t)
SS_STUB_LAUNCH(launch_mfma_dq, const KP&, hipStream_t)
SS_STUB_LAUNCH(launch_mfma_dkdv, const KP&, hipStream_t)
SS_STUB_LAUNCH(launch_mfma_dbias, const KP&, hipStream_t)
SS_STUB_LAUNCH(launch_mfma_dq_dkdv, const KP&, hipStream_t)
SS_STUB_LAUNCH(launch_mfma_recompute_dq, const KP&, hipStream_t)
SS_STUB_LAUNCH(launch_bias_transpose, const void*, void*, int, int, int, hipStream_t)
SS_STUB_LAUNCH(launch_gemm, const GemmArgs&, bool, bool, int, hipStream_t)
SS_STUB_LAUNCH(launch_colsum, const void*, int64_t, int, int, void*, hipStream_t)
bool small_supported(const KP& p, bool bf16) { return bf16 && p.D == 32 && p.S <= 64 && !p.gated; }
bool mfma_supported(const KP& p, bool bf16) { return bf16 && (p.D == 32 || p.D == 64 || p.D == 128); }
bool mfma_fuses_dq_dkdv(const KP&) { return false; }
bool mfma_fuses_recompute_dq(const KP&) { return false; }
bool mfma_wants_bias_transpose(const KP& p) { return p.bias_kind == 1 && p.bias_bf16; }
int mfma_dbias_group_rows(const KP& p) { return p.bias_kind == 1 ? 64 : 0; }
size_t gemm_acc_bytes(int M, int N) { return (size_t)((M + 255) / 256) * ((N + 255) / 256) * 256 * 256 * sizeof(float); }
}  // namespace ssa

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static uint64_t rnd() {
  rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
  return rng_state;
}
static int pick(int lo, int hi) { return lo + (int)(rnd() % (uint64_t)(hi - lo + 1)); }

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main() {
  // attention descriptors: boundary values and seeded random fields, valid and invalid alike
  long ok = 0, bad = 0;
  for (int it = 0; it < 20000; ++it) {
    ss_attn_desc d;
    std::memset(&d, 0, sizeof d);
    d.B = pick(-1, 70); d.H = pick(0, 20); d.S = pick(0, 300); d.D = 8 * pick(0, 34);
    if (it % 7 == 0) d.D = pick(0, 300);
    d.dtype = pick(-1, 2); d.scale = 0.125f;
    d.stride_h = d.D + 8 * pick(-1, 2); d.stride_s = (int64_t)d.H * d.stride_h; d.stride_b = (int64_t)d.S * d.stride_s;
    if (it % 11 == 0) d.stride_b = pick(0, 64);
    d.bias_kind = pick(-1, 3); d.bias_dtype = pick(0, 1);
    d.win_h = pick(0, 17); d.win_w = d.win_h > 0 && it % 3 ? d.S / (d.win_h) : pick(0, 17);
    d.mask_kind = pick(-1, 3); d.mask_period = pick(0, 300); d.gated = pick(0, 1);
    d.shard_axis = pick(0, 1);
    const int ext = d.shard_axis == SS_AXIS_HEAD ? d.H : d.B;
    d.lo = pick(-1, ext > 0 ? ext : 1); d.hi = pick(0, ext + 1); d.k = pick(0, 9);
    d.flags = it % 13 == 0 ? (uint32_t)rnd() : (uint32_t)pick(0, 1);
    size_t f = 0, b = 0;
    const int rc = ss_attn_workspace_bytes(&d, &f, &b);
    if (rc == SS_OK) {
      ++ok;
      CHECK(b % 256 == 0);
      CHECK(ss_attn_kernel_family(&d) != nullptr);
      int prev = d.lo;
      for (int c = 0; c < d.k; ++c) {
        int32_t a = 0, e = 0;
        CHECK(ss_attn_chunk_range(&d, c, &a, &e) == SS_OK);
        CHECK(a == prev && e > a);
        prev = e;
      }
      CHECK(prev == d.hi);
      int32_t a, e;
      CHECK(ss_attn_chunk_range(&d, d.k, &a, &e) == SS_ERR_BAD_K);
      // every entry point rejects missing pointers / workspace before it would launch anything
      CHECK(ss_attn_fwd(&d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == SS_ERR_NULL);
      char* one = (char*)256;
      CHECK(ss_attn_bwd(&d, one, one, one, one, (const int32_t*)one, one, one, nullptr, one, one, one, nullptr, one, nullptr, 0, nullptr) == SS_ERR_WORKSPACE);
    } else {
      ++bad;
      CHECK(rc < 0 && rc >= SS_ERR_STATIC_SCRATCH);
      CHECK(ss_attn_kernel_family(&d) == nullptr);
      CHECK(std::strlen(ss_strerror(rc)) > 0);
    }
  }
  CHECK(ok > 100 && bad > 100);
  CHECK(ss_attn_workspace_bytes(nullptr, nullptr, nullptr) == SS_ERR_NULL);

  // feed-forward descriptors
  ok = bad = 0;
  for (int it = 0; it < 20000; ++it) {
    ss_ffn_desc d;
    std::memset(&d, 0, sizeof d);
    d.T = pick(0, 3000); d.dm = 8 * pick(0, 200) + (it % 17 == 0); d.dh = 8 * pick(0, 400);
    d.dtype = it % 19 == 0 ? SS_F32 : SS_BF16; d.act = pick(0, 1 + (it % 23 == 0));
    d.ld_x = d.dm + 8 * pick(0, 2) - (it % 29 == 0); d.ld_w1 = d.dh + 8 * pick(0, 2); d.ld_w2 = d.dm + 8 * pick(0, 2);
    d.lo = 8 * pick(0, 20); d.hi = 8 * pick(0, 400); d.k = pick(0, 12); d.flags = pick(0, 1) + 2 * (it % 31 == 0);
    size_t f = 0, b = 0;
    const int rc = ss_ffn_workspace_bytes(&d, &f, &b);
    if (rc == SS_OK) {
      ++ok;
      CHECK(f % 256 == 0 && b % 256 == 0 && b >= f);
      int prev = d.lo;
      for (int c = 0; c < d.k; ++c) {
        int32_t a = 0, e = 0;
        CHECK(ss_ffn_chunk_range(&d, c, &a, &e) == SS_OK);
        CHECK(a == prev && e >= a && (a - d.lo) % 16 == 0);
        prev = e;
      }
      CHECK(prev == d.hi);
      CHECK(ss_ffn_fwd(&d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == SS_ERR_NULL);
      char* one = (char*)256;
      CHECK(ss_ffn_bwd(&d, one, one, one, one, one, one, one, one, one, one, nullptr, 0, nullptr) == SS_ERR_WORKSPACE);
    } else {
      ++bad;
      CHECK(rc < 0);
    }
  }
  CHECK(ok > 100 && bad > 100);

  // planner: dependencies, validation, layout search on random inputs, tight and short output buffers
  for (int it = 0; it < 300; ++it) {
    const int np = pick(0, 12), nc = pick(0, 12);
    std::vector<ss_vtensor> P(np), C(nc);
    auto fill = [&](ss_vtensor& v) {
      v.op = pick(0, 9); v.tensor = pick(0, 3); v.ndim = pick(it % 37 == 0 ? 0 : 1, it % 41 == 0 ? 5 : SS_PLAN_MAX_DIMS);
      for (int a = 0; a < SS_PLAN_MAX_DIMS; ++a) { v.lo[a] = pick(0, 8); v.hi[a] = v.lo[a] + pick(it % 43 == 0 ? -1 : 0, 8); }
    };
    for (auto& v : P) fill(v);
    for (auto& v : C) fill(v);
    const int cap = pick(0, np * nc + 1);
    std::vector<int32_t> edges(2 * (size_t)cap + 2, -7);
    int32_t n = -1;
    const int rc = ss_plan_dependencies(P.data(), np, C.data(), nc, edges.data(), cap, &n);
    CHECK(rc == SS_OK || rc == SS_ERR_WORKSPACE || rc == SS_ERR_BAD_SHAPE);
    CHECK(edges[2 * (size_t)cap] == -7 && edges[2 * (size_t)cap + 1] == -7);
    const int n_ops = pick(1, 10), n_fixed = pick(0, 14), n_groups = pick(0, 4);
    std::vector<int32_t> fixed(2 * (size_t)n_fixed + 1), sizes(n_groups + 1), alts;
    for (int i = 0; i < 2 * n_fixed; ++i) fixed[i] = pick(it % 47 == 0 ? -1 : 0, n_ops - (it % 53 == 0 ? 0 : 1));
    for (int g = 0; g < n_groups; ++g) {
      sizes[g] = pick(1, 3);
      for (int e = 0; e < 2 * sizes[g]; ++e) alts.push_back(pick(0, n_ops - 1));
    }
    alts.push_back(0);
    int32_t feasible = -1;
    std::vector<int32_t> choice(n_groups + 1, -7), order(n_ops + 1, -7);
    const int rv = ss_plan_validate(n_ops, fixed.data(), n_fixed, alts.data(), sizes.data(), n_groups, &feasible, choice.data(), order.data());
    CHECK(rv == SS_OK || rv == SS_ERR_BAD_RANGE);
    CHECK(choice[n_groups] == -7 && order[n_ops] == -7);
    if (rv == SS_OK && feasible) {
      std::vector<int> seen(n_ops, 0);
      for (int i = 0; i < n_ops; ++i) { CHECK(order[i] >= 0 && order[i] < n_ops && !seen[order[i]]); seen[order[i]] = 1; }
    }
  }
  {
    const int facs[] = {1, 2, 4, 8};
    const ss_link_model model = {2000, 153000, 500};
    for (int it = 0; it < 200; ++it) {
      const int ndim = pick(1, 2);
      int32_t src[2 + SS_PLAN_MAX_DIMS] = {0}, dst[2 + SS_PLAN_MAX_DIMS] = {0};
      for (int i = 0; i < 2 + ndim; ++i) { src[i] = facs[pick(0, 2)]; dst[i] = facs[pick(0, 2)]; }
      const int cap = pick(0, 8);
      std::vector<ss_rvd_step> steps((size_t)cap + 1);
      std::memset(steps.data(), 0x5a, steps.size() * sizeof(ss_rvd_step));
      int32_t n = -1; int64_t total = -1;
      const int rc = ss_rvd_search(src, dst, ndim, 1 << 24, &model, steps.data(), cap, &n, &total);
      CHECK(rc == SS_OK || rc == SS_ERR_BAD_SHAPE || rc == SS_ERR_UNSUPPORTED || rc == SS_ERR_WORKSPACE);
      CHECK(steps[cap].primitive == 0x5a5a5a5a);
      if (rc == SS_OK) CHECK(n >= 0 && n <= cap && total >= 0);
    }
  }
  std::printf("host sanitizer driver: all checks passed\n");
  return 0;
}
