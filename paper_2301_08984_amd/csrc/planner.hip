// Host-side planner pieces: dependency extraction, schedule validation and completion, and the
// shortest chain of collectives between two RVD layouts.  Plain C++, no device code.
#include "../../include/ss_plan.h"

#include <algorithm>
#include <array>
#include <functional>
#include <map>
#include <queue>
#include <set>
#include <utility>
#include <vector>

namespace {

using Edge = std::pair<int32_t, int32_t>;

bool masks_overlap(const ss_vtensor& a, const ss_vtensor& b) {
  if (a.tensor != b.tensor || a.ndim != b.ndim) return false;
  for (int d = 0; d < a.ndim; ++d)
    if (std::max(a.lo[d], b.lo[d]) >= std::min(a.hi[d], b.hi[d])) return false;
  return true;
}

bool well_formed(const ss_vtensor& t) {
  if (t.ndim < 1 || t.ndim > SS_PLAN_MAX_DIMS) return false;
  for (int d = 0; d < t.ndim; ++d)
    if (t.lo[d] > t.hi[d]) return false;
  return true;
}

// Kahn's algorithm with a min-heap of ready operators; false if a cycle is left over
bool smallest_first_order(int n, const std::vector<Edge>& edges, std::vector<int32_t>* order) {
  std::vector<Edge> e(edges);
  std::sort(e.begin(), e.end());
  e.erase(std::unique(e.begin(), e.end()), e.end());
  std::vector<std::vector<int32_t>> out(n);
  std::vector<int32_t> indeg(n, 0);
  for (const Edge& x : e) {
    out[x.first].push_back(x.second);
    ++indeg[x.second];
  }
  std::priority_queue<int32_t, std::vector<int32_t>, std::greater<int32_t>> ready;
  for (int u = 0; u < n; ++u)
    if (indeg[u] == 0) ready.push(u);
  order->clear();
  while (!ready.empty()) {
    const int32_t u = ready.top();
    ready.pop();
    order->push_back(u);
    for (int32_t v : out[u])
      if (--indeg[v] == 0) ready.push(v);
  }
  return (int)order->size() == n;
}

// ---- RVD
using State = std::array<int32_t, 2 + SS_PLAN_MAX_DIMS>;  // unused axes hold 1
struct Move {
  int32_t prim, axis, axis2, g;
  State next;
};
using Key = std::array<int32_t, 4>;

void for_each_divisor(int32_t x, const std::function<void(int32_t)>& f) {
  for (int32_t g = 2; g <= x; ++g)
    if (x % g == 0) f(g);
}

std::vector<Move> moves_from(const State& s, int ndim) {
  std::vector<Move> m;
  for_each_divisor(s[1], [&](int32_t g) {
    State n = s;
    n[0] *= g; n[1] /= g;
    m.push_back({SS_RVD_ALL_REDUCE, -1, -1, g, n});
    for (int a = 0; a < ndim; ++a) {
      State t = s;
      t[1] /= g; t[2 + a] *= g;
      m.push_back({SS_RVD_REDUCE_SCATTER, a, -1, g, t});
    }
  });
  for (int a = 0; a < ndim; ++a)
    for_each_divisor(s[2 + a], [&](int32_t g) {
      State n = s;
      n[0] *= g; n[2 + a] /= g;
      m.push_back({SS_RVD_ALL_GATHER, a, -1, g, n});
      for (int b = 0; b < ndim; ++b) {
        if (b == a) continue;
        State t = s;
        t[2 + a] /= g; t[2 + b] *= g;
        m.push_back({SS_RVD_ALL_TO_ALL, a, b, g, t});
      }
    });
  for_each_divisor(s[0], [&](int32_t g) {
    State n = s;
    n[0] /= g; n[1] *= g;
    m.push_back({SS_RVD_VCHUNK, -1, -1, g, n});
    for (int a = 0; a < ndim; ++a) {
      State t = s;
      t[0] /= g; t[2 + a] *= g;
      m.push_back({SS_RVD_SCHUNK, a, -1, g, t});
    }
  });
  return m;
}

int64_t move_time(const Move& mv, const State& from, int ndim, int64_t tensor_bytes, const ss_link_model& lm) {
  if (mv.prim == SS_RVD_SCHUNK || mv.prim == SS_RVD_VCHUNK) return lm.local_ns;
  int64_t m = tensor_bytes;
  for (int a = 0; a < ndim; ++a) m /= from[2 + a];
  if (mv.prim == SS_RVD_ALL_GATHER) return lm.alpha_ns + m * 1000 / lm.link_bytes_per_us;
  const int64_t piece = (m / mv.g) * 1000 / lm.link_bytes_per_us;
  return lm.alpha_ns + (mv.prim == SS_RVD_ALL_REDUCE ? 2 * piece : piece);
}

}  // namespace

extern "C" {

int ss_plan_dependencies(const ss_vtensor* produced, int32_t n_produced, const ss_vtensor* consumed, int32_t n_consumed,
                         int32_t* edges, int32_t capacity, int32_t* n_edges) {
  if (!n_edges || (n_produced > 0 && !produced) || (n_consumed > 0 && !consumed) || (capacity > 0 && !edges)) return SS_ERR_NULL;
  if (n_produced < 0 || n_consumed < 0 || capacity < 0) return SS_ERR_BAD_SHAPE;
  for (int i = 0; i < n_produced; ++i)
    if (!well_formed(produced[i])) return SS_ERR_BAD_SHAPE;
  for (int i = 0; i < n_consumed; ++i)
    if (!well_formed(consumed[i])) return SS_ERR_BAD_SHAPE;
  std::set<Edge> found;
  for (int i = 0; i < n_produced; ++i)
    for (int j = 0; j < n_consumed; ++j)
      if (produced[i].op != consumed[j].op && masks_overlap(produced[i], consumed[j])) found.insert({produced[i].op, consumed[j].op});
  *n_edges = (int32_t)found.size();
  int k = 0;
  for (const Edge& e : found) {
    if (k >= capacity) break;
    edges[2 * k] = e.first;
    edges[2 * k + 1] = e.second;
    ++k;
  }
  return (int)found.size() > capacity ? SS_ERR_WORKSPACE : SS_OK;
}

int ss_plan_validate(int32_t n_ops, const int32_t* fixed_edges, int32_t n_fixed, const int32_t* alt_edges,
                     const int32_t* alt_group_sizes, int32_t n_groups, int32_t* feasible, int32_t* choice, int32_t* order) {
  if (!feasible || (n_fixed > 0 && !fixed_edges) || (n_groups > 0 && (!alt_edges || !alt_group_sizes || !choice)) ||
      (n_ops > 0 && !order))
    return SS_ERR_NULL;
  if (n_ops < 0 || n_fixed < 0 || n_groups < 0) return SS_ERR_BAD_SHAPE;
  auto inside = [&](int32_t op) { return op >= 0 && op < n_ops; };
  std::vector<Edge> fixed;
  for (int i = 0; i < n_fixed; ++i) {
    if (!inside(fixed_edges[2 * i]) || !inside(fixed_edges[2 * i + 1])) return SS_ERR_BAD_RANGE;
    fixed.push_back({fixed_edges[2 * i], fixed_edges[2 * i + 1]});
  }
  std::vector<std::vector<Edge>> groups(n_groups);
  int64_t combos = 1;
  int at = 0;
  for (int gidx = 0; gidx < n_groups; ++gidx) {
    if (alt_group_sizes[gidx] < 1) return SS_ERR_BAD_SHAPE;
    for (int i = 0; i < alt_group_sizes[gidx]; ++i, ++at) {
      if (!inside(alt_edges[2 * at]) || !inside(alt_edges[2 * at + 1])) return SS_ERR_BAD_RANGE;
      groups[gidx].push_back({alt_edges[2 * at], alt_edges[2 * at + 1]});
    }
    combos *= alt_group_sizes[gidx];
    if (combos > (1 << 20)) return SS_ERR_UNSUPPORTED;
  }
  // choices in lexicographic order: the last group's index runs fastest
  std::vector<int32_t> pick(n_groups, 0), ord;
  for (int64_t c = 0; c < combos; ++c) {
    std::vector<Edge> edges(fixed);
    for (int gidx = 0; gidx < n_groups; ++gidx) edges.push_back(groups[gidx][pick[gidx]]);
    if (smallest_first_order(n_ops, edges, &ord)) {
      *feasible = 1;
      for (int gidx = 0; gidx < n_groups; ++gidx) choice[gidx] = pick[gidx];
      for (int i = 0; i < n_ops; ++i) order[i] = ord[i];
      return SS_OK;
    }
    for (int gidx = n_groups - 1; gidx >= 0; --gidx) {
      if (++pick[gidx] < alt_group_sizes[gidx]) break;
      pick[gidx] = 0;
    }
  }
  *feasible = 0;
  return SS_OK;
}

int ss_rvd_search(const int32_t* src, const int32_t* dst, int32_t ndim, int64_t tensor_bytes, const ss_link_model* model,
                  ss_rvd_step* steps, int32_t capacity, int32_t* n_steps, int64_t* total_ns) {
  if (!src || !dst || !model || !n_steps || !total_ns || (capacity > 0 && !steps)) return SS_ERR_NULL;
  if (ndim < 1 || ndim > SS_PLAN_MAX_DIMS || capacity < 0 || tensor_bytes < 0 || model->link_bytes_per_us < 1)
    return SS_ERR_BAD_SHAPE;
  State s0, s1;
  s0.fill(1);
  s1.fill(1);
  int64_t n0 = 1, n1 = 1;
  for (int i = 0; i < 2 + ndim; ++i) {
    if (src[i] < 1 || dst[i] < 1) return SS_ERR_BAD_SHAPE;
    s0[i] = src[i];
    s1[i] = dst[i];
    n0 *= src[i];
    n1 *= dst[i];
    if (n0 > 4096 || n1 > 4096) return SS_ERR_BAD_SHAPE;
  }
  if (n0 != n1) return SS_ERR_BAD_SHAPE;

  // Dijkstra over (time, sequence of move keys): the sequence makes the result unique among ties
  struct Label {
    int64_t t;
    std::vector<Key> path;
    bool operator<(const Label& o) const { return t != o.t ? t < o.t : path < o.path; }
  };
  std::map<State, Label> best;
  auto cmp = [](const std::pair<Label, State>& a, const std::pair<Label, State>& b) {
    return b.first < a.first || (!(a.first < b.first) && b.second < a.second);
  };
  std::priority_queue<std::pair<Label, State>, std::vector<std::pair<Label, State>>, decltype(cmp)> heap(cmp);
  best[s0] = Label{0, {}};
  heap.push({best[s0], s0});
  while (!heap.empty()) {
    const std::pair<Label, State> top = heap.top();
    heap.pop();
    const Label& cur = best[top.second];
    if (cur < top.first || top.first < cur) continue;  // stale entry
    if (top.second == s1) {
      *n_steps = (int32_t)top.first.path.size();
      *total_ns = top.first.t;
      if (*n_steps > capacity) return SS_ERR_WORKSPACE;
      State at = s0;
      for (int i = 0; i < *n_steps; ++i) {
        const Key& k = top.first.path[i];
        for (const Move& mv : moves_from(at, ndim))
          if (mv.prim == k[0] && mv.axis == k[1] && mv.axis2 == k[2] && mv.g == k[3]) {
            steps[i].primitive = mv.prim; steps[i].axis = mv.axis; steps[i].axis2 = mv.axis2; steps[i].group = mv.g;
            steps[i].time_ns = move_time(mv, at, ndim, tensor_bytes, *model);
            for (int j = 0; j < 2 + SS_PLAN_MAX_DIMS; ++j) steps[i].state[j] = mv.next[j];
            at = mv.next;
            break;
          }
      }
      return SS_OK;
    }
    for (const Move& mv : moves_from(top.second, ndim)) {
      Label nl{top.first.t + move_time(mv, top.second, ndim, tensor_bytes, *model), top.first.path};
      nl.path.push_back(Key{mv.prim, mv.axis, mv.axis2, mv.g});
      auto it = best.find(mv.next);
      if (it == best.end() || nl < it->second) {
        best[mv.next] = nl;
        heap.push({nl, mv.next});
      }
    }
  }
  return SS_ERR_UNSUPPORTED;
}

}  // extern "C"
