/* ss_plan.h -- C ABI of the host-side planner pieces.  No GPU work: every pointer is HOST memory,
 * nothing is allocated for the caller, nothing is kept between calls.
 *
 * Two pieces of the method that surround the co-sharded operators:
 *
 *  - schedule validation and completion (Section 3.2, "Scheduling validation and completion";
 *    the mask intersection is that of Section 3.3, "Dependency materialization"): data
 *    dependencies between operators are the non-empty intersections of the index masks of produced
 *    and consumed vTensors of the same pTensor; with the happen-before pairs of op-order they form
 *    the dependency graph; the schedule is feasible iff the graph is acyclic, where a consumer that
 *    may read any one of several replicated producers needs one acyclic choice only; a
 *    topological sort completes the order.
 *  - communication primitive search (Section 5, "RVD representation" and "Communication primitive
 *    search over RVD graph"): a tensor laid out over a device group as R(i)V(j)D(k1..kn); every
 *    collective is a transition between layouts, weighted with its time; Dijkstra's algorithm
 *    gives the cheapest chain from the producers' layout to the consumers'.  Same-group (intra-RVD)
 *    primitives only.
 *
 * Error codes are those of ss_attn.h.
 */
#ifndef SS_PLAN_H
#define SS_PLAN_H

#include <stdint.h>

#include "ss_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

#define SS_PLAN_MAX_DIMS 4

/* One vTensor: the operator that produces or consumes it, the pTensor it is a view of, and its mask:
 * a half-open index range [lo, hi) per dimension, 1 <= ndim <= SS_PLAN_MAX_DIMS. */
typedef struct {
  int32_t op, tensor, ndim;
  int64_t lo[SS_PLAN_MAX_DIMS], hi[SS_PLAN_MAX_DIMS];
} ss_vtensor;

/* Data dependencies: every (producer op, consumer op), producer != consumer, whose masks on the
 * same pTensor intersect; sorted ascending, no duplicates.  edges: room for `capacity` pairs
 * (2 * capacity int32).  *n_edges receives the number found; SS_ERR_WORKSPACE if it exceeds
 * capacity (nothing past capacity is written).  SS_ERR_BAD_SHAPE for an ndim out of range or a
 * range with lo > hi. */
int ss_plan_dependencies(const ss_vtensor* produced, int32_t n_produced, const ss_vtensor* consumed, int32_t n_consumed,
                         int32_t* edges, int32_t capacity, int32_t* n_edges);

/* Validation and completion.  Operators are 0 .. n_ops-1.  fixed_edges: n_fixed pairs (before,
 * after) that must all hold (data dependencies and happen-before pairs).  Alternatives: n_groups
 * groups; group i has alt_group_sizes[i] >= 1 candidate pairs, stored one group after the other in
 * alt_edges; exactly one pair of every group is taken.  Choices are tried in lexicographic order of
 * their indices (at most 1 << 20 combinations, else SS_ERR_UNSUPPORTED).
 * Outputs: *feasible 1/0; choice[n_groups] the first acyclic choice; order[n_ops] the topological
 * order that always takes the smallest ready operator.  choice and order are written only when
 * feasible.  SS_ERR_BAD_RANGE for an operator index outside 0 .. n_ops-1. */
int ss_plan_validate(int32_t n_ops, const int32_t* fixed_edges, int32_t n_fixed, const int32_t* alt_edges,
                     const int32_t* alt_group_sizes, int32_t n_groups, int32_t* feasible, int32_t* choice, int32_t* order);

/* Same-group collectives as layout transitions.  A layout is int32 state[2 + ndim] = {r, v, d1..dn}.
 *   all-reduce      V(v) -> R: (r g, v / g, d)            groups of g | v
 *   all-gather      D on `axis` -> R: (r g, v, d_axis / g)
 *   reduce-scatter  V -> D on `axis`: (r, v / g, d_axis g)
 *   all-to-all      D on `axis` -> D on `axis2`: (d_axis / g, d_axis2 g)
 *   schunk          R -> D on `axis`, a local slice: (r / g, v, d_axis g)
 *   vchunk          R -> V, local: (r / g, v g, d)
 * The text names the first four and schunk; vchunk is this library's reading of the sixth. */
typedef enum {
  SS_RVD_ALL_REDUCE = 0, SS_RVD_ALL_GATHER = 1, SS_RVD_REDUCE_SCATTER = 2, SS_RVD_ALL_TO_ALL = 3, SS_RVD_SCHUNK = 4,
  SS_RVD_VCHUNK = 5
} ss_rvd_primitive;

/* Edge weights, integer nanoseconds: with m = tensor_bytes / (d1 .. dn) of the layout before the
 * primitive (integer divisions, in that order), on a group whose members each have a link to every
 * other (xGMI): reduce-scatter and all-to-all alpha + (m / g) * 1000 / link_bytes_per_us,
 * all-gather alpha + m * 1000 / link_bytes_per_us, all-reduce alpha + 2 * ((m / g) * 1000 /
 * link_bytes_per_us), schunk and vchunk local_ns.  MI355X: 153000 bytes per microsecond and link. */
typedef struct {
  int64_t alpha_ns, link_bytes_per_us, local_ns;
} ss_link_model;

typedef struct {
  int32_t primitive, axis, axis2, group; /* axis / axis2 = -1 where they do not apply */
  int32_t state[2 + SS_PLAN_MAX_DIMS];   /* the layout after the step */
  int64_t time_ns;                       /* of this step */
} ss_rvd_step;

/* Cheapest chain of primitives from layout src to layout dst (ndim tensor axes each, the same
 * number of devices r v d1 .. dn on both sides, at most 4096 devices).  Among chains of equal time
 * the lexicographically smallest sequence of (primitive, axis, axis2, group) is returned.
 * steps: room for `capacity` steps; *n_steps and *total_ns receive the result (0 steps when
 * src == dst).  SS_ERR_BAD_SHAPE: a factor < 1, ndim out of range, different device counts;
 * SS_ERR_UNSUPPORTED: dst cannot be reached; SS_ERR_WORKSPACE: capacity too small. */
int ss_rvd_search(const int32_t* src, const int32_t* dst, int32_t ndim, int64_t tensor_bytes, const ss_link_model* model,
                  ss_rvd_step* steps, int32_t capacity, int32_t* n_steps, int64_t* total_ns);

#ifdef __cplusplus
}
#endif
#endif /* SS_PLAN_H */
