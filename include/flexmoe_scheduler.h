/*
 * flexmoe_scheduler.h -- C ABI of the host-side placement scheduler of FlexMoE (arXiv 2304.03946):
 * balance ratio (Section 3.3, Eq. 6), Policy Maker (Section 3.4, Alg. 2, with the cost of Eq. 5
 * built from Eq. 7 and optionally Eq. 9), Scheduler (Section 3.3, Alg. 1 with the Expand, Shrink
 * and Migrate primitives), and the export of a placement as the table flexmoe_route consumes.
 *
 * Everything here is plain host arithmetic on HOST pointers owned by the caller: no device is
 * touched, nothing is allocated beyond the call's own temporaries, and every decision is taken
 * in integers, so results are reproducible bit for bit.
 *
 * Cluster model (Section 3.2): G GPUs with S vExpert slots each; slot s = g*S + i lives on GPU
 * g.  A placement is slot_owner[G*S]: the expert a slot replicates, or FLEXMOE_SLOT_FREE.  Every
 * expert owns at least one slot.  The tokens[e] = I_e tokens of an expert are partitioned evenly
 * over its vExperts: floor(I_e/n_e) each, one more for the first I_e mod n_e in ascending slot
 * id -- the shares flexmoe_route hands out for the exported table.
 *
 * Cost of a training step (Eq. 5): max over GPUs of the sum over the experts placed there of
 *   T_C    = (tokens of the expert computed on that GPU) * token_cost      (Eq. 7, token_cost = 1/TPS)
 *   T_Sync = sync_cost[m], m = number of GPUs that hold the expert          (Eq. 9; 0 when sync_cost is NULL)
 * in the caller's integer time unit.  The All-to-All term (Eq. 8) is not modelled.
 *
 * Choices the paper leaves open:
 *   - Alg. 2 expands the expert with the largest capacity I_e/n_e and shrinks the one with the
 *     smallest capacity among those that own two or more vExperts (ties: lowest expert id; fractions
 *     are compared exactly).  No such expert, or the same expert: empty plan.
 *   - Every vExpert of the shrunk expert is tried as the one to release; the new vExpert goes into
 *     the released slot or into the lowest free slot of any GPU; the pair with the smallest
 *     estimated cost wins, the first in (released, target) order among equals; it is returned only
 *     if that cost is below the current one.
 *   - Migrate exchanges the owners of two slots so that an expert leaves a GPU where it holds one
 *     vExpert for a GPU where it already has one; at most one exchange per flexmoe_schedule call,
 *     the one with the smallest estimated cost, and only if that is below the current cost.
 *   - A cluster without tokens has balance ratio 1.
 *
 * Return value: a flexmoe_status code (flexmoe.h).  FLEXMOE_INVALID_ARG for null pointers, sizes
 * out of range (1 <= E <= FLEXMOE_MAX_EXPERTS, 1 <= G, 1 <= S, G*S <= FLEXMOE_MAX_SLOTS), negative
 * tokens or costs, or a cost that could overflow 62 bits; FLEXMOE_BAD_PLACEMENT for an owner
 * outside [-1, E) or an expert without a slot.  On an error nothing is written.
 */
#ifndef FLEXMOE_SCHEDULER_H
#define FLEXMOE_SCHEDULER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FLEXMOE_SLOT_FREE (-1)
#define FLEXMOE_MAX_SLOTS 65536

enum flexmoe_primitive { FLEXMOE_EXPAND = 0, FLEXMOE_SHRINK = 1, FLEXMOE_MIGRATE = 2 };

/*
 * Eq. 6: the largest per-GPU token load under the placement divided by the mean per-GPU load.
 *   tokens [E], slot_owner [G*S] -> *ratio;  gpu_load [G] (tokens each GPU computes) or NULL.
 */
int flexmoe_balance_ratio(const int64_t* tokens, const int32_t* slot_owner, int E, int G, int S,
                          double* ratio, int64_t* gpu_load);

/* Eq. 5 for the placement: *cost in the unit of token_cost / sync_cost [G+1] (or NULL). */
int flexmoe_step_cost(const int64_t* tokens, const int32_t* slot_owner, int E, int G, int S,
                      int64_t token_cost, const int64_t* sync_cost, int64_t* cost);

/*
 * Alg. 2, MakeSchedulingPlan.  *has_plan = 0: the empty plan.  Otherwise
 *   plan[0] = e0 (expert to expand)   plan[1] = source slot (a vExpert of e0: on the target's GPU
 *   if there is one, else its lowest slot)   plan[2] = target slot
 *   plan[3] = e1 (expert to shrink)   plan[4] = released slot
 *   t[0], t[1] = estimated cost before and after (t[1] < t[0]).
 * The release comes first when the plan is applied: the target may be the released slot.
 */
int flexmoe_make_scheduling_plan(const int64_t* tokens, const int32_t* slot_owner, int E, int G, int S,
                                 int64_t token_cost, const int64_t* sync_cost,
                                 int32_t plan[5], int64_t t[2], int* has_plan);

/*
 * One pass of Alg. 1's outer loop for the token assignment `tokens`: while the balance ratio is
 * above `threshold`, ask the Policy Maker for a plan and apply it; then one Migrate.
 *   slot_owner [G*S]  IN/OUT: the placement, modified in place
 *   ops [max_ops*4]   the primitives in the order they must run, 4 ints each:
 *                       FLEXMOE_SHRINK,  e1, released slot, -1
 *                       FLEXMOE_EXPAND,  e0, source slot,   target slot
 *                       FLEXMOE_MIGRATE, owner of slot a before, slot a, slot b
 *   *n_ops            how many were written (a Shrink/Expand pair needs room for two)
 *   *ratio_before, *ratio_after   Eq. 6 on entry and on return.
 */
int flexmoe_schedule(const int64_t* tokens, int32_t* slot_owner, int E, int G, int S,
                     int64_t token_cost, const int64_t* sync_cost, double threshold, int max_ops,
                     int32_t* ops, int* n_ops, double* ratio_before, double* ratio_after);

/*
 * The placement as the CSR table of flexmoe_route: occupied slots become vExperts 0..V-1 in
 * ascending slot id; rep_ids lists every expert's vExperts in that order.
 *   slot_owner [n_slots] -> rep_off [E+1], rep_ids [n_slots] (the first *V entries are written), *V.
 */
int flexmoe_placement_table(const int32_t* slot_owner, int E, int n_slots,
                            int32_t* rep_off, int32_t* rep_ids, int* V);

#ifdef __cplusplus
}
#endif
#endif /* FLEXMOE_SCHEDULER_H */
