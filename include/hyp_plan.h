/*
 * hyp_plan.h - C ABI of the two scheduling algorithms that decide which blocks a
 * stage gets and which node runs a task: host code, no device memory involved.
 *
 *   hypsplit_dp        offline inter-tier partitioning, Sec. IV-A, Algorithm 1
 *   hypsched_rt        online intra-tier node selection, Sec. IV-B, Algorithm 2
 *   hypsched_simulate  the per-node FIFO queue model of Sec. IV-B that produces the
 *                      scheduler's inputs (T_wait of a node = remaining workload of
 *                      its running task plus the workloads waiting, over C), driven
 *                      by a list of task arrival times
 *
 * Blocks are numbered 1..N and tiers 1..T as in the paper; arrays are 0-based, so
 * f[i-1] is f_i.  Every pointer is host memory owned by the caller for the duration
 * of the call; nothing is retained.  No call allocates device memory, throws or
 * prints; failures are status codes (hyp_stage.h).
 *
 * Points the paper leaves open and this library fixes (the CPU oracle fixes the same):
 *   - the binary search starts from tau_low = 0, tau_high = S_f(N) / min_j C_j, and the
 *     upper bound itself is checked once first, so that "no partition" is reported
 *     exactly when the memory limits M_j admit none;
 *   - among several feasible predecessors k the check keeps the smallest;
 *   - every tier receives at least one block (the transition's k < n);
 *   - Algorithm 2 breaks ties in favour of the node listed first;
 *   - in the queue model a task holds m_act of its node's memory from the moment it is
 *     assigned until it completes, and a node serves its queue without idling.
 */
#ifndef HYP_PLAN_H
#define HYP_PLAN_H

#include <stddef.h>
#include <stdint.h>

#include "hyp_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * HypSplit-DP (Algorithm 1): the partition vector p* = (p_1 .. p_{T-1}) that minimises
 * max_j L_j(p), L_j(p) = (1 / C_j) sum_{i = p_{j-1}+1}^{p_j} f_i, subject to
 * sum m_i <= M_j per tier, by binary search on the target latency tau around the
 * feasibility check DP(j, n) (the state-transition equation of Sec. IV-A with prefix
 * sums S_f, S_m), to precision eps: the returned tau* is at most eps above the optimum.
 *
 *   f, m   host [n_blocks]  computing load and memory need of each block, >= 0, finite
 *   C, M   host [n_tiers]   computing capacity (> 0) and memory capacity of each tier
 *   eps                     > 0, in the unit of f / C
 *   p_out  host [n_tiers-1] p_1 .. p_{T-1}: tier j runs blocks p_{j-1}+1 .. p_j, i.e. the
 *                           0-based range [p_{j-1}, p_j) for stage_create; untouched if
 *                           infeasible; may be null when n_tiers == 1
 *   tau_out                 tau* (the last feasible target; the initial upper bound if
 *                           the search never met a feasible one)
 *   feasible_out            1 if a partition exists, else 0 (then the status is still HYP_OK)
 *
 * HYP_EINVAL: null pointer, n_tiers < 1, n_blocks < n_tiers, eps <= 0, a negative or
 * non-finite f / m, a non-positive or non-finite C, a NaN M.
 */
HYP_API hyp_status_t hypsplit_dp(int32_t n_blocks, int32_t n_tiers, const double *f, const double *m,
                                 const double *C, const double *M, double eps, int32_t *p_out,
                                 double *tau_out, int32_t *feasible_out);

/*
 * HypSched-RT (Algorithm 2): among the nodes of one tier that are available and have
 * M_avail >= m_act, the one with the smallest (F_run_rem + F_wait + F_new) / C, i.e. the
 * earliest expected completion (the k* equation of Sec. IV-B).
 *
 *   C, M_avail, F_run_rem, F_wait  host [n_nodes]; available host [n_nodes] of 0 / 1
 *   k_out                          index of k*, or -1 if no node is eligible
 *
 * HYP_EINVAL: null pointer with n_nodes > 0, n_nodes < 0, null k_out.
 */
HYP_API hyp_status_t hypsched_rt(int32_t n_nodes, const double *C, const double *M_avail,
                                 const uint8_t *available, const double *F_run_rem, const double *F_wait,
                                 double F_new, double m_act, int32_t *k_out);

/*
 * Queue model: n_tasks tasks arrive at tier 1 at arrivals[q] (any order) and pass
 * through tiers 1..T.  On arrival at tier j the node is chosen by hypsched_rt from the
 * node states at that instant; the task joins that node's FIFO queue, needs F[j] / C of
 * the node once it is served, and reaches tier j+1 transfer[j] after it completes.
 * Events are processed in time order, lower task index first at equal times.
 *
 *   F, m_act        host [n_tiers]      workload and memory of a task at each tier
 *   nodes_per_tier  host [n_tiers]      K_j >= 1
 *   C, M            host [sum K_j]      per node, tier after tier
 *   available       host [sum K_j] of 0 / 1, or null for "all available"
 *   transfer        host [n_tiers - 1]  (null allowed when n_tiers == 1)
 *   node_out        host [n_tasks * n_tiers]  chosen node per task and tier, -1 where the
 *                                       task found no eligible node (it is dropped there)
 *   finish_out      host [n_tasks * n_tiers]  completion times, +inf where dropped
 *
 * HYP_EINVAL: null pointer, non-positive counts, K_j < 1, non-positive C.
 */
HYP_API hyp_status_t hypsched_simulate(int32_t n_tasks, const double *arrivals, int32_t n_tiers,
                                       const double *F, const double *m_act, const int32_t *nodes_per_tier,
                                       const double *C, const double *M, const uint8_t *available,
                                       const double *transfer, int32_t *node_out, double *finish_out);

#ifdef __cplusplus
}
#endif
#endif /* HYP_PLAN_H */
