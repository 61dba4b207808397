/*
 * prism_placement.h -- scheduler-side placement pipeline of Prism (arXiv
 * 2508.12851, Sec. III-C "Activation-Aware Expert Placement"): it consumes the
 * per-expert activation counts that the MoE layer of prism.h accumulates
 * (counts_accum) for N servers x L layers and produces the per-server,
 * per-layer local_mask arrays that layer takes, plus the two cost figures the
 * migration rule compares.
 *
 * Host code only: every pointer is HOST memory, nothing here touches the GPU,
 * allocates device memory or synchronises.  Arrays are dense, row-major:
 *   f          int64 [N][L][E]   activation counts f_n^l(e) (raw, >= 0)
 *   v          double[N][L]      activation entropy in bits
 *   counts     int32 [N][L]      N_{n,l}: experts of layer l to hold on server n
 *   placement  uint8 [N][L][E]   1 iff server n holds expert e of layer l
 *                                (= sum_g z_{n,g}^e >= 1); row [n][l] is the
 *                                local_mask of prism_moe_layer for that layer
 * Errors: PRISM_ERR_INVALID_ARG for NULL pointers, sizes < 1, negative counts,
 * non-positive memory sizes or speeds; nothing is written in that case.
 * Where the paper's listings leave a choice open (ties, the donor layer, what a
 * duplicate is, termination), the rule taken is stated at the function.
 */
#ifndef PRISM_PLACEMENT_H_
#define PRISM_PLACEMENT_H_

#include <stddef.h>
#include <stdint.h>

#include "prism.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Activation entropy (formula printed with Alg. 1):
 *   v[n][l] = - sum_e p_e log2 p_e,  p_e = f[n][l][e] / sum_e' f[n][l][e'].
 * Terms with p_e = 0 contribute 0; a (server, layer) with no observation gets 0.
 */
prism_status prism_activation_entropy(const int64_t* f, int32_t n_servers, int32_t n_layers,
                                      int32_t n_experts, double* v);

/*
 * Alg. 1, layer-wise expert count allocation.
 * Step 1: counts[n][l] = min(E, floor(server_mem[n] / expert_mem * v[n][l] / sum_l v[n][l]));
 *         a server whose entropies are all zero splits evenly (share 1/L).
 * Step 2: for l = 0..L-1, while the layer's total over the servers is below E:
 *         visit the servers in order of descending server_mem (index order among
 *         equals); for each, the donor l' is the layer other than l with the
 *         largest total among those with total > E (lowest index on ties); if
 *         counts[n][l'] > 0 and counts[n][l] < E move one expert from l' to l on
 *         that server; stop the pass when the total reaches E.  A pass that
 *         moves nothing leaves the layer short and sets *feasible = 0.
 *   server_mem [N] (M_n, any unit), expert_mem (m_e, same unit), feasible: host int.
 */
prism_status prism_expert_count_allocation(const double* v, const double* server_mem,
                                           double expert_mem, int32_t n_servers,
                                           int32_t n_layers, int32_t n_experts, int32_t* counts,
                                           int32_t* feasible);

/*
 * Alg. 2, expert-to-server assignment.
 * Every server takes its counts[n][l] most frequent experts of layer l
 * (descending f, lower index first on ties).  Then, per layer, while some
 * expert is held by nobody: servers are visited by ascending number of
 * duplicates (experts they hold that another server holds too; index order among
 * equals, order fixed per pass, servers without duplicates skipped); the server
 * takes the unassigned expert it uses most (lower index on ties) in place of its
 * least used duplicate (higher index on ties); the sets are updated after every
 * replacement; a pass without a replacement ends the loop with *covered = 0.
 */
prism_status prism_expert_assignment(const int64_t* f, const int32_t* counts, int32_t n_servers,
                                     int32_t n_layers, int32_t n_experts, uint8_t* placement,
                                     int32_t* covered);

/*
 * Eq. 2, the communication-aware proxy objective:
 *   *cost = sum_{n,l,e} f[n][l][e] * [placement[n][l][e] == 0].
 * For one server and one layer this is the n_remote the layer's dispatch reports.
 */
prism_status prism_proxy_cost(const int64_t* f, const uint8_t* placement, int32_t n_servers,
                              int32_t n_layers, int32_t n_experts, int64_t* cost);

/*
 * Eq. 3, migration cost between two placements, on the server-level indicator:
 *   *seconds = sum over entries with old != new of expert_mem / speed[n],
 *   *flips   = number of such entries (removals count like additions, as printed).
 *   speed [N]: I/O bandwidth of server n in expert_mem units per second.
 */
prism_status prism_migration_cost(const uint8_t* old_placement, const uint8_t* new_placement,
                                  int32_t n_servers, int32_t n_layers, int32_t n_experts,
                                  double expert_mem, const double* speed, double* seconds,
                                  int64_t* flips);

/*
 * Eq. 4, the migration rule, with the proxy costs converted to time by the
 * historical seconds per remote invocation (Sec. IV-A, system parameter settings):
 *   *adopt = [ cost_new * seconds_per_remote_call + t_mig < cost_old * seconds_per_remote_call ].
 */
prism_status prism_migration_decision(int64_t cost_old, int64_t cost_new, double t_mig,
                                      double seconds_per_remote_call, int32_t* adopt);

/*
 * The pipeline entropy -> Alg. 1 -> Alg. 2 in one call.  v and counts may be NULL
 * when the caller does not want them; *ok = feasible && covered.
 */
prism_status prism_placement_plan(const int64_t* f, const double* server_mem, double expert_mem,
                                  int32_t n_servers, int32_t n_layers, int32_t n_experts,
                                  double* v, int32_t* counts, uint8_t* placement, int32_t* ok);

#ifdef __cplusplus
}
#endif
#endif /* PRISM_PLACEMENT_H_ */
