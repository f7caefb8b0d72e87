/*
 * moe_planner.h - C ABI of the host-side load-balancing planner (paper section 4,
 * "Load Balancing Planner": problem formulation, Alg. 1 expert relocation, Alg. 2
 * expert layout; appendix: lite routing algorithm, replica allocation algorithm).
 *
 * The planner runs on the CPU by design (the paper delegates the layout search to
 * the host and overlaps it with the layer's GPU work), so every pointer here is
 * HOST memory owned by the caller; nothing is allocated on a device and no stream
 * is involved.  Calls are re-entrant and keep no state.
 *
 * Notation: N devices in nodes of D consecutive devices, E experts, C expert slots
 * per device;
 *     R [N][E]     int64   tokens held by device i that the gate routed to expert j
 *     A [N][E]     int32   replicas of expert j restored on device i (the layout)
 *     S [N][E][N]  int64   tokens of device i for expert j that are sent to device k
 * all dense row-major.
 *
 * Where the paper leaves a choice open the library takes these readings (the same
 * the test oracle takes, so results are comparable bit for bit):
 *   - loads and times are IEEE doubles; per-replica load = load / replicas;
 *     a device's load is the running sum of what was placed on it;
 *   - ties go to the lower expert index and the lower device index;
 *   - relocation: nodes with no eligible device are left out before the node with
 *     the fewest replicas of the expert is chosen; a device that already holds the
 *     expert is eligible only when no other device has a free slot;
 *   - lite routing: integer shares that differ by at most one, the larger ones to
 *     the lower-indexed replicas; a device with m replicas counts m times; if the
 *     sender's node holds a replica nothing leaves the node;
 *   - a device sending to itself costs no communication time;
 *   - even allocation when N*C is not a multiple of E: the remainder goes to the
 *     lowest-indexed experts;
 *   - a random perturbation moves one replica from a random expert that has more
 *     than one to another random expert; random numbers are splitmix64(seed) % n.
 *
 * Errors: MOE_ERR_INVALID_ARG for NULL pointers, N,E,C,D < 1, N % D != 0, N*C < E,
 * replica counts that are < 1 or exceed the N*C slots, negative token counts;
 * the message is available from moe_last_error().
 */
#ifndef PAPER_2602_11686_MOE_PLANNER_H
#define PAPER_2602_11686_MOE_PLANNER_H

#include "moe.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t N; /* devices                       */
    int32_t E; /* experts                       */
    int32_t C; /* expert slots per device       */
    int32_t D; /* devices per node (divides N)  */
} moe_plan_shape;

/* Constants of the cost model (section 4, problem formulation). */
typedef struct {
    double v_comm;  /* communication volume per token            */
    double b_intra; /* bandwidth between devices of one node     */
    double b_inter; /* bandwidth between devices of two nodes    */
    double v_comp;  /* computation volume per token              */
    double b_comp;  /* computational power of a device           */
    int32_t f_ckpt; /* 1 if activations are recomputed, else 0   */
} moe_plan_cost;

/* Appendix, replica allocation algorithm: expert_rep[E], every expert >= 1, sum = N*C;
 * the expert with the highest load per replica receives the next replica. */
moe_status moe_plan_replica_allocation(const moe_plan_shape* s, const int64_t* R, int32_t* expert_rep);

/* Alg. 1, expert relocation: places expert_rep[j] replicas of every expert (sum <= N*C),
 * heaviest per-replica load first, each on the least-loaded eligible device of the nodes
 * that hold the fewest replicas of that expert.  expert_loads[E] = column sums of R.
 * A[N][E] is overwritten. */
moe_status moe_plan_expert_relocation(const moe_plan_shape* s, const int32_t* expert_rep, const int64_t* expert_loads,
                                      int32_t* A);

/* Appendix, lite routing algorithm, for every sending device: S[N][E][N] is overwritten.
 * An expert with tokens but no replica anywhere is an error. */
moe_status moe_plan_lite_routing(const moe_plan_shape* s, const int64_t* R, const int32_t* A, int64_t* S);

/* Section 4, problem formulation: T[0] = T_comm + T_comp, T[1] = T_comm =
 * 4 V_comm sum S[i][j][k] / bw(i,k), T[2] = T_comp = (3 + F_ckpt) max_i V_comp sum_{j,k} S[k][j][i] / B_comp. */
moe_status moe_plan_time_cost(const moe_plan_shape* s, const moe_plan_cost* c, const int64_t* S, double* T);

/* Alg. 2, expert layout: builds eps >= 1 candidate replica vectors (load-proportional; even, if
 * eps >= 2; then random perturbations of earlier candidates), places each with Alg. 1, routes it
 * with the lite routing and prices it with the cost model - without materialising S, in
 * O(eps N^2 C) - and returns the cheapest layout (the first one on ties).
 * A[N][E], *T and *best_index are overwritten; replicas_set[eps][E] too if it is not NULL. */
moe_status moe_plan_expert_layout(const moe_plan_shape* s, const moe_plan_cost* c, const int64_t* R, int32_t eps,
                                  uint64_t seed, int32_t* A, double* T, int32_t* best_index, int32_t* replicas_set);

/* The table the token dispatcher of device `rank` needs (moe_permute_lite, moe_grouped_ffn_fwd_groups):
 * groups = replica slots numbered by (device, expert index on that device, copy); G = sum of A.
 *   expert_of_group[g], device_of_group[g]   (capacity N*C each)
 *   rep_begin[E+1], rep_group[<= N*C]: for expert j the groups `rank` routes to, ascending - the replicas
 *   inside rank's node if it has any, else all replicas (appendix, lite routing algorithm).
 * *G_out and *n_rep_out receive G and rep_begin[E]. */
moe_status moe_plan_dispatch_table(const moe_plan_shape* s, const int32_t* A, int32_t rank, int32_t* G_out,
                                   int32_t* n_rep_out, int32_t* expert_of_group, int32_t* device_of_group,
                                   int32_t* rep_begin, int32_t* rep_group);

#ifdef __cplusplus
}
#endif
#endif
