/*
 * moe_fsep.h - the parameter layout of fully sharded expert parallelism (paper section 3.1,
 * executor: "shard", "unshard", "reshard"), as device kernels over the buffers of N ranks held
 * side by side in one device's memory.  In the real system unshard and reshard are balanced
 * All-to-All exchanges (every rank sends C chunks of 1/N of an expert to every other rank); here
 * the same index arithmetic runs as copy / reduce kernels, which is what one GPU can show.
 *
 * psi = values per expert (all of an expert's matrices flattened and concatenated), a multiple
 * of 8*N (16-byte pieces of bf16 per chunk; 4*N suffices for fp32).  chunk = psi / N.
 *   experts      [E][psi]        el   the unsharded parameters
 *   shards       [N][E][chunk]   el   rank n holds chunk n of every expert
 *   hosted       [N][C]          i32  DEVICE array: the expert restored in slot c of rank i, or -1
 *                                     (entries outside [-1, E) are treated as -1)
 *   restored     [N][C][psi]     el   what unshard produces: the C full experts of every rank
 *   grads        [N][C][psi]     el   full gradients of the hosted experts
 *   grad_shards  [N][E][chunk]   el   what reshard produces
 * Pointers are device memory, 16-byte aligned, owned by the caller; calls only enqueue.
 * N, E, C >= 1, N*C <= 4096.  dtype as in moe.h.
 */
#ifndef PAPER_2602_11686_MOE_FSEP_H
#define PAPER_2602_11686_MOE_FSEP_H

#include "moe.h"

#ifdef __cplusplus
extern "C" {
#endif

/* shards[n][e][:] = experts[e][n*chunk : (n+1)*chunk]   (model initialisation) */
moe_status moe_fsep_shard(int32_t N, int32_t E, int64_t psi, int32_t dtype, const void* experts, void* shards,
                          void* stream);

/* restored[i][c][n*chunk + o] = shards[n][hosted[i][c]][o]; an empty slot is filled with zeros. */
moe_status moe_fsep_unshard(int32_t N, int32_t E, int32_t C, int64_t psi, int32_t dtype, const void* shards,
                            const int32_t* hosted, void* restored, void* stream);

/* grad_shards[n][e][o] = sum over the slots (i, c) with hosted[i][c] == e, in ascending (i, c) order, of
 * grads[i][c][n*chunk + o]; fp32 accumulation, one rounding; an expert that no rank hosts gets zeros. */
moe_status moe_fsep_reshard(int32_t N, int32_t E, int32_t C, int64_t psi, int32_t dtype, const void* grads,
                            const int32_t* hosted, void* grad_shards, void* stream);

#ifdef __cplusplus
}
#endif
#endif
