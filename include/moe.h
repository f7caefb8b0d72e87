/*
 * moe.h - C ABI of the single-device MoE-layer hot path on MI355X (gfx950).
 *
 * The layer is the mixture of experts of the paper's Preliminary section,
 *     y = sum_i g(x)_i * f_i(x),     g(x) = Softmax(TopK(x * W_g)),
 * with SwiGLU experts without bias (section 3.1, overlap analysis:
 * H = silu(x*W1) (.) (x*W3), y = H*W2, 6*H*H' FLOPs per routed token) and
 * dropless routing (experimental setup): an expert takes every token routed to
 * it, possibly none.  The calls below are the stages of that layer on one
 * device's share of T tokens:
 *
 *     moe_gate_topk -> moe_permute -> moe_grouped_ffn_fwd -> moe_unpermute_combine
 *     moe_combine_bwd -> moe_grouped_ffn_bwd -> moe_unpermute_combine (unit
 *     weights) -> moe_gate_topk_bwd
 *
 * Conventions common to every call
 *   - Every pointer is DEVICE memory owned by the caller (inputs, outputs and
 *     the workspace).  The library never allocates, frees or keeps a pointer
 *     after the call returns.  Pointers must be 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Every call only enqueues kernels on it and returns; there is no host
 *     synchronisation and no device-to-host copy anywhere (the paper's
 *     "host bound optimization": routing counts never visit the CPU).  Calls
 *     on one stream are ordered; calls that share a workspace must not overlap.
 *   - All tensors are dense row-major.  `el` is the storage type named by
 *     shape->dtype (bf16 or fp32).  All arithmetic accumulates in fp32.
 *       x        [T, d]  el      tokens
 *       w_gate   [d, E]  el      gate weight,          logits = x * w_gate (+ bias)
 *       w1, w3   [E, d, f] el    expert up projections (w1 is the silu branch)
 *       w2       [E, f, d] el    expert down projection
 *     R = T*k routed rows; the flat index of (token t, slot s) is p = t*k + s.
 *   - Validation is host-side and argument-only: NULL pointers, alignment,
 *     T,d,f,E,k >= 1, k <= E <= MOE_MAX_EXPERTS, d and f multiples of 8 (bf16)
 *     or 4 (fp32), T*k*max(d,f) < 2^31 * 64, workspace size.  A failed check
 *     returns an error code, launches nothing, and leaves a message for
 *     moe_last_error().  Data-dependent faults (non-finite values, expert ids
 *     out of range, offsets that do not describe R rows) are undefined
 *     behaviour and are not checked on the device.
 *   - Device: the grouped-GEMM calls (moe_grouped_ffn_fwd, _fwd_groups, _fwd_products, _bwd, _bwd_groups,
 *     _bwd_products and, for bf16, moe_gate_topk_bwd) are laid out for a whole MI355X (gfx950, 256 compute units: one persistent
 *     workgroup per unit, dealt round-robin to the 8 XCDs).  They look the current device up once and
 *     return MOE_ERR_UNSUPPORTED on any other architecture or under a compute-unit mask, and
 *     MOE_ERR_DEVICE if no device can be queried; nothing is launched in either case.  One-time kernel
 *     attributes are set under a lock, once per kernel and device: calls may come from several threads.
 *   - Same inputs give bit-identical outputs from run to run (no floating
 *     point atomics; integer atomics only where the order cannot matter).
 */
#ifndef PAPER_2602_11686_MOE_H
#define PAPER_2602_11686_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_MAX_EXPERTS 256

typedef enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = 1,
    MOE_ERR_UNSUPPORTED = 2,
    MOE_ERR_WORKSPACE_TOO_SMALL = 3,
    MOE_ERR_DEVICE = 4 /* a HIP launch reported an error */
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;

/* Problem shape of one call; passed by const pointer, read on the host only. */
typedef struct {
    int32_t T; /* tokens on this device            */
    int32_t d; /* hidden size            (paper: H)  */
    int32_t f; /* SwiGLU intermediate    (paper: H') */
    int32_t E; /* experts                          */
    int32_t k; /* experts per token (top-k)        */
    int32_t dtype; /* moe_dtype of x and all weights   */
} moe_shape;

/* Static strings; never freed.  moe_last_error() is thread-local and describes
 * the most recent failed call of the calling thread ("" if none). */
const char* moe_status_string(moe_status s);
const char* moe_last_error(void);
int moe_abi_version(void);

/* Upper bound, in bytes, of the workspace any call below needs for this shape
 * (0 if the shape itself is invalid).  The workspace needs no initialisation
 * and carries nothing from one call to the next. */
size_t moe_workspace_bytes(const moe_shape* shape);

/* Gate (Preliminary section, g = Softmax(TopK(x W_g))).
 *   logits[t,e] = sum_c x[t,c] * w_gate[c,e] + bias[e]      (fp32 accumulate)
 *   topk_ids[t,0..k-1] = the k experts of largest logit, in descending order of
 *                        logit; equal logits: the lower expert index first
 *   topk_w[t,s] = exp(l_s - l_0) / sum_j exp(l_j - l_0) over the k selected
 * bias [E] fp32 may be NULL (zero).  logits_out [T,E] fp32 may be NULL.
 * Workspace: used. */
moe_status moe_gate_topk(const moe_shape* shape, const void* x, const void* w_gate,
                         const float* bias, int32_t* topk_ids /*[T,k]*/, float* topk_w /*[T,k]*/,
                         float* logits_out /*[T,E] or NULL*/, void* ws, size_t ws_bytes,
                         void* stream);

/* Token rearrangement by expert (the paper's implementation section names a
 * dedicated kernel for it; here: histogram -> prefix sum -> stable rank ->
 * row scatter, all on the device).
 *   counts[e]      = number of pairs p with topk_ids[p] == e          (sum = R)
 *   offsets[0] = 0, offsets[e+1] = offsets[e] + counts[e]
 *   row_of_pair[p] = offsets[e] + #{p' < p : topk_ids[p'] == e},  e = topk_ids[p]
 *                    (stable counting sort of p by expert)
 *   pair_of_row    = inverse permutation of row_of_pair
 *   x_perm[row_of_pair[p], :] = x[p / k, :]                (bitwise copy)
 * x_perm may be NULL (indices only).  Workspace: used. */
moe_status moe_permute(const moe_shape* shape, const void* x, const int32_t* topk_ids,
                       int32_t* counts /*[E]*/, int32_t* offsets /*[E+1]*/,
                       int32_t* row_of_pair /*[R]*/, int32_t* pair_of_row /*[R]*/,
                       void* x_perm /*[R,d] el or NULL*/, void* ws, size_t ws_bytes, void* stream);

/* moe_permute for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs and
 * kernels as moe_permute, without `ws`: the per-chunk histograms of the counting sort live in a
 * file-scope device array inside the library (256 KiB on every GPU that runs the library, held until the
 * process ends).  The call allocates nothing and frees nothing; the first call on a device looks the
 * array's address up once (hipGetSymbolAddress) and later calls reuse it.
 * Limit: chunks(T*k) * E <= moe_permute_static_max_hist_entries() (65536), where the T*k pairs are cut
 * into chunks of 128 pairs, doubled until at most 256 chunks remain; all shapes with T*k <= 2^21 and
 * E <= 256 fit.  A larger problem returns MOE_ERR_UNSUPPORTED and launches nothing.
 * All calls on one GPU share the array, which keeps the previous call's contents (nothing in it has to
 * start at zero: every entry read is written first by the same call): two calls that overlap in time on
 * one GPU - different streams, different host threads - race; calls on one stream are ordered. */
size_t moe_permute_static_max_hist_entries(void);
moe_status moe_permute_static(const moe_shape* shape, const void* x, const int32_t* topk_ids,
                              int32_t* counts /*[E]*/, int32_t* offsets /*[E+1]*/,
                              int32_t* row_of_pair /*[R]*/, int32_t* pair_of_row /*[R]*/,
                              void* x_perm /*[R,d] el or NULL*/, void* stream);

/* Expert computation, forward (section 3.1: SwiGLU MLP; per device the work is
 * 6*d*f FLOPs per routed row).  For every expert e and its rows
 * r in [offsets[e], offsets[e+1]):
 *   A = x_perm[r,:] * w1[e],  B = x_perm[r,:] * w3[e],  H = silu(A) (.) B,
 *   y_perm[r,:] = H * w2[e]
 * a_save / b_save [R,f] el receive A and B (the activations backward needs);
 * both may be NULL.  Workspace: used (holds H). */
moe_status moe_grouped_ffn_fwd(const moe_shape* shape, const void* x_perm, const int32_t* offsets,
                               const void* w1, const void* w3, const void* w2,
                               void* y_perm /*[R,d] el*/, void* a_save, void* b_save, void* ws,
                               size_t ws_bytes, void* stream);

/* The token dispatcher of one device: the lite routing of the paper's appendix (Lite Routing
 * Algorithm) folded into the permutation.  Experts may be replicated; a replica slot is a "group"
 * g in [0, G), G <= MOE_MAX_EXPERTS, numbered so that the groups of one destination device are
 * consecutive (the caller - the planner - numbers them; see moe_plan_dispatch_table).  For expert e
 * the sending device may use the groups rep_group[rep_begin[e] .. rep_begin[e+1]) (its node's replicas
 * if there are any, else all).  The n_e pairs of expert e, in stable order (ascending p), are cut into
 * len = rep_begin[e+1] - rep_begin[e] consecutive blocks of n_e / len pairs, the first n_e % len
 * blocks one pair longer; block r belongs to group rep_group[rep_begin[e] + r].
 *   expert_counts[e] = n_e;   group_counts[g] = pairs of group g (0 for groups not listed);
 *   group_offsets = exclusive prefix sum of group_counts, group_offsets[G] = R;
 *   row_of_pair[p] = group_offsets[g(p)] + (position of p inside its block); pair_of_row = inverse;
 *   x_perm[row_of_pair[p], :] = x[p / k, :].
 * Rows are therefore ordered by group: one contiguous send region per destination device.
 * rep_begin, rep_group are DEVICE arrays and are checked on the device (list bounds against n_rep,
 * a list for every expert that has pairs, group ids inside [0, G), no group listed twice).  If a check
 * fails, *table_errors (device, may be NULL) receives a non-zero bit mask, every pair is counted in
 * group 0 and the rows are in plain expert order: no index ever leaves [0, R).  A valid table writes 0.
 * x_perm may be NULL.  Workspace: used. */
moe_status moe_permute_lite(const moe_shape* shape, int32_t G, int32_t n_rep, const void* x,
                            const int32_t* topk_ids, const int32_t* rep_begin /*[E+1]*/,
                            const int32_t* rep_group /*[n_rep]*/, int32_t* expert_counts /*[E]*/,
                            int32_t* group_counts /*[G]*/, int32_t* group_offsets /*[G+1]*/,
                            int32_t* row_of_pair /*[R]*/, int32_t* pair_of_row /*[R]*/,
                            void* x_perm /*[R,d] el or NULL*/, int32_t* table_errors /*[1] or NULL*/,
                            void* ws, size_t ws_bytes, void* stream);

/* moe_grouped_ffn_fwd over replica groups: the rows [group_offsets[g], group_offsets[g+1]) are
 * multiplied with the weights of expert expert_of_group[g] (DEVICE array [G]; entries are clamped
 * into [0, E-1]).  Replicas of one expert share its weights, so with the rows of moe_permute_lite
 * the layer output equals that of the plain path bit for bit.  Everything else as moe_grouped_ffn_fwd. */
moe_status moe_grouped_ffn_fwd_groups(const moe_shape* shape, int32_t G, const int32_t* expert_of_group,
                                      const void* x_perm, const int32_t* group_offsets, const void* w1,
                                      const void* w3, const void* w2, void* y_perm, void* a_save,
                                      void* b_save, void* ws, size_t ws_bytes, void* stream);

/* moe_grouped_ffn_bwd over replica groups (appendix, lite routing; section 3.1, executor: a device
 * computes on the replica slots it hosts and the reshard step sums the slots' gradients per expert).
 * The rows [group_offsets[g], group_offsets[g+1]) are differentiated against the weights of expert
 * expert_of_group[g] (DEVICE array [G], entries clamped into [0, E-1]); dx_perm is per row as in
 * moe_grouped_ffn_bwd.  The weight gradients are written PER GROUP:
 *   dw1_groups, dw3_groups [G, d, f] el,  dw2_groups [G, f, d] el   (a group without rows gets zeros);
 * the gradient of an expert is the sum over its groups, which is what moe_fsep_reshard forms from the
 * slots of all devices.  G <= MOE_MAX_EXPERTS.  Everything else as moe_grouped_ffn_bwd. */
moe_status moe_grouped_ffn_bwd_groups(const moe_shape* shape, int32_t G, const int32_t* expert_of_group,
                                      const void* x_perm, const int32_t* group_offsets, const void* w1,
                                      const void* w3, const void* w2, const void* a_save,
                                      const void* b_save, const void* dy_perm, void* dx_perm /*[R,d]*/,
                                      void* dw1_groups, void* dw3_groups, void* dw2_groups, void* ws,
                                      size_t ws_bytes, void* stream);

/* Expert computation, backward (section 3.2 prices it at twice the forward).
 *   dH = dy_perm * w2[e]^T,  dA = dH (.) B (.) silu'(A),  dB = dH (.) silu(A)
 *   dx_perm = dA * w1[e]^T + dB * w3[e]^T
 *   dw2[e] = H^T * dy_perm,  dw1[e] = x_perm^T * dA,  dw3[e] = x_perm^T * dB
 * (sums over the rows of expert e; an expert without rows gets exact zeros).
 * a_save and b_save as written by the forward call; if either is NULL, A and
 * B are recomputed from x_perm (expert-only recomputation, section 4).
 * dw1, dw3 [E,d,f] and dw2 [E,f,d] are el and are overwritten.
 * Workspace: used (H, dA, dB and, when recomputing, A and B). */
moe_status moe_grouped_ffn_bwd(const moe_shape* shape, const void* x_perm, const int32_t* offsets,
                               const void* w1, const void* w3, const void* w2, const void* a_save,
                               const void* b_save, const void* dy_perm, void* dx_perm /*[R,d]*/,
                               void* dw1, void* dw3, void* dw2, void* ws, size_t ws_bytes,
                               void* stream);

/* The same pair of calls with the activations saved as products (section 3.1: the SwiGLU expert;
 * section 3.2: backward priced at twice the forward).  What the backward pass needs of A and B is
 *   H = silu(A) (.) B  (for dw2),   P = B (.) silu'(A)  (dA = dH (.) P),   Q = silu(A)  (dB = dH (.) Q),
 * so the forward call keeps H (which it computes anyway) and writes P and Q where the plain call writes A
 * and B: h_save, p_save, q_save [R,f] el, all required.  The backward call then spends two multiplications
 * per element where the plain one recomputes a sigmoid, at the price of a third saved tensor.  P and Q are
 * rounded to el once; everything else as in moe_grouped_ffn_fwd / moe_grouped_ffn_bwd.
 * Workspace: none in the forward call; the backward call uses it (dA, dB), size as for moe_grouped_ffn_bwd. */
moe_status moe_grouped_ffn_fwd_products(const moe_shape* shape, const void* x_perm, const int32_t* offsets,
                                        const void* w1, const void* w3, const void* w2,
                                        void* y_perm /*[R,d] el*/, void* h_save, void* p_save, void* q_save,
                                        void* stream);
moe_status moe_grouped_ffn_bwd_products(const moe_shape* shape, const void* x_perm, const int32_t* offsets,
                                        const void* w1, const void* w3, const void* w2, const void* h_save,
                                        const void* p_save, const void* q_save, const void* dy_perm,
                                        void* dx_perm /*[R,d]*/, void* dw1, void* dw3, void* dw2, void* ws,
                                        size_t ws_bytes, void* stream);

/* Weighted combine ("a weighted sum of the outputs from the selected experts",
 * introduction; the mixture formula of the Preliminary section).
 *   y[t,:] = sum_{s<k} topk_w[t,s] * y_perm[row_of_pair[t*k+s], :]
 * summed in slot order in fp32, rounded once.  topk_w == NULL means unit
 * weights: the backward of the row scatter of moe_permute. */
moe_status moe_unpermute_combine(const moe_shape* shape, const void* y_perm,
                                 const int32_t* row_of_pair, const float* topk_w,
                                 void* y /*[T,d] el*/, void* stream);

/* Backward of the weighted combine.
 *   dy_perm[row_of_pair[t*k+s], :] = topk_w[t,s] * dy[t,:]
 *   dtopk_w[t,s] = <dy[t,:], y_perm[row_of_pair[t*k+s], :]> */
moe_status moe_combine_bwd(const moe_shape* shape, const void* dy /*[T,d] el*/, const void* y_perm,
                           const int32_t* row_of_pair, const float* topk_w,
                           void* dy_perm /*[R,d] el*/, float* dtopk_w /*[T,k]*/, void* stream);

/* Backward of the gate through the k selected logits (the selection itself
 * carries no gradient).
 *   dl[t,s] = topk_w[t,s] * (dtopk_w[t,s] - sum_j topk_w[t,j] * dtopk_w[t,j])
 *   dw_gate[c,e] = sum_t x[t,c] * dL[t,e],   dL[t, topk_ids[t,s]] = dl[t,s]
 *   dx_inout[t,c] += sum_s dl[t,s] * w_gate[c, topk_ids[t,s]]
 * dx_inout [T,d] el is read, updated and written (it arrives holding the
 * gradient that came through the experts); it may be NULL.  dw_gate [d,E] is
 * fp32 whatever the dtype.  Workspace: used. */
moe_status moe_gate_topk_bwd(const moe_shape* shape, const void* x, const void* w_gate,
                             const int32_t* topk_ids, const float* topk_w, const float* dtopk_w,
                             void* dx_inout, float* dw_gate /*[d,E] fp32*/, void* ws,
                             size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PAPER_2602_11686_MOE_H */
