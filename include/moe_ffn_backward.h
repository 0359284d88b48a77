/*
 * moe_ffn_backward.h - C ABI of the backward pass of the routed-expert MoE FFN block declared in
 * moe_ffn.h, for AMD gfx950 (MI355X), one GPU.
 *
 * The trainer maximises the objective of Section 2.2 (Eq. 2-3) with AdamW (Section 4.1, "Training
 * Details"), which differentiates every layer of the policy, this block included.  The paper does not spell
 * the gradient out; what is implemented is the chain rule through the operation moe_ffn.h defines, with
 * the top-K selection held fixed (it is piecewise constant and carries no gradient):
 *
 *   out_t = sum_k w_k y_k               dw_k  = <d_out_t, y_k>
 *   w = softmax(l over the selection)   dl_k  = w_k (dw_k - sum_j w_j dw_j)
 *   (renormalize == 0: w_k = p_{e_k}, p the softmax over all E logits, and every logit of the token has a gradient,
 *    dl_e = p_e ([e selected] dw_e - sum_j w_j dw_j); the three router sums below then run over all experts / tokens)
 *   l_e = <x_t, Wr_e> + b_e             dx_t += sum_k dl_k Wr_e;  dWr_e += dl x_t;  db_e += dl
 *   y = Wd a, a = silu(g) u             da = w_k Wd^T d_out_t;  dWd_e += (w_k d_out_t) a^T
 *   g = Wg x, u = Wu x                  dg = da u silu'(g), du = da silu(g), silu'(g) = s (1 + g (1 - s)), s = 1/(1+e^-g)
 *                                       dWg_e += dg x_t^T;  dWu_e += du x_t^T;  dx_t += Wg^T dg + Wu^T du
 *
 * Conventions: those of moe_ffn.h (device pointers unless marked host, dense row-major tensors, caller-owned
 * buffers and stream, nothing allocated or kept, arguments validated on the host before anything is enqueued,
 * every data pointer 16-byte aligned, outputs overwritten in full, T == 0 gives zero weight gradients).
 * Storage types: shape->dtype names the type of x, the weights, d_out, d_x and the row gradients, as in moe_ffn.h.  The
 * GEMMs multiply bf16 either way: with MOE_F32 the router still reads the float values (it has to select what the forward
 * pass selected), every other input is rounded once to bf16 into the workspace (which grows by those copies) and d_x is
 * widened on the way out.  moe_forward_saving / moe_backward_saved are MOE_BF16 only (else MOE_ERR_DTYPE).
 * Both kinds of routing weights are taken (shape->renormalize); the un-renormalised kind needs T*E more floats of
 * workspace and its router gradients are plain dense sums (not tuned: it is not the configuration of the model the
 * paper trains).  Every weight gradient is float and is written, not accumulated into (an expert that received no row
 * gets zeros).
 * Nothing is kept from a forward call: routing, permutation and the expert pre-activations are recomputed (what
 * activation recomputation does for long sequences).  The pair moe_forward_saving / moe_backward_saved is the other
 * choice: the forward pass keeps the pre-activations g and u of every expert-sorted row, the backward pass reads them.
 * Intermediates are rounded to bf16, sums run in float on the matrix cores.
 */
#ifndef MOE_FFN_BACKWARD_H
#define MOE_FFN_BACKWARD_H

#include "moe_ffn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Host only.  Bytes of scratch that the two entry points below need for `shape`; a multiple of 256. */
moe_status_t moe_backward_workspace_bytes(const moe_shape_t *shape, size_t *out_bytes);

/*
 * Backward of moe_grouped_swiglu over expert-sorted rows (the data- and weight-gradient grouped GEMMs).
 *   x_perm   [T*K,H] dtype    expert_offsets [E+1] int32     w_gate, w_up [E,I,H] dtype    w_down [E,H,I] dtype
 *   dy_perm  [T*K,H] dtype: dL/dy for every row
 *   d_x_perm [T*K,H] dtype out      d_w_gate, d_w_up [E,I,H] float out       d_w_down [E,H,I] float out
 */
moe_status_t moe_grouped_swiglu_backward(const moe_shape_t *shape, const void *x_perm, const int32_t *expert_offsets,
                                         const void *w_gate, const void *w_up, const void *w_down, const void *dy_perm,
                                         void *d_x_perm, float *d_w_gate, float *d_w_up, float *d_w_down,
                                         void *ws, size_t ws_bytes, void *stream);

/*
 * Backward of moe_forward: all gradients of <out, d_out> in one call.
 *   x [T,H], w_router [E,H], w_gate, w_up [E,I,H], w_down [E,H,I]: dtype; router_bias [E] float or NULL
 *   d_out [T,H] dtype
 *   d_x [T,H] dtype out     d_w_router [E,H] float out      d_router_bias [E] float out or NULL
 *   d_w_gate, d_w_up [E,I,H] float out      d_w_down [E,H,I] float out
 * Sums over the rows of an expert run in row order and sums over a token's K slots in slot order, so two calls
 * on the same inputs give the same bits.
 */
moe_status_t moe_backward(const moe_shape_t *shape, const void *x, const void *w_router, const float *router_bias,
                          const void *w_gate, const void *w_up, const void *w_down, const void *d_out,
                          void *d_x, float *d_w_router, float *d_router_bias, float *d_w_gate, float *d_w_up,
                          float *d_w_down, void *ws, size_t ws_bytes, void *stream);

/*
 * moe_forward that also keeps what the backward pass would otherwise recompute (the trainer of Section 4.1 runs the
 * policy's forward pass and then its backward pass over the same tokens).
 *   x, w_router, router_bias, w_gate, w_up, w_down, out: as for moe_forward
 *   g_rows, u_rows [T*K, I] bf16 out: g = W_gate[e] x_t and u = W_up[e] x_t of expert-sorted row r (the row order of
 *                                     moe_permute; a pure function of the routing, so moe_backward_saved finds it again)
 *   topk_idx_out [T,K] int32, topk_w_out [T,K] float out, or NULL: the routing, as from moe_forward
 *   ws: a forward workspace (the size that moe_workspace_bytes gives for `shape`)
 * The activations are formed from the rounded g and u (one rounding more than in moe_forward: same tolerance).
 * Restrictions: MOE_BF16 (else MOE_ERR_DTYPE); H a multiple of 256 and I a multiple of 128 (else MOE_ERR_SHAPE): the
 * large-batch kernels do all the work, whatever T is.
 */
moe_status_t moe_forward_saving(const moe_shape_t *shape, const void *x, const void *w_router, const float *router_bias,
                                const void *w_gate, const void *w_up, const void *w_down, void *out, void *g_rows,
                                void *u_rows, int32_t *topk_idx_out, float *topk_w_out, void *ws, size_t ws_bytes,
                                void *stream);

/*
 * moe_backward with the pre-activations supplied instead of recomputed.
 *   g_rows, u_rows [T*K, I] bf16: as written by moe_forward_saving for the same x, router and expert weights
 *   topk_idx [T,K] int32, topk_w [T,K] float: the routing that moe_forward_saving wrote, or both NULL (then it is recomputed)
 * Everything else as for moe_backward (same workspace size, same results: with g_rows and u_rows from
 * moe_forward_saving the gradients are bit for bit those of moe_backward, whose recomputation yields the same g and u).
 */
moe_status_t moe_backward_saved(const moe_shape_t *shape, const void *x, const void *w_router, const float *router_bias,
                                const void *w_gate, const void *w_up, const void *w_down, const void *d_out,
                                const void *g_rows, const void *u_rows, const int32_t *topk_idx, const float *topk_w, void *d_x,
                                float *d_w_router, float *d_router_bias, float *d_w_gate, float *d_w_up, float *d_w_down,
                                void *ws, size_t ws_bytes, void *stream);

/*
 * moe_backward with a HIP event recorded on `stream` at every stage boundary, for attributing the time of one
 * call to its kernels.  Unlike the other entry points this one blocks until the call has finished on the device.
 *   stage_ms  host float[MOE_BW_NUM_STAGES] out: elapsed milliseconds of
 *             [0] routing (recomputed)   [1] permutation + copies of x and d_out into expert-sorted rows
 *             [2] row-tile list   [3] g = x Wg^T   [4] u = x Wu^T (nothing when one launch, counted under [3], yields both)
 *             [5] dq = d_out Wd   [6] row-wise SwiGLU backward
 *             [7] dx rows = dg Wg + du Wu   [8] dWd   [9] dWg   [10] dWu   [11] softmax backward, dx, router gradients
 *             [12] an empty interval (two events back to back): what the measurement itself adds to a stage
 * Same arguments, results and errors as moe_backward otherwise.
 */
#define MOE_BW_NUM_STAGES 13
moe_status_t moe_backward_stage_times(const moe_shape_t *shape, const void *x, const void *w_router, const float *router_bias,
                                      const void *w_gate, const void *w_up, const void *w_down, const void *d_out,
                                      void *d_x, float *d_w_router, float *d_router_bias, float *d_w_gate, float *d_w_up,
                                      float *d_w_down, void *ws, size_t ws_bytes, void *stream, float *stage_ms);

#ifdef __cplusplus
}
#endif
#endif /* MOE_FFN_BACKWARD_H */
