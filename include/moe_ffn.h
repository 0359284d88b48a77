/*
 * moe_ffn.h - C ABI of the routed-expert mixture-of-experts FFN block for
 * AMD gfx950 (MI355X), one GPU.
 *
 * The block is the MoE feed-forward layer of the Qwen3-30B-A3B-class policy
 * that the paper trains (Section 4.1, "Training Details", names the model).  It
 * is evaluated for every generated token during rollout decode (Section 2.3,
 * segment rollouts) and for every token of a trajectory when the trainer
 * recomputes token probabilities for the importance ratio (Section 2.2, Eq. 3).
 * The paper does not spell the layer out; the operation implemented is the
 * standard dropless top-K mixture of SwiGLU experts:
 *
 *   T tokens, H hidden size, E experts, K experts per token, I expert
 *   intermediate size.  Assignment id a = t*K + k (token t, slot k).
 *
 *   logits   l[t,e] = float( sum_h x[t,h]*Wr[e,h] + b[e] ), sum carried wide enough
 *            that the one rounding to float is (practically) order independent
 *   select   experts ordered by (logit descending, index ascending); first K
 *   weights  softmax over the K selected logits (== full softmax renormalised
 *            over the selection); or, with renormalize = 0, the entries of the
 *            full softmax over all E logits
 *   permute  stable counting sort of the assignments by expert
 *   expert   y = Wd[e] * ( silu(Wg[e]*v) .* (Wu[e]*v) ),  silu(g) = g/(1+exp(-g))
 *   combine  out[t,:] = sum_k w[t,k] * y[row(t*K+k),:]
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers (HIP global memory) unless marked
 *     "host".  The shape struct and `out_bytes` are host memory.
 *   - All tensors are dense row-major with the last index contiguous.
 *   - The caller owns every buffer and the stream.  The library allocates
 *     nothing, frees nothing and keeps no pointer after a call returns.  Scratch
 *     memory is the caller's `ws` buffer, at least moe_workspace_bytes() long;
 *     calls that run concurrently must use disjoint workspaces.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it and the call returns without synchronising; no
 *     device-to-host copy happens inside any call.
 *   - Inputs are read-only.  Outputs are overwritten in full.
 *   - Arguments are validated on the host before any HIP call is made; a
 *     failed validation enqueues nothing.  T == 0 is MOE_OK and enqueues nothing:
 *     every output that has elements is then left as it was, which only concerns
 *     moe_permute's expert_offsets (E+1 values whatever T is; all zero in meaning).
 *   - The one thing any entry point creates is the set of HIP events of the two
 *     stage-timing calls, destroyed before they return.
 *   - Every data pointer must be 16-byte aligned.  H and I must be multiples
 *     of 8.  Non-finite inputs give undefined results.
 *   - dtype names the storage type of x, of every weight, of x_perm/y_perm and
 *     of out: MOE_BF16 (bfloat16) or MOE_F32 (float).  With MOE_F32 the router
 *     consumes the float values as they are; the expert GEMMs round x and the
 *     weights to bf16 (nearest even) on load.  Products are bf16 x bf16 on the
 *     matrix cores with float accumulation in either case.
 */
#ifndef MOE_FFN_H
#define MOE_FFN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_ERR_NULL = 1,       /* a required pointer is NULL */
    MOE_ERR_SHAPE = 2,      /* T<0, H/E/K/I < 1, K > E, H or I not a multiple of 8, T*K or T*E overflow */
    MOE_ERR_DTYPE = 3,      /* dtype is neither MOE_BF16 nor MOE_F32 */
    MOE_ERR_WORKSPACE = 4,  /* ws is NULL or ws_bytes is below moe_workspace_bytes() */
    MOE_ERR_ALIGN = 5,      /* a data pointer is not 16-byte aligned */
    MOE_ERR_HIP = 6,        /* a kernel launch (or another HIP call) reported an error */
    MOE_ERR_STATIC_LIMIT = 7 /* moe_forward_noalloc: the shape needs more than MOE_NOALLOC_SCRATCH_BYTES of scratch */
} moe_status_t;

typedef enum { MOE_BF16 = 0, MOE_F32 = 1 } moe_dtype_t;

typedef struct {
    int32_t T;            /* tokens in the batch (>= 0) */
    int32_t H;            /* hidden size */
    int32_t E;            /* routed experts */
    int32_t K;            /* experts per token, 1 <= K <= E */
    int32_t I;            /* expert intermediate size */
    int32_t dtype;        /* moe_dtype_t */
    int32_t renormalize;  /* nonzero: weights sum to one over the selected K */
} moe_shape_t;

/* Static, NUL-terminated description of a status code (host). */
const char *moe_status_string(moe_status_t status);

/* Host only.  Bytes of scratch that any entry point below may need for `shape`
 * (one figure covers them all).  *out_bytes is a multiple of 256. */
moe_status_t moe_workspace_bytes(const moe_shape_t *shape, size_t *out_bytes);

/*
 * Router: logits, top-K selection and routing weights (definition above).
 *   x          [T,H] dtype            w_router  [E,H] dtype
 *   router_bias[E] float or NULL      (added to the logit; affects selection and weights)
 *   topk_idx   [T,K] int32 out: expert ids, slot 0 = arg-max, ties to the lower id
 *   topk_w     [T,K] float out
 * The logit sum is carried in double (every bf16*bf16 and float*float product is
 * exact in double), then rounded once to float; selection compares those floats.
 */
moe_status_t moe_route_topk(const moe_shape_t *shape, const void *x, const void *w_router,
                            const float *router_bias, int32_t *topk_idx, float *topk_w,
                            void *ws, size_t ws_bytes, void *stream);

/*
 * Expert-sorted permutation: stable counting sort of the T*K assignments by expert.
 *   topk_idx       [T,K] int32, every value in [0,E) (values outside are undefined behaviour)
 *   x              [T,H] dtype or NULL (only read when x_perm is given)
 *   expert_offsets [E+1] int32 out: rows of expert e are [off[e], off[e+1]); off[E] = T*K
 *   row_to_assign  [T*K] int32 out: assignment id held by each sorted row
 *   assign_to_row  [T*K] int32 out: inverse map
 *   x_perm         [T*K,H] dtype out or NULL: x_perm[row(a),:] = x[a / K,:] (bit copy)
 * Within an expert's segment rows keep increasing assignment id (stability), so the
 * result is unique.
 */
moe_status_t moe_permute(const moe_shape_t *shape, const int32_t *topk_idx, const void *x,
                         int32_t *expert_offsets, int32_t *row_to_assign, int32_t *assign_to_row,
                         void *x_perm, void *ws, size_t ws_bytes, void *stream);

/*
 * Grouped SwiGLU expert FFN over expert-sorted rows.
 *   x_perm  [T*K,H] dtype           expert_offsets [E+1] int32 (as written by moe_permute)
 *   w_gate  [E,I,H] dtype           w_up [E,I,H] dtype        w_down [E,H,I] dtype
 *   y_perm  [T*K,H] dtype out
 * For each expert e and row r of its segment:
 *   g = Wg[e] x_r, u = Wu[e] x_r (float accumulation), a = bf16(silu(g)*u),
 *   y_r = Wd[e] a (float accumulation), rounded once to dtype.
 * Experts with no rows cost nothing.
 */
moe_status_t moe_grouped_swiglu(const moe_shape_t *shape, const void *x_perm,
                                const int32_t *expert_offsets, const void *w_gate,
                                const void *w_up, const void *w_down, void *y_perm,
                                void *ws, size_t ws_bytes, void *stream);

/*
 * Weighted combine: out[t,:] = sum_{k=0..K-1} topk_w[t,k] * y_perm[assign_to_row[t*K+k],:]
 * accumulated in float in increasing k, rounded once to dtype.
 *   y_perm [T*K,H] dtype   assign_to_row [T*K] int32   topk_w [T,K] float   out [T,H] dtype
 */
moe_status_t moe_combine(const moe_shape_t *shape, const void *y_perm, const int32_t *assign_to_row,
                         const float *topk_w, void *out, void *stream);

/*
 * The whole block: route, permute, grouped SwiGLU, combine, in one call.  Same
 * routing and permutation as the separate calls; the token rows are gathered
 * inside the first GEMM instead of being copied to x_perm.
 *   out           [T,H] dtype out
 *   topk_idx_out  [T,K] int32 out or NULL     topk_w_out [T,K] float out or NULL
 */
moe_status_t moe_forward(const moe_shape_t *shape, const void *x, const void *w_router,
                         const float *router_bias, const void *w_gate, const void *w_up,
                         const void *w_down, void *out, int32_t *topk_idx_out, float *topk_w_out,
                         void *ws, size_t ws_bytes, void *stream);

/*
 * moe_forward for callers that cannot allocate device memory or hand over a workspace: code running under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus ws / ws_bytes),
 * kernels, results and errors as moe_forward; the scratch is a buffer of MOE_NOALLOC_SCRATCH_BYTES that is part of
 * the loaded library (one copy per GPU, held until the process ends).  The call allocates and frees nothing.
 *   - A shape whose moe_workspace_bytes() exceeds MOE_NOALLOC_SCRATCH_BYTES is rejected with
 *     MOE_ERR_STATIC_LIMIT before anything is enqueued (32 MiB covers decode batches of up to 512 tokens at
 *     H 2048, E 128, K 8, I 768).
 *   - The first call on a GPU looks up that GPU's copy of the buffer (hipGetSymbolAddress); a failure there is
 *     MOE_ERR_HIP.
 *   - All calls on one GPU share that GPU's buffer, which keeps the previous call's contents: calls that overlap
 *     in time on one GPU (different streams, different threads) race.  Calls on one stream are ordered and safe.
 */
#define MOE_NOALLOC_SCRATCH_BYTES (32u << 20)
moe_status_t moe_forward_noalloc(const moe_shape_t *shape, const void *x, const void *w_router,
                                 const float *router_bias, const void *w_gate, const void *w_up,
                                 const void *w_down, void *out, int32_t *topk_idx_out, float *topk_w_out,
                                 void *stream);

/*
 * moe_forward with a HIP event recorded on `stream` at every stage boundary, for
 * attributing the time of one call to its kernels.  Unlike every other entry
 * point this one blocks until the call has finished on the device.
 *   stage_ms  host float[MOE_NUM_STAGES] out: elapsed milliseconds of
 *             [0] router logits  [1] top-K + weights  [2] permutation (3 kernels)
 *             [3] row-tile list  [4] gate/up GEMM + SiLU*mul  [5] down GEMM  [6] combine
 *             [7] an empty interval (two events back to back): what the measurement itself adds to a stage
 * Same arguments, results and errors as moe_forward otherwise.
 */
#define MOE_NUM_STAGES 8
moe_status_t moe_forward_stage_times(const moe_shape_t *shape, const void *x, const void *w_router,
                                     const float *router_bias, const void *w_gate, const void *w_up,
                                     const void *w_down, void *out, void *ws, size_t ws_bytes,
                                     void *stream, float *stage_ms);

#ifdef __cplusplus
}
#endif
#endif /* MOE_FFN_H */
