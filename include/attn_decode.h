/*
 * attn_decode.h - C ABI of single-token (decode) grouped-query attention over a paged key/value cache, for AMD gfx950
 * (MI355X), one GPU.
 *
 * The policy the paper trains generates up to 64k tokens on top of 32k-token inputs (Section 4.1, "Training Details"),
 * one token at a time; at those lengths reading the key/value cache is the other large cost of rollout next to the MoE
 * block.  The paper does not spell the operation out; it is the textbook one:
 *
 *   sequence b, query head j, key/value head h = j / (Hq / Hkv), context length n_b = seq_lens[b]:
 *     s[t] = <q[b,j,:], K_b[t,h,:]> / sqrt(D),  p = softmax(s over t < n_b),  out[b,j,:] = sum_t p[t] V_b[t,h,:]
 *
 * Cache layout (chosen for the hardware: every page of a head is one contiguous 64 KB block that is read exactly once
 * and front to back).  The context of sequence b is cut into pages of 256 positions; page i of the sequence is page
 * block_table[b * max_pages + i] of the pools:
 *   k_pages [n_pages, Hkv, 256, D]   position-major: K[t, h, :] of a page are D contiguous elements
 *   v_pages [n_pages, Hkv, D, 256]   feature-major: V[t0 .. t0+255, h, d] of a page are 256 contiguous elements
 * (the values are stored transposed because their product reduces over positions; appending a token writes D scattered
 * elements, once, against thousands of reads).
 *
 * Conventions: all data pointers are DEVICE pointers, 16-byte aligned, bf16 unless stated; the caller owns every buffer
 * and the stream; nothing is allocated or kept; arguments are validated on the host before anything is enqueued.
 * Restrictions: D = 128, page = 256 positions, Hq a multiple of Hkv with Hq / Hkv <= 16.  B == 0 enqueues nothing.  A
 * sequence of length 0 gives zeros.  Positions at or beyond seq_lens[b] are never read through (their pages need not
 * exist: block_table entries past the last used page are ignored).
 */
#ifndef ATTN_DECODE_H
#define ATTN_DECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t B;          /* sequences */
    int32_t Hq, Hkv;    /* query heads, key/value heads */
    int32_t D;          /* head size: 128 */
    int32_t max_pages;  /* row length of block_table: every seq_lens[b] <= 256 * max_pages */
    int32_t n_pages;    /* pages in the pools (bound for block_table entries) */
} attn_shape_t;

/* 0 ok, 1 NULL pointer, 2 unsupported shape, 4 workspace missing or too small, 5 misaligned pointer, 6 HIP launch error */
int attn_decode_workspace_bytes(const attn_shape_t *shape, size_t *out_bytes);

/*
 *   q [B, Hq, D]    k_pages, v_pages as above    block_table [B, max_pages] int32    seq_lens [B] int32
 *   out [B, Hq, D] bf16 out
 * All 64-position steps of all (sequence, key/value head) pairs form one list that is cut into equal contiguous shares,
 * one per resident wave (8 per compute unit of the current device); a wave keeps a running maximum and sum (float
 * accumulation on the matrix cores) and writes a partial result per pair it touches, and the partial results of a pair
 * are merged in position order.  The split depends on the lengths and the device only, so results do not depend on
 * timing.  The workspace holds the step counts and the partial results; its contents mean nothing between calls.
 */
int attn_decode(const attn_shape_t *shape, const void *q, const void *k_pages, const void *v_pages,
                const int32_t *block_table, const int32_t *seq_lens, void *out, void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ATTN_DECODE_H */
