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
 * Cache layout (chosen for the hardware: every page of a head is one contiguous 64 KB block that is read exactly once,
 * front to back, by load instructions that each fetch eight whole 128-byte lines).  The context of sequence b is cut
 * into pages of 256 positions; page i of the sequence is page block_table[b * max_pages + i] of the pools:
 *   k_pages [n_pages, Hkv, 32768]   v_pages [n_pages, Hkv, 32768]
 * Inside the 32768 elements of a page and head, each block of 64 positions is 8192 contiguous elements made of 16 tiles
 * of 512 elements (16 rows of 32 elements).  With p the position inside the block (0..63) and f the feature (0..127):
 *   K[p, f] is element ((4 t + f / 32) * 16 + r) * 32 + f % 32 of the block,
 *           where t = 2 (p / 32) + (p % 8) / 4 and r = 4 ((p % 32) / 8) + p % 4;
 *   V[p, f] is element ((2 (f / 16) + p / 32) * 16 + f % 16) * 32 + p % 32 of the block
 * (keys: tiles of 16 positions x 32 features; values: tiles of 16 features x 32 positions, i.e. stored transposed, because
 * their product reduces over positions).  Appending a token writes 4 pieces of 64 bytes of K and 128 single elements of
 * V, once, against thousands of reads.  paper_2511_11373_amd/workloads.py has the same maps as array reshapes
 * (attn_tile_keys, attn_tile_values and their inverses).
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
