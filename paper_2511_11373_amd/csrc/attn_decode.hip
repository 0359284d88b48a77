// Single-token grouped-query attention over a paged key/value cache (bf16, head size 128): HBM-bound, every byte of the
// cache is read once, in 64 KB pages that are contiguous per head and tiled for the load instructions below.
//
// The work is the list of all 64-position steps of all (sequence, key/value head) pairs, in that order; it is cut into
// equal contiguous shares, one per wave, as many waves as the chip holds at once (8 per CU: the registers of a step's keys
// and values limit it to that).  A wave streams through its share with the next step's keys and values always in
// flight, keeps a running maximum / sum / output, and writes them out as a partial result whenever its share leaves a
// (sequence, head) pair; no wave waits for another, and there is one cold start per wave instead of one per block.  A
// second kernel merges the partial results of a pair in position order.  A tiny first kernel counts the steps.
//
// One step on v_mfma_f32_16x16x32_bf16 (lane l = (c, q) = (l % 16, l / 16) feeds row or column c, reduction slots
// 8q .. 8q+7; result register j is D[4q + j][c]), without LDS and without any transposition:
//   scores, transposed:  S^T = K Q^T.  A = 16 positions of K (rows), B = the group's query heads (columns, zero beyond
//     the group), 4 MFMAs over the 128 features.  Which position a row stands for is free: row r of tile t is position
//     8 (r / 4) + r % 4 + 4 (t % 2) + 32 (t / 2) of the step, so that lane (c, q) ends up with the scores of head c at
//     positions 8 q .. 8 q + 7 (tiles 0, 1) and 32 + 8 q .. + 7 (tiles 2, 3; registers j = 0..3 each).
//   softmax: per lane over its 16 scores, across the four q groups by two shuffles; running maximum per head, sums kept
//     per lane and added across q when a partial result is written.
//   output: O = P V.  A = P (row = head c, the lane's own exponentials: positions 32 u + 8 q .. + 7 for MFMA u = 0, 1),
//     B = V stored feature-major (column = feature 16 c8 + c, the same 8 consecutive positions = one 16-byte load, the
//     four q groups of a feature reading 64 contiguous bytes), 8 feature tiles x 2 MFMAs.  The reduction slots of an
//     MFMA may be any positions as long as A and B agree.
// Storage inside a page of one head (32768 elements), in blocks of 64 positions (8192 elements each):
//   keys:   tile (t, i) = 512 elements at (4 t + i) * 512: row r of score tile t (the position given above), features
//           32 i .. + 31, rows 32 elements apart;
//   values: tile (c8, u) = 512 elements at (2 c8 + u) * 512: feature 16 c8 + c in row c, positions 32 u .. + 31 of the block.
#include "moe_internal.hpp"

#include <type_traits>

#include "attn_decode.h"

namespace moe {
namespace attn {

constexpr int D = 128, PAGE = 256, STEP = 64, MAXG = 16, MAX_WAVES = 4096;
constexpr float kNegBig = -1e30f;

__device__ __forceinline__ u32x4 ld16(const bf16_t *p) { return *reinterpret_cast<const u32x4 *>(p); }
// a length as the kernels use it: never negative, never beyond the block table's row
__device__ __forceinline__ int usable_length(int n, int max_pages) { return min(max(n, 0), max_pages * PAGE); }
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// first[b] = number of steps of the sequences before b (per key/value head), first[B] = that of all
__global__ __launch_bounds__(1024) void attn_plan_kernel(const int32_t *__restrict__ seq_lens, int32_t *__restrict__ first, int B,
                                                         int max_pages) {
    __shared__ int wave_sum[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int carry = 0;
    for (int b0 = 0; b0 < B; b0 += 1024) {
        const int b = b0 + threadIdx.x;
        const int v = b < B ? (usable_length(seq_lens[b], max_pages) + STEP - 1) / STEP : 0;
        int inc = v;                                                    // inclusive prefix within the wave
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_up(inc, d, 64);
            if (lane >= d) inc += o;
        }
        if (lane == 63) wave_sum[wave] = inc;
        __syncthreads();
        int before = 0, all = 0;
        for (int i = 0; i < 16; ++i) {
            const int t = wave_sum[i];
            if (i < wave) before += t;
            all += t;
        }
        if (b < B) first[b] = carry + before + inc - v;
        carry += all;
        __syncthreads();
    }
    if (threadIdx.x == 0) first[B] = carry;
}

// steps per wave when `total` steps are shared among n_waves
__device__ __forceinline__ int share_of(int total, int n_waves) { return max(1, (total + n_waves - 1) / n_waves); }

// Partial results: slot (wave + pair index) holds [head of the group][D + 2] floats: output (unnormalised), maximum (log2
// domain), sum.  Wave and pair index both grow along the list of steps and one of them changes from one partial result to
// the next, so the slots are distinct, and those of a pair are consecutive.
__global__ __launch_bounds__(256, 2) void attn_stream_kernel(const bf16_t *__restrict__ qp, const bf16_t *__restrict__ k_pages,
                                                             const bf16_t *__restrict__ v_pages, const int32_t *__restrict__ block_table,
                                                             const int32_t *__restrict__ seq_lens, const int32_t *__restrict__ first,
                                                             float *__restrict__ part, int B, int Hq, int Hkv, int max_pages,
                                                             float scale_log2) {
    const int lane = threadIdx.x & 63, c = lane & 15, q = lane >> 4;
    const int w = uniform(blockIdx.x * 4 + (threadIdx.x >> 6));
    const int group = Hq / Hkv;
    const int total = first[B] * Hkv;
    const int per = share_of(total, gridDim.x * 4);
    const int begin = w * per;
    if (begin >= total) return;
    const int count = min(per, total - begin);

    // the pair and step the share begins in: the last sequence whose first step is not after `begin`
    int lo = 0, hi = B;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (first[mid] * Hkv <= begin) lo = mid;
        else hi = mid;
    }
    int b = lo, nsteps = uniform(first[b + 1] - first[b]), n = uniform(usable_length(seq_lens[b], max_pages));
    int h = (begin - first[b] * Hkv) / nsteps, s = (begin - first[b] * Hkv) - h * nsteps;

    u32x4 qop[4], kr[4][4], vr[8][2];
    // the group's queries as the B operand: column c = head c of the group, features 32 i + 8 q .. + 7
    auto load_queries = [&](int b, int h) {
        int l = lane;
        asm volatile("" : "+v"(l));                                    // the lane's offset is formed here, not kept in registers
        const int c = l & 15, q = l >> 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            qop[i] = u32x4{0u, 0u, 0u, 0u};
            if (c < group) qop[i] = ld16(qp + ((size_t)b * Hq + h * group + c) * D + 32 * i + 8 * q);
        }
    };
    auto page_of = [&](int b, int s) { return uniform(block_table[(size_t)b * max_pages + (s >> 2)]); };
    // Both caches are stored in 1 KB tiles of 16 rows x 64 bytes, exactly what one load instruction of a wave reads (lane
    // (c, q): row c, bytes 16 q .. + 15), so every instruction reads eight whole 128-byte lines and can be non-temporal.
    auto load_keys = [&](int page, int h, int s) {
        const bf16_t *kp = k_pages + ((size_t)page * Hkv + h) * PAGE * D + (size_t)(s & 3) * STEP * D + c * 32 + 8 * q;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) kr[t][i] = load_once(kp + (t * 4 + i) * 512);      // tile (t, i): rows of tile t, features 32 i .. + 31
    };
    auto load_values = [&](int page, int h, int s) {
        const bf16_t *vp = v_pages + ((size_t)page * Hkv + h) * D * PAGE + (size_t)(s & 3) * STEP * D + c * 32 + 8 * q;
#pragma unroll
        for (int c8 = 0; c8 < 8; ++c8)
#pragma unroll
            for (int u = 0; u < 2; ++u) vr[c8][u] = load_once(vp + (c8 * 2 + u) * 512);      // tile (c8, u): features 16 c8 .. + 15, positions 32 u .. + 31
    };

    float m = kNegBig, lsum = 0.f;                 // of head c; lsum covers this lane's positions only
    f32x4 acc[8];
#pragma unroll
    for (int c8 = 0; c8 < 8; ++c8) acc[c8] = f32x4{0.f, 0.f, 0.f, 0.f};
    load_queries(b, h);
    {
        const int page = page_of(b, s);
        load_keys(page, h, s);
        __builtin_amdgcn_sched_barrier(0);                              // keys first, as in the loop: the first wait is for them alone
        load_values(page, h, s);
    }
    // Keys and values of a step are loaded one step ahead, each as soon as its registers are free (the keys' when the
    // scores are formed, the values' after the value product): 16 KB of each per wave.  The share's last step loads
    // nothing; it is a copy of the body of its own, because a load that is issued on one path only makes the compiler wait
    // for every load in flight where the paths meet.
    auto step = [&](auto more_tag) __attribute__((always_inline)) {
        constexpr bool more = decltype(more_tag)::value;
        // the step after this one
        int b2 = b, h2 = h, s2 = s + 1, nsteps2 = nsteps, n2 = n;
        if (s2 == nsteps) {
            s2 = 0;
            if (++h2 == Hkv && more) {                                 // on to the next sequence that has a step
                h2 = 0;
                do {
                    ++b2;
                    nsteps2 = uniform(first[b2 + 1] - first[b2]);
                } while (nsteps2 == 0 && b2 < B - 1);
                n2 = uniform(usable_length(seq_lens[b2], max_pages));
            }
        }
        const bool pair_ends = !more || s2 == 0;
        const int page2 = more ? page_of(b2, s2) : 0;
        const int t0 = s * STEP;                                        // first position of the step

        // scores of head c at positions t0 + 8 q + j + 4 (t % 2) + 32 (t / 2)
        f32x4 st[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            st[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                st[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kr[t][i]), __builtin_bit_cast(bf16x8, qop[i]),
                                                                st[t], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);                              // the loads stay behind the last use of their registers
        if (more) {                                                     // query and key registers are free
            if (s2 == 0) load_queries(b2, h2);
            load_keys(page2, h2, s2);
        }
        __builtin_amdgcn_sched_barrier(0);
        const int left = n - (t0 + 8 * q);                              // position 8 q + e of the step is valid iff e < left
        float smax = kNegBig;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float v = (j + 4 * (t & 1) + 32 * (t >> 1) < left) ? st[t][j] * scale_log2 : kNegBig;
                st[t][j] = v;
                smax = fmaxf(smax, v);
            }
        smax = fmaxf(smax, __shfl_xor(smax, 16, 64));
        smax = fmaxf(smax, __shfl_xor(smax, 32, 64));
        const float m_new = fmaxf(m, smax);                             // finite: position t0 is valid for every head
        const float alpha = exp2f(m - m_new);
        m = m_new;
        float psum = 0.f;
        u32x4 pop[2];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            float p[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                p[j] = (j + 4 * (t & 1) + 32 * (t >> 1) < left) ? exp2f(st[t][j] - m_new) : 0.f;
                psum += p[j];
            }
            pop[t >> 1][2 * (t & 1)] = pack_bf16x2(p[0], p[1]);
            pop[t >> 1][2 * (t & 1) + 1] = pack_bf16x2(p[2], p[3]);
        }
        lsum = lsum * alpha + psum;
        // values at positions the sequence has not reached may hold anything (0 * NaN = NaN): zero them in the last step
        if (t0 + STEP > n) {
#pragma unroll
            for (int c8 = 0; c8 < 8; ++c8)
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int w4 = 0; w4 < 4; ++w4) {
                        const int e = 32 * u + 2 * w4;                  // positions 8 q + e, + 1 of the step
                        const unsigned int keep = (e < left ? 0xFFFFu : 0u) | (e + 1 < left ? 0xFFFF0000u : 0u);
                        vr[c8][u][w4] &= keep;
                    }
        }
        // rescale what has been accumulated: output register j belongs to head 4 q + j, whose factor lane 4 q + j holds
        float a4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) a4[j] = __shfl(alpha, 4 * q + j, 64);
#pragma unroll
        for (int c8 = 0; c8 < 8; ++c8) {
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[c8][j] *= a4[j];
#pragma unroll
            for (int u = 0; u < 2; ++u)
                acc[c8] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pop[u]), __builtin_bit_cast(bf16x8, vr[c8][u]),
                                                                  acc[c8], 0, 0, 0);
        }
        if (pair_ends) {                                                // the share leaves the pair: its partial result
            float l = lsum;
            l += __shfl_xor(l, 16, 64);
            l += __shfl_xor(l, 32, 64);
            float *dst = part + (size_t)(w + b * Hkv + h) * group * (D + 2);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (4 * q + j < group) {
#pragma unroll
                    for (int c8 = 0; c8 < 8; ++c8) dst[(4 * q + j) * (D + 2) + 16 * c8 + c] = acc[c8][j];
                }
            if (q == 0 && c < group) {
                dst[c * (D + 2) + D] = m;
                dst[c * (D + 2) + D + 1] = l;
            }
            m = kNegBig;
            lsum = 0.f;
#pragma unroll
            for (int c8 = 0; c8 < 8; ++c8) acc[c8] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        __builtin_amdgcn_sched_barrier(0);
        if (more) load_values(page2, h2, s2);                           // the value registers are free
        __builtin_amdgcn_sched_barrier(0);
        b = b2, h = h2, s = s2, nsteps = nsteps2, n = n2;
    };
    for (int i = 1; i < count; ++i) step(std::true_type{});
    step(std::false_type{});
}

// out[b, head, :] from the partial results of the head's pair, in position order
__global__ __launch_bounds__(128) void attn_merge_kernel(const float *__restrict__ part, const int32_t *__restrict__ first,
                                                         bf16_t *__restrict__ out, int B, int Hq, int Hkv, int n_waves) {
    const int b = blockIdx.x / Hq, jh = blockIdx.x - b * Hq, group = Hq / Hkv;
    const int h = jh / group, head = jh - h * group, d = threadIdx.x;
    const int nsteps = first[b + 1] - first[b];
    float o = 0.f;
    if (nsteps > 0) {
        const int per = share_of(first[B] * Hkv, n_waves);
        const int s0 = first[b] * Hkv + h * nsteps;                     // the pair's steps in the list: s0 .. s0 + nsteps - 1
        const int w0 = s0 / per, w1 = (s0 + nsteps - 1) / per, used = w1 - w0 + 1;
        const float *p = part + ((size_t)(w0 + b * Hkv + h) * group + head) * (D + 2);
        const size_t stride = (size_t)group * (D + 2);
        float M = kNegBig;
        for (int ch = 0; ch < used; ++ch) M = fmaxf(M, p[ch * stride + D]);
        float num = 0.f, den = 0.f;
        for (int ch = 0; ch < used; ++ch) {
            const float wgt = exp2f(p[ch * stride + D] - M);
            num = fmaf(p[ch * stride + d], wgt, num);
            den = fmaf(p[ch * stride + D + 1], wgt, den);
        }
        o = num / den;
    }
    out[(size_t)blockIdx.x * D + d] = (bf16_t)float_to_bf16_bits(o);
}

int check(const attn_shape_t *s) {
    if (!s) return 1;
    if (s->B < 0 || s->Hq < 1 || s->Hkv < 1 || s->Hq % s->Hkv != 0 || s->Hq / s->Hkv > MAXG || s->D != D || s->max_pages < 1 ||
        s->n_pages < 1)
        return 2;
    // the list of steps is indexed with int: B * Hkv * (steps of a full row of the block table) stays below 2^30
    if ((long long)s->B * s->Hkv * ((long long)s->max_pages * (PAGE / STEP)) > 0x3FFFFFFFLL) return 2;
    return 0;
}
size_t plan_bytes_of(const attn_shape_t &s) { return align256(((size_t)s.B + 1) * sizeof(int32_t)); }
size_t ws_bytes_of(const attn_shape_t &s) {
    return plan_bytes_of(s) + align256(((size_t)MAX_WAVES + (size_t)s.B * s.Hkv) * (s.Hq / s.Hkv) * (D + 2) * sizeof(float));
}
bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

}  // namespace attn
}  // namespace moe

using namespace moe;

extern "C" {

int attn_decode_workspace_bytes(const attn_shape_t *shape, size_t *out_bytes) {
    const int st = attn::check(shape);
    if (st) return st;
    if (!out_bytes) return 1;
    *out_bytes = attn::ws_bytes_of(*shape);
    return 0;
}

int attn_decode(const attn_shape_t *shape, const void *q, const void *k_pages, const void *v_pages,
                const int32_t *block_table, const int32_t *seq_lens, void *out, void *ws, size_t ws_bytes, void *stream) {
    const int st = attn::check(shape);
    if (st) return st;
    if (!q || !k_pages || !v_pages || !block_table || !seq_lens || !out) return 1;
    if (attn::misaligned(q) || attn::misaligned(k_pages) || attn::misaligned(v_pages) || attn::misaligned(block_table) ||
        attn::misaligned(seq_lens) || attn::misaligned(out))
        return 5;
    if (!ws) return 4;
    if (attn::misaligned(ws)) return 5;
    if (ws_bytes < attn::ws_bytes_of(*shape)) return 4;
    const attn_shape_t &s = *shape;
    if (s.B == 0) return 0;
    hipStream_t hs = (hipStream_t)stream;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return 6;
    const int n_blocks = std::min(2 * cus, attn::MAX_WAVES / 4);       // two blocks of four waves per CU: all resident at once
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)attn::D);
    int32_t *first = (int32_t *)ws;
    float *part = (float *)((char *)ws + attn::plan_bytes_of(s));
    hipLaunchKernelGGL(attn::attn_plan_kernel, dim3(1), dim3(1024), 0, hs, seq_lens, first, s.B, s.max_pages);
    if (hipGetLastError() != hipSuccess) return 6;
    hipLaunchKernelGGL(attn::attn_stream_kernel, dim3(n_blocks), dim3(256), 0, hs, (const bf16_t *)q, (const bf16_t *)k_pages,
                       (const bf16_t *)v_pages, block_table, seq_lens, (const int32_t *)first, part, s.B, s.Hq, s.Hkv, s.max_pages,
                       scale_log2);
    if (hipGetLastError() != hipSuccess) return 6;
    hipLaunchKernelGGL(attn::attn_merge_kernel, dim3(s.B * s.Hq), dim3(attn::D), 0, hs, (const float *)part, (const int32_t *)first,
                       (bf16_t *)out, s.B, s.Hq, s.Hkv, 4 * n_blocks);
    return hipGetLastError() == hipSuccess ? 0 : 6;
}

}  // extern "C"
