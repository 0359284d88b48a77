// Single-token grouped-query attention over a paged key/value cache (bf16, head size 128): HBM-bound, every byte of the
// cache is read once, in 64 KB pages that are contiguous per head.
//
// Block = (sequence, key/value head, 2048-position chunk), 4 waves; wave w takes the 64-position steps w, w+4, ... of
// the chunk with its own running maximum / sum / output and the four are merged through LDS at the end; a second kernel
// merges the chunks of a sequence in position order.
//
// One step on v_mfma_f32_16x16x32_bf16 (lane l = (c, q) = (l % 16, l / 16) feeds row or column c, reduction slots
// 8q .. 8q+7; result register j is D[4q + j][c]), without LDS and without any transposition:
//   scores, transposed:  S^T = K Q^T.  A = 16 positions of K (rows), B = the group's query heads (columns, zero beyond
//     the group), 4 MFMAs over the 128 features.  Which position a row stands for is free: row r of tile t is position
//     8 (r / 4) + r % 4 + 4 (t % 2) + 32 (t / 2) of the step, so that lane (c, q) ends up with the scores of head c at
//     positions 8 q .. 8 q + 7 (tiles 0, 1) and 32 + 8 q .. + 7 (tiles 2, 3; registers j = 0..3 each).
//   softmax: per lane over its 16 scores, across the four q groups by two shuffles; running maximum per head, sums kept
//     per lane and added across q at the very end.
//   output: O = P V.  A = P (row = head c, the lane's own exponentials: positions 32 u + 8 q .. + 7 for MFMA u = 0, 1),
//     B = V stored feature-major (column = feature 16 c8 + c, the same 8 consecutive positions = one 16-byte load, the
//     four q groups of a feature reading 64 contiguous bytes), 8 feature tiles x 2 MFMAs.  The reduction slots of an
//     MFMA may be any positions as long as A and B agree.
#include "moe_internal.hpp"

#include "attn_decode.h"

namespace moe {
namespace attn {

constexpr int D = 128, PAGE = 256, STEP = 64, CHUNK = 2048, MAXG = 16;
constexpr float kNegBig = -1e30f;

__device__ __forceinline__ u32x4 ld16(const bf16_t *p) { return *reinterpret_cast<const u32x4 *>(p); }

// partial results of a chunk: [bh][chunk][head of the group][D + 2] floats: output (unnormalised), maximum (log2 domain), sum
__global__ __launch_bounds__(256, 2) void attn_chunk_kernel(const bf16_t *__restrict__ qp, const bf16_t *__restrict__ k_pages,
                                                            const bf16_t *__restrict__ v_pages, const int32_t *__restrict__ block_table,
                                                            const int32_t *__restrict__ seq_lens, float *__restrict__ part,
                                                            int Hq, int Hkv, int max_pages, int n_chunks, float scale_log2) {
    __shared__ float red[4][MAXG][D + 2];
    const int bh = blockIdx.x, b = bh / Hkv, h = bh - b * Hkv, chunk = blockIdx.y;
    const int n = seq_lens[b];
    const int tok0 = chunk * CHUNK;
    if (tok0 >= n) return;
    const int group = Hq / Hkv;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, c = lane & 15, q = lane >> 4;

    // the group's queries as the B operand: column c = head c of the group, features 32 i + 8 q .. + 7
    u32x4 qop[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        qop[i] = u32x4{0u, 0u, 0u, 0u};
        if (c < group) qop[i] = ld16(qp + ((size_t)b * Hq + h * group + c) * D + 32 * i + 8 * q);
    }
    float m = kNegBig, lsum = 0.f;                 // of head c; lsum covers this lane's positions only
    f32x4 acc[8];
#pragma unroll
    for (int c8 = 0; c8 < 8; ++c8) acc[c8] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int steps = min(CHUNK, n - tok0 + STEP - 1) / STEP;         // steps of this chunk that hold a valid position
    // A wave's steps are 256 positions apart, i.e. one page each.  The keys of a step are loaded one step ahead (their
    // registers are free as soon as the scores are formed), its values at the start of the step: 16 KB of each per wave.
    u32x4 kr[4][4], vr[8][2];
    auto page_of = [&](int s) { return block_table[(size_t)b * max_pages + ((tok0 + s * STEP) >> 8)]; };
    auto load_keys = [&](int s, int page) {
        const bf16_t *kp = k_pages + ((size_t)page * Hkv + h) * PAGE * D + (size_t)((tok0 + s * STEP) & (PAGE - 1)) * D;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) kr[t][i] = ld16(kp + (size_t)(8 * (c >> 2) + (c & 3) + 4 * (t & 1) + 32 * (t >> 1)) * D + 32 * i + 8 * q);
    };
    int page = wave < steps ? page_of(wave) : 0;
    if (wave < steps) load_keys(wave, page);
    for (int s = wave; s < steps; s += 4) {
        const int t0 = tok0 + s * STEP;                                // first position of the step
        const bf16_t *vp = v_pages + ((size_t)page * Hkv + h) * D * PAGE + (t0 & (PAGE - 1));
#pragma unroll
        for (int c8 = 0; c8 < 8; ++c8)
#pragma unroll
            for (int u = 0; u < 2; ++u) vr[c8][u] = ld16(vp + (size_t)(16 * c8 + c) * PAGE + 32 * u + 8 * q);
        const int page_next = s + 4 < steps ? page_of(s + 4) : 0;

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
        if (s + 4 < steps) load_keys(s + 4, page_next);                // the key registers are free: next step's keys
        page = page_next;
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
                    for (int w = 0; w < 4; ++w) {
                        const int e = 32 * u + 2 * w;                   // positions 8 q + e, + 1 of the step
                        const unsigned int keep = (e < left ? 0xFFFFu : 0u) | (e + 1 < left ? 0xFFFF0000u : 0u);
                        vr[c8][u][w] &= keep;
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
    }
    // this lane's share of the sums -> the head's sum
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);

    // ---- merge the four waves ------------------------------------------------------------------------------------
#pragma unroll
    for (int c8 = 0; c8 < 8; ++c8)
#pragma unroll
        for (int j = 0; j < 4; ++j) red[wave][4 * q + j][16 * c8 + c] = acc[c8][j];
    if (q == 0) {
        red[wave][c][D] = m;
        red[wave][c][D + 1] = lsum;
    }
    __syncthreads();
    float *dst = part + ((size_t)bh * n_chunks + chunk) * group * (D + 2);
    for (int idx = threadIdx.x; idx < group * (D + 2); idx += 256) {
        const int head = idx / (D + 2), d = idx - head * (D + 2);
        const float m0 = red[0][head][D], m1 = red[1][head][D], m2 = red[2][head][D], m3 = red[3][head][D];
        const float M = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));          // wave 0 always has a step, so M is finite
        float v;
        if (d == D) v = M;
        else v = ((red[0][head][d] * exp2f(m0 - M) + red[1][head][d] * exp2f(m1 - M)) + red[2][head][d] * exp2f(m2 - M)) +
                 red[3][head][d] * exp2f(m3 - M);                      // d == D + 1: the sums, same weights
        dst[idx] = v;
    }
}

// out[b, head, :] from the chunk partials, in chunk order
__global__ __launch_bounds__(128) void attn_merge_kernel(const float *__restrict__ part, const int32_t *__restrict__ seq_lens,
                                                         bf16_t *__restrict__ out, int Hq, int Hkv, int n_chunks) {
    const int b = blockIdx.x / Hq, jh = blockIdx.x - b * Hq, group = Hq / Hkv;
    const int h = jh / group, head = jh - h * group, d = threadIdx.x;
    const int n = seq_lens[b];
    const int used = (n + CHUNK - 1) / CHUNK;
    float o = 0.f;
    if (used > 0) {
        const float *p = part + (((size_t)(b * Hkv + h) * n_chunks) * group + head) * (D + 2);
        const size_t stride = (size_t)group * (D + 2);
        float M = kNegBig;
        for (int ch = 0; ch < used; ++ch) M = fmaxf(M, p[ch * stride + D]);
        float num = 0.f, den = 0.f;
        for (int ch = 0; ch < used; ++ch) {
            const float w = exp2f(p[ch * stride + D] - M);
            num = fmaf(p[ch * stride + d], w, num);
            den = fmaf(p[ch * stride + D + 1], w, den);
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
    if ((long long)s->B * s->Hkv > 0x7FFFFFFFLL || (long long)s->max_pages * PAGE > 0x7FFFFFFFLL) return 2;
    return 0;
}
int chunks_of(const attn_shape_t &s) { return (s.max_pages * PAGE + CHUNK - 1) / CHUNK; }
size_t ws_bytes_of(const attn_shape_t &s) {
    return align256((size_t)s.B * s.Hkv * chunks_of(s) * (s.Hq / s.Hkv) * (D + 2) * sizeof(float));
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
    const int nch = attn::chunks_of(s);
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)attn::D);
    hipLaunchKernelGGL(attn::attn_chunk_kernel, dim3(s.B * s.Hkv, nch), dim3(256), 0, hs, (const bf16_t *)q, (const bf16_t *)k_pages,
                       (const bf16_t *)v_pages, block_table, seq_lens, (float *)ws, s.Hq, s.Hkv, s.max_pages, nch, scale_log2);
    if (hipGetLastError() != hipSuccess) return 6;
    hipLaunchKernelGGL(attn::attn_merge_kernel, dim3(s.B * s.Hq), dim3(attn::D), 0, hs, (const float *)ws, seq_lens, (bf16_t *)out, s.Hq,
                       s.Hkv, nch);
    return hipGetLastError() == hipSuccess ? 0 : 6;
}

}  // extern "C"
