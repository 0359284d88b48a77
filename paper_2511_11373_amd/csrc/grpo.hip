// Token log-probability and GRPO objective (Section 2.2, Eq. 1-3): one streaming pass over the logits with an
// online log-sum-exp, the per-token surrogate in the same kernel, and small fixed-order reductions for the
// response means and the objective.  The logits pass is bound by HBM: N*V stored elements read exactly once.
#include <float.h>

#include "grpo_loss.h"
#include "moe_internal.hpp"

namespace moe {

constexpr float kNegHuge = -3.0e38f;   // stands in for -inf: exp(kNegHuge - x) underflows to 0 and never makes a NaN

__device__ __forceinline__ void unpack8(const bf16_t *p, float (&v)[8]) {
    const u32x4 r = load_once(p);                    // the logits are read once
#pragma unroll
    for (int j = 0; j < 4; ++j) { v[2 * j] = __uint_as_float(r[j] << 16); v[2 * j + 1] = __uint_as_float(r[j] & 0xFFFF0000u); }
}
__device__ __forceinline__ void unpack8(const float *p, float (&v)[8]) {
    const f32x4 a = *reinterpret_cast<const f32x4 *>(p), b = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
    for (int j = 0; j < 4; ++j) { v[j] = a[j]; v[4 + j] = b[j]; }
}
__device__ __forceinline__ float load1(const bf16_t *p) { return __uint_as_float((unsigned int)*p << 16); }
__device__ __forceinline__ float load1(const float *p) { return *p; }

// running (maximum, sum of exp(v - maximum)) absorbs 8 more values
__device__ __forceinline__ void absorb8(float &m, float &s, const float (&v)[8]) {
    float mx = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
    const float mn = fmaxf(m, mx);
    float acc = s * __expf(m - mn);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc += __expf(v[j] - mn);
    s = acc;
    m = mn;
}
__device__ __forceinline__ void merge(float &m, float &s, float m2, float s2) {
    const float mn = fmaxf(m, m2);
    s = s * __expf(m - mn) + s2 * __expf(m2 - mn);
    m = mn;
}

// Eq. 2's inner bracket for one token
__device__ __forceinline__ float surrogate_term(float logp, float old, float ref, float adv, float clip_eps, float beta) {
    const float ratio = expf(logp - old);
    const float clipped = fminf(fmaxf(ratio, 1.0f - clip_eps), 1.0f + clip_eps);
    const float d = ref - logp;
    const float kl = expf(d) - d - 1.0f;
    return fminf(ratio * adv, clipped * adv) - beta * kl;
}
// response that owns token t: the last i with off[i] <= t (empty responses are skipped by construction)
__device__ __forceinline__ int response_of(const int32_t *__restrict__ off, int G, int t) {
    int lo = 0, hi = G;            // invariant: off[lo] <= t < off[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

// One block per token row.  Every thread keeps four 16-byte loads in flight.
template <typename S, bool WITH_TERM>
__global__ __launch_bounds__(256) void logprob_kernel(const S *__restrict__ logits, const int32_t *__restrict__ target,
                                                      float *__restrict__ logp_out, int V, const float *__restrict__ logp_old,
                                                      const float *__restrict__ logp_ref, const float *__restrict__ adv,
                                                      const int32_t *__restrict__ off, int G, float clip_eps, float beta,
                                                      float *__restrict__ term_out) {
    __shared__ float red_m[4], red_s[4];
    const int t = blockIdx.x, tid = threadIdx.x;
    const S *row = logits + (size_t)t * V;
    const int nchunk = V >> 3;
    float m = kNegHuge, s = 0.f;
    int c = tid;
    for (; c + 768 < nchunk; c += 1024) {
        float v0[8], v1[8], v2[8], v3[8];
        unpack8(row + (size_t)c * 8, v0);
        unpack8(row + (size_t)(c + 256) * 8, v1);
        unpack8(row + (size_t)(c + 512) * 8, v2);
        unpack8(row + (size_t)(c + 768) * 8, v3);
        absorb8(m, s, v0);
        absorb8(m, s, v1);
        absorb8(m, s, v2);
        absorb8(m, s, v3);
    }
    for (; c < nchunk; c += 256) {
        float v0[8];
        unpack8(row + (size_t)c * 8, v0);
        absorb8(m, s, v0);
    }
#pragma unroll
    for (int k = 32; k >= 1; k >>= 1) merge(m, s, __shfl_xor(m, k, 64), __shfl_xor(s, k, 64));
    if ((tid & 63) == 0) { red_m[tid >> 6] = m; red_s[tid >> 6] = s; }
    __syncthreads();
    if (tid == 0) {
        m = red_m[0]; s = red_s[0];
#pragma unroll
        for (int w = 1; w < 4; ++w) merge(m, s, red_m[w], red_s[w]);
        int tg = target[t];
        tg = tg < 0 ? 0 : (tg >= V ? V - 1 : tg);
        const float lp = (load1(row + tg) - m) - logf(s);     // subtract the maximum first: no cancellation at large offsets
        logp_out[t] = lp;
        if (WITH_TERM) {
            const int i = response_of(off, G, t);
            term_out[t] = surrogate_term(lp, logp_old[t], logp_ref[t], adv[i], clip_eps, beta);
        }
    }
}

// Eq. 1 for one group: population mean and standard deviation, fixed summation order.
__global__ __launch_bounds__(256) void advantage_kernel(const float *__restrict__ rewards, int G, float adv_eps,
                                                        float *__restrict__ adv) {
    __shared__ float red[256];
    const int tid = threadIdx.x;
    float a = 0.f;
    for (int i = tid; i < G; i += 256) a += rewards[i];
    red[tid] = a;
    __syncthreads();
    for (int k = 128; k >= 1; k >>= 1) { if (tid < k) red[tid] += red[tid + k]; __syncthreads(); }
    const float mean = red[0] / (float)G;
    __syncthreads();
    float q = 0.f;
    for (int i = tid; i < G; i += 256) { const float d = rewards[i] - mean; q += d * d; }
    red[tid] = q;
    __syncthreads();
    for (int k = 128; k >= 1; k >>= 1) { if (tid < k) red[tid] += red[tid + k]; __syncthreads(); }
    const float sd = sqrtf(red[0] / (float)G);
    for (int i = tid; i < G; i += 256) adv[i] = (rewards[i] - mean) / (sd + adv_eps);
}

// token terms from given log-probabilities (the stand-alone objective entry point)
__global__ __launch_bounds__(256) void term_kernel(const float *__restrict__ logp, const float *__restrict__ logp_old,
                                                   const float *__restrict__ logp_ref, const float *__restrict__ adv,
                                                   const int32_t *__restrict__ off, int N, int G, float clip_eps, float beta,
                                                   float *__restrict__ term_out) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= N) return;
    term_out[t] = surrogate_term(logp[t], logp_old[t], logp_ref[t], adv[response_of(off, G, t)], clip_eps, beta);
}

// response means and the objective: one block of 16 waves.  W waves share a response (W = 16 for one response,
// 1 from 16 responses on); every lane strides over its share of the response's tokens, a butterfly adds the 64
// partial sums, the W wave sums are added in wave order, and thread 0 adds the means in response order.
__global__ __launch_bounds__(1024) void objective_kernel(const float *__restrict__ term, const int32_t *__restrict__ off, int G,
                                                         float *__restrict__ resp_mean, float *__restrict__ objective) {
    __shared__ float part[16];
    __shared__ float jsum;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int W = 16;
    while (W > 1 && 16 / W < G) W >>= 1;
    const int per_round = 16 / W, sub = wave % W;
    if (threadIdx.x == 0) jsum = 0.f;
    for (int i0 = 0; i0 < G; i0 += per_round) {
        const int i = i0 + wave / W;
        float a = 0.f;
        int b = 0, e = 0;
        if (i < G) {
            b = off[i];
            e = off[i + 1];
            for (int t = b + sub * 64 + lane; t < e; t += W * 64) a += term[t];
#pragma unroll
            for (int k = 32; k >= 1; k >>= 1) a += __shfl_xor(a, k, 64);
        }
        if (lane == 0) part[wave] = a;
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int r = 0; r < per_round && i0 + r < G; ++r) {
                float sum = 0.f;
                for (int j = 0; j < W; ++j) sum += part[r * W + j];
                const int n = off[i0 + r + 1] - off[i0 + r];
                const float mean = n > 0 ? sum / (float)n : 0.f;
                resp_mean[i0 + r] = mean;
                jsum += mean;
            }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) objective[0] = G > 0 ? jsum / (float)G : 0.f;
}

static moe_status_t check_grpo(const grpo_shape_t *s) {
    if (!s) return MOE_ERR_NULL;
    if (s->dtype != MOE_BF16 && s->dtype != MOE_F32) return MOE_ERR_DTYPE;
    if (s->N < 0 || s->G < 0 || s->V < 8 || s->V % 8 != 0) return MOE_ERR_SHAPE;
    return MOE_OK;
}
static bool bad_align(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

}  // namespace moe

using namespace moe;

extern "C" {

moe_status_t grpo_token_logprob(const grpo_shape_t *shape, const void *logits, const int32_t *target,
                                float *logp, void *stream) {
    moe_status_t st = check_grpo(shape);
    if (st != MOE_OK) return st;
    if (!logits || !target || !logp) return MOE_ERR_NULL;
    if (bad_align(logits) || bad_align(target) || bad_align(logp)) return MOE_ERR_ALIGN;
    if (shape->N == 0) return MOE_OK;
    hipStream_t hs = (hipStream_t)stream;
    if (shape->dtype == MOE_BF16)
        hipLaunchKernelGGL((logprob_kernel<bf16_t, false>), dim3(shape->N), dim3(256), 0, hs, (const bf16_t *)logits, target, logp,
                           shape->V, nullptr, nullptr, nullptr, nullptr, 0, 0.f, 0.f, nullptr);
    else
        hipLaunchKernelGGL((logprob_kernel<float, false>), dim3(shape->N), dim3(256), 0, hs, (const float *)logits, target, logp,
                           shape->V, nullptr, nullptr, nullptr, nullptr, 0, 0.f, 0.f, nullptr);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status_t grpo_objective(const grpo_shape_t *shape, const float *logp, const float *logp_old,
                            const float *logp_ref, const float *rewards, const int32_t *resp_offsets,
                            float *advantage, float *token_term, float *resp_mean, float *objective,
                            void *stream) {
    moe_status_t st = check_grpo(shape);
    if (st != MOE_OK) return st;
    if (!logp || !logp_old || !logp_ref || !rewards || !resp_offsets || !advantage || !resp_mean || !objective || !token_term)
        return MOE_ERR_NULL;
    if (bad_align(logp) || bad_align(logp_old) || bad_align(logp_ref) || bad_align(rewards) || bad_align(resp_offsets) ||
        bad_align(advantage) || bad_align(token_term) || bad_align(resp_mean) || bad_align(objective))
        return MOE_ERR_ALIGN;
    if (shape->N == 0 || shape->G == 0) return MOE_OK;
    hipStream_t hs = (hipStream_t)stream;
    hipLaunchKernelGGL(advantage_kernel, dim3(1), dim3(256), 0, hs, rewards, shape->G, shape->adv_eps, advantage);
    if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
    hipLaunchKernelGGL(term_kernel, dim3((shape->N + 255) / 256), dim3(256), 0, hs, logp, logp_old, logp_ref, advantage,
                       resp_offsets, shape->N, shape->G, shape->clip_eps, shape->beta, token_term);
    if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
    hipLaunchKernelGGL(objective_kernel, dim3(1), dim3(1024), 0, hs, token_term, resp_offsets, shape->G, resp_mean, objective);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status_t grpo_logprob_objective(const grpo_shape_t *shape, const void *logits, const int32_t *target,
                                    const float *logp_old, const float *logp_ref, const float *rewards,
                                    const int32_t *resp_offsets, float *logp, float *advantage,
                                    float *token_term, float *resp_mean, float *objective, void *stream) {
    moe_status_t st = check_grpo(shape);
    if (st != MOE_OK) return st;
    if (!logits || !target || !logp_old || !logp_ref || !rewards || !resp_offsets || !logp || !advantage || !token_term ||
        !resp_mean || !objective)
        return MOE_ERR_NULL;
    if (bad_align(logits) || bad_align(target) || bad_align(logp_old) || bad_align(logp_ref) || bad_align(rewards) ||
        bad_align(resp_offsets) || bad_align(logp) || bad_align(advantage) || bad_align(token_term) || bad_align(resp_mean) ||
        bad_align(objective))
        return MOE_ERR_ALIGN;
    if (shape->N == 0 || shape->G == 0) return MOE_OK;
    hipStream_t hs = (hipStream_t)stream;
    hipLaunchKernelGGL(advantage_kernel, dim3(1), dim3(256), 0, hs, rewards, shape->G, shape->adv_eps, advantage);
    if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
    if (shape->dtype == MOE_BF16)
        hipLaunchKernelGGL((logprob_kernel<bf16_t, true>), dim3(shape->N), dim3(256), 0, hs, (const bf16_t *)logits, target, logp,
                           shape->V, logp_old, logp_ref, advantage, resp_offsets, shape->G, shape->clip_eps, shape->beta, token_term);
    else
        hipLaunchKernelGGL((logprob_kernel<float, true>), dim3(shape->N), dim3(256), 0, hs, (const float *)logits, target, logp,
                           shape->V, logp_old, logp_ref, advantage, resp_offsets, shape->G, shape->clip_eps, shape->beta, token_term);
    if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
    hipLaunchKernelGGL(objective_kernel, dim3(1), dim3(1024), 0, hs, token_term, resp_offsets, shape->G, resp_mean, objective);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // extern "C"
