// Router: logits on the fp64 matrix cores, then top-K selection and routing
// weights with one wavefront per token.
//
// The logit of (token, expert) is the dot product of two rows of bf16 (or float)
// numbers.  Every such product is exact in double, and for inputs of ordinary
// dynamic range so is their sum, so the float the sum is rounded to does not
// depend on the order of summation.  That is what lets an independently written
// reference reproduce the selection bit for bit.
#include "moe_internal.hpp"

namespace moe {

// ---- operand loads: 8 consecutive stored elements widened to double -----------------------
__device__ __forceinline__ void load8_as_double(const bf16_t *p, bool ok, double (&d)[8]) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (ok) v = *reinterpret_cast<const u32x4 *>(p);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        d[2 * j]     = (double)__uint_as_float(v[j] << 16);
        d[2 * j + 1] = (double)__uint_as_float(v[j] & 0xFFFF0000u);
    }
}
__device__ __forceinline__ void load8_as_double(const float *p, bool ok, double (&d)[8]) {
    f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
    if (ok) {
        a = *reinterpret_cast<const f32x4 *>(p);
        b = *reinterpret_cast<const f32x4 *>(p + 4);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) { d[j] = (double)a[j]; d[4 + j] = (double)b[j]; }
}

// One wave: 16 tokens x 32 experts (two 16x16 accumulators) over a range of 32-wide k chunks.
// v_mfma_f64_16x16x4_f64 operand layout: lane l supplies A[l%16][l/16] and B[l/16][l%16]; result
// register r of lane l is D[4*r + l/16][l%16].  Which four k values share one instruction is free as
// long as A and B agree: lane (row, q) loads 8 consecutive elements at k = 32*c + 8*q and feeds
// element j to the j-th instruction of the chunk.
template <typename S>
__global__ __launch_bounds__(256) void router_logits_kernel(const S *__restrict__ x, const S *__restrict__ wr,
                                                            double *__restrict__ part, int T, int H, int E,
                                                            int chunks_per_split) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int pair = blockIdx.y * 4 + wave;
    const int npairs = (E + 31) >> 5;
    if (pair >= npairs) return;
    const int row = lane & 15, q = lane >> 4;
    const int nchunks = (H + 31) >> 5;
    const int c0 = blockIdx.z * chunks_per_split;
    const int c1 = min(c0 + chunks_per_split, nchunks);

    const int tok = min(blockIdx.x * 16 + row, T - 1);
    const int ea = min(pair * 32 + row, E - 1);
    const int eb = min(pair * 32 + 16 + row, E - 1);
    const S *px = x + (size_t)tok * H + q * 8;
    const S *pa = wr + (size_t)ea * H + q * 8;
    const S *pb = wr + (size_t)eb * H + q * 8;

    f64x4 acc0 = {0., 0., 0., 0.}, acc1 = {0., 0., 0., 0.};
    for (int c = c0; c < c1; ++c) {
        const bool ok = (c * 32 + q * 8) < H;   // H is a multiple of 8
        double dx[8], da[8], db[8];
        load8_as_double(px + c * 32, ok, dx);
        load8_as_double(pa + c * 32, ok, da);
        load8_as_double(pb + c * 32, ok, db);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(dx[j], da[j], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(dx[j], db[j], acc1, 0, 0, 0);
        }
    }
    double *dst = part + (size_t)blockIdx.z * T * E;
    const int e_lo = pair * 32 + row;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int t = blockIdx.x * 16 + 4 * r + q;
        if (t < T) {
            if (e_lo < E) dst[(size_t)t * E + e_lo] = acc0[r];
            if (e_lo + 16 < E) dst[(size_t)t * E + e_lo + 16] = acc1[r];
        }
    }
}

// ---- top-K and weights ---------------------------------------------------------------------
__device__ __forceinline__ unsigned int float_order_bits(float f) {
    if (f == 0.0f) f = 0.0f;   // -0 and +0 compare equal
    unsigned int u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float order_bits_float(unsigned int o) {
    return __uint_as_float((o & 0x80000000u) ? (o ^ 0x80000000u) : ~o);
}
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        unsigned long long o = __shfl_xor(v, m, 64);
        v = o > v ? o : v;
    }
    return v;
}
__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// logit of (t, e): the partial sums of the k splits added in split order, plus the bias, in double,
// rounded once to float.
__device__ __forceinline__ float final_logit(const double *__restrict__ part, int ksplit, size_t split_stride,
                                             size_t pos, const float *__restrict__ bias, int e) {
    double s = 0.0;
    int z = 0;
    for (; z + 4 <= ksplit; z += 4) {
        const double a = part[pos + (size_t)z * split_stride], b = part[pos + (size_t)(z + 1) * split_stride];
        const double c = part[pos + (size_t)(z + 2) * split_stride], d = part[pos + (size_t)(z + 3) * split_stride];
        s = (((s + a) + b) + c) + d;
    }
    for (; z < ksplit; ++z) s += part[pos + (size_t)z * split_stride];
    if (bias) s += (double)bias[e];
    return (float)s;
}

// Weights from the selected logits sel[0..K) (descending) of one token; all lanes of the wave call it.
__device__ __forceinline__ void write_weights(const float *sel, int K, int renorm, float denom_all,
                                              float *__restrict__ dst, int lane) {
    const float m = sel[0];
    float denom = denom_all;
    if (renorm) {
        float part_sum = 0.f;
        for (int k = lane; k < K; k += 64) part_sum += expf(sel[k] - m);
        denom = wave_sum_f32(part_sum);
    }
    for (int k = lane; k < K; k += 64) dst[k] = expf(sel[k] - m) / denom;
}

// One wave per token.  Lane l holds the logits of experts l, l+64, ...  Each of the K rounds takes
// the wave-wide maximum of the key (ordered logit bits, ~expert id), so equal logits go to the lower id.
template <int R>
__global__ __launch_bounds__(256) void topk_kernel(const double *__restrict__ part, int ksplit,
                                                   const float *__restrict__ bias, int32_t *__restrict__ topk_idx,
                                                   float *__restrict__ topk_w, int T, int E, int K, int renorm) {
    extern __shared__ float sel_all[];   // [4][K] selected logits, one row per wave
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + wave;
    if (t >= T) return;
    float *sel = sel_all + (size_t)wave * K;

    float logit[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int e = lane + 64 * r;
        logit[r] = e < E ? final_logit(part, ksplit, (size_t)T * E, (size_t)t * E + e, bias, e) : 0.f;
    }
    unsigned int taken = 0;
    for (int k = 0; k < K; ++k) {
        unsigned long long best = 0ull;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int e = lane + 64 * r;
            if (e < E && !((taken >> r) & 1u)) {
                unsigned long long key = ((unsigned long long)float_order_bits(logit[r]) << 32) |
                                         (unsigned long long)(0xFFFFFFFFu - (unsigned int)e);
                best = key > best ? key : best;
            }
        }
        best = wave_max_u64(best);
        const int e_win = (int)(0xFFFFFFFFu - (unsigned int)(best & 0xFFFFFFFFull));
        if ((e_win & 63) == lane) taken |= 1u << (e_win >> 6);
        if (lane == 0) {
            topk_idx[(size_t)t * K + k] = e_win;
            sel[k] = order_bits_float((unsigned int)(best >> 32));
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float denom_all = 0.f;
    if (!renorm) {
        const float m = sel[0];
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (lane + 64 * r < E) denom_all += expf(logit[r] - m);
        denom_all = wave_sum_f32(denom_all);
    }
    write_weights(sel, K, renorm, denom_all, topk_w + (size_t)t * K, lane);
}

// Same result for E <= 64*R <= 256 without a serial chain: every lane counts, for each of its
// logits, how many (logit, id) pairs of the token precede it; that count is its slot.
template <int R>
__global__ __launch_bounds__(256) void topk_rank_kernel(const double *__restrict__ part, int ksplit,
                                                        const float *__restrict__ bias, int32_t *__restrict__ topk_idx,
                                                        float *__restrict__ topk_w, int T, int E, int K, int renorm) {
    __shared__ __attribute__((aligned(16))) unsigned int keys_all[4][R * 64];
    __shared__ float sel_all[4][R * 64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + wave;
    if (t >= T) return;
    unsigned int *keys = keys_all[wave];
    float *sel = sel_all[wave];
    float logit[R];
    unsigned int key[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int e = lane + 64 * r;
        logit[r] = e < E ? final_logit(part, ksplit, (size_t)T * E, (size_t)t * E + e, bias, e) : 0.f;
        key[r] = e < E ? float_order_bits(logit[r]) : 0u;     // 0 sorts below every finite float
        keys[e] = key[r];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    int rank[R];
#pragma unroll
    for (int r = 0; r < R; ++r) rank[r] = 0;
    for (int e4 = 0; e4 < R * 64; e4 += 4) {
        const u32x4 k4 = *reinterpret_cast<const u32x4 *>(&keys[e4]);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int e = lane + 64 * r;
                rank[r] += (k4[j] > key[r]) || (k4[j] == key[r] && (e4 + j) < e);
            }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int e = lane + 64 * r;
        if (e < E && rank[r] < K) {
            topk_idx[(size_t)t * K + rank[r]] = e;
            sel[rank[r]] = logit[r];
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float denom_all = 0.f;
    if (!renorm) {
        const float m = sel[0];
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (lane + 64 * r < E) denom_all += expf(logit[r] - m);
        denom_all = wave_sum_f32(denom_all);
    }
    write_weights(sel, K, renorm, denom_all, topk_w + (size_t)t * K, lane);
}

int router_ksplit(const moe_shape_t &s) {
    const long waves = (long)((s.T + 15) / 16) * ((s.E + 31) / 32);
    const int nchunks = (s.H + 31) / 32;
    long ks = waves >= 1024 ? 1 : (1024 + waves - 1) / (waves > 0 ? waves : 1);
    if (ks > kMaxLogitSplit) ks = kMaxLogitSplit;
    if (ks > nchunks) ks = nchunks;
    const int cps = (nchunks + (int)ks - 1) / (int)ks;
    return (nchunks + cps - 1) / cps;
}

hipError_t launch_route(const moe_shape_t &s, const void *x, const void *w_router, const float *bias,
                        double *logit_part, int32_t *topk_idx, float *topk_w, hipStream_t st, Probe *probe) {
    const int ks = router_ksplit(s);
    const int nchunks = (s.H + 31) / 32;
    const int cps = (nchunks + ks - 1) / ks;
    const int npairs = (s.E + 31) / 32;
    dim3 grid((s.T + 15) / 16, (npairs + 3) / 4, ks);
    if (s.dtype == MOE_BF16)
        hipLaunchKernelGGL(router_logits_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t *)x,
                           (const bf16_t *)w_router, logit_part, s.T, s.H, s.E, cps);
    else
        hipLaunchKernelGGL(router_logits_kernel<float>, grid, dim3(256), 0, st, (const float *)x,
                           (const float *)w_router, logit_part, s.T, s.H, s.E, cps);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    probe_mark(probe);

    dim3 g2((s.T + 3) / 4);
    const size_t smem = (size_t)4 * s.K * sizeof(float);
    const int r = (s.E + 63) / 64;
#define MOE_TOPK(RR)                                                                                   \
    hipLaunchKernelGGL(topk_kernel<RR>, g2, dim3(256), smem, st, logit_part, ks, bias, topk_idx, topk_w, \
                       s.T, s.E, s.K, s.renormalize)
#define MOE_TOPK_RANK(RR)                                                                              \
    hipLaunchKernelGGL(topk_rank_kernel<RR>, g2, dim3(256), 0, st, logit_part, ks, bias, topk_idx, topk_w, \
                       s.T, s.E, s.K, s.renormalize)
    if (r <= 1) MOE_TOPK_RANK(1);
    else if (r <= 2) MOE_TOPK_RANK(2);
    else if (r <= 4) MOE_TOPK_RANK(4);
#undef MOE_TOPK_RANK
    else if (r <= 8) MOE_TOPK(8);
    else MOE_TOPK(16);
#undef MOE_TOPK
    return hipGetLastError();
}

}  // namespace moe
