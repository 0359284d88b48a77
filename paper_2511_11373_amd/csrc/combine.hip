// Weighted combine: out[t,:] = sum_k w[t,k] * y_perm[assign_to_row[t*K+k],:], float accumulation in
// increasing k, one rounding to the storage type.
#include "moe_internal.hpp"

namespace moe {

__device__ __forceinline__ void load8f(const bf16_t *p, float (&v)[8]) {
    const u32x4 r = load_once(p);                    // every expert output row is read once
#pragma unroll
    for (int j = 0; j < 4; ++j) { v[2 * j] = __uint_as_float(r[j] << 16); v[2 * j + 1] = __uint_as_float(r[j] & 0xFFFF0000u); }
}
__device__ __forceinline__ void load8f(const float *p, float (&v)[8]) {
    const f32x4 a = *reinterpret_cast<const f32x4 *>(p), b = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
    for (int j = 0; j < 4; ++j) { v[j] = a[j]; v[4 + j] = b[j]; }
}
__device__ __forceinline__ void store8f(bf16_t *p, const float (&v)[8]) {
    u32x4 r = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
    *reinterpret_cast<u32x4 *>(p) = r;
}
__device__ __forceinline__ void store8f(float *p, const float (&v)[8]) {
    f32x4 a = {v[0], v[1], v[2], v[3]}, b = {v[4], v[5], v[6], v[7]};
    *reinterpret_cast<f32x4 *>(p) = a;
    *reinterpret_cast<f32x4 *>(p + 4) = b;
}

// One block per (token, slab of 2048 features); each thread owns 8 consecutive features.  The K row
// ids and weights of a group of 8 slots are fetched first so that the 8 row loads are independent.
template <typename S>
__global__ __launch_bounds__(256) void combine_kernel(const S *__restrict__ y, const int32_t *__restrict__ a2r,
                                                      const float *__restrict__ w, S *__restrict__ out, int T, int H, int K) {
    const int t = blockIdx.x;
    const int h = (blockIdx.y * 256 + threadIdx.x) * 8;
    if (t >= T || h >= H) return;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const int32_t *rows = a2r + (size_t)t * K;
    const float *wk = w + (size_t)t * K;
    for (int k0 = 0; k0 < K; k0 += 8) {
        int row[8]; float wt[8]; float v[8][8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool ok = k0 + j < K;
            row[j] = ok ? rows[k0 + j] : rows[0];
            wt[j] = ok ? wk[k0 + j] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) load8f(y + (size_t)row[j] * H + h, v[j]);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (k0 + j < K) {
#pragma unroll
                for (int f = 0; f < 8; ++f) acc[f] = fmaf(wt[j], v[j][f], acc[f]);
            }
    }
    store8f(out + (size_t)t * H + h, acc);
}

hipError_t launch_combine(const moe_shape_t &s, const void *y_perm, const int32_t *assign_to_row,
                          const float *topk_w, void *out, hipStream_t st) {
    dim3 grid(s.T, (s.H + 2047) / 2048);
    if (s.dtype == MOE_BF16)
        hipLaunchKernelGGL(combine_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t *)y_perm, assign_to_row,
                           topk_w, (bf16_t *)out, s.T, s.H, s.K);
    else
        hipLaunchKernelGGL(combine_kernel<float>, grid, dim3(256), 0, st, (const float *)y_perm, assign_to_row,
                           topk_w, (float *)out, s.T, s.H, s.K);
    return hipGetLastError();
}

}  // namespace moe
