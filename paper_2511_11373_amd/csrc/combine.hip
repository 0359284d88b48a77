// Weighted combine: out[t,:] = sum_k w[t,k] * y_perm[assign_to_row[t*K+k],:], float accumulation in
// increasing k, one rounding to the storage type.  One wave per token, 8 features per lane per step.
#include "moe_internal.hpp"

namespace moe {

__device__ __forceinline__ void load8f(const bf16_t *p, float (&v)[8]) {
    const u32x4 r = *reinterpret_cast<const u32x4 *>(p);
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

template <typename S>
__global__ __launch_bounds__(256) void combine_kernel(const S *__restrict__ y, const int32_t *__restrict__ a2r,
                                                      const float *__restrict__ w, S *__restrict__ out, int T, int H, int K) {
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const int lane = threadIdx.x & 63;
    for (int h = lane * 8; h < H; h += 64 * 8) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int k = 0; k < K; ++k) {
            const int row = a2r[(size_t)t * K + k];
            const float wk = w[(size_t)t * K + k];
            float v[8];
            load8f(y + (size_t)row * H + h, v);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = fmaf(wk, v[j], acc[j]);
        }
        store8f(out + (size_t)t * H + h, acc);
    }
}

hipError_t launch_combine(const moe_shape_t &s, const void *y_perm, const int32_t *assign_to_row,
                          const float *topk_w, void *out, hipStream_t st) {
    dim3 grid((s.T + 3) / 4);
    if (s.dtype == MOE_BF16)
        hipLaunchKernelGGL(combine_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t *)y_perm, assign_to_row,
                           topk_w, (bf16_t *)out, s.T, s.H, s.K);
    else
        hipLaunchKernelGGL(combine_kernel<float>, grid, dim3(256), 0, st, (const float *)y_perm, assign_to_row,
                           topk_w, (float *)out, s.T, s.H, s.K);
    return hipGetLastError();
}

}  // namespace moe
