// Backward pass of the MoE FFN block (bf16 storage, renormalised routing weights): entry points, the row-wise
// kernels around the grouped GEMMs of backward_gemm.hip, and the workspace.
//
// With the selection S_t held fixed (it is piecewise constant), for d_out = dL/d_out:
//   out_t = sum_k w_k y_k            dw_k = <d_out_t, y_k> = <d_out_t Wd, a_k>      (no need to rebuild y)
//   w = softmax(l[S_t])              dl_k = w_k (dw_k - sum_j w_j dw_j)
//   l_e = <x_t, Wr_e> + b_e          dx_t += sum_k dl_k Wr_e,  dWr_e += dl x_t,  db_e += dl
//   y = Wd a, a = silu(g) u          da = w_k (d_out_t Wd),  dWd_e += d_out_t (x) (w_k a)
//   g = Wg x, u = Wu x               dg = da u silu'(g),  du = da silu(g),  silu'(g) = s (1 + g (1 - s)),  s = 1/(1+e^-g)
//                                    dWg_e += dg (x) x_t,  dWu_e += du (x) x_t,  dx_t += dg Wg + du Wu
// moe_backward recomputes g, u from x (it takes nothing from a forward call); moe_backward_saved reads the g, u that
// moe_forward_saving wrote.  Intermediates are bf16, sums are float.
#include <type_traits>

#include "moe_internal.hpp"

#include "moe_ffn_backward.h"

namespace moe {

hipError_t launch_bw_rows_kfast(const bf16_t *rows, const bf16_t *w, const int32_t *off, const int32_t *tile_map, int max_tiles,
                                bf16_t *out, int KD, int N, hipStream_t st);
hipError_t launch_bw_rows_kslow(const bf16_t *a0, const bf16_t *a1, const bf16_t *w0, const bf16_t *w1, const int32_t *off,
                                const int32_t *tile_map, int max_tiles, bf16_t *out, int KD, int N, hipStream_t st);
hipError_t launch_bw_wgrad(const bf16_t *P, const bf16_t *Q, const int32_t *off, int E, float *out, int M, int N, hipStream_t st);
bool big_pre_activations_applicable(int H, int I);
hipError_t launch_big_tile_list(const moe_shape_t &s, const int32_t *off, void *list, hipStream_t st);
hipError_t launch_big_pre_activations(const moe_shape_t &s, const bf16_t *rows, const int32_t *row_token, int row_div,
                                      const void *list, const bf16_t *wg, const bf16_t *wu, bf16_t *g, bf16_t *u, hipStream_t st);
bool bw_lds_applicable(const moe_shape_t &s);
hipError_t launch_bw_lds_rows(const moe_shape_t &s, const bf16_t *a0, const bf16_t *a1, const bf16_t *w0, const bf16_t *w1,
                              const void *list, const bf16_t *zeros, const int32_t *a0_token, bf16_t *out, int KD, int N,
                              hipStream_t st);
hipError_t launch_bw_lds_wgrad(const moe_shape_t &s, const bf16_t *P, const bf16_t *Q, const int32_t *off, const bf16_t *zeros,
                               const int32_t *p_token, const int32_t *q_token, float *out, int M, int N, hipStream_t st);
hipError_t launch_build_tile_map(const int32_t *off, int E, int tile_rows, int max_tiles, int32_t *tile_map, hipStream_t st);

namespace {

constexpr int kBwTile = 256;       // row tile of the backward GEMMs

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// One wave per expert-sorted row r: from g, u and dq = d_out_t Wd (all [n][I] bf16) and the row's routing weight w,
//   a = silu(g) u,  dw_row[r] = <dq, a>,  da = w dq,  dg = da u silu'(g),  du = da silu(g),  aw = w a.
__global__ __launch_bounds__(256) void bw_swiglu_kernel(const bf16_t *__restrict__ g, const bf16_t *__restrict__ u,
                                                        const bf16_t *__restrict__ dq, const float *__restrict__ topk_w,
                                                        const int32_t *__restrict__ row_to_assign, bf16_t *__restrict__ dg,
                                                        bf16_t *__restrict__ du, bf16_t *__restrict__ aw,
                                                        float *__restrict__ dw_row, int n, int I) {
    const int lane = threadIdx.x & 63, r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= n) return;
    const float w = topk_w ? topk_w[row_to_assign ? row_to_assign[r] : r] : 1.0f;
    float dot = 0.f;
    for (int p = lane; p < (I >> 3); p += 64) {
        const size_t at = (size_t)r * I + p * 8;
        const u32x4 gv = load_once(g + at), uv = load_once(u + at), qv = load_once(dq + at);      // each read once
        float odg[8], odu[8], oaw[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float gf = __uint_as_float((j & 1) ? (gv[j >> 1] & 0xFFFF0000u) : (gv[j >> 1] << 16));
            const float uf = __uint_as_float((j & 1) ? (uv[j >> 1] & 0xFFFF0000u) : (uv[j >> 1] << 16));
            const float qf = __uint_as_float((j & 1) ? (qv[j >> 1] & 0xFFFF0000u) : (qv[j >> 1] << 16));
            const float s = 1.0f / (1.0f + __expf(-gf));
            const float a = gf * s * uf;
            dot = fmaf(qf, a, dot);
            const float da = w * qf;
            odg[j] = da * uf * (s * (1.0f + gf * (1.0f - s)));
            odu[j] = da * (gf * s);
            oaw[j] = w * a;
        }
        *reinterpret_cast<u32x4 *>(dg + at) = u32x4{pack_bf16x2(odg[0], odg[1]), pack_bf16x2(odg[2], odg[3]), pack_bf16x2(odg[4], odg[5]), pack_bf16x2(odg[6], odg[7])};
        *reinterpret_cast<u32x4 *>(du + at) = u32x4{pack_bf16x2(odu[0], odu[1]), pack_bf16x2(odu[2], odu[3]), pack_bf16x2(odu[4], odu[5]), pack_bf16x2(odu[6], odu[7])};
        *reinterpret_cast<u32x4 *>(aw + at) = u32x4{pack_bf16x2(oaw[0], oaw[1]), pack_bf16x2(oaw[2], oaw[3]), pack_bf16x2(oaw[4], oaw[5]), pack_bf16x2(oaw[6], oaw[7])};
    }
    dot = wave_sum(dot);
    if (lane == 0 && dw_row) dw_row[r] = dot;
}

// One thread per token: dl_k = w_k (dw_k - sum_j w_j dw_j), written per assignment and, over the dw it came from, per row.
__global__ __launch_bounds__(256) void bw_softmax_kernel(const float *__restrict__ topk_w, float *__restrict__ dw_row,
                                                         const int32_t *__restrict__ assign_to_row, float *__restrict__ dl,
                                                         int T, int K) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= T) return;
    float mean = 0.f;
    for (int k = 0; k < K; ++k) mean = fmaf(topk_w[(size_t)t * K + k], dw_row[assign_to_row[(size_t)t * K + k]], mean);
    for (int k = 0; k < K; ++k) {
        const size_t a = (size_t)t * K + k;
        const int row = assign_to_row[a];
        const float v = topk_w[a] * (dw_row[row] - mean);
        dl[a] = v;
        dw_row[row] = v;        // only this thread touches the rows of its token
    }
}

// Un-renormalised routing weights (w_k = p_{e_k}, p the softmax over all E logits): every logit of a token receives a
// gradient, dl_e = p_e ([e selected] dw_e - sum_k w_k dw_k).  One thread per token; probs [T][E] is overwritten by dl.
__global__ __launch_bounds__(256) void bw_softmax_dense_kernel(const float *__restrict__ topk_w, const float *__restrict__ dw_row,
                                                               const int32_t *__restrict__ assign_to_row,
                                                               const int32_t *__restrict__ topk_idx, float *__restrict__ probs,
                                                               int T, int K, int E) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= T) return;
    float mean = 0.f;
    for (int k = 0; k < K; ++k) mean = fmaf(topk_w[(size_t)t * K + k], dw_row[assign_to_row[(size_t)t * K + k]], mean);
    float *p = probs + (size_t)t * E;
    for (int e = 0; e < E; ++e) p[e] = -p[e] * mean;
    // the selected experts' extra term, with their probability taken from the routing weights (the same number)
    for (int k = 0; k < K; ++k) {
        const size_t a = (size_t)t * K + k;
        p[topk_idx[a]] = fmaf(topk_w[a], dw_row[assign_to_row[a]], p[topk_idx[a]]);
    }
}

// One block per token: dx_t = sum_k dxp[row(t,k)] + sum_k dl_k Wr[e_k], float sums in k order, rounded once.
// With dl_full (un-renormalised weights) the router term runs over all E experts, coefficients dl_full[t][e], instead of
// the K selected ones.
__global__ __launch_bounds__(256) void bw_dx_kernel(const bf16_t *__restrict__ dxp, const int32_t *__restrict__ assign_to_row,
                                                    const float *__restrict__ dl, const int32_t *__restrict__ topk_idx,
                                                    const bf16_t *__restrict__ wr, bf16_t *__restrict__ dx, int H, int K,
                                                    const float *__restrict__ dl_full, int E) {
    const int t = blockIdx.x;
    for (int p = threadIdx.x; p < (H >> 3); p += 256) {
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.f;
        // groups of 8 slots: row numbers, expert ids and coefficients first, then the 16 row loads (8 of dxp, 8 of Wr)
        // together, then the sums in k order.  Every load is unconditional: a missing slot reads slot 0's rows and enters
        // with the factor 0.
        for (int k0 = 0; k0 < K; k0 += 8) {
            int row[8], e[8];
            float c[8], live[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const bool ok = k0 + i < K;
                const size_t a = (size_t)t * K + (ok ? k0 + i : 0);
                row[i] = assign_to_row[a];
                e[i] = topk_idx[a];
                c[i] = ok ? dl[a] : 0.f;
                live[i] = ok ? 1.f : 0.f;
            }
            if (dl_full) {
#pragma unroll
                for (int i = 0; i < 8; ++i) { e[i] = 0; c[i] = 0.f; }      // the router term follows below, over all experts
            }
            u32x4 v[8], r[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = load_once(dxp + (size_t)row[i] * H + p * 8);
#pragma unroll
            for (int i = 0; i < 8; ++i) r[i] = *reinterpret_cast<const u32x4 *>(wr + (size_t)e[i] * H + p * 8);
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[2 * j] = fmaf(live[i], __uint_as_float(v[i][j] << 16), acc[2 * j]);
                    acc[2 * j + 1] = fmaf(live[i], __uint_as_float(v[i][j] & 0xFFFF0000u), acc[2 * j + 1]);
                }
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[2 * j] = fmaf(c[i], __uint_as_float(r[i][j] << 16), acc[2 * j]);
                    acc[2 * j + 1] = fmaf(c[i], __uint_as_float(r[i][j] & 0xFFFF0000u), acc[2 * j + 1]);
                }
        }
        if (dl_full) {
            for (int e0 = 0; e0 < E; e0 += 8) {
                float c[8];
                u32x4 r[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int e = min(e0 + i, E - 1);
                    c[i] = e0 + i < E ? dl_full[(size_t)t * E + e] : 0.f;
                    r[i] = *reinterpret_cast<const u32x4 *>(wr + (size_t)e * H + p * 8);
                }
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        acc[2 * j] = fmaf(c[i], __uint_as_float(r[i][j] << 16), acc[2 * j]);
                        acc[2 * j + 1] = fmaf(c[i], __uint_as_float(r[i][j] & 0xFFFF0000u), acc[2 * j + 1]);
                    }
            }
        }
        *reinterpret_cast<u32x4 *>(dx + (size_t)t * H + p * 8) =
            u32x4{pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]), pack_bf16x2(acc[4], acc[5]), pack_bf16x2(acc[6], acc[7])};
    }
}

// Router weight gradient: dWr[e][h] = sum over the rows r of expert e of dl_row[r] x_perm[r][h] (x_perm[r] = x[row_token[r]] with a map).  Block (e, 512-wide slice
// of h), 4 waves: wave w sums rows r0 + w, r0 + w + 4, ... in that order, four rows in flight, and the four partial sums are
// added in wave order, so the result does not depend on timing.
// With off == nullptr (un-renormalised weights: every token has a logit gradient for every expert) the rows are all T
// tokens of x itself and the coefficient of row t is dl_row[t * coef_stride + e].
__global__ __launch_bounds__(256) void bw_router_wgrad_kernel(const bf16_t *__restrict__ x_perm, const int32_t *__restrict__ row_token,
                                                              const float *__restrict__ dl_row, const int32_t *__restrict__ off,
                                                              float *__restrict__ dwr, float *__restrict__ dbias, int H,
                                                              int n_all, int coef_stride) {
    __shared__ float part[4][64][9];
    const int e = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int h0 = blockIdx.y * 512 + lane * 8;
    const bool live = h0 < H;
    const int r0 = off ? off[e] : 0, r1 = off ? off[e + 1] : n_all;
    if (!off) dl_row += e;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    float bsum = 0.f;
    auto add = [&](float c, const u32x4 &v) {
        bsum += c;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[2 * j] = fmaf(c, __uint_as_float(v[j] << 16), acc[2 * j]);
            acc[2 * j + 1] = fmaf(c, __uint_as_float(v[j] & 0xFFFF0000u), acc[2 * j + 1]);
        }
    };
    const u32x4 zero = {0u, 0u, 0u, 0u};
    // row r of the expert-sorted order is row row_token[r] of the matrix passed when a map is given
    auto row_of = [&](int r) { return (size_t)(row_token ? row_token[r] : r); };
    auto row_at = [&](int r) { return live ? *reinterpret_cast<const u32x4 *>(x_perm + row_of(r) * H + h0) : zero; };
    int r = r0 + wave;
    for (; r + 12 < r1; r += 16) {          // four rows in flight per wave: the loop is a chain of memory round trips
        const float c0 = dl_row[(size_t)r * coef_stride], c1 = dl_row[(size_t)(r + 4) * coef_stride],
                    c2 = dl_row[(size_t)(r + 8) * coef_stride], c3 = dl_row[(size_t)(r + 12) * coef_stride];
        const u32x4 v0 = row_at(r), v1 = row_at(r + 4), v2 = row_at(r + 8), v3 = row_at(r + 12);
        add(c0, v0);
        add(c1, v1);
        add(c2, v2);
        add(c3, v3);
    }
    for (; r < r1; r += 4) add(dl_row[(size_t)r * coef_stride], row_at(r));
#pragma unroll
    for (int j = 0; j < 8; ++j) part[wave][lane][j] = acc[j];
    part[wave][lane][8] = bsum;
    __syncthreads();
    if (wave == 0) {
        float tot[9];
#pragma unroll
        for (int j = 0; j < 9; ++j) tot[j] = ((part[0][lane][j] + part[1][lane][j]) + part[2][lane][j]) + part[3][lane][j];
        if (live) {
            *reinterpret_cast<f32x4 *>(dwr + (size_t)e * H + h0) = f32x4{tot[0], tot[1], tot[2], tot[3]};
            *reinterpret_cast<f32x4 *>(dwr + (size_t)e * H + h0 + 4) = f32x4{tot[4], tot[5], tot[6], tot[7]};
        }
        if (dbias && blockIdx.y == 0 && lane == 0) dbias[e] = tot[8];
    }
}

// token of every expert-sorted row
__global__ __launch_bounds__(256) void bw_row_token_kernel(const int32_t *__restrict__ row_to_assign, int K, int n,
                                                           int32_t *__restrict__ row_token) {
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r < n) row_token[r] = row_to_assign[r] / K;
}

__global__ __launch_bounds__(256) void bw_zero_kernel(float *__restrict__ p, size_t count) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256) p[i] = 0.f;
}
// zero-fill by a kernel (safe to record into a HIP graph)
hipError_t zero_floats(float *p, size_t count, hipStream_t st) {
    if (!p || count == 0) return hipSuccess;
    const size_t blocks = (count + 255) / 256;
    hipLaunchKernelGGL(bw_zero_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, st, p, count);
    return hipGetLastError();
}

// Float storage: the GEMMs of this pass multiply bf16 (as the forward pass does, which rounds float inputs on load), so
// float inputs are rounded once into bf16 copies in the workspace, and row gradients are widened on the way out.
__global__ __launch_bounds__(256) void bw_to_bf16_kernel(const float *__restrict__ in, bf16_t *__restrict__ out, size_t n8) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
        const f32x4 a = *reinterpret_cast<const f32x4 *>(in + i * 8), b = *reinterpret_cast<const f32x4 *>(in + i * 8 + 4);
        *reinterpret_cast<u32x4 *>(out + i * 8) =
            u32x4{pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(b[0], b[1]), pack_bf16x2(b[2], b[3])};
    }
}
__global__ __launch_bounds__(256) void bw_to_float_kernel(const bf16_t *__restrict__ in, float *__restrict__ out, size_t n8) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
        const u32x4 v = *reinterpret_cast<const u32x4 *>(in + i * 8);
        *reinterpret_cast<f32x4 *>(out + i * 8) = f32x4{__uint_as_float(v[0] << 16), __uint_as_float(v[0] & 0xFFFF0000u),
                                                        __uint_as_float(v[1] << 16), __uint_as_float(v[1] & 0xFFFF0000u)};
        *reinterpret_cast<f32x4 *>(out + i * 8 + 4) = f32x4{__uint_as_float(v[2] << 16), __uint_as_float(v[2] & 0xFFFF0000u),
                                                            __uint_as_float(v[3] << 16), __uint_as_float(v[3] & 0xFFFF0000u)};
    }
}
hipError_t to_bf16(const void *in, bf16_t *out, size_t count, hipStream_t st) {      // count is a multiple of 8
    if (count == 0) return hipSuccess;
    const size_t n8 = count / 8, blocks = (n8 + 255) / 256;
    hipLaunchKernelGGL(bw_to_bf16_kernel, dim3((unsigned)(blocks < 8192 ? blocks : 8192)), dim3(256), 0, st, (const float *)in, out, n8);
    return hipGetLastError();
}
hipError_t to_float(const bf16_t *in, void *out, size_t count, hipStream_t st) {
    if (count == 0) return hipSuccess;
    const size_t n8 = count / 8, blocks = (n8 + 255) / 256;
    hipLaunchKernelGGL(bw_to_float_kernel, dim3((unsigned)(blocks < 8192 ? blocks : 8192)), dim3(256), 0, st, in, (float *)out, n8);
    return hipGetLastError();
}

// Optional stage timer of the backward call: an event at every stage boundary.
struct BwProbe {
    hipEvent_t ev[MOE_BW_NUM_STAGES + 1];
    int n = 0;
    hipStream_t st = nullptr;
    void mark() { if (n <= MOE_BW_NUM_STAGES) (void)hipEventRecord(ev[n++], st); }
};
inline void bw_mark(BwProbe *p) { if (p) p->mark(); }

struct BwWorkspace {
    Workspace fwd;          // routing, permutation, tile list; fwd.act holds g, fwd.y_perm holds the row gradients dxp
    bf16_t *u, *dq, *dg, *du, *aw;      // [n][I] each
    bf16_t *x_perm, *up_perm;           // [n][H] each: x and d_out copied into expert-sorted row order
    float *dw_row, *dl;                 // [n] each: <dq, a> per row (later dl per row), dl per assignment
    void *big_list;                     // per-XCD row-tile list of the forward pass's large-batch GEMM
    bf16_t *zeros;                      // 512 zero bytes: what the large-batch GEMMs read past an expert's last row
    int32_t *row_token;                 // [n]: the token each expert-sorted row belongs to
    float *probs;                       // [T][E], un-renormalised weights only: the full softmax, later every logit's gradient
    // float storage only: bf16 copies of the inputs, and the row gradients before they are widened
    bf16_t *x16, *up16, *dx16;          // [T][H] each (for moe_grouped_swiglu_backward: [n][H] each)
    bf16_t *wr16, *wg16, *wu16, *wd16;  // [E][H], [E][I][H], [E][I][H], [E][H][I]
    size_t total;
};

BwWorkspace carve_bw(const moe_shape_t &s, void *base) {
    BwWorkspace b;
    b.fwd = carve_workspace(s, base);
    uintptr_t cur = reinterpret_cast<uintptr_t>(base) + b.fwd.total;      // integers: the base is null when only sizing
    const size_t n = (size_t)s.T * s.K;
    auto take = [&](auto *&field, size_t bytes) {
        field = reinterpret_cast<std::remove_reference_t<decltype(field)>>(cur);
        cur += align256(bytes);
    };
    take(b.u, n * s.I * 2);
    take(b.dq, n * s.I * 2);
    take(b.dg, n * s.I * 2);
    take(b.du, n * s.I * 2);
    take(b.aw, n * s.I * 2);
    take(b.x_perm, n * s.H * 2);
    take(b.up_perm, n * s.H * 2);
    take(b.dw_row, n * 4);
    take(b.dl, n * 4);
    take(b.big_list, big_tile_list_bytes(s));
    take(b.zeros, 512);
    take(b.row_token, n * 4);
    take(b.probs, s.renormalize ? 0 : (size_t)s.T * s.E * 4);
    const size_t f = s.dtype == MOE_F32 ? 2 : 0;      // bytes per element of the bf16 copies, none for bf16 storage
    take(b.x16, n * s.H * f);
    take(b.up16, n * s.H * f);
    take(b.dx16, n * s.H * f);
    take(b.wr16, (size_t)s.E * s.H * f);
    take(b.wg16, (size_t)s.E * s.I * s.H * f);
    take(b.wu16, (size_t)s.E * s.I * s.H * f);
    take(b.wd16, (size_t)s.E * s.H * s.I * f);
    b.total = (size_t)(cur - reinterpret_cast<uintptr_t>(base));
    return b;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

moe_status_t check_bw_shape(const moe_shape_t *s) {
    if (!s) return MOE_ERR_NULL;
    if (s->T < 0 || s->H < 1 || s->E < 1 || s->K < 1 || s->I < 1 || s->K > s->E || s->E > kMaxExperts) return MOE_ERR_SHAPE;
    if ((s->H & 7) || (s->I & 7)) return MOE_ERR_SHAPE;
    if ((long long)s->T * s->K > 0x7FFFFFFFLL || (long long)s->T * s->E > 0x7FFFFFFFLL) return MOE_ERR_SHAPE;
    if (s->dtype != MOE_BF16 && s->dtype != MOE_F32) return MOE_ERR_DTYPE;
    return MOE_OK;
}

// Shapes that every LDS-pipelined GEMM takes: those GEMMs can fetch a row through a map, so the block's
// backward pass hands them x and d_out as they are instead of copies in expert-sorted order.
bool rows_through_map(const moe_shape_t &s) {
    return big_pre_activations_applicable(s.H, s.I) && bw_lds_applicable(s);
}

// The expert part over expert-sorted rows: x_rows [n][H], up_rows [n][H] = the upstream gradient of each row's y
// (without the routing weight when topk_w is given: the weight of row r is then topk_w[row_to_assign[r]]).
// With row_token (only if rows_through_map(s)): expert-sorted row r is row row_token[r] of x_rows and of up_rows.
hipError_t expert_backward(const moe_shape_t &s, const bf16_t *x_rows, const bf16_t *up_rows, const int32_t *row_token,
                           const int32_t *row_to_assign, const float *topk_w, const int32_t *off, const bf16_t *wg,
                           const bf16_t *wu, const bf16_t *wd, BwWorkspace &b, bf16_t *dxp, float *d_wg, float *d_wu,
                           float *d_wd, hipStream_t st, BwProbe *probe = nullptr, const bf16_t *g_saved = nullptr,
                           const bf16_t *u_saved = nullptr) {
    const int n = s.T * s.K, H = s.H, I = s.I, E = s.E;
    const int max_tiles = n / kBwTile + (E < n ? E : n);
    int32_t *tiles = b.fwd.tile_map;
    // the pre-activations: the caller's (kept from the forward pass), or recomputed into the workspace
    const bool saved = g_saved && u_saved;
    bf16_t *g_new = b.fwd.act;
    const bf16_t *g = saved ? g_saved : g_new, *u = saved ? u_saved : b.u;
    hipError_t err;
#define MOE_TRY(call) do { err = (call); if (err != hipSuccess) return err; } while (0)
    MOE_TRY(launch_build_tile_map(off, E, kBwTile, max_tiles, tiles, st));
    // the pre-activations are forward-form products: the forward pass's large-batch kernel takes them when the shape allows
    const bool fwd_kernel = big_pre_activations_applicable(H, I);
    const bool lds_kernels = bw_lds_applicable(s);      // the LDS-pipelined GEMMs, whenever the shape allows
    if (fwd_kernel || lds_kernels) MOE_TRY(launch_big_tile_list(s, off, b.big_list, st));
    if (lds_kernels) MOE_TRY(zero_floats(reinterpret_cast<float *>(b.zeros), 128, st));
    bw_mark(probe);
    if (!saved) {
        if (fwd_kernel) MOE_TRY(launch_big_pre_activations(s, x_rows, row_token, 1, b.big_list, wg, wu, g_new, b.u, st));      // both from one launch
        else MOE_TRY(launch_bw_rows_kfast(x_rows, wg, off, tiles, max_tiles, g_new, H, I, st));
    }
    bw_mark(probe);
    if (!saved && !fwd_kernel) MOE_TRY(launch_bw_rows_kfast(x_rows, wu, off, tiles, max_tiles, b.u, H, I, st));
    bw_mark(probe);
    if (lds_kernels) MOE_TRY(launch_bw_lds_rows(s, up_rows, nullptr, wd, nullptr, b.big_list, b.zeros, row_token, b.dq, H, I, st));
    else MOE_TRY(launch_bw_rows_kslow(up_rows, nullptr, wd, nullptr, off, tiles, max_tiles, b.dq, H, I, st));
    bw_mark(probe);
    hipLaunchKernelGGL(bw_swiglu_kernel, dim3((n + 3) / 4), dim3(256), 0, st, g, u, b.dq, topk_w, row_to_assign, b.dg, b.du, b.aw,
                       b.dw_row, n, I);
    MOE_TRY(hipGetLastError());
    bw_mark(probe);
    if (lds_kernels) MOE_TRY(launch_bw_lds_rows(s, b.dg, b.du, wg, wu, b.big_list, b.zeros, nullptr, dxp, I, H, st));
    else MOE_TRY(launch_bw_rows_kslow(b.dg, b.du, wg, wu, off, tiles, max_tiles, dxp, I, H, st));
    bw_mark(probe);
    if (lds_kernels) MOE_TRY(launch_bw_lds_wgrad(s, up_rows, b.aw, off, b.zeros, row_token, nullptr, d_wd, H, I, st));
    else MOE_TRY(launch_bw_wgrad(up_rows, b.aw, off, E, d_wd, H, I, st));
    bw_mark(probe);
    if (lds_kernels) MOE_TRY(launch_bw_lds_wgrad(s, b.dg, x_rows, off, b.zeros, nullptr, row_token, d_wg, I, H, st));
    else MOE_TRY(launch_bw_wgrad(b.dg, x_rows, off, E, d_wg, I, H, st));
    bw_mark(probe);
    if (lds_kernels) MOE_TRY(launch_bw_lds_wgrad(s, b.du, x_rows, off, b.zeros, nullptr, row_token, d_wu, I, H, st));
    else MOE_TRY(launch_bw_wgrad(b.du, x_rows, off, E, d_wu, I, H, st));
    bw_mark(probe);
#undef MOE_TRY
    return hipSuccess;
}

}  // namespace
}  // namespace moe

using namespace moe;

extern "C" {

moe_status_t moe_backward_workspace_bytes(const moe_shape_t *shape, size_t *out_bytes) {
    moe_status_t st = check_bw_shape(shape);
    if (st != MOE_OK) return st;
    if (!out_bytes) return MOE_ERR_NULL;
    *out_bytes = carve_bw(*shape, nullptr).total;
    return MOE_OK;
}

moe_status_t moe_grouped_swiglu_backward(const moe_shape_t *shape, const void *x_perm, const int32_t *expert_offsets,
                                         const void *w_gate, const void *w_up, const void *w_down, const void *dy_perm,
                                         void *d_x_perm, float *d_w_gate, float *d_w_up, float *d_w_down,
                                         void *ws, size_t ws_bytes, void *stream) {
    moe_status_t st = check_bw_shape(shape);
    if (st != MOE_OK) return st;
    if (!x_perm || !expert_offsets || !w_gate || !w_up || !w_down || !dy_perm || !d_x_perm || !d_w_gate || !d_w_up || !d_w_down)
        return MOE_ERR_NULL;
    if (misaligned(x_perm) || misaligned(expert_offsets) || misaligned(w_gate) || misaligned(w_up) || misaligned(w_down) ||
        misaligned(dy_perm) || misaligned(d_x_perm) || misaligned(d_w_gate) || misaligned(d_w_up) || misaligned(d_w_down))
        return MOE_ERR_ALIGN;
    if (!ws) return MOE_ERR_WORKSPACE;
    if (misaligned(ws)) return MOE_ERR_ALIGN;
    if (ws_bytes < carve_bw(*shape, nullptr).total) return MOE_ERR_WORKSPACE;
    hipStream_t hs = (hipStream_t)stream;
    const moe_shape_t &s = *shape;
    BwWorkspace b = carve_bw(s, ws);
    if (s.T == 0) {      // no rows: the weight gradients are zero
        const size_t cnt = (size_t)s.E * s.I * s.H;
        if (zero_floats(d_w_gate, cnt, hs) != hipSuccess || zero_floats(d_w_up, cnt, hs) != hipSuccess ||
            zero_floats(d_w_down, cnt, hs) != hipSuccess)
            return MOE_ERR_HIP;
        return MOE_OK;
    }
    if (s.dtype == MOE_F32) {
        const size_t nh = (size_t)s.T * s.K * s.H, wn = (size_t)s.E * s.I * s.H;
        if (to_bf16(x_perm, b.x16, nh, hs) != hipSuccess || to_bf16(dy_perm, b.up16, nh, hs) != hipSuccess ||
            to_bf16(w_gate, b.wg16, wn, hs) != hipSuccess || to_bf16(w_up, b.wu16, wn, hs) != hipSuccess ||
            to_bf16(w_down, b.wd16, wn, hs) != hipSuccess)
            return MOE_ERR_HIP;
        moe_shape_t sb = s;
        sb.dtype = MOE_BF16;
        if (expert_backward(sb, b.x16, b.up16, nullptr, nullptr, nullptr, expert_offsets, b.wg16, b.wu16, b.wd16, b, b.dx16, d_w_gate,
                            d_w_up, d_w_down, hs) != hipSuccess)
            return MOE_ERR_HIP;
        return to_float(b.dx16, d_x_perm, nh, hs) == hipSuccess ? MOE_OK : MOE_ERR_HIP;
    }
    return expert_backward(s, (const bf16_t *)x_perm, (const bf16_t *)dy_perm, nullptr, nullptr, nullptr, expert_offsets,
                           (const bf16_t *)w_gate, (const bf16_t *)w_up, (const bf16_t *)w_down, b, (bf16_t *)d_x_perm,
                           d_w_gate, d_w_up, d_w_down, hs) == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// Host-side checks of moe_backward's arguments (no HIP call).
static moe_status_t check_backward_args(const moe_shape_t *shape, const void *x, const void *w_router, const float *router_bias,
                                        const void *w_gate, const void *w_up, const void *w_down, const void *d_out,
                                        const void *d_x, const float *d_w_router, const float *d_router_bias,
                                        const float *d_w_gate, const float *d_w_up, const float *d_w_down, const void *ws,
                                        size_t ws_bytes) {
    moe_status_t st = check_bw_shape(shape);
    if (st != MOE_OK) return st;
    if (!x || !w_router || !w_gate || !w_up || !w_down || !d_out || !d_x || !d_w_router || !d_w_gate || !d_w_up || !d_w_down)
        return MOE_ERR_NULL;
    if (misaligned(x) || misaligned(w_router) || misaligned(router_bias) || misaligned(w_gate) || misaligned(w_up) ||
        misaligned(w_down) || misaligned(d_out) || misaligned(d_x) || misaligned(d_w_router) || misaligned(d_router_bias) ||
        misaligned(d_w_gate) || misaligned(d_w_up) || misaligned(d_w_down))
        return MOE_ERR_ALIGN;
    if (!ws) return MOE_ERR_WORKSPACE;
    if (misaligned(ws)) return MOE_ERR_ALIGN;
    if (ws_bytes < carve_bw(*shape, nullptr).total) return MOE_ERR_WORKSPACE;
    return MOE_OK;
}

static moe_status_t backward_impl(const moe_shape_t *shape, const void *x, const void *w_router, const float *router_bias,
                                  const void *w_gate, const void *w_up, const void *w_down, const void *d_out,
                                  void *d_x, float *d_w_router, float *d_router_bias, float *d_w_gate, float *d_w_up,
                                  float *d_w_down, void *ws, size_t ws_bytes, void *stream, BwProbe *probe,
                                  const void *g_rows = nullptr, const void *u_rows = nullptr,
                                  const int32_t *topk_idx_saved = nullptr, const float *topk_w_saved = nullptr) {
    moe_status_t st = check_backward_args(shape, x, w_router, router_bias, w_gate, w_up, w_down, d_out, d_x, d_w_router,
                                          d_router_bias, d_w_gate, d_w_up, d_w_down, ws, ws_bytes);
    if (st != MOE_OK) return st;
    if (misaligned(g_rows) || misaligned(u_rows) || misaligned(topk_idx_saved) || misaligned(topk_w_saved)) return MOE_ERR_ALIGN;
    hipStream_t hs = (hipStream_t)stream;
    const moe_shape_t &s = *shape;
    BwWorkspace b = carve_bw(s, ws);
    Workspace &w = b.fwd;
    if (s.T == 0) {
        const size_t cnt = (size_t)s.E * s.I * s.H;
        if (zero_floats(d_w_gate, cnt, hs) != hipSuccess || zero_floats(d_w_up, cnt, hs) != hipSuccess ||
            zero_floats(d_w_down, cnt, hs) != hipSuccess || zero_floats(d_w_router, (size_t)s.E * s.H, hs) != hipSuccess ||
            zero_floats(d_router_bias, (size_t)s.E, hs) != hipSuccess)
            return MOE_ERR_HIP;
        return MOE_OK;
    }
    bf16_t *dxp = (bf16_t *)w.y_perm;
    if (probe) { probe->st = hs; probe->mark(); }
    // Float storage: the router below still sees the float values (so that it selects what the forward pass selected);
    // everything after it works on bf16 copies, under a shape that says so.
    const void *x_in = x, *w_router_in = w_router;
    const moe_shape_t s_in = s;
    moe_shape_t sb = s;
    sb.dtype = MOE_BF16;
    void *d_x_out = d_x;
    if (s_in.dtype == MOE_F32) {
        if (g_rows || u_rows) return MOE_ERR_DTYPE;      // the saving pair is bf16 only
        const size_t th = (size_t)s.T * s.H, wn = (size_t)s.E * s.I * s.H;
        if (to_bf16(x, b.x16, th, hs) != hipSuccess || to_bf16(d_out, b.up16, th, hs) != hipSuccess ||
            to_bf16(w_router, b.wr16, (size_t)s.E * s.H, hs) != hipSuccess || to_bf16(w_gate, b.wg16, wn, hs) != hipSuccess ||
            to_bf16(w_up, b.wu16, wn, hs) != hipSuccess || to_bf16(w_down, b.wd16, wn, hs) != hipSuccess)
            return MOE_ERR_HIP;
        x = b.x16; d_out = b.up16; w_router = b.wr16; w_gate = b.wg16; w_up = b.wu16; w_down = b.wd16;
        d_x = b.dx16;
    }
    // the routing: the caller's (kept from the forward pass), or recomputed
    const bool routed = topk_idx_saved && topk_w_saved;
    const int32_t *topk_idx = routed ? topk_idx_saved : w.topk_idx;
    const float *topk_w = routed ? topk_w_saved : w.topk_w;
    // Un-renormalised weights need the softmax over all experts: the router runs even when the routing was handed over
    // (its partial logit sums are what the probabilities are computed from).
    const bool dense = !s.renormalize;
    if ((!routed || dense) && launch_route(s_in, x_in, w_router_in, router_bias, w.logit_part, w.topk_idx, w.topk_w, hs) != hipSuccess)
        return MOE_ERR_HIP;
    if (dense && launch_router_probs(s_in, w.logit_part, router_bias, b.probs, hs) != hipSuccess) return MOE_ERR_HIP;
    bw_mark(probe);
    if (launch_permute(sb, topk_idx, w.expert_offsets, w.row_to_assign, w.assign_to_row, w.chunk_base, hs) != hipSuccess)
        return MOE_ERR_HIP;
    // Shapes the LDS-pipelined GEMMs take: they fetch the rows of x and d_out through a row -> token map (both then stay
    // in the caches instead of being streamed back K times over).  Otherwise: copies of x and d_out in expert-sorted row
    // order, so that the LDS-free GEMMs address their rows by plain arithmetic.
    const bool mapped = rows_through_map(sb);
    const bf16_t *x_rows = mapped ? (const bf16_t *)x : b.x_perm, *up_rows = mapped ? (const bf16_t *)d_out : b.up_perm;
    const int32_t *row_token = mapped ? b.row_token : nullptr;
    if (mapped) {
        hipLaunchKernelGGL(bw_row_token_kernel, dim3((s.T * s.K + 255) / 256), dim3(256), 0, hs, w.row_to_assign, s.K, s.T * s.K,
                           b.row_token);
        if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
    } else if (launch_gather_rows(sb, x, w.row_to_assign, b.x_perm, hs) != hipSuccess ||
               launch_gather_rows(sb, d_out, w.row_to_assign, b.up_perm, hs) != hipSuccess) {
        return MOE_ERR_HIP;
    }
    bw_mark(probe);
    if (expert_backward(sb, x_rows, up_rows, row_token, w.row_to_assign, topk_w, w.expert_offsets, (const bf16_t *)w_gate,
                        (const bf16_t *)w_up, (const bf16_t *)w_down, b, dxp, d_w_gate, d_w_up, d_w_down, hs, probe,
                        (const bf16_t *)g_rows, (const bf16_t *)u_rows) != hipSuccess)
        return MOE_ERR_HIP;
    if (dense) {
        hipLaunchKernelGGL(bw_softmax_dense_kernel, dim3((s.T + 255) / 256), dim3(256), 0, hs, topk_w, b.dw_row, w.assign_to_row, topk_idx,
                           b.probs, s.T, s.K, s.E);
        if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
        hipLaunchKernelGGL(bw_dx_kernel, dim3(s.T), dim3(256), 0, hs, dxp, w.assign_to_row, b.dl, topk_idx, (const bf16_t *)w_router,
                           (bf16_t *)d_x, s.H, s.K, b.probs, s.E);
        if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
        // every token contributes to every expert's router row: the sums run over the tokens of x in token order
        hipLaunchKernelGGL(bw_router_wgrad_kernel, dim3(s.E, (s.H + 511) / 512), dim3(256), 0, hs, (const bf16_t *)x, (const int32_t *)nullptr,
                           b.probs, (const int32_t *)nullptr, d_w_router, d_router_bias, s.H, s.T, s.E);
        if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
    } else {
        hipLaunchKernelGGL(bw_softmax_kernel, dim3((s.T + 255) / 256), dim3(256), 0, hs, topk_w, b.dw_row, w.assign_to_row, b.dl, s.T, s.K);
        if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
        hipLaunchKernelGGL(bw_dx_kernel, dim3(s.T), dim3(256), 0, hs, dxp, w.assign_to_row, b.dl, topk_idx, (const bf16_t *)w_router,
                           (bf16_t *)d_x, s.H, s.K, (const float *)nullptr, s.E);
        if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
        hipLaunchKernelGGL(bw_router_wgrad_kernel, dim3(s.E, (s.H + 511) / 512), dim3(256), 0, hs, x_rows, row_token, b.dw_row, w.expert_offsets,
                           d_w_router, d_router_bias, s.H, 0, 1);
        if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
    }
    if (s_in.dtype == MOE_F32 && to_float(b.dx16, d_x_out, (size_t)s.T * s.H, hs) != hipSuccess) return MOE_ERR_HIP;
    bw_mark(probe);
    bw_mark(probe);       // closes the empty calibration interval
    return MOE_OK;
}

moe_status_t moe_backward(const moe_shape_t *shape, const void *x, const void *w_router, const float *router_bias,
                          const void *w_gate, const void *w_up, const void *w_down, const void *d_out,
                          void *d_x, float *d_w_router, float *d_router_bias, float *d_w_gate, float *d_w_up,
                          float *d_w_down, void *ws, size_t ws_bytes, void *stream) {
    return backward_impl(shape, x, w_router, router_bias, w_gate, w_up, w_down, d_out, d_x, d_w_router, d_router_bias, d_w_gate,
                         d_w_up, d_w_down, ws, ws_bytes, stream, nullptr);
}

moe_status_t moe_backward_saved(const moe_shape_t *shape, const void *x, const void *w_router, const float *router_bias,
                                const void *w_gate, const void *w_up, const void *w_down, const void *d_out,
                                const void *g_rows, const void *u_rows, const int32_t *topk_idx, const float *topk_w, void *d_x,
                                float *d_w_router, float *d_router_bias, float *d_w_gate, float *d_w_up, float *d_w_down,
                                void *ws, size_t ws_bytes, void *stream) {
    if (!g_rows || !u_rows || (topk_idx == nullptr) != (topk_w == nullptr)) return MOE_ERR_NULL;
    return backward_impl(shape, x, w_router, router_bias, w_gate, w_up, w_down, d_out, d_x, d_w_router, d_router_bias, d_w_gate,
                         d_w_up, d_w_down, ws, ws_bytes, stream, nullptr, g_rows, u_rows, topk_idx, topk_w);
}

moe_status_t moe_backward_stage_times(const moe_shape_t *shape, const void *x, const void *w_router, const float *router_bias,
                                      const void *w_gate, const void *w_up, const void *w_down, const void *d_out,
                                      void *d_x, float *d_w_router, float *d_router_bias, float *d_w_gate, float *d_w_up,
                                      float *d_w_down, void *ws, size_t ws_bytes, void *stream, float *stage_ms) {
    if (!stage_ms) return MOE_ERR_NULL;
    for (int i = 0; i < MOE_BW_NUM_STAGES; ++i) stage_ms[i] = 0.f;
    // arguments are checked before the first HIP call; the events are destroyed before the call returns
    moe_status_t st = check_backward_args(shape, x, w_router, router_bias, w_gate, w_up, w_down, d_out, d_x, d_w_router,
                                          d_router_bias, d_w_gate, d_w_up, d_w_down, ws, ws_bytes);
    if (st != MOE_OK) return st;
    BwProbe probe;
    const bool timed = shape->T > 0;
    for (int i = 0; timed && i <= MOE_BW_NUM_STAGES; ++i)
        if (hipEventCreate(&probe.ev[i]) != hipSuccess) {
            while (--i >= 0) (void)hipEventDestroy(probe.ev[i]);
            return MOE_ERR_HIP;
        }
    st = backward_impl(shape, x, w_router, router_bias, w_gate, w_up, w_down, d_out, d_x, d_w_router, d_router_bias,
                                    d_w_gate, d_w_up, d_w_down, ws, ws_bytes, stream, timed ? &probe : nullptr);
    if (timed && st == MOE_OK && probe.n == MOE_BW_NUM_STAGES + 1) {
        if (hipEventSynchronize(probe.ev[MOE_BW_NUM_STAGES]) != hipSuccess) st = MOE_ERR_HIP;
        for (int i = 0; i < MOE_BW_NUM_STAGES && st == MOE_OK; ++i)
            if (hipEventElapsedTime(&stage_ms[i], probe.ev[i], probe.ev[i + 1]) != hipSuccess) st = MOE_ERR_HIP;
    }
    for (int i = 0; timed && i <= MOE_BW_NUM_STAGES; ++i) (void)hipEventDestroy(probe.ev[i]);
    return st;
}

}  // extern "C"
