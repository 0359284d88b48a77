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
    // all partials are fetched before the first add so that the loads overlap (ksplit <= kMaxLogitSplit)
    double v[kMaxLogitSplit];
#pragma unroll
    for (int z = 0; z < kMaxLogitSplit; ++z) v[z] = z < ksplit ? part[pos + (size_t)z * split_stride] : 0.0;
    double s = 0.0;
#pragma unroll
    for (int z = 0; z < kMaxLogitSplit; ++z) s += v[z];      // adding 0.0 for the unused splits changes nothing
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

// ---- fast router (bf16 storage, renormalised weights, E <= 128, H <= 2048) -------------------------------------
// The selection must equal the one made on exactly summed logits, but only the logits near the top matter.
// Step 1 gets every logit cheaply on the bf16 matrix cores (float accumulation) together with a rigorous error
// radius; step 2 recomputes in double only the candidates that could be among the K largest, and ranks those.
//
// Error radius.  |fast - exact| <= kGamma * |x_t|_2 * |w_e|_2 + 4e-7 * (1 + |fast|): the fast logit is a sum of
// H products (each exact in float) reduced by up to 8 chained 32-term MFMAs per k eighth, seven float adds and the
// bias add.  Allowing each MFMA an error of 2^-21 of the magnitude it handles gives 2^-17 * sum|x_h w_h| in all;
// Cauchy-Schwarz bounds that sum by the norms; kGamma = 2^-16 doubles it.
// Candidates.  With lo_e = fast_e - r_e and hi_e = fast_e + r_e, the K-th largest lo is a lower bound tau of the
// K-th largest exact logit, so every member of the exact top K (ties included) has hi_e >= tau.
constexpr float kGamma = 1.52587890625e-05f;

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// ranks[r] = number of (key, expert) pairs of this token that precede the lane's r-th expert; keys in LDS.
template <int R>
__device__ __forceinline__ void rank_by_count(const unsigned int *keys, const unsigned int (&key)[R], int lane, int (&rank)[R]) {
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
}
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Block = 16 tokens, 16 waves.  Step 1: wave w multiplies k eighth w%8 of expert tiles w/8, w/8+2, ...
// (v_mfma_f32_16x16x32_bf16, experts as rows, tokens as columns).  Step 2: wave w owns token w.
template <int R>
__global__ __launch_bounds__(1024) void router_fast_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ wr,
                                                           const float *__restrict__ bias, int32_t *__restrict__ topk_idx,
                                                           float *__restrict__ topk_w, int T, int H, int E, int K) {
    constexpr int EP = 64 * R;
    __shared__ __attribute__((aligned(16))) float partial[8][16][EP];
    __shared__ float wn2[8][EP];
    __shared__ __attribute__((aligned(16))) unsigned int keys_all[16][EP];
    __shared__ float sel_all[16][EP];
    __shared__ int cid_all[16][EP];
    __shared__ u32x4 xrow_all[16][256];          // the block's 16 token rows (H <= 2048), packed bf16
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t0 = blockIdx.x * 16;
    {
        const int kq = wave & 7, tg = wave >> 3;
        const int n = lane & 15, q = lane >> 4;
        const int hq = H >> 3, steps = hq >> 5;            // H % 256 == 0, steps <= 8
        const bf16_t *xp = x + (size_t)min(t0 + n, T - 1) * H + kq * hq + q * 8;
        u32x4 xop[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) xop[s] = *reinterpret_cast<const u32x4 *>(xp + min(s, steps - 1) * 32);
        const int ntiles = (E + 15) >> 4;
        for (int et = tg; et < ntiles; et += 2) {
            const bf16_t *wp = wr + (size_t)min(et * 16 + n, E - 1) * H + kq * hq + q * 8;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            float ss = 0.f;
            u32x4 a[8];
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                a[s] = *reinterpret_cast<const u32x4 *>(wp + min(s, steps - 1) * 32);
                if (s >= steps) a[s] = u32x4{0u, 0u, 0u, 0u};      // a zero weight piece contributes nothing
            }
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[s]),
                                                              __builtin_bit_cast(bf16x8, xop[s]), acc, 0, 0, 0);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float lo = __uint_as_float(a[s][j] << 16), hi = __uint_as_float(a[s][j] & 0xFFFF0000u);
                    ss = fmaf(lo, lo, ss);
                    ss = fmaf(hi, hi, ss);
                }
            }
            // result register j of lane (n, q) is expert et*16 + 4q + j, token n
            *reinterpret_cast<f32x4 *>(&partial[kq][n][et * 16 + 4 * q]) = acc;
            ss += __shfl_xor(ss, 16, 64);
            ss += __shfl_xor(ss, 32, 64);
            if (q == 0) wn2[kq][et * 16 + n] = ss;
        }
    }
    __syncthreads();

    const int t = t0 + wave;
    if (t >= T) return;
    unsigned int *ckey = keys_all[wave];     // candidate list: ordered exact-logit bits ...
    int *cid = cid_all[wave];                // ... and expert ids
    float *sel = sel_all[wave];              // selected logits by slot
    // The wave works as 4 groups of 16 lanes so that four candidates are re-evaluated at a time; the token row
    // sits in LDS (piece p = 8 values) and lane li of a group handles pieces li, li+16, ...
    const int grp = lane >> 4, li = lane & 15;
    const int npp = H >> 7;                  // pieces per lane: H/8/16 <= 16
    u32x4 *xrow = xrow_all[wave];
    float xsq = 0.f;
    for (int p = lane; p < (H >> 3); p += 64) {
        const u32x4 v = *reinterpret_cast<const u32x4 *>(x + (size_t)t * H + p * 8);
        xrow[p] = v;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float lo = __uint_as_float(v[i] << 16), hi = __uint_as_float(v[i] & 0xFFFF0000u);
            xsq = fmaf(lo, lo, xsq);
            xsq = fmaf(hi, hi, xsq);
        }
    }
    const float xnorm = sqrtf(wave_sum_f32(xsq)) * 1.0001f;

    float fast[R], rad[R];
    unsigned int lokey[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int e = lane + 64 * r;
        float f = 0.f, w2 = 0.f;
        if (e < E) {
#pragma unroll
            for (int z = 0; z < 8; ++z) { f += partial[z][wave][e]; w2 += wn2[z][e]; }
            if (bias) f += bias[e];
        }
        fast[r] = f;
        rad[r] = kGamma * xnorm * (sqrtf(w2) * 1.0001f) + 4e-7f * (1.0f + fabsf(f));
        lokey[r] = e < E ? float_order_bits(f - rad[r]) : 0u;       // 0 sorts below every finite float
    }
    // tau = K-th largest lower bound, by radix selection on the ordered bits (ballots only)
    unsigned int prefix = 0u;
    int remaining = K;
    for (int bit = 31; bit >= 0; --bit) {
        const unsigned int want = prefix | (1u << bit), mask = ~((1u << bit) - 1u);
        int cnt = 0;
#pragma unroll
        for (int r = 0; r < R; ++r) cnt += __popcll(__ballot((lokey[r] & mask) == want));
        if (cnt >= remaining) prefix = want; else remaining -= cnt;
    }
    const float tau = order_bits_float(prefix);

    // candidate list, in expert order
    int nc = 0;
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const bool cand = lane + 64 * r < E && fast[r] + rad[r] >= tau;
        const unsigned long long m = __ballot(cand);
        if (cand) cid[nc + __popcll(m & below)] = lane + 64 * r;
        nc += __popcll(m);
    }
    wave_lds_sync();
    // exact logits of the candidates, four at a time: the sum in double (products exact), one rounding to float
    for (int c0 = 0; c0 < nc; c0 += 4) {
        const int ci = c0 + grp;
        const int e = cid[ci < nc ? ci : c0];
        const bf16_t *wrow = wr + (size_t)e * H + li * 8;
        double s = 0.0;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            u32x4 wv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (half * 8 + j < npp) v = *reinterpret_cast<const u32x4 *>(wrow + (half * 8 + j) * 128);
                wv[j] = v;
            }
            u32x4 xv4[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) xv4[j] = xrow[li + 16 * min(half * 8 + j, npp - 1)];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const unsigned int xv = xv4[j][i], ww = wv[j][i];
                    s = fma((double)__uint_as_float(xv << 16), (double)__uint_as_float(ww << 16), s);
                    s = fma((double)__uint_as_float(xv & 0xFFFF0000u), (double)__uint_as_float(ww & 0xFFFF0000u), s);
                }
                __builtin_amdgcn_sched_barrier(0);      // keeps the widening to double from being hoisted (registers)
            }
        }
#pragma unroll
        for (int m = 8; m >= 1; m >>= 1) s += __shfl_xor(s, m, 64);
        if (bias) s += (double)bias[e];
        if (li == 0 && ci < nc) ckey[ci] = float_order_bits((float)s);
    }
    wave_lds_sync();
    // order the candidates: (exact logit descending, expert id ascending); the first K are the selection
    for (int ci = lane; ci < nc; ci += 64) {
        const unsigned int mykey = ckey[ci];
        const int myid = cid[ci];
        int rank = 0;
        for (int cj = 0; cj < nc; ++cj) rank += (ckey[cj] > mykey) || (ckey[cj] == mykey && cid[cj] < myid);
        if (rank < K) {
            topk_idx[(size_t)t * K + rank] = myid;
            sel[rank] = order_bits_float(mykey);
        }
    }
    wave_lds_sync();
    write_weights(sel, K, 1, 0.f, topk_w + (size_t)t * K, lane);
}

static bool router_fast_applicable(const moe_shape_t &s) {
    // one block works through 16 tokens for tens of microseconds, so the path pays off only when there are
    // enough blocks to fill the chip several times; small batches keep the two-kernel fp64 path
    return s.dtype == MOE_BF16 && s.renormalize != 0 && s.E <= 128 && s.H % 256 == 0 && s.H <= 2048 && s.T >= 1024;
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
    if (router_fast_applicable(s)) {
        dim3 grid((s.T + 15) / 16);
        const bf16_t *xb = (const bf16_t *)x, *wb = (const bf16_t *)w_router;
        if (s.E <= 64) hipLaunchKernelGGL(router_fast_kernel<1>, grid, dim3(1024), 0, st, xb, wb, bias, topk_idx, topk_w, s.T, s.H, s.E, s.K);
        else hipLaunchKernelGGL(router_fast_kernel<2>, grid, dim3(1024), 0, st, xb, wb, bias, topk_idx, topk_w, s.T, s.H, s.E, s.K);
        probe_mark(probe);
        return hipGetLastError();
    }
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
