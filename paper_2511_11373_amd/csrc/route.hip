// Router: logits on the fp64 matrix cores, then top-K selection and routing
// weights with one wavefront per token.
//
// The logit of (token, expert) is the dot product of two rows of bf16 (or float)
// numbers.  Every bf16 x bf16 product is exact in double (16 significant bits),
// and for bf16 inputs whose magnitudes span less than about 2^18 a sum of 2048
// of them still fits the 53 bits, so the float the sum is rounded to does not
// depend on the order of summation; that is what lets an independently written
// reference reproduce the selection bit for bit.  Outside that range (float
// storage, whose products have up to 48 bits, or bf16 values of very different
// magnitudes in one row) the additions round at 2^-53 relative and two orders
// of summation can, rarely, land on different sides of a float rounding
// boundary: the result is then one of the two neighbouring floats.
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

// Same result for E <= 64*R <= 256 without a serial chain: a logit's slot is the number of (logit, id) pairs of the
// token that precede it.  One block of four waves per token.  Every wave holds all the token's logits (lane l: experts
// l, l + 64, ...), packed with the expert id into 64-bit keys that are all different (ordered logit bits high, ~id
// low: a larger key is a larger logit or the same logit with a lower id); each wave counts, for each of its lanes' keys,
// the larger ones among a quarter of the token's keys (read from LDS, the same address in every lane), the four
// counts meet in LDS, and the first wave writes the selection and its weights.
typedef __attribute__((ext_vector_type(2))) unsigned long long u64x2;
template <int R>
__global__ __launch_bounds__(256) void topk_rank_kernel(const double *__restrict__ part, int ksplit,
                                                        const float *__restrict__ bias, int32_t *__restrict__ topk_idx,
                                                        float *__restrict__ topk_w, int T, int E, int K, int renorm) {
    constexpr int EP = R * 64, QK = EP / 4;
    __shared__ __attribute__((aligned(16))) unsigned long long keys[EP];
    __shared__ int part_rank[4][EP];
    __shared__ float sel[EP];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t = blockIdx.x;                                  // the grid has one block per token
    float logit[R];
    unsigned long long key[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int e = lane + 64 * r;
        logit[r] = e < E ? final_logit(part, ksplit, (size_t)T * E, (size_t)t * E + e, bias, e) : 0.f;
        // 0 sorts below every real expert's key
        key[r] = e < E ? ((unsigned long long)float_order_bits(logit[r]) << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned int)e) : 0ull;
        if (wave == 0) keys[e] = key[r];
    }
    __syncthreads();
    int rank[R];
#pragma unroll
    for (int r = 0; r < R; ++r) rank[r] = 0;
    for (int j = 0; j < QK; j += 2) {
        const u64x2 k2 = *reinterpret_cast<const u64x2 *>(&keys[wave * QK + j]);
#pragma unroll
        for (int r = 0; r < R; ++r) rank[r] += (int)(k2[0] > key[r]) + (int)(k2[1] > key[r]);
    }
#pragma unroll
    for (int r = 0; r < R; ++r) part_rank[wave][lane + 64 * r] = rank[r];
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int e = lane + 64 * r;
        const int rk = part_rank[0][e] + part_rank[1][e] + part_rank[2][e] + part_rank[3][e];
        if (e < E && rk < K) {
            topk_idx[(size_t)t * K + rk] = e;
            sel[rk] = logit[r];
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

// ---- fast router (bf16 storage, renormalised weights, E <= 128, H <= 2048, many tokens) ------------------------
// The selection must equal the one made on exactly summed logits, but only the logits near the top matter.
// Kernel 1 gets every logit cheaply on the bf16 matrix cores (float accumulation), with the squared norms of the
// router rows that a rigorous error radius needs; kernel 2 recomputes in double only the candidates that could be
// among the K largest, and ranks those.
//
// Error radius.  |fast - exact| <= kGamma * |x_t|_2 * |w_e|_2 + 4e-7 * (1 + |fast|).  The fast logit is a chain of
// H/32 <= 64 matrix-core instructions, each adding 32 products (exact in float: 16 significant bits) to the running
// float sum.  How the hardware adds those 33 numbers is not documented; the bound assumes no more than that each of
// them is kept to 24 bits below the largest of the instruction (aligned to the largest exponent and cut), i.e. an
// error of at most 33 * 2^-23 * (sum of the magnitudes seen so far) per instruction, final rounding included.  Over
// 64 instructions that is 64 * 33 * 2^-23 = 2^-11.96 times sum_h |x_h w_h|, which Cauchy-Schwarz bounds by the
// product of the norms; kGamma = 2^-11.5 leaves a third on top.  The second term covers the bias add and the float
// arithmetic of the radius itself.  Random rounding errors stay orders of magnitude below this (a float emulation of
// the chain on rows built for heavy cancellation: 1e-8 of the norms' product), so the price is a few per cent more
// candidates, not correctness resting on a guess.
// Candidates.  With lo_e = fast_e - r_e and hi_e = fast_e + r_e, the K-th largest lo is a lower bound tau of the
// K-th largest exact logit, so every member of the exact top K (ties included) has hi_e >= tau.
constexpr float kGamma = 3.4526698300124393e-04f;      // 2^-11.5

// Butterfly partners inside a row of 16 lanes through the data-parallel-primitive lane permutations: lanes l^1 and
// l^2 (quad permutations), then the mirror images inside 8 and 16 lanes, which pair every group of 4 (8) lanes
// holding equal values with the other group of its half row (row).  The rows are paired by ordinary shuffles.
template <int CTRL>
__device__ __forceinline__ unsigned int dpp_u32(unsigned int v) {
    return (unsigned int)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

__device__ __forceinline__ unsigned int wave_max_u32(unsigned int v) {
    v = max(v, dpp_u32<kDppXor1>(v));
    v = max(v, dpp_u32<kDppXor2>(v));
    v = max(v, dpp_u32<kDppHalfMirror>(v));
    v = max(v, dpp_u32<kDppMirror>(v));
    v = max(v, (unsigned int)__shfl_xor((int)v, 16, 64));
    v = max(v, (unsigned int)__shfl_xor((int)v, 32, 64));
    return v;
}
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    const unsigned long long u = __builtin_bit_cast(unsigned long long, v);
    const unsigned long long o = (unsigned long long)dpp_u32<CTRL>((unsigned int)u) |
                                 ((unsigned long long)dpp_u32<CTRL>((unsigned int)(u >> 32)) << 32);
    return __builtin_bit_cast(double, o);
}
__device__ __forceinline__ double wave_sum_f64(double v) {
    v += dpp_f64<kDppXor1>(v);
    v += dpp_f64<kDppXor2>(v);
    v += dpp_f64<kDppHalfMirror>(v);
    v += dpp_f64<kDppMirror>(v);
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    return v;
}

// K-th largest of the wave's keys (lane l holds key[r] of expert l + 64 r; 0 = no expert), counting equal keys
// as often as they occur: K rounds, each taking the maximum of what is left and striking out one holder of it.
template <int R>
__device__ __forceinline__ unsigned int kth_largest_key(const unsigned int (&key)[R], int K, int lane) {
    unsigned int taken = 0u, kth = 0u;
    for (int k = 0; k < K; ++k) {
        unsigned int best = 0u;
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (!((taken >> r) & 1u)) best = max(best, key[r]);
        kth = wave_max_u32(best);
        const unsigned long long holders = __ballot(best == kth);
        if (lane == __ffsll((long long)holders) - 1) {
            bool done = false;
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (!done && !((taken >> r) & 1u) && key[r] == kth) { taken |= 1u << r; done = true; }
        }
    }
    return kth;
}

__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Kernel 1: fast[t][e] for 64 tokens x EP = 64*R experts per block, k in steps of 128 through two LDS stages.
// 8 waves: wave w owns expert tile w % (EP/16) and EP/32 of the four 16-token tiles (v_mfma_f32_16x16x32_bf16,
// experts as rows, tokens as columns: lane (n, q) = (l%16, l/16) feeds row n, k = 8q..8q+7, and gets experts
// 4q..4q+3 of token n).  LDS rows are 256 bytes; the 16-byte piece p of row r is stored at p ^ (r % 16) so that
// the 16 rows read together at one k fall on different banks.
template <int R>
__global__ __launch_bounds__(512) void router_fast_logits_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ wr,
                                                                 float *__restrict__ fast, float *__restrict__ wn2,
                                                                 int T, int H, int E) {
    constexpr int EP = 64 * R, NT = EP / 16, TPW = NT / 2;      // expert tiles, token tiles per wave
    constexpr int BK = 128, ROWB = BK * 2, WP = EP * 16 / 512, XP = 64 * 16 / 512;   // pieces per thread and stage
    __shared__ __attribute__((aligned(16))) unsigned char Ws[2][EP * ROWB];
    __shared__ __attribute__((aligned(16))) unsigned char Xs[2][64 * ROWB];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 15, q = lane >> 4;
    const int et = wave % NT, th = wave / NT;
    const int t0 = blockIdx.x * 64;

    // global sources and LDS targets of this thread's pieces (rows past the end are clamped: their results are unused)
    const bf16_t *wsrc[WP], *xsrc[XP];
    int wdst[WP], xdst[XP];
#pragma unroll
    for (int i = 0; i < WP; ++i) {
        const int g = tid + i * 512, r = g >> 4, pc = g & 15;
        wsrc[i] = wr + (size_t)min(r, E - 1) * H + pc * 8;
        wdst[i] = r * ROWB + ((pc ^ (r & 15)) << 4);
    }
#pragma unroll
    for (int i = 0; i < XP; ++i) {
        const int g = tid + i * 512, r = g >> 4, pc = g & 15;
        xsrc[i] = x + (size_t)min(t0 + r, T - 1) * H + pc * 8;
        xdst[i] = r * ROWB + ((pc ^ (r & 15)) << 4);
    }
    // two register sets: the k tiles of the next two stages are in flight while one is multiplied
    u32x4 wreg[2][WP], xreg[2][XP];
    auto fetch = [&](int set, int k0) {
#pragma unroll
        for (int i = 0; i < WP; ++i) wreg[set][i] = *reinterpret_cast<const u32x4 *>(wsrc[i] + k0);
#pragma unroll
        for (int i = 0; i < XP; ++i) xreg[set][i] = *reinterpret_cast<const u32x4 *>(xsrc[i] + k0);
    };
    auto stash = [&](int set, int buf) {
#pragma unroll
        for (int i = 0; i < WP; ++i) *reinterpret_cast<u32x4 *>(&Ws[buf][wdst[i]]) = wreg[set][i];
#pragma unroll
        for (int i = 0; i < XP; ++i) *reinterpret_cast<u32x4 *>(&Xs[buf][xdst[i]]) = xreg[set][i];
    };

    f32x4 acc[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    float ss = 0.f;
    auto multiply = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < BK / 32; ++ks) {
            const int pc = ((ks * 4 + q) ^ n) << 4;
            const u32x4 a = *reinterpret_cast<const u32x4 *>(&Ws[buf][(et * 16 + n) * ROWB + pc]);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float lo = __uint_as_float(a[j] << 16), hi = __uint_as_float(a[j] & 0xFFFF0000u);
                ss = fmaf(lo, lo, ss);
                ss = fmaf(hi, hi, ss);
            }
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const u32x4 b = *reinterpret_cast<const u32x4 *>(&Xs[buf][((th * TPW + i) * 16 + n) * ROWB + pc]);
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                                 acc[i], 0, 0, 0);
            }
        }
    };
    const int nk = H / BK;          // H is a multiple of 256: an even number of stages, two per turn of the loop
    fetch(0, 0);
    fetch(1, BK);
    stash(0, 0);
    __syncthreads();
    for (int kt = 0; kt < nk; kt += 2) {
        if (kt + 2 < nk) fetch(0, (kt + 2) * BK);
        multiply(0);
        stash(1, 1);                              // stage kt+1; buffer 1 was last read before the previous barrier
        __syncthreads();
        if (kt + 3 < nk) fetch(1, (kt + 3) * BK);
        multiply(1);
        if (kt + 2 < nk) stash(0, 0);
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int t = t0 + (th * TPW + i) * 16 + n;
        if (t < T) *reinterpret_cast<f32x4 *>(fast + (size_t)t * EP + et * 16 + 4 * q) = acc[i];
    }
    ss += __shfl_xor(ss, 16, 64);
    ss += __shfl_xor(ss, 32, 64);
    if (blockIdx.x == 0 && th == 0 && q == 0) wn2[et * 16 + n] = ss;
}

// Kernel 2: one wave per token.  Lane l keeps the token's values 8*(l + 64 j) .. +7 as doubles, so a candidate's
// exact logit costs one load, one widening and one fused multiply-add per element and a wave-wide sum.
template <int R>
__global__ __launch_bounds__(256, 4) void router_fast_select_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ wr,
                                                                 const float *__restrict__ bias, const float *__restrict__ fast,
                                                                 const float *__restrict__ wn2, int32_t *__restrict__ topk_idx,
                                                                 float *__restrict__ topk_w, int T, int H, int E, int K) {
    constexpr int EP = 64 * R;
    __shared__ __attribute__((aligned(16))) unsigned int keys_all[4][EP];
    __shared__ float sel_all[4][EP];
    __shared__ int cid_all[4][EP];
    __shared__ float cbias_all[4][EP];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + wave;
    if (t >= T) return;
    unsigned int *ckey = keys_all[wave];     // the candidates' exact-logit bits
    int *cid = cid_all[wave];                // candidate expert ids
    float *cbias = cbias_all[wave];          // and their biases (read here, not between the row loads of the loop below)
    float *sel = sel_all[wave];              // selected logits by slot

    // the token row: pieces lane, lane+64, ... of 8 values (H <= 2048: at most 4 per lane), widened once
    const int npieces = H >> 3;
    double xd[4][8];
    float xsq = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int pc = lane + 64 * j;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (pc < npieces) v = *reinterpret_cast<const u32x4 *>(x + (size_t)t * H + pc * 8);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float lo = __uint_as_float(v[i] << 16), hi = __uint_as_float(v[i] & 0xFFFF0000u);
            xsq = fmaf(lo, lo, xsq);
            xsq = fmaf(hi, hi, xsq);
            xd[j][2 * i] = (double)lo;
            xd[j][2 * i + 1] = (double)hi;
        }
    }
    const float xnorm = sqrtf(wave_sum_f32(xsq)) * 1.0001f;

    float fst[R], rad[R], bia[R];
    unsigned int lokey[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int e = lane + 64 * r;
        float f = 0.f, w2 = 0.f;
        bia[r] = 0.f;
        if (e < E) {
            f = fast[(size_t)t * EP + e];
            w2 = wn2[e];
            if (bias) bia[r] = bias[e];
            f += bia[r];
        }
        fst[r] = f;
        rad[r] = kGamma * xnorm * (sqrtf(w2) * 1.0001f) + 4e-7f * (1.0f + fabsf(f));
        lokey[r] = e < E ? float_order_bits(f - rad[r]) : 0u;       // 0 sorts below every finite float
    }
    const float tau = order_bits_float(kth_largest_key<R>(lokey, K, lane));     // K <= E: a real expert's bound

    // candidate list, in expert order
    int nc = 0;
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const bool cand = lane + 64 * r < E && fst[r] + rad[r] >= tau;
        const unsigned long long m = __ballot(cand);
        if (cand) {
            cid[nc + __popcll(m & below)] = lane + 64 * r;
            cbias[nc + __popcll(m & below)] = bia[r];
        }
        nc += __popcll(m);
    }
    wave_lds_sync();
    // exact logits of the candidates: the sum in double (products exact), one rounding to float
    // The rows of two candidates are in flight at any time (a row comes from L2 in about the time it takes to sum a few).
    // Every load is unconditional, so that the compiler's waits count exactly: past the last candidate the last row is
    // fetched again, and a lane whose piece lies beyond H re-reads piece 0, which its zero x values cancel.
    u32x4 wv[2][4];
    const int pc_of[4] = {lane < npieces ? lane : 0, lane + 64 < npieces ? lane + 64 : 0, lane + 128 < npieces ? lane + 128 : 0,
                          lane + 192 < npieces ? lane + 192 : 0};
    auto fetch_row = [&](u32x4 (&row)[4], int ci) {
        const int e = cid[min(ci, nc - 1)];                  // K >= 1, so there is at least one candidate
#pragma unroll
        for (int j = 0; j < 4; ++j) row[j] = *reinterpret_cast<const u32x4 *>(wr + (size_t)e * H + pc_of[j] * 8);
    };
    auto exact_logit = [&](const u32x4 (&row)[4], int ci) {
        double s0 = 0.0, s1 = 0.0;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                s0 = fma(xd[j][2 * i], (double)__uint_as_float(row[j][i] << 16), s0);
                s1 = fma(xd[j][2 * i + 1], (double)__uint_as_float(row[j][i] & 0xFFFF0000u), s1);
            }
        double s = wave_sum_f64(s0 + s1);
        if (bias) s += (double)cbias[ci];
        if (lane == 0) ckey[ci] = float_order_bits((float)s);
    };
    fetch_row(wv[0], 0);
    fetch_row(wv[1], 1);
    for (int ci = 0; ci < nc; ci += 2) {
        exact_logit(wv[0], ci);
        fetch_row(wv[0], ci + 2);
        if (ci + 1 < nc) exact_logit(wv[1], ci + 1);
        fetch_row(wv[1], ci + 3);
    }
    wave_lds_sync();
    // order the candidates: (exact logit descending, expert id ascending); the first K are the selection
    for (int ci = lane; ci < nc; ci += 64) {
        const unsigned int mykey = ckey[ci];
        const int myid = cid[ci];
        int rk = 0;
        for (int cj = 0; cj < nc; ++cj) rk += (ckey[cj] > mykey) || (ckey[cj] == mykey && cid[cj] < myid);
        if (rk < K) {
            topk_idx[(size_t)t * K + rk] = myid;
            sel[rk] = order_bits_float(mykey);
        }
    }
    wave_lds_sync();
    write_weights(sel, K, 1, 0.f, topk_w + (size_t)t * K, lane);
}

// Full softmax over all E logits of a token, p[t][e] = exp(l_e - max) / sum, from the partial logit sums the fp64 path
// leaves behind (the backward pass of un-renormalised routing weights needs every expert's probability).  One wave per token.
__global__ __launch_bounds__(256) void router_probs_kernel(const double *__restrict__ part, int ksplit, const float *__restrict__ bias,
                                                           float *__restrict__ probs, int T, int E) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + wave;
    if (t >= T) return;
    float m = -3.0e38f;
    for (int e = lane; e < E; e += 64) m = fmaxf(m, final_logit(part, ksplit, (size_t)T * E, (size_t)t * E + e, bias, e));
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
    float z = 0.f;
    for (int e = lane; e < E; e += 64) z += expf(final_logit(part, ksplit, (size_t)T * E, (size_t)t * E + e, bias, e) - m);
    z = wave_sum_f32(z);
    for (int e = lane; e < E; e += 64)
        probs[(size_t)t * E + e] = expf(final_logit(part, ksplit, (size_t)T * E, (size_t)t * E + e, bias, e) - m) / z;
}

// Only after launch_route on the same shape and workspace, and only for shapes that take the fp64 path (every shape with
// renormalize == 0 does).
hipError_t launch_router_probs(const moe_shape_t &s, const double *logit_part, const float *bias, float *probs, hipStream_t st) {
    hipLaunchKernelGGL(router_probs_kernel, dim3((s.T + 3) / 4), dim3(256), 0, st, logit_part, router_ksplit(s), bias, probs, s.T, s.E);
    return hipGetLastError();
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

// Bytes of scratch launch_route needs: the k-split partial sums in double, or the fast path's float logits and norms.
size_t router_scratch_bytes(const moe_shape_t &s) {
    const size_t part = sizeof(double) * (size_t)router_ksplit(s) * s.T * s.E;
    const size_t fast = router_fast_applicable(s) ? sizeof(float) * ((size_t)s.T + 1) * 128 : 0;
    return part > fast ? part : fast;
}

hipError_t launch_route(const moe_shape_t &s, const void *x, const void *w_router, const float *bias,
                        double *logit_part, int32_t *topk_idx, float *topk_w, hipStream_t st, Probe *probe) {
    if (router_fast_applicable(s)) {
        const bf16_t *xb = (const bf16_t *)x, *wb = (const bf16_t *)w_router;
        const int ep = s.E <= 64 ? 64 : 128;
        float *fast = reinterpret_cast<float *>(logit_part), *wn2 = fast + (size_t)s.T * ep;
        dim3 g1((s.T + 63) / 64), g2((s.T + 3) / 4);
        if (ep == 64) hipLaunchKernelGGL(router_fast_logits_kernel<1>, g1, dim3(512), 0, st, xb, wb, fast, wn2, s.T, s.H, s.E);
        else hipLaunchKernelGGL(router_fast_logits_kernel<2>, g1, dim3(512), 0, st, xb, wb, fast, wn2, s.T, s.H, s.E);
        hipError_t e1 = hipGetLastError();
        if (e1 != hipSuccess) return e1;
        probe_mark(probe);
        if (ep == 64) hipLaunchKernelGGL(router_fast_select_kernel<1>, g2, dim3(256), 0, st, xb, wb, bias, fast, wn2, topk_idx, topk_w, s.T, s.H, s.E, s.K);
        else hipLaunchKernelGGL(router_fast_select_kernel<2>, g2, dim3(256), 0, st, xb, wb, bias, fast, wn2, topk_idx, topk_w, s.T, s.H, s.E, s.K);
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
    hipLaunchKernelGGL(topk_rank_kernel<RR>, dim3(s.T), dim3(256), 0, st, logit_part, ks, bias, topk_idx, topk_w, \
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
