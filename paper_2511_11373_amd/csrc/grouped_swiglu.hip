// Grouped SwiGLU expert FFN on the bf16 matrix cores.
//
// Two GEMM passes over the expert-sorted rows, both with the weight rows as the
// MFMA "A" operand and the token rows as the "B" operand, so that a lane ends
// up holding four consecutive output features of one token:
//   pass 1: act[r, i]  = bf16( silu(Wg[e,i,:] . x_r) * (Wu[e,i,:] . x_r) )
//   pass 2: y[r, j]    = Wd[e,j,:] . act[r,:]
// Row tiles never straddle two experts: a small kernel turns expert_offsets into
// a list of (expert, first row) tiles on the device, and the GEMM grids are
// sized from an upper bound so the host never reads the offsets.
#include "moe_internal.hpp"

#include <type_traits>

namespace moe {

// ---- tile list -----------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void build_tile_map_kernel(const int32_t *__restrict__ off, int E, int BT,
                                                              int max_tiles, int32_t *__restrict__ tile_map) {
    __shared__ int first[kMaxExperts + 1];
    for (int e = threadIdx.x; e < E; e += 1024) first[e] = (off[e + 1] - off[e] + BT - 1) / BT;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int e = 0; e < E; ++e) { const int v = first[e]; first[e] = run; run += v; }
        first[E] = run;
        tile_map[2 * max_tiles] = run < max_tiles ? run : max_tiles;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += 1024) {
        const int r0 = off[e];
        for (int t = first[e], i = 0; t < first[e + 1] && t < max_tiles; ++t, ++i) {
            tile_map[2 * t] = e;
            tile_map[2 * t + 1] = r0 + i * BT;
        }
    }
}

hipError_t launch_build_tile_map(const int32_t *off, int E, int tile_rows, int max_tiles, int32_t *tile_map, hipStream_t st) {
    hipLaunchKernelGGL(build_tile_map_kernel, dim3(1), dim3(1024), 0, st, off, E, tile_rows, max_tiles, tile_map);
    return hipGetLastError();
}

// ---- global -> register staging of 8 consecutive elements as packed bf16 -------------------
__device__ __forceinline__ u32x4 load8_bf16(const bf16_t *p, bool ok) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (ok) v = *reinterpret_cast<const u32x4 *>(p);
    return v;
}
__device__ __forceinline__ u32x4 load8_bf16(const float *p, bool ok) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (ok) {
        const f32x4 a = *reinterpret_cast<const f32x4 *>(p);
        const f32x4 b = *reinterpret_cast<const f32x4 *>(p + 4);
        v[0] = pack_bf16x2(a[0], a[1]); v[1] = pack_bf16x2(a[2], a[3]);
        v[2] = pack_bf16x2(b[0], b[1]); v[3] = pack_bf16x2(b[2], b[3]);
    }
    return v;
}
// weights: eight lanes read one whole line of a row, and at the batch sizes this kernel serves an expert's weights are
// read by one or two token tiles: non-temporal
__device__ __forceinline__ u32x4 load8_weights(const bf16_t *p) { return load_once(p); }
__device__ __forceinline__ u32x4 load8_weights(const float *p) { return load8_bf16(p, true); }
__device__ __forceinline__ void store4(bf16_t *p, float a, float b, float c, float d) {
    u32x2 v = {pack_bf16x2(a, b), pack_bf16x2(c, d)};
    *reinterpret_cast<u32x2 *>(p) = v;
}
__device__ __forceinline__ void store4(float *p, float a, float b, float c, float d) {
    f32x4 v = {a, b, c, d};
    *reinterpret_cast<f32x4 *>(p) = v;
}
__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + __expf(-g)) * u; }

// ---- tiled grouped GEMM --------------------------------------------------------------------
// Block = WW x WT waves; each wave owns MW x MT tiles of 32 weight rows x 32 tokens
// (v_mfma_f32_32x32x16_bf16: lane l feeds row l%32, k = 8*(l/32)..+7 of both operands; result
// register r is D[8*(r/4) + 4*(l/32) + r%4][l%32]).
//   GATE_UP: weight tile = BW rows of Wg and the same BW rows of Wu, output act (bf16).
//   else   : weight tile = BW rows of Wd, output y in the storage type SO.
// SX/SW: storage type of the token rows / of the weights (bf16 bits or float, rounded on load).
// Small batches are bound by the weight stream, so what matters is bytes in flight: the k tiles of
// the next TWO steps sit in registers (global loads issued, not yet waited for) while the current one
// is multiplied out of LDS.
template <typename SX, typename SW, typename SO, bool GATE_UP, int WW, int WT, int MW, int MT, int BK>
__global__ __launch_bounds__(WW * WT * 64) void grouped_gemm_kernel(
    const SX *__restrict__ xrows, const int32_t *__restrict__ row_map, int K_assign,
    const int32_t *__restrict__ off, const int32_t *__restrict__ tile_map, int max_tiles,
    const SW *__restrict__ w0, const SW *__restrict__ w1, SO *__restrict__ outp,
    int KD /* reduction length */, int NW /* weight rows per expert */) {
    constexpr int NT = WW * WT * 64;
    constexpr int BW = WW * MW * 32, BT = WT * MT * 32, LDK = BK + 8, CPR = BK / 8;   // 16-byte chunks per row
    constexpr int NMAT = GATE_UP ? 2 : 1;
    constexpr int WCH = NMAT * BW * CPR, XCH = BT * CPR;                              // chunks per k tile
    constexpr int WPT = (WCH + NT - 1) / NT, XPT = (XCH + NT - 1) / NT;
    __shared__ __attribute__((aligned(16))) bf16_t Ws[NMAT * BW * LDK];
    __shared__ __attribute__((aligned(16))) bf16_t Xs[BT * LDK];

    const int tile = blockIdx.x;
    if (tile >= tile_map[2 * max_tiles]) return;
    const int e = tile_map[2 * tile], row0 = tile_map[2 * tile + 1];
    const int row_end = off[e + 1];
    const int wrow0 = blockIdx.y * BW;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ww = wave % WW, wt = wave / WW;

    // staging assignments: chunk c -> (row c/CPR, k piece c%CPR); NT is a multiple of CPR, so a thread stages the same k
    // piece of every row it has.  Every load of the main loop is unconditional (a load on one path only would make the
    // compiler wait for all loads in flight where the paths meet): rows that do not exist are replaced by one that does
    // (their results are never stored), a k piece past the end of the rows re-reads the last one and is zeroed when staged.
    static_assert(NT % CPR == 0, "a thread stages one k piece");
    const int kcol = (tid % CPR) * 8;
    const SW *wsrc[WPT]; int wdst[WPT];
#pragma unroll
    for (int i = 0; i < WPT; ++i) {
        const int c = min(tid + i * NT, WCH - 1);
        const int mat = c / (BW * CPR), r = (c / CPR) % BW;
        const int wr = min(wrow0 + r, NW - 1);
        const SW *base = (GATE_UP && mat == 1) ? w1 : w0;
        wsrc[i] = base + ((size_t)e * NW + wr) * KD;
        wdst[i] = (mat * BW + r) * LDK + kcol;
    }
    const SX *xsrc[XPT]; int xdst[XPT];
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
        const int c = min(tid + i * NT, XCH - 1);
        const int r = c / CPR;
        int src = min(row0 + r, row_end - 1);
        if (row_map) src = row_map[src] / K_assign;
        xsrc[i] = xrows + (size_t)src * KD;
        xdst[i] = r * LDK + kcol;
    }

    f32x16 acc[NMAT][MW][MT];
#pragma unroll
    for (int m = 0; m < NMAT; ++m)
#pragma unroll
        for (int a = 0; a < MW; ++a)
#pragma unroll
            for (int b = 0; b < MT; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[m][a][b][r] = 0.f;

    u32x4 wreg[2][WPT], xreg[2][XPT];
    auto fetch = [&](int k0, int set) {
        const int kk = min(k0 + kcol, KD - 8);
#pragma unroll
        for (int i = 0; i < WPT; ++i) wreg[set][i] = load8_weights(wsrc[i] + kk);
#pragma unroll
        for (int i = 0; i < XPT; ++i) xreg[set][i] = load8_bf16(xsrc[i] + kk, true);
    };
    const int arow = lane & 31, akq = (lane >> 5) * 8;
    auto step = [&](int k0, int set, auto fetch_tag) __attribute__((always_inline)) {      // k tile at k0 is in registers `set`
        __syncthreads();
        const bool past = k0 + kcol >= KD;
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < WPT; ++i)
            if (tid + i * NT < WCH) *reinterpret_cast<u32x4 *>(&Ws[wdst[i]]) = past ? zero : wreg[set][i];
#pragma unroll
        for (int i = 0; i < XPT; ++i)
            if (tid + i * NT < XCH) *reinterpret_cast<u32x4 *>(&Xs[xdst[i]]) = past ? zero : xreg[set][i];
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (decltype(fetch_tag)::value) fetch(k0 + 2 * BK, set);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 bop[MT];
#pragma unroll
            for (int b = 0; b < MT; ++b)
                bop[b] = *reinterpret_cast<const bf16x8 *>(&Xs[((wt * MT + b) * 32 + arow) * LDK + ks * 16 + akq]);
#pragma unroll
            for (int m = 0; m < NMAT; ++m)
#pragma unroll
                for (int a = 0; a < MW; ++a) {
                    const bf16x8 aop = *reinterpret_cast<const bf16x8 *>(
                        &Ws[(m * BW + (ww * MW + a) * 32 + arow) * LDK + ks * 16 + akq]);
#pragma unroll
                    for (int b = 0; b < MT; ++b)
                        acc[m][a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop, bop[b], acc[m][a][b], 0, 0, 0);
                }
        }
    };
    // Two k tiles are always in flight in registers.  The last steps, which load nothing, are copies of the loop body of
    // their own, so that inside the loop the loads are unconditional and the waits count exactly.
    const std::true_type loads;
    const std::false_type no_load;
    const int n_steps = (KD + BK - 1) / BK;
    fetch(0, 0);
    if (n_steps == 1) {
        step(0, 0, no_load);
    } else {
        fetch(BK, 1);
        int i = 0;
        for (; i + 3 < n_steps; i += 2) {
            step(i * BK, 0, loads);
            step((i + 1) * BK, 1, loads);
        }
        if (n_steps - i == 3) {
            step(i * BK, 0, loads);
            step((i + 1) * BK, 1, no_load);
            step((i + 2) * BK, 0, no_load);
        } else {
            step(i * BK, 0, no_load);
            step((i + 1) * BK, 1, no_load);
        }
    }

    // epilogue: lane holds token (l%32), features 8*(r/4) + 4*(l/32) + 0..3
#pragma unroll
    for (int a = 0; a < MW; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b) {
            const int row = row0 + (wt * MT + b) * 32 + (lane & 31);
            if (row >= row_end) continue;
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int f = wrow0 + (ww * MW + a) * 32 + 8 * rq + 4 * (lane >> 5);
                if (f >= NW) continue;
                float v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (GATE_UP) v[j] = silu_mul(acc[0][a][b][4 * rq + j], acc[NMAT - 1][a][b][4 * rq + j]);
                    else v[j] = acc[0][a][b][4 * rq + j];
                }
                store4(outp + (size_t)row * NW + f, v[0], v[1], v[2], v[3]);
            }
        }
}

// large-batch bf16 variant (grouped_swiglu_big.hip); builds its own per-XCD row-tile list in `tile_map`
bool big_gemm_applicable(const moe_shape_t &s);
hipError_t launch_grouped_swiglu_big(const moe_shape_t &s, const bf16_t *x_rows, const int32_t *row_map,
                                     const int32_t *off, const bf16_t *wg, const bf16_t *wu, const bf16_t *wd,
                                     bf16_t *act, int32_t *tile_map, bf16_t *y_perm, hipStream_t st, Probe *probe);

// decode-sized bf16 variant (grouped_swiglu_stream.hip); needs no row-tile list
bool stream_gemm_applicable(const moe_shape_t &s);
hipError_t launch_grouped_swiglu_stream(const moe_shape_t &s, const bf16_t *x_rows, const int32_t *row_map,
                                        const int32_t *off, const bf16_t *wg, const bf16_t *wu, const bf16_t *wd,
                                        bf16_t *act, bf16_t *y_perm, hipStream_t st, Probe *probe);

constexpr int kWW = 2, kWT = 2, kMW = 1, kMT = 1;      // wave grid and MFMA tiles per wave of the tiled kernel
constexpr int kBK = 64;                                 // k tile of the tiled kernel
int gemm_tile_rows(const moe_shape_t &s) {
    if (stream_gemm_applicable(s) || big_gemm_applicable(s)) return 0;      // no tile list, or one of their own
    return kWT * kMT * 32;
}
int gemm_max_tiles(const moe_shape_t &s) {
    const int n = s.T * s.K;
    const int rows = gemm_tile_rows(s);
    return rows ? n / rows + (s.E < n ? s.E : n) : 0;
}

template <typename S>
static hipError_t launch_typed(const moe_shape_t &s, const S *x_rows, const int32_t *row_map,
                               const int32_t *off, const S *wg, const S *wu, const S *wd, bf16_t *act,
                               int32_t *tile_map, S *y_perm, hipStream_t st, Probe *probe, bool tile_map_ready) {
    constexpr int WW = kWW, WT = kWT, MW = kMW, MT = kMT;
    constexpr int BW = WW * MW * 32;
    if constexpr (sizeof(S) == 2) {
        if (stream_gemm_applicable(s)) {
            probe_mark(probe);
            return launch_grouped_swiglu_stream(s, x_rows, row_map, off, wg, wu, wd, act, y_perm, st, probe);
        }
        if (big_gemm_applicable(s))
            return launch_grouped_swiglu_big(s, x_rows, row_map, off, wg, wu, wd, act, tile_map, y_perm, st, probe);
    }
    const int max_tiles = gemm_max_tiles(s);
    hipError_t err = hipSuccess;
    if (!tile_map_ready) {
        hipLaunchKernelGGL(build_tile_map_kernel, dim3(1), dim3(1024), 0, st, off, s.E, gemm_tile_rows(s), max_tiles, tile_map);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    probe_mark(probe);
    hipLaunchKernelGGL((grouped_gemm_kernel<S, S, bf16_t, true, WW, WT, MW, MT, kBK>), dim3(max_tiles, (s.I + BW - 1) / BW),
                       dim3(WW * WT * 64), 0, st, x_rows, row_map, s.K, off, tile_map, max_tiles, wg, wu, act, s.H, s.I);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
    probe_mark(probe);
    // the down pass takes 128 weight rows per block (two MFMA tiles per wave): its rows are short (I elements), so a block of
    // 64 rows streams too little between start-up and epilogue (512 tokens at H 2048, I 768: 91 -> 84 us)
    constexpr int MWD = 2, BWD = WW * MWD * 32;
    hipLaunchKernelGGL((grouped_gemm_kernel<bf16_t, S, S, false, WW, WT, MWD, MT, kBK>), dim3(max_tiles, (s.H + BWD - 1) / BWD),
                       dim3(WW * WT * 64), 0, st, (const bf16_t *)act, (const int32_t *)nullptr, 1, off, tile_map,
                       max_tiles, wd, wd, y_perm, s.I, s.H);
    return hipGetLastError();
}

hipError_t launch_grouped_swiglu(const moe_shape_t &s, const void *x_rows, const int32_t *row_map,
                                 const int32_t *expert_offsets, const void *w_gate, const void *w_up,
                                 const void *w_down, bf16_t *act, int32_t *tile_map, void *y_perm,
                                 hipStream_t st, Probe *probe, bool tile_map_ready) {
    if (s.dtype == MOE_BF16)
        return launch_typed<bf16_t>(s, (const bf16_t *)x_rows, row_map, expert_offsets, (const bf16_t *)w_gate,
                                    (const bf16_t *)w_up, (const bf16_t *)w_down, act, tile_map, (bf16_t *)y_perm, st, probe, tile_map_ready);
    return launch_typed<float>(s, (const float *)x_rows, row_map, expert_offsets, (const float *)w_gate,
                               (const float *)w_up, (const float *)w_down, act, tile_map, (float *)y_perm, st, probe, tile_map_ready);
}

}  // namespace moe
