// Large-batch grouped GEMM for bf16 storage: 256 weight rows x 256 token rows per block, direct
// global->LDS loads (no register staging), two LDS stages, 32x32x16 bf16 MFMA.
//
// Block = 4 waves in a 2 (weight) x 2 (token) grid; a wave owns 4 weight tiles x 4 token tiles of
// 32x32, i.e. 16 accumulators (256 VGPRs).  For the gate/up pass the 256 weight rows are 128 rows of
// Wg and the same 128 rows of Wu, so that silu(g)*u is formed in registers.
//
// LDS stage layout (per operand): 256 rows x 128 bytes (64 bf16 of the reduction axis), dense.
// A global_load_lds_dwordx4 writes 64 lanes x 16 B = 8 rows contiguously; to keep the later MFMA
// operand reads (ds_read_b128 by 16 consecutive rows at the same k) off the same banks, the 16-byte
// piece j of row r is stored at position j ^ ((r >> 1) & 7) of the row; the lane that fills a
// position fetches the matching piece from global memory, so every 8 lanes still read one full
// 128-byte line.
//
// Row tiles are walked in a list (expert, first row); the flattened (row tile, weight tile) index is
// remapped so that each XCD (blocks are dealt round-robin to the 8 XCDs) works on a contiguous range
// of the list: the blocks that share an expert's weights and a row tile's tokens share one L2.
#include "moe_internal.hpp"

namespace moe {

namespace big {
constexpr int BW = 256, BT = 256, BK = 64;
constexpr int ROWB = BK * 2;                  // bytes per LDS row
constexpr int OPB = 256 * ROWB;               // bytes per operand stage (32 KB)
}  // namespace big

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void gbl_void;

// The compiler tracks LDS writes made by global_load_lds conservatively: an ordinary LDS read that
// follows would wait for every load in flight, including the next stage's.  The MFMA operand reads of
// the main loop are therefore issued as inline asm and the counters are waited on by hand:
//   vmcnt   - global->LDS loads of this wave (complete in order)
//   lgkmcnt - LDS reads of this wave (complete in order)
// The wait that guards a set of operand registers names them as in/out operands so that the MFMAs
// consuming them cannot be scheduled above it.
#define MOE_WAIT_VMCNT(N) asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory")

__device__ __forceinline__ bf16x8 lds_read_b128(unsigned addr, int) = delete;
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128(unsigned addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return v;
}
template <int N>
__device__ __forceinline__ void wait_lds_reads(bf16x8 (&a)[4], bf16x8 (&b)[4]) {
    asm volatile("s_waitcnt lgkmcnt(%8)"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3])
                 : "n"(N)
                 : "memory");
}
__device__ __forceinline__ unsigned lds_addr(const void *p) {
    return (unsigned)(size_t)(const __attribute__((address_space(3))) void *)p;
}

template <bool B>
struct FullTile { static constexpr bool value = B; };

// Which of the next stage's 16 global->LDS loads follows MFMA m of k step ks (-1: none).
#ifndef MOE_BIG_LOADPLAN
#define MOE_BIG_LOADPLAN 3
#endif
// Plans 0-2 load the next stage during the first k steps of the current one; plan 3 loads the stage after
// the next during the last k step, right behind the barrier that frees the buffer, which leaves three k steps
// for the data to arrive instead of one or two.
__device__ constexpr int big_load_slot(int ks, int m) {
#if MOE_BIG_LOADPLAN == 0
    return ks == 0 ? m : -1;
#elif MOE_BIG_LOADPLAN == 1
    return (ks < 2 && m >= 8) ? ks * 8 + m - 8 : -1;
#elif MOE_BIG_LOADPLAN == 2
    return (ks < 2 && (m & 1)) ? ks * 8 + (m >> 1) : -1;
#else
    return ks == 3 ? m : -1;
#endif
}
constexpr bool big_load_two_ahead = MOE_BIG_LOADPLAN == 3;

__device__ __forceinline__ float silu_mul_f(float g, float u) { return g / (1.0f + __expf(-g)) * u; }

template <bool GATE_UP>
__global__ __launch_bounds__(256, 1) void grouped_gemm_big_kernel(
    const bf16_t *__restrict__ xrows, const int32_t *__restrict__ row_map, int K_assign,
    const int32_t *__restrict__ off, const int32_t *__restrict__ tile_map, int max_tiles,
    const bf16_t *__restrict__ w0, const bf16_t *__restrict__ w1, bf16_t *__restrict__ outp, int KD, int NW,
    int n_wtiles) {
    using namespace big;
    __shared__ __attribute__((aligned(1024))) unsigned char WsA[OPB];
    __shared__ __attribute__((aligned(1024))) unsigned char XsA[OPB];
    __shared__ __attribute__((aligned(1024))) unsigned char WsB[OPB];
    __shared__ __attribute__((aligned(1024))) unsigned char XsB[OPB];

    // ---- which tile --------------------------------------------------------------------------
    const int total = tile_map[2 * max_tiles] * n_wtiles;
    const int per_xcd = (total + 7) >> 3;
    const int slot = blockIdx.x >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + slot;
    if (slot >= per_xcd || logical >= total) return;
    const int rtile = logical / n_wtiles, wtile = logical - rtile * n_wtiles;
    const int e = tile_map[2 * rtile], row0 = tile_map[2 * rtile + 1];
    const int row_end = off[e + 1];
    const int wrow0 = wtile * (GATE_UP ? BW / 2 : BW);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // uniform: LDS destinations stay in scalar registers
    const int ww = wave & 1, wt = wave >> 1;
    // The 256 token rows are 8 sub-tiles of 32; token-wave wt owns sub-tiles wt, wt+2, wt+4, wt+6, so a
    // short (ragged) tile is split evenly between the two token waves.  nb = live sub-tiles of this wave.
    const int nsub = min(8, (row_end - row0 + 31) >> 5);
    const int nb = max(0, min(4, (nsub - wt + 1) >> 1));

    // ---- global sources of this thread's 16 pieces per stage ------------------------------------
    // load 2*i (weights) and 2*i+1 (tokens) of this wave fill LDS rows (i*4 + wave)*8 .. +8 of their operand;
    // lane -> (row lane/8, position lane%8).  (row >> 1) & 7 does not depend on i, so neither does the piece
    // a lane fetches.
    const int lrow = wave * 8 + (lane >> 3);                      // LDS row of pair 0
    const int piece = (lane & 7) ^ ((lrow >> 1) & 7);
    const bf16_t *src[16];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // weights: rows are a fixed stride apart (the launcher guarantees whole weight tiles)
        const bf16_t *wm = GATE_UP && i >= 4 ? w1 : w0;
        const int wr = GATE_UP ? (i & 3) * 32 + lrow : i * 32 + lrow;
        src[2 * i] = wm + ((size_t)e * NW + wrow0 + wr) * KD + piece * 8;
        // token rows: gathered, clamped to the expert's last row (results of clamped rows are never stored)
        int xr = row0 + i * 32 + lrow;
        xr = xr < row_end ? xr : row_end - 1;
        src[2 * i + 1] = xrows + (size_t)(row_map ? row_map[xr] / K_assign : xr) * KD + piece * 8;
    }

    f32x16 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    auto issue = [&](unsigned char *Ws, unsigned char *Xs, int k0, int j) {
        unsigned char *dst = ((j & 1) ? Xs : Ws) + ((j >> 1) * 4 + wave) * 1024;
        __builtin_amdgcn_global_load_lds((gbl_void *)(src[j] + k0), (lds_void *)dst, 16, 0, 0);
    };
    // operand addresses inside a stage: lane (row l%32, half l/32); k step ks uses pieces 2*ks + half.
    // Tile bases are multiples of 32 rows, so the swizzle term only depends on the lane.
    const int orow = lane & 31, ohalf = lane >> 5, sw = (orow >> 1) & 7;
    unsigned kpos[BK / 16];
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) kpos[ks] = orow * ROWB + (((2 * ks + ohalf) ^ sw) << 4);
    const unsigned a_base = (GATE_UP ? ww * 64 : ww * 128) * ROWB;
    const unsigned b_base = wt * 32 * ROWB;
    constexpr int A1 = 32 * ROWB, A2 = GATE_UP ? 128 * ROWB : 64 * ROWB, A3 = GATE_UP ? 160 * ROWB : 96 * ROWB;
    bf16x8 aop[2][4], bop[2][4];
    // the 8 operand reads of a k step, in the order the MFMAs first need them
    auto read_one = [&](unsigned wa, unsigned xa, int set, int q) {
        switch (q) {
            case 0: aop[set][0] = lds_read_b128<0>(wa); break;
            case 1: bop[set][0] = lds_read_b128<0>(xa); break;
            case 2: aop[set][1] = lds_read_b128<A1>(wa); break;
            case 3: aop[set][2] = lds_read_b128<A2>(wa); break;
            case 4: aop[set][3] = lds_read_b128<A3>(wa); break;
            case 5: bop[set][1] = lds_read_b128<64 * ROWB>(xa); break;
            case 6: bop[set][2] = lds_read_b128<128 * ROWB>(xa); break;
            default: bop[set][3] = lds_read_b128<192 * ROWB>(xa); break;
        }
    };
    // One 16-wide k step: 16 MFMAs out of operand set ks&1.  A wave is alone on its SIMD, so an instruction
    // that is not an MFMA only comes for free in the shadow of the MFMA issued just before it (the matrix
    // pipe is busy for 8 passes per MFMA): the 8 operand reads of the following k step and this k step's
    // share of the next stage's 16 global->LDS loads are therefore dealt out one per MFMA.
    auto kstep = [&](auto full_c, int ks, unsigned wrd, unsigned xrd, int ks_rd, unsigned char *Wn,
                     unsigned char *Xn, int k_next) {
        constexpr bool FULL = decltype(full_c)::value;
        const int set = ks & 1;
        const unsigned wa = wrd + a_base + kpos[ks_rd], xa = xrd + b_base + kpos[ks_rd];
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const int b = m >> 2, a = m & 3;
            if (FULL) {
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[set][a], bop[set][b], acc[a][b], 0, 0, 0);
            } else if (a == 0 && b < nb) {
#pragma unroll
                for (int a2 = 0; a2 < 4; ++a2)
                    acc[a2][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[set][a2], bop[set][b], acc[a2][b], 0, 0, 0);
            }
            if (m < 8) read_one(wa, xa, set ^ 1, m);
            const int j = big_load_slot(ks, m);
            if (j >= 0) issue(Wn, Xn, k_next, j);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop ------------------------------------------------------------------------------------
    // Two LDS stages, one block barrier per stage.  Operand registers are double-buffered per 16-wide k step.
    // The barrier sits in front of the last k step of a stage: by then this wave has read everything it needs
    // from the current buffer and its own loads into the other buffer have landed, so behind the barrier the
    // current buffer is free in every wave and the other one is complete.  The last k step therefore reads the
    // first operands of the next stage and issues the 16 loads of the stage after the next into the buffer
    // just freed; they have the three following k steps (about a microsecond) to arrive, which is what a miss
    // to HBM takes under load.  The last two stages reload the final k tile instead of branching around the loads.
    const int nk = KD / BK;      // KD is a multiple of BK (checked by the launcher)
    const int k_last = KD - BK;
    const unsigned wsA = lds_addr(WsA), xsA = lds_addr(XsA), wsB = lds_addr(WsB), xsB = lds_addr(XsB);
#pragma unroll
    for (int j = 0; j < 16; ++j) issue(WsA, XsA, 0, j);
    if (big_load_two_ahead) {
#pragma unroll
        for (int j = 0; j < 16; ++j) issue(WsB, XsB, min(BK, k_last), j);
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    } else {
        MOE_WAIT_VMCNT(0);
    }
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int q = 0; q < 8; ++q) read_one(wsA + a_base + kpos[0], xsA + b_base + kpos[0], 0, q);
    auto run = [&](auto full_c) {
#pragma unroll 1
        for (int kt = 0; kt < nk; ++kt) {
            const bool odd = kt & 1;
            const unsigned wcur = odd ? wsB : wsA, xcur = odd ? xsB : xsA;
            const unsigned wnxt = odd ? wsA : wsB, xnxt = odd ? xsA : xsB;
            // destination and k offset of the loads issued in this iteration
            unsigned char *Wl = (odd != big_load_two_ahead) ? WsA : WsB, *Xl = (odd != big_load_two_ahead) ? XsA : XsB;
            const int k_load = min((kt + (big_load_two_ahead ? 2 : 1)) * BK, k_last);
            wait_lds_reads<0>(aop[0], bop[0]);
            kstep(full_c, 0, wcur, xcur, 1, Wl, Xl, k_load);
            wait_lds_reads<0>(aop[1], bop[1]);
            kstep(full_c, 1, wcur, xcur, 2, Wl, Xl, k_load);
            wait_lds_reads<0>(aop[0], bop[0]);
            kstep(full_c, 2, wcur, xcur, 3, Wl, Xl, k_load);
            wait_lds_reads<0>(aop[1], bop[1]);
            MOE_WAIT_VMCNT(0);
            __builtin_amdgcn_s_barrier();
            kstep(full_c, 3, wnxt, xnxt, 0, Wl, Xl, k_load);
        }
    };
    if (nsub == 8) run(FullTile<true>{});
    else run(FullTile<false>{});
    wait_lds_reads<0>(aop[0], bop[0]);
    MOE_WAIT_VMCNT(0);
    __builtin_amdgcn_s_barrier();

    // ---- epilogue -----------------------------------------------------------------------------------
    // The accumulators of one 32-token sub-tile go through this wave's 32 KB of LDS (the stage buffers are
    // free now) and come back with 8 consecutive features of one token per lane, so that results leave as
    // 16-byte pieces forming 128 (gate/up) or 256 (down) contiguous bytes per token row.
    unsigned char *region = wave == 0 ? WsA : wave == 1 ? XsA : wave == 2 ? WsB : XsB;
    constexpr int TROW = 32 * 4 + 16;                    // bytes per token row of a 32x32 float tile (padded)
    constexpr int TILEB = 32 * TROW;
    constexpr int LPR = GATE_UP ? 8 : 16;                // lanes per token row on the way out
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        if (b >= nb) continue;
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                f32x4 v = {acc[a][b][4 * rq], acc[a][b][4 * rq + 1], acc[a][b][4 * rq + 2], acc[a][b][4 * rq + 3]};
                *reinterpret_cast<f32x4 *>(region + a * TILEB + (lane & 31) * TROW + (8 * rq + 4 * (lane >> 5)) * 4) = v;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int p = 0; p < 32 * LPR / 64; ++p) {
            const int n = p * (64 / LPR) + lane / LPR;    // token inside the 32-token sub-tile
            const int c = lane % LPR;                     // 8-feature piece
            const int at = c >> 2, fi = (c & 3) * 8;      // accumulator tile and first feature inside it
            const unsigned char *gp = region + at * TILEB + n * TROW + fi * 4;
            const f32x4 g0 = *reinterpret_cast<const f32x4 *>(gp), g1 = *reinterpret_cast<const f32x4 *>(gp + 16);
            const int row = row0 + (2 * b + wt) * 32 + n;
            u32x4 pk;
            int f;
            if (GATE_UP) {
                const f32x4 u0 = *reinterpret_cast<const f32x4 *>(gp + 2 * TILEB), u1 = *reinterpret_cast<const f32x4 *>(gp + 2 * TILEB + 16);
                pk = u32x4{pack_bf16x2(silu_mul_f(g0[0], u0[0]), silu_mul_f(g0[1], u0[1])),
                           pack_bf16x2(silu_mul_f(g0[2], u0[2]), silu_mul_f(g0[3], u0[3])),
                           pack_bf16x2(silu_mul_f(g1[0], u1[0]), silu_mul_f(g1[1], u1[1])),
                           pack_bf16x2(silu_mul_f(g1[2], u1[2]), silu_mul_f(g1[3], u1[3]))};
                f = wrow0 + ww * 64 + c * 8;
            } else {
                pk = u32x4{pack_bf16x2(g0[0], g0[1]), pack_bf16x2(g0[2], g0[3]), pack_bf16x2(g1[0], g1[1]), pack_bf16x2(g1[2], g1[3])};
                f = wrow0 + ww * 128 + c * 8;
            }
            if (row < row_end && f < NW) *reinterpret_cast<u32x4 *>(outp + (size_t)row * NW + f) = pk;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

bool big_gemm_applicable(const moe_shape_t &s) {
    // whole weight tiles in both passes, whole k tiles, and enough rows per expert to fill 256-row tiles
    return s.dtype == MOE_BF16 && s.H % big::BW == 0 && s.I % (big::BW / 2) == 0 && (long)s.T * s.K >= 128L * s.E;
}
int big_tile_rows() { return big::BT; }

hipError_t launch_grouped_swiglu_big(const moe_shape_t &s, const bf16_t *x_rows, const int32_t *row_map,
                                     const int32_t *off, const bf16_t *wg, const bf16_t *wu, const bf16_t *wd,
                                     bf16_t *act, const int32_t *tile_map, int max_tiles, bf16_t *y_perm,
                                     hipStream_t st, Probe *probe) {
    using namespace big;
    const int nw1 = (s.I + BW / 2 - 1) / (BW / 2), nw2 = (s.H + BW - 1) / BW;
    const int g1 = ((max_tiles * nw1 + 7) / 8) * 8, g2 = ((max_tiles * nw2 + 7) / 8) * 8;
    hipLaunchKernelGGL(grouped_gemm_big_kernel<true>, dim3(g1), dim3(256), 0, st, x_rows, row_map, s.K, off, tile_map,
                       max_tiles, wg, wu, act, s.H, s.I, nw1);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    probe_mark(probe);
    hipLaunchKernelGGL(grouped_gemm_big_kernel<false>, dim3(g2), dim3(256), 0, st, (const bf16_t *)act,
                       (const int32_t *)nullptr, 1, off, tile_map, max_tiles, wd, wd, y_perm, s.I, s.H, nw2);
    return hipGetLastError();
}

}  // namespace moe
