// Large-batch grouped GEMMs of the backward pass: the forward pass's 256 x 256 x 64 LDS pipeline with operands
// that are stored ACROSS the reduction axis transposed on their way into LDS.
//
// out[x][f] = sum_k X[x][k] * W[f][k], 32x32x16 bf16 MFMAs, 4 waves in a 2 x 2 grid, 16 accumulators per wave, two LDS
// stages of 256 rows x 128 bytes per operand (16-byte piece j of row r at position j ^ ((r >> 1) & 7)), one block
// barrier per stage in front of its last k step, one memory instruction per MFMA slot - all as in
// grouped_swiglu_big.hip.  What differs is where an operand comes from:
//   * stored along k (the token-row operand of the data gradients): global_load_lds straight into LDS, as there;
//   * stored across k (W[e] as [k][f] for the data gradients; both operands of a weight gradient, where k runs over the
//     expert's token rows): thread (kg, rg) loads the 8 x 8 block of k = 8 kg .. +7 by rows 8 rg .. +7 (16 bytes per k,
//     128 contiguous bytes per 8 lanes) into registers right behind the barrier, transposes it with 32 byte
//     permutes one stage later and writes each row's 8 consecutive k as one 16-byte piece into its swizzled place.
// Both kinds arrive in the same buffer at the same time: loaded behind barrier t, complete at barrier t + 1.
#include "moe_internal.hpp"

namespace moe {
namespace bwl {

constexpr int BT = 256, BK = 64, ROWB = BK * 2, OPB = 256 * ROWB;

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void gbl_void;

template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128(unsigned addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return v;
}
template <int OFF>
__device__ __forceinline__ void lds_write_b128(unsigned addr, u32x4 v) {
    asm volatile("ds_write_b128 %0, %1 offset:%2" : : "v"(addr), "v"(v), "n"(OFF) : "memory");
}
// waits for every LDS access of this wave; names the operand registers so that their MFMAs stay behind it
__device__ __forceinline__ void wait_lds(bf16x8 (&a)[4], bf16x8 (&b)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3])
                 :
                 : "memory");
}
__device__ __forceinline__ unsigned lds_addr(const void *p) {
    return (unsigned)(size_t)(const __attribute__((address_space(3))) void *)p;
}
__device__ __forceinline__ u32x4 load16(const bf16_t *p, bool ok) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (ok) v = *reinterpret_cast<const u32x4 *>(p);
    return v;
}

// WGRAD = false: out[r][f] = sum over pairs p and k of xa_p[r][k] * w_p[e][k][f]   (rows r of expert e, bf16 out)
// WGRAD = true : out[e][m][f] = sum over the rows r of expert e of xa_0[r][m] * w_0[r][f]   (float out)
template <bool WGRAD, typename OutT>
__global__ __launch_bounds__(256, 1) void bw_lds_kernel(const bf16_t *__restrict__ xa0, const bf16_t *__restrict__ xa1,
                                                        const bf16_t *__restrict__ w0, const bf16_t *__restrict__ w1,
                                                        const i32x4 *__restrict__ tile_list, int tiles_per_xcd,
                                                        const int32_t *__restrict__ off, OutT *__restrict__ outp, int KD, int XN,
                                                        int N, int n_xtiles, int n_wtiles, int E, int n_rows) {
    __shared__ __attribute__((aligned(1024))) unsigned char WsA[OPB];
    __shared__ __attribute__((aligned(1024))) unsigned char XsA[OPB];
    __shared__ __attribute__((aligned(1024))) unsigned char WsB[OPB];
    __shared__ __attribute__((aligned(1024))) unsigned char XsB[OPB];

    // ---- which tile: blocks go round-robin to the 8 XCDs ------------------------------------------------------
    const int slot = blockIdx.x >> 3;
    int e, row0, row_end, wcol0, k_begin, k_end;
    if (WGRAD) {                                   // all tiles of an expert on one XCD
        const int tiles = n_xtiles * n_wtiles;
        e = (slot / tiles) * 8 + (blockIdx.x & 7);
        if (e >= E) return;
        const int tile = slot % tiles;
        row0 = (tile / n_wtiles) * BT;             // first output row (a column of xa_0)
        row_end = XN;
        wcol0 = (tile % n_wtiles) * BT;
        k_begin = off[e];
        k_end = off[e + 1];
    } else {                                       // the forward pass's per-XCD row-tile list, row tile fastest
        const i32x4 *entry = tile_list + 2 * ((blockIdx.x & 7) * tiles_per_xcd + slot / n_wtiles);
        const i32x4 ea = entry[0], eb = entry[1];
        e = ea[0];
        if (e < 0) return;
        row_end = ea[2];
        const int in_run = slot - ea[3] * n_wtiles;
        wcol0 = (in_run / eb[0]) * BT;
        row0 = ea[1] + (eb[1] + in_run % eb[0]) * BT;
        k_begin = 0;
        k_end = KD;
    }
    const int n_pairs = (!WGRAD && xa1) ? 2 : 1;
    const int per_pair = (k_end - k_begin + BK - 1) / BK;
    const int nst = per_pair * n_pairs;            // stages; 0 for an expert without rows (its gradient is zero)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ww = wave & 1, wt = wave >> 1;

    // ---- producers ---------------------------------------------------------------------------------------------
    // register path: thread (kg, rg) = (lane % 8, lane / 8 + 8 wave); LDS row 8 rg + c gets piece kg at position
    // kg ^ (((8 rg + c) >> 1) & 7) = kg ^ (4 (rg & 1) + c / 2)
    const int kg = lane & 7, rg = (lane >> 3) + 8 * wave;
    unsigned put_at[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) put_at[h] = rg * 8 * ROWB + ((kg ^ (4 * (rg & 1) + h)) << 4);
    const int wcol = wcol0 + 8 * rg;               // this thread's 8 weight-side rows (columns of the stored operand)
    const bool wcol_ok = wcol < N;
    const int xcol = row0 + 8 * rg;                // WGRAD: its 8 x-side rows likewise
    const bool xcol_ok = xcol < XN;
    u32x4 wraw[8], xraw[8];
    auto stage_k = [&](int s) { return k_begin + (s % per_pair) * BK; };
    auto load_w = [&](int s, int jj) {
        const int k = stage_k(s) + 8 * kg + jj;
        const bf16_t *base = WGRAD ? w0 : (s >= per_pair ? w1 : w0) + (size_t)e * KD * N;
        wraw[jj] = load16(base + (size_t)k * N + wcol, wcol_ok && k < k_end);
    };
    auto load_x = [&](int s, int jj) {             // WGRAD only
        const int k = stage_k(s) + 8 * kg + jj;
        xraw[jj] = load16(xa0 + (size_t)k * XN + xcol, xcol_ok && k < k_end);
    };
    auto put = [&](unsigned buf, const u32x4 (&raw)[8], int c) {     // row 8 rg + c: its 8 consecutive k, one 16-byte piece
        const int w = c >> 1;
        u32x4 t;
#pragma unroll
        for (int rp = 0; rp < 4; ++rp) {
            const unsigned int a = raw[2 * rp][w], b = raw[2 * rp + 1][w];
            t[rp] = (c & 1) ? ((a >> 16) | (b & 0xFFFF0000u)) : ((a & 0xFFFFu) | (b << 16));
        }
        const unsigned at = buf + put_at[w];
        switch (c) {
            case 0: lds_write_b128<0 * ROWB>(at, t); break;
            case 1: lds_write_b128<1 * ROWB>(at, t); break;
            case 2: lds_write_b128<2 * ROWB>(at, t); break;
            case 3: lds_write_b128<3 * ROWB>(at, t); break;
            case 4: lds_write_b128<4 * ROWB>(at, t); break;
            case 5: lds_write_b128<5 * ROWB>(at, t); break;
            case 6: lds_write_b128<6 * ROWB>(at, t); break;
            default: lds_write_b128<7 * ROWB>(at, t); break;
        }
    };
    // direct path (token rows stored along k): load i of this wave fills LDS rows (4 i + wave) * 8 .. +8, lane ->
    // (row lane / 8, position lane % 8); rows past the last one there is are clamped (their results are never stored)
    const int lrow = wave * 8 + (lane >> 3);
    const int piece = (lane & 7) ^ ((lrow >> 1) & 7);
    size_t xsrc[8];
    if (!WGRAD) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int xr = row0 + i * 32 + lrow;
            xr = xr < n_rows ? xr : n_rows - 1;
            xsrc[i] = (size_t)xr * KD + piece * 8;
        }
    }
    auto dma_x = [&](unsigned char *Xs, int s, int i) {
        const bf16_t *base = s >= per_pair ? xa1 : xa0;
        __builtin_amdgcn_global_load_lds((gbl_void *)(base + xsrc[i] + stage_k(s)), (lds_void *)(Xs + (i * 4 + wave) * 1024), 16, 0, 0);
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // ---- consumers: as in the forward kernel ------------------------------------------------------------------
    const int orow = lane & 31, ohalf = lane >> 5, sw = (orow >> 1) & 7;
    unsigned kpos[BK / 16];
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) kpos[ks] = orow * ROWB + (((2 * ks + ohalf) ^ sw) << 4);
    const unsigned a_base = ww * 128 * ROWB, b_base = wt * 32 * ROWB;
    bf16x8 aop[2][4], bop[2][4];
    auto read_one = [&](unsigned wa, unsigned xa, int set, int q) {
        switch (q) {
            case 0: aop[set][0] = lds_read_b128<0>(wa); break;
            case 1: bop[set][0] = lds_read_b128<0>(xa); break;
            case 2: aop[set][1] = lds_read_b128<32 * ROWB>(wa); break;
            case 3: aop[set][2] = lds_read_b128<64 * ROWB>(wa); break;
            case 4: aop[set][3] = lds_read_b128<96 * ROWB>(wa); break;
            case 5: bop[set][1] = lds_read_b128<64 * ROWB>(xa); break;
            case 6: bop[set][2] = lds_read_b128<128 * ROWB>(xa); break;
            default: bop[set][3] = lds_read_b128<192 * ROWB>(xa); break;
        }
    };
    const unsigned wsA = lds_addr(WsA), xsA = lds_addr(XsA), wsB = lds_addr(WsB), xsB = lds_addr(XsB);

    // One k step: 16 MFMAs out of operand set ks & 1, each followed by at most one read of the next k step's operands and
    // one producer action.  ks 2: the blocks loaded one stage ago are transposed into the buffer that the coming barrier
    // completes (`wput`/`xput`).  ks 3 (behind the barrier): loads of stage `s_load` (into the buffer just freed, `Xl`).
    auto kstep = [&](int ks, unsigned wrd, unsigned xrd, int ks_rd, unsigned wput, unsigned xput, unsigned char *Xl, int s_load) {
        const int set = ks & 1;
        const unsigned wa = wrd + a_base + kpos[ks_rd], xa = xrd + b_base + kpos[ks_rd];
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const int b = m >> 2, a = m & 3;
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[set][a], bop[set][b], acc[a][b], 0, 0, 0);
            if (m < 8) read_one(wa, xa, set ^ 1, m);
            if (ks == 2) {
                if (m >= 8) put(wput, wraw, m - 8);
                else if (WGRAD) put(xput, xraw, m);
            }
            if (ks == 3) {
                if (m >= 8) load_w(s_load, m - 8);
                else if (WGRAD) load_x(s_load, m);
                else dma_x(Xl, s_load, m);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    if (nst > 0) {
        // stage 0 into buffer A in full; stage 1: direct loads into buffer B, register blocks stay in registers until
        // the first pass of the loop writes them
        const int s1 = nst > 1 ? 1 : 0;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            load_w(0, jj);
            if (WGRAD) load_x(0, jj);
            else dma_x(XsA, 0, jj);
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            put(wsA, wraw, c);
            if (WGRAD) put(xsA, xraw, c);
        }
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            load_w(s1, jj);
            if (WGRAD) load_x(s1, jj);
            else dma_x(XsB, s1, jj);
        }
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int q = 0; q < 8; ++q) read_one(wsA + a_base + kpos[0], xsA + b_base + kpos[0], 0, q);
#pragma unroll 1
        for (int kt = 0; kt < nst; ++kt) {
            const bool odd = kt & 1;
            const unsigned wcur = odd ? wsB : wsA, xcur = odd ? xsB : xsA;
            const unsigned wnxt = odd ? wsA : wsB, xnxt = odd ? xsA : xsB;
            unsigned char *Xl = odd ? XsB : XsA;                       // direct loads of stage kt + 2 land in the current buffer
            const int s_load = min(kt + 2, nst - 1);                   // past the end: the last stage again, never read
            wait_lds(aop[0], bop[0]);
            kstep(0, wcur, xcur, 1, 0, 0, Xl, s_load);
            wait_lds(aop[1], bop[1]);
            kstep(1, wcur, xcur, 2, 0, 0, Xl, s_load);
            wait_lds(aop[0], bop[0]);
            kstep(2, wcur, xcur, 3, wnxt, xnxt, Xl, s_load);            // register blocks of stage kt + 1 -> the other buffer
            wait_lds(aop[1], bop[1]);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            kstep(3, wnxt, xnxt, 0, 0, 0, Xl, s_load);
        }
        wait_lds(aop[0], bop[0]);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
    }

    // ---- epilogue: accumulators through this wave's 32 KB of LDS, out as 8 consecutive outputs of one row per lane ----
    unsigned char *region = wave == 0 ? WsA : wave == 1 ? XsA : wave == 2 ? WsB : XsB;
    constexpr int TROW = 32 * 4 + 16, TILEB = 32 * TROW;
    const int c = lane & 15, at = c >> 2, fi = (c & 3) * 8;
    const int f = wcol0 + ww * 128 + c * 8;
    OutT *obase = WGRAD ? outp + (size_t)e * XN * N : outp;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
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
        for (int p = 0; p < 8; ++p) {
            const int n = p * 4 + (lane >> 4);                  // row inside the 32-row sub-tile
            const unsigned char *gp = region + at * TILEB + n * TROW + fi * 4;
            const f32x4 g0 = *reinterpret_cast<const f32x4 *>(gp), g1 = *reinterpret_cast<const f32x4 *>(gp + 16);
            const int row = row0 + (2 * b + wt) * 32 + n;
            if (row < row_end && f < N) {
                OutT *dst = obase + (size_t)row * N + f;
                if constexpr (sizeof(OutT) == 4) {
                    *reinterpret_cast<f32x4 *>(dst) = g0;
                    *reinterpret_cast<f32x4 *>(dst + 4) = g1;
                } else {
                    *reinterpret_cast<u32x4 *>(dst) = u32x4{pack_bf16x2(g0[0], g0[1]), pack_bf16x2(g0[2], g0[3]),
                                                            pack_bf16x2(g1[0], g1[1]), pack_bf16x2(g1[2], g1[3])};
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

}  // namespace bwl

// Shapes the LDS kernels take: whole 64-wide reduction tiles for the data gradients (their reduction length is a
// multiple of 64), row counts that are multiples of 8 (every H and I is), and enough rows per expert to fill tiles.
bool bw_lds_applicable(const moe_shape_t &s) {
    return s.H % bwl::BK == 0 && s.I % bwl::BK == 0 && (long)s.T * s.K >= 128L * s.E;
}

// out[r][f] = sum_k a0[r][k] w0[e][k][f] (+ a1, w1), rows expert-sorted; `list` is the forward pass's per-XCD row-tile list
hipError_t launch_bw_lds_rows(const moe_shape_t &s, const bf16_t *a0, const bf16_t *a1, const bf16_t *w0, const bf16_t *w1,
                              const void *list, bf16_t *out, int KD, int N, hipStream_t st) {
    const int max_tiles = s.T * s.K / bwl::BT + s.E, tiles_per_xcd = (max_tiles + 7) / 8;
    const int nw = (N + bwl::BT - 1) / bwl::BT;
    hipLaunchKernelGGL((bwl::bw_lds_kernel<false, bf16_t>), dim3(8 * tiles_per_xcd * nw), dim3(256), 0, st, a0, a1, w0, w1,
                       reinterpret_cast<const i32x4 *>(list), tiles_per_xcd, (const int32_t *)nullptr, out, KD, 0, N, 0, nw, s.E,
                       s.T * s.K);
    return hipGetLastError();
}

// out[e][m][f] = sum over the rows r of expert e of P[r][m] Q[r][f]
hipError_t launch_bw_lds_wgrad(const moe_shape_t &s, const bf16_t *P, const bf16_t *Q, const int32_t *off, float *out, int M, int N,
                               hipStream_t st) {
    const int tm = (M + bwl::BT - 1) / bwl::BT, tn = (N + bwl::BT - 1) / bwl::BT;
    hipLaunchKernelGGL((bwl::bw_lds_kernel<true, float>), dim3(8 * ((s.E + 7) / 8) * tm * tn), dim3(256), 0, st, P, (const bf16_t *)nullptr,
                       Q, (const bf16_t *)nullptr, (const i32x4 *)nullptr, 0, off, out, 0, M, N, tm, tn, s.E, s.T * s.K);
    return hipGetLastError();
}

}  // namespace moe
