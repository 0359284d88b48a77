// Large-batch grouped GEMMs of the backward pass: the forward pass's 256 x 256 x 64 LDS pipeline with operands that
// are stored ACROSS the reduction axis read out of LDS by the transposing LDS load.
//
// out[x][f] = sum_k X[x][k] * W[f][k], 32x32x16 bf16 MFMAs, 4 waves in a 2 x 2 grid, 16 accumulators per wave, LDS
// stages of 32 KB per operand (a ring of three for the operand whose loads go out early, of two for the other), every
// operand brought in by global_load_lds two stages ahead with the loads spread over three k steps, one block barrier per
// stage in front of its last k step - all as in grouped_swiglu_big.hip.  What differs is how an operand lies in LDS:
//   * stored along k (the token-row operand of the data gradients): 256 rows x 128 bytes, 16-byte piece j of row r at
//     position j ^ ((r >> 1) & 7), read with ds_read_b128, as there;
//   * stored across k (W[e] as [k][f] for the data gradients; both operands of a weight gradient, where k runs over
//     the expert's token rows): 64 k-rows x 512 bytes exactly as they lie in memory (a load instruction copies two
//     whole k-rows), the 16-byte piece p of k-row k at position p ^ ((k & 3) << 2).  ds_read_b64_tr_b16 turns that
//     into MFMA operands: in every group of 16 lanes, lane i receives as element j the halfword i % 4 of the 8 bytes
//     that lane 4 j + i / 4 points at; with lane s of a group pointing at k-row s / 4 (of the 4 this instruction covers)
//     and rows 4 (s % 4) .. +3, lane i ends up with its row's 4 consecutive k.  Two such reads make the 8 k values
//     of a lane.  The swizzle puts the four k-rows a half-wave reads on different banks.
// Rows past an expert's last one (weight gradients only) are fetched from a zero-filled line instead.
#include "moe_internal.hpp"

namespace moe {
namespace bwl {

constexpr int BT = 256, BK = 64, ROWB = BK * 2, OPB = 256 * ROWB;
constexpr int KROWB = 512;                        // bytes per k-row of an operand stored across k

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void gbl_void;

template <int OFF>
__device__ __forceinline__ u32x4 lds_read_b128(unsigned addr) {
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return v;
}
template <int OFF>
__device__ __forceinline__ u32x2 lds_read_tr_b64(unsigned addr) {
    u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return v;
}
// waits for every LDS access of this wave; names the operand registers so that their MFMAs stay behind it
__device__ __forceinline__ void wait_lds(u32x4 (&a)[4], u32x4 (&b)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3])
                 :
                 : "memory");
}
__device__ __forceinline__ unsigned lds_addr(const void *p) {
    return (unsigned)(size_t)(const __attribute__((address_space(3))) void *)p;
}

// WGRAD = false: out[r][f] = sum over pairs p and k of xa_p[r][k] * w_p[e][k][f]   (rows r of expert e, bf16 out)
// WGRAD = true : out[e][m][f] = sum over the rows r of expert e of xa_0[r][m] * w_0[r][f]   (float out)
// zeros: 512 zero bytes.  x_token (w_token, weight gradients only), when given: row r of xa_0 (w_0) is not stored in
// expert-sorted order but is row x_token[r] of the matrix passed, e.g. the token a row is a copy of.
// MAPPED (weight gradients): 0 no map, 1 the rows of xa_0 through x_token, 2 the rows of w_0 through w_token.
template <bool WGRAD, int MAPPED, typename OutT>
__global__ __launch_bounds__(256, 1) void bw_lds_kernel(const bf16_t *__restrict__ xa0, const bf16_t *__restrict__ xa1,
                                                        const bf16_t *__restrict__ w0, const bf16_t *__restrict__ w1,
                                                        const i32x4 *__restrict__ tile_list, int tiles_per_xcd,
                                                        const int32_t *__restrict__ off, const bf16_t *__restrict__ zeros,
                                                        const int32_t *__restrict__ x_token, const int32_t *__restrict__ w_token,
                                                        OutT *__restrict__ outp, int KD, int XN, int N, int n_xtiles,
                                                        int n_wtiles, int E, int n_rows) {
    __shared__ __attribute__((aligned(1024))) unsigned char WsA[OPB];
    __shared__ __attribute__((aligned(1024))) unsigned char XsA[OPB];
    __shared__ __attribute__((aligned(1024))) unsigned char WsB[OPB];
    __shared__ __attribute__((aligned(1024))) unsigned char XsB[OPB];
    __shared__ __attribute__((aligned(1024))) unsigned char ThirdS[OPB];      // third stage of the operand that is loaded early

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
        k_begin = __builtin_amdgcn_readfirstlane(off[e]);
        k_end = __builtin_amdgcn_readfirstlane(off[e + 1]);
    } else {                                       // the forward pass's per-XCD row-tile list, row tile fastest
        const i32x4 *entry = tile_list + 2 * ((blockIdx.x & 7) * tiles_per_xcd + slot / n_wtiles);
        const i32x4 ea = entry[0], eb = entry[1];
        e = __builtin_amdgcn_readfirstlane(ea[0]);
        if (e < 0) return;
        row_end = __builtin_amdgcn_readfirstlane(ea[2]);
        const int run_tiles = __builtin_amdgcn_readfirstlane(eb[0]);
        const int in_run = slot - __builtin_amdgcn_readfirstlane(ea[3]) * n_wtiles;
        wcol0 = (in_run / run_tiles) * BT;
        row0 = __builtin_amdgcn_readfirstlane(ea[1]) + (__builtin_amdgcn_readfirstlane(eb[1]) + in_run % run_tiles) * BT;
        k_begin = 0;
        k_end = KD;
    }
    const int n_pairs = (!WGRAD && xa1) ? 2 : 1;
    const int per_pair = (k_end - k_begin + BK - 1) / BK;
    const int nst = per_pair * n_pairs;            // stages; 0 for an expert without rows (its gradient is zero)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ww = wave & 1, wt = wave >> 1;

    // ---- producers: 16 loads per wave and stage, even ones for the weight-side operand ---------------------------
    // Operand stored across k: load i of this wave copies k-rows 8 i + 2 wave, + 1 of the stage; lane -> (k-row lane / 32,
    // position lane % 32).  (k & 3) does not depend on i, so neither does the piece a lane fetches; a piece past the
    // operand's last column is replaced by the last one there is (its products are never stored).
    const int kl0 = 2 * wave + (lane >> 5), pos = lane & 31;
    const int gpiece = pos ^ ((kl0 & 3) << 2);
    const int col_w = min(wcol0 + gpiece * 8, N - 8), col_x = WGRAD ? min(row0 + gpiece * 8, XN - 8) : 0;
    auto stage_k = [&](int s) { return k_begin + (s % per_pair) * BK; };
    // a weight gradient with one operand addressed through a token map keeps the 8 row numbers of the stage it loads
    // next in registers; they are fetched one stage before the loads that use them
    const int32_t *tok_map = MAPPED == 1 ? x_token : w_token;
    int tk[8];
    auto load_tokens = [&](int s, int (&t)[8], int i) { t[i] = tok_map[min(stage_k(s) + 8 * i + kl0, n_rows - 1)]; };
    // Operand stored along k (token rows of the data gradients): load i fills LDS rows (4 i + wave) * 8 .. + 8, lane ->
    // (row lane / 8, position lane % 8); rows past the last one there is are clamped (their results are never stored)
    const int lrow = wave * 8 + (lane >> 3);
    const int piece = (lane & 7) ^ ((lrow >> 1) & 7);
    size_t xsrc[8];
    if (!WGRAD) {
        int xr[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) xr[i] = min(row0 + i * 32 + lrow, min(row_end, n_rows) - 1);      // rows past the expert's end: its last row again (one line for all of them)
        if (x_token) {                                                 // the eight row numbers in one round trip
            int token[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) token[i] = x_token[xr[i]];
#pragma unroll
            for (int i = 0; i < 8; ++i) xr[i] = token[i];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) xsrc[i] = (size_t)xr[i] * KD + piece * 8;
    }
    auto issue = [&](int s, unsigned char *Wl, unsigned char *Xl, int j, const int (&t)[8]) {
        const int i = j >> 1, k0 = stage_k(s);
        const bool second = s >= per_pair;
        const int k = k0 + 8 * i + kl0;
        if (!(j & 1)) {
            const bf16_t *base = WGRAD ? w0 : (second ? w1 : w0) + (size_t)e * KD * N;
            const bf16_t *src = base + (size_t)(MAPPED == 2 ? t[i] : k) * N + col_w;
            if (WGRAD && k >= k_end) src = zeros + pos * 8;
            __builtin_amdgcn_global_load_lds((gbl_void *)src, (lds_void *)(Wl + (i * 4 + wave) * 1024), 16, 0, 0);
        } else if (WGRAD) {
            const bf16_t *src = xa0 + (size_t)(MAPPED == 1 ? t[i] : k) * XN + col_x;
            if (k >= k_end) src = zeros + pos * 8;
            __builtin_amdgcn_global_load_lds((gbl_void *)src, (lds_void *)(Xl + (i * 4 + wave) * 1024), 16, 0, 0);
        } else {
            const bf16_t *base = second ? xa1 : xa0;
            __builtin_amdgcn_global_load_lds((gbl_void *)(base + xsrc[i] + k0), (lds_void *)(Xl + (i * 4 + wave) * 1024), 16, 0, 0);
        }
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // ---- consumers --------------------------------------------------------------------------------------------
    // along-k operand: lane (row l % 32, half l / 32); k step ks uses pieces 2 ks + half
    const int orow = lane & 31, ohalf = lane >> 5, sw = (orow >> 1) & 7;
    unsigned kpos[BK / 16];
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) kpos[ks] = orow * ROWB + (((2 * ks + ohalf) ^ sw) << 4);
    const unsigned xb_base = wt * 32 * ROWB;
    // across-k operand: group g = l / 16 holds rows 16 (g & 1) .. + 16 of a 32-row tile and k 8 (g / 2) .. + 8; lane s of the
    // group points at k-row s / 4 (+ 4 for the second read) and rows 4 (s % 4) .. + 3.  Tile t of this wave begins at piece
    // 4 t' (t' = 4 ww + t on the weight side, 2 t + wt on the other); the swizzle flips the low two bits of t'.
    const int g4 = lane >> 4, s16 = lane & 15, kq = s16 >> 2;
    const unsigned tr_lane = (8 * (g4 >> 1) + kq) * KROWB + ((2 * (g4 & 1) + ((s16 & 3) >> 1)) << 4) + 8 * (s16 & 1);
    unsigned a_tr[4], b_tr[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        a_tr[t] = tr_lane + ((4 * ww + (t ^ kq)) << 6);
        b_tr[t] = tr_lane + (((2 * t + wt) ^ kq) << 6);
    }
    u32x4 aop[2][4], bop[2][4];
    // the operand reads of a k step, in the order the MFMAs first need them: 16 for a weight gradient (both operands
    // across k), 12 for a data gradient
    auto read_one = [&](unsigned wbuf, unsigned xbuf, int ks_rd, int set, int q) {
        const unsigned wk = wbuf + ks_rd * 16 * KROWB, xk = xbuf + ks_rd * 16 * KROWB, xa = xbuf + xb_base + kpos[ks_rd];
        auto tr = [&](u32x4 &dst, unsigned at, int hi) {
            if (hi) dst.hi = lds_read_tr_b64<4 * KROWB>(at);
            else dst.lo = lds_read_tr_b64<0>(at);
        };
        if (WGRAD) {
            switch (q) {
                case 0: tr(aop[set][0], wk + a_tr[0], 0); break;
                case 1: tr(aop[set][0], wk + a_tr[0], 1); break;
                case 2: tr(bop[set][0], xk + b_tr[0], 0); break;
                case 3: tr(bop[set][0], xk + b_tr[0], 1); break;
                case 4: tr(aop[set][1], wk + a_tr[1], 0); break;
                case 5: tr(aop[set][1], wk + a_tr[1], 1); break;
                case 6: tr(aop[set][2], wk + a_tr[2], 0); break;
                case 7: tr(aop[set][2], wk + a_tr[2], 1); break;
                case 8: tr(aop[set][3], wk + a_tr[3], 0); break;
                case 9: tr(aop[set][3], wk + a_tr[3], 1); break;
                case 10: tr(bop[set][1], xk + b_tr[1], 0); break;
                case 11: tr(bop[set][1], xk + b_tr[1], 1); break;
                case 12: tr(bop[set][2], xk + b_tr[2], 0); break;
                case 13: tr(bop[set][2], xk + b_tr[2], 1); break;
                case 14: tr(bop[set][3], xk + b_tr[3], 0); break;
                default: tr(bop[set][3], xk + b_tr[3], 1); break;
            }
        } else {
            switch (q) {
                case 0: tr(aop[set][0], wk + a_tr[0], 0); break;
                case 1: tr(aop[set][0], wk + a_tr[0], 1); break;
                case 2: bop[set][0] = lds_read_b128<0>(xa); break;
                case 3: tr(aop[set][1], wk + a_tr[1], 0); break;
                case 4: tr(aop[set][1], wk + a_tr[1], 1); break;
                case 5: tr(aop[set][2], wk + a_tr[2], 0); break;
                case 6: tr(aop[set][2], wk + a_tr[2], 1); break;
                case 7: tr(aop[set][3], wk + a_tr[3], 0); break;
                case 8: tr(aop[set][3], wk + a_tr[3], 1); break;
                case 9: bop[set][1] = lds_read_b128<64 * ROWB>(xa); break;
                case 10: bop[set][2] = lds_read_b128<128 * ROWB>(xa); break;
                case 11: bop[set][3] = lds_read_b128<192 * ROWB>(xa); break;
                default: break;
            }
        }
    };
    constexpr int NREAD = WGRAD ? 16 : 12;
    const unsigned wsA = lds_addr(WsA), xsA = lds_addr(XsA), wsB = lds_addr(WsB), xsB = lds_addr(XsB);

    // One k step: 16 MFMAs out of operand set ks & 1, each followed by one read of the next k step's operands; the loads
    // of stage `s_load` are dealt out at most one per two MFMAs (back to back they hold up the MFMAs behind them).
    // The operand that is NOT addressed through a row map is the early one: its loads of stage s_load go out during the
    // first two k steps (one per four MFMAs) into the third buffer of its ring; the other operand's loads follow in the
    // last k step (one per two MFMAs), into the buffer the barrier has just freed, with the row numbers fetched in k step 0.
    constexpr bool EARLY_W = MAPPED != 2;
    auto kstep = [&](int ks, unsigned wrd, unsigned xrd, int ks_rd, unsigned char *early_buf, unsigned char *late_buf, int s_load) {
        const int set = ks & 1;
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const int b = m >> 2, a = m & 3;
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, aop[set][a]),
                                                                __builtin_bit_cast(bf16x8, bop[set][b]), acc[a][b], 0, 0, 0);
            if (m < NREAD) read_one(wrd, xrd, ks_rd, set ^ 1, m);
            if (ks < 2 && (m & 3) == 3) issue(s_load, early_buf, early_buf, 2 * (ks * 4 + (m >> 2)) + (EARLY_W ? 0 : 1), tk);
            if (ks == 3 && (m & 1)) issue(s_load, late_buf, late_buf, 2 * (m >> 1) + (EARLY_W ? 1 : 0), tk);
            if (MAPPED && ks == 0 && m < 8) load_tokens(s_load, tk, m);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    if (nst > 0) {
        // stages 0 and 1 (the last stage again if there is only one; it is never read) into buffers A and B
        const int s1 = nst > 1 ? 1 : 0;
        int tk1[8];
        if (MAPPED) {
#pragma unroll
            for (int i = 0; i < 8; ++i) { load_tokens(0, tk, i); load_tokens(s1, tk1, i); }
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) issue(0, WsA, XsA, j, tk);
#pragma unroll
        for (int j = 0; j < 16; ++j) issue(s1, WsB, XsB, j, tk1);
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int q = 0; q < NREAD; ++q) read_one(wsA, xsA, 0, 0, q);
        // rings: three buffers for the early operand, two for the late one
        unsigned char *e_cur = EARLY_W ? WsA : XsA, *e_nxt = EARLY_W ? WsB : XsB, *e_aft = ThirdS;
        unsigned char *l_cur = EARLY_W ? XsA : WsA, *l_nxt = EARLY_W ? XsB : WsB;
#pragma unroll 1
        for (int kt = 0; kt < nst; ++kt) {
            const unsigned wcur = lds_addr(EARLY_W ? e_cur : l_cur), xcur = lds_addr(EARLY_W ? l_cur : e_cur);
            const unsigned wnxt = lds_addr(EARLY_W ? e_nxt : l_nxt), xnxt = lds_addr(EARLY_W ? l_nxt : e_nxt);
            const int s_load = min(kt + 2, nst - 1);                        // past the end: the last stage again, never read
            wait_lds(aop[0], bop[0]);
            kstep(0, wcur, xcur, 1, e_aft, l_cur, s_load);
            wait_lds(aop[1], bop[1]);
            kstep(1, wcur, xcur, 2, e_aft, l_cur, s_load);
            wait_lds(aop[0], bop[0]);
            kstep(2, wcur, xcur, 3, e_aft, l_cur, s_load);
            wait_lds(aop[1], bop[1]);
            // stage kt + 1 has landed; what may still be under way is what this stage issued: the early operand's 8 loads
            // and, with a row map, the 8 row numbers (for those the compiler adds a wait of its own in front of their first
            // use in the last k step, which also waits for the early loads: with a row map the ring only spreads the loads)
            if (MAPPED) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            kstep(3, wnxt, xnxt, 0, e_aft, l_cur, s_load);
            unsigned char *t = e_cur;
            e_cur = e_nxt; e_nxt = e_aft; e_aft = t;
            t = l_cur; l_cur = l_nxt; l_nxt = t;
        }
        wait_lds(aop[0], bop[0]);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }

    // ---- epilogue: straight from the accumulators ---------------------------------------------------------------
    // Of each 32x32 tile a lane holds output row lane % 32 (a token row, or a row m of a weight gradient) and columns
    // 8 rq + 4 (lane / 32) .. + 3, rq = 0..3.  Float results leave as they are, 16 bytes per lane and rq; bf16 results
    // are paired up first: exchanging the upper half-wave of an even rq's packed pair with the lower half-wave of the
    // following odd one's leaves every lane with 8 consecutive columns.  Either way the stores of a tile complete whole
    // 128-byte lines in L2.
    const int lane_now = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));      // taken afresh: see grouped_swiglu_big.hip
    const int orow_e = lane_now & 31, half = lane_now >> 5;
    OutT *obase = WGRAD ? outp + (size_t)e * XN * N : outp;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int row = row0 + (2 * b + wt) * 32 + orow_e;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int f0 = wcol0 + ww * 128 + a * 32;
            if constexpr (sizeof(OutT) == 4) {
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    const int f = f0 + 8 * rq + 4 * half;
                    if (row < row_end && f < N)
                        *reinterpret_cast<f32x4 *>(obase + (size_t)row * N + f) =
                            f32x4{acc[a][b][4 * rq], acc[a][b][4 * rq + 1], acc[a][b][4 * rq + 2], acc[a][b][4 * rq + 3]};
                }
            } else {
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    const int r0 = 8 * p;
                    const u32x2 s0 = __builtin_amdgcn_permlane32_swap(pack_bf16x2(acc[a][b][r0], acc[a][b][r0 + 1]),
                                                                      pack_bf16x2(acc[a][b][r0 + 4], acc[a][b][r0 + 5]), false, false);
                    const u32x2 s1 = __builtin_amdgcn_permlane32_swap(pack_bf16x2(acc[a][b][r0 + 2], acc[a][b][r0 + 3]),
                                                                      pack_bf16x2(acc[a][b][r0 + 6], acc[a][b][r0 + 7]), false, false);
                    const int f = f0 + 16 * p + 8 * half;
                    if (row < row_end && f < N)
                        *reinterpret_cast<u32x4 *>(obase + (size_t)row * N + f) = u32x4{s0[0], s1[0], s0[1], s1[1]};
                }
            }
        }
    }
}

}  // namespace bwl

// Shapes the LDS kernels take: whole 64-wide reduction tiles for the data gradients (their reduction length is a
// multiple of 64) and row counts that are multiples of 8 (every H and I is).  No batch is too small for them: measured
// at H = 2048, I = 768, 128 experts they beat the LDS-free kernels from 4 tokens on (0.67 against 0.86 ms) - a backward
// pass streams every weight and writes every gradient whatever the batch, and these kernels stream better.
bool bw_lds_applicable(const moe_shape_t &s) { return s.H % bwl::BK == 0 && s.I % bwl::BK == 0; }

// out[r][f] = sum_k a0[r][k] w0[e][k][f] (+ a1, w1), rows expert-sorted (row r of a0 and a1 is row a0_token[r] of the matrix
// passed when a map is given); `list` is the forward pass's per-XCD row-tile list
hipError_t launch_bw_lds_rows(const moe_shape_t &s, const bf16_t *a0, const bf16_t *a1, const bf16_t *w0, const bf16_t *w1,
                              const void *list, const bf16_t *zeros, const int32_t *a0_token, bf16_t *out, int KD, int N,
                              hipStream_t st) {
    const int tiles_per_xcd = big_tiles_per_xcd(s);
    const int nw = (N + bwl::BT - 1) / bwl::BT;
    hipLaunchKernelGGL((bwl::bw_lds_kernel<false, 0, bf16_t>), dim3(8 * tiles_per_xcd * nw), dim3(256), 0, st, a0, a1, w0, w1,
                       reinterpret_cast<const i32x4 *>(list), tiles_per_xcd, (const int32_t *)nullptr, zeros, a0_token, (const int32_t *)nullptr, out, KD, 0, N, 0, nw, s.E,
                       s.T * s.K);
    return hipGetLastError();
}

// out[e][m][f] = sum over the rows r of expert e of P[r][m] Q[r][f]; at most one of the two through a row map
hipError_t launch_bw_lds_wgrad(const moe_shape_t &s, const bf16_t *P, const bf16_t *Q, const int32_t *off, const bf16_t *zeros,
                               const int32_t *p_token, const int32_t *q_token, float *out, int M, int N, hipStream_t st) {
    const int tm = (M + bwl::BT - 1) / bwl::BT, tn = (N + bwl::BT - 1) / bwl::BT;
    const dim3 grid(8 * ((s.E + 7) / 8) * tm * tn);
#define MOE_BW_WGRAD(MAPPED)                                                                                                         \
    hipLaunchKernelGGL((bwl::bw_lds_kernel<true, MAPPED, float>), grid, dim3(256), 0, st, P, (const bf16_t *)nullptr, Q,              \
                       (const bf16_t *)nullptr, (const i32x4 *)nullptr, 0, off, zeros, p_token, q_token, out, 0, M, N, tm, tn, s.E, \
                       s.T * s.K)
    if (p_token) MOE_BW_WGRAD(1);
    else if (q_token) MOE_BW_WGRAD(2);
    else MOE_BW_WGRAD(0);
#undef MOE_BW_WGRAD
    return hipGetLastError();
}

}  // namespace moe
