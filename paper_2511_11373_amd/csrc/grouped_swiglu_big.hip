// Large-batch grouped GEMM for bf16 storage: 256 weight rows x 256 token rows per block, direct
// global->LDS loads (no register staging), 64-wide k stages in LDS rings (three for the weights, two for the token rows),
// 32x32x16 bf16 MFMA.
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
// A row tile that holds at most 128 rows (the tail of an expert, or an expert with few rows) takes a variant of the
// main loop with a ring of three smaller LDS stages instead of two: it has a quarter of the arithmetic per stage or
// less, so with two stages every stage would wait out a whole memory round trip; with three, two stages' loads
// are in flight while one is multiplied, and such a tile costs little more than streaming its weights.
//
// Row tiles (expert, first row, end of the expert's rows) come from a list that a small kernel writes
// once per call, already split per XCD: blocks are dealt round-robin to the 8 XCDs, block b is slot b/8
// of XCD b%8, and XCD x owns a contiguous eighth of the row tiles, each with all its weight tiles, so
// that the blocks sharing an expert's weights and a row tile's tokens run behind one L2.  A block finds
// its tile with one 16-byte load at an address that depends on the block index alone.
#include "moe_internal.hpp"

namespace moe {

namespace big {
constexpr int BW = 256, BT = 256, BK = 64;
constexpr int ROWB = BK * 2;                  // bytes per LDS row
constexpr int OPB = 256 * ROWB;               // bytes per operand stage (32 KB)
constexpr int SHORT_ROWS = 128;               // row tiles of at most this many rows take the three-stage loop
constexpr int SHORT_STAGE = OPB + SHORT_ROWS * ROWB;      // its stage: 256 weight rows + 128 token rows (48 KB)
constexpr int LDS_BYTES = 5 * OPB;            // 160 KB: three weight stages and two token stages of long tiles (3 * SHORT_STAGE fits too)
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

// How a row tile is worked through: whole tiles take a branch-free loop; NX > 0 is the three-stage loop of short tiles,
// which always loads NX token sub-tiles of 32 rows (so that the number of loads in flight is known to the waits).
template <bool FULL, int NX>
struct TileMode { static constexpr bool full = FULL; static constexpr int nx = NX; };

// silu(g)*u with the hardware reciprocal (1 ulp): far inside the bf16 rounding that follows
__device__ __forceinline__ float silu_mul_f(float g, float u) { return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u; }

// What a block's 256 weight rows are and what leaves it: 256 rows of one matrix and their products (the down pass, or
// any plain grouped GEMM); 128 rows of W_gate and the same 128 of W_up and silu(gate)*up; or those rows and both
// products, each to a matrix of its own (the backward pass recomputes the pre-activations with it).
enum BigMode { kBigPlain = 0, kBigGateUp = 1, kBigGateUpRaw = 2 };

template <int MODE>
__global__ __launch_bounds__(256, 1) void grouped_gemm_big_kernel(
    const bf16_t *__restrict__ xrows, const int32_t *__restrict__ row_map, int K_assign,
    const i32x4 *__restrict__ tile_list, int tiles_per_xcd,
    const bf16_t *__restrict__ w0, const bf16_t *__restrict__ w1, bf16_t *__restrict__ outp, bf16_t *__restrict__ outp2,
    int KD, int NW, int n_wtiles, int n_rows) {
    using namespace big;
    constexpr bool GATE_UP = MODE != kBigPlain;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];

    // ---- which tile --------------------------------------------------------------------------
    // Slot s of an XCD falls into row tile s / n_wtiles of that XCD's list; the entry there describes the run of
    // consecutive row tiles of the same expert around it.  The run's blocks are walked weight tile fastest in
    // the gate/up pass (neighbours share their token rows) and row tile fastest in the down pass (neighbours
    // share their weights): measured, the passes differ by about a percent either way.
    const int slot = blockIdx.x >> 3;
    const i32x4 *entry = tile_list + 2 * ((blockIdx.x & 7) * tiles_per_xcd + slot / n_wtiles);
    const i32x4 ea = entry[0], eb = entry[1];
    // the same in every lane: kept in scalar registers
    const int e = __builtin_amdgcn_readfirstlane(ea[0]), row_end = __builtin_amdgcn_readfirstlane(ea[2]);
    if (e < 0) return;
    const int run_tiles = __builtin_amdgcn_readfirstlane(eb[0]);                     // row tiles in the run
    const int in_run = slot - __builtin_amdgcn_readfirstlane(ea[3]) * n_wtiles;      // ea[3]: first row tile of the run in this XCD's list
    const int wtile = GATE_UP ? in_run % n_wtiles : in_run / run_tiles;
    const int rt = GATE_UP ? in_run / n_wtiles : in_run % run_tiles;
    // ea[1]: the expert's first row, eb[1]: the run's first tile in the expert
    const int row0 = __builtin_amdgcn_readfirstlane(ea[1]) + (__builtin_amdgcn_readfirstlane(eb[1]) + rt) * BT;
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
    // token rows: gathered.  Rows past the expert's end are replaced by its last row: they are multiplied like the
    // others and never stored, and all lanes that stand for such a row fetch the same line, so a ragged tile takes in
    // little more than the rows it has (the expert's end comes with the tile's list entry, at no extra round trip).
    // The eight row numbers are fetched together, under one test of the map pointer: one round trip, not eight in a row.
    int xr[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) xr[i] = min(row0 + i * 32 + lrow, min(row_end, n_rows) - 1);
    if (row_map) {
        int assignment[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) assignment[i] = row_map[xr[i]];
#pragma unroll
        for (int i = 0; i < 8; ++i) xr[i] = assignment[i] / K_assign;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // weights: rows are a fixed stride apart (the launcher guarantees whole weight tiles)
        const bf16_t *wm = GATE_UP && i >= 4 ? w1 : w0;
        const int wr = GATE_UP ? (i & 3) * 32 + lrow : i * 32 + lrow;
        src[2 * i] = wm + ((size_t)e * NW + wrow0 + wr) * KD + piece * 8;
        src[2 * i + 1] = xrows + (size_t)xr[i] * KD + piece * 8;
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
    // A ragged tile skips the operand reads and the products of token sub-tiles it does not have; a wave left without any
    // reads nothing.  (The loads are issued all the same, so that the number in flight is known.)
    auto read_live = [&](int q) { return q == 5 ? nb > 1 : q == 6 ? nb > 2 : q == 7 ? nb > 3 : nb > 0; };
    // One 16-wide k step: 16 MFMAs out of operand set ks&1.  A wave is alone on its SIMD, so an instruction
    // that is not an MFMA only comes for free in the shadow of the MFMA issued just before it (the matrix
    // pipe is busy for 8 passes per MFMA): the 8 operand reads of the following k step are therefore dealt out one per
    // MFMA, and the global->LDS loads at most one per two MFMAs - issued back to back they queue up in front of the
    // texture unit and hold up the MFMAs behind them (all 16 of a stage in one k step: 7 % slower).
    auto kstep = [&](auto mode_c, int ks, unsigned wrd, unsigned xrd, int ks_rd, unsigned char *Wn,
                     unsigned char *Xn, int k_w, int k_x) {
        constexpr bool FULL = decltype(mode_c)::full;
        constexpr int NX = decltype(mode_c)::nx;
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
            if (m < 8 && (FULL || read_live(m))) read_one(wa, xa, set ^ 1, m);
            if (NX > 0) {
                // short tiles: all loads in the last k step, weight and token loads alternating
                if (ks == 3 && (!(m & 1) || (m >> 1) < NX)) issue(Wn, Xn, (m & 1) ? k_x : k_w, m);
            } else {
                // long tiles: the 8 token loads in the last k step (one per two MFMAs), the 8 weight loads in the first two
                // k steps (one per four MFMAs); the wait in front of the barrier lets exactly the weight loads stay under way
                if (ks == 3 && (m & 1)) issue(Wn, Xn, k_x, 2 * (m >> 1) + 1);
                if (ks < 2 && (m & 3) == 3) issue(Wn, Xn, k_w, 2 * (ks * 4 + (m >> 2)));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop ------------------------------------------------------------------------------------
    // One block barrier per 64-wide stage.  Operand registers are double-buffered per 16-wide k step.  The barrier sits
    // in front of the last k step of a stage: by then this wave has read everything it needs from the current buffers
    // and its own loads of the next stage have landed, so behind the barrier the current buffers are free in every wave
    // and the next ones complete.  The last k step therefore reads the first operands of the next stage and issues
    // loads into the buffers just freed.
    // Long tiles keep the weights in a ring of three stages and the token rows in a ring of two.  The token rows of the
    // stage after the next are issued in that last k step, into the buffer just freed (three k steps to arrive: they
    // come from L2 or the last-level cache, each row being read by 48 blocks).  The WEIGHTS of the stage after the next
    // are issued earlier, during the first two k steps of the current stage, into the third weight buffer, which the
    // stage before this one left: they have six to seven k steps to arrive - a weight tile is read by four blocks only
    // and often comes from HBM - and the loads of a stage are spread over three k steps instead of one.  The last stages
    // reload the final k tile instead of branching around the loads.  Every wave issues all 16 loads of a stage, live
    // token rows or not (rows past the tile's end are the expert's last row again), so the waits can count.
    const int nk = KD / BK;      // KD is a multiple of BK (checked by the launcher)
    const int k_last = KD - BK;
    const unsigned wsA = lds_addr(lds);
    auto all_loads = [&](unsigned char *Ws, unsigned char *Xs, int k0, int kind) {      // kind 0: weights, 1: token rows
#pragma unroll
        for (int i = 0; i < 8; ++i) issue(Ws, Xs, k0, 2 * i + kind);
    };
    auto run = [&](auto mode_c) {
        unsigned char *w_cur = lds, *w_nxt = lds + OPB, *w_aft = lds + 2 * OPB;
        unsigned char *x_cur = lds + 3 * OPB, *x_nxt = lds + 4 * OPB;
        all_loads(w_cur, x_cur, 0, 0);
        all_loads(w_cur, x_cur, 0, 1);
        all_loads(w_nxt, x_nxt, min(BK, k_last), 0);
        all_loads(w_nxt, x_nxt, min(BK, k_last), 1);
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");      // stage 0 has landed
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (read_live(q)) read_one(lds_addr(w_cur) + a_base + kpos[0], lds_addr(x_cur) + b_base + kpos[0], 0, q);
#pragma unroll 1
        for (int kt = 0; kt < nk; ++kt) {
            const unsigned wcur = lds_addr(w_cur), xcur = lds_addr(x_cur), wnxt = lds_addr(w_nxt), xnxt = lds_addr(x_nxt);
            // weights of stage kt + 2: during k steps 0 and 1, into the buffer that stage kt - 1 left (w_aft); token rows of
            // stage kt + 2: during k step 3, into this stage's buffer
            const int k_w = min((kt + 2) * BK, k_last), k_x = min((kt + 2) * BK, k_last);
            wait_lds_reads<0>(aop[0], bop[0]);
            kstep(mode_c, 0, wcur, xcur, 1, w_aft, x_cur, k_w, k_x);
            wait_lds_reads<0>(aop[1], bop[1]);
            kstep(mode_c, 1, wcur, xcur, 2, w_aft, x_cur, k_w, k_x);
            wait_lds_reads<0>(aop[0], bop[0]);
            kstep(mode_c, 2, wcur, xcur, 3, w_cur, x_cur, k_w, k_x);
            wait_lds_reads<0>(aop[1], bop[1]);
            asm volatile("s_waitcnt vmcnt(8)" ::: "memory");      // all but the newest weight stage has landed
            __builtin_amdgcn_s_barrier();
            kstep(mode_c, 3, wnxt, xnxt, 0, w_cur, x_cur, k_w, k_x);
            unsigned char *t = w_cur;
            w_cur = w_nxt; w_nxt = w_aft; w_aft = t;
            t = x_cur; x_cur = x_nxt; x_nxt = t;
        }
    };
    // Short tiles: a ring of three stages (weights at the start of a stage, token rows behind them).  The loads of stage
    // kt + 3 are issued during the last k step of stage kt into the buffer that stage just left, so two stages' loads
    // are in flight while a stage is multiplied.  Every wave issues exactly 8 + NX loads per stage (token rows past the
    // tile's end are the expert's last row again: loaded, multiplied into accumulators that are never stored), which is
    // what lets the wait in front of the barrier name the number of loads that may still be under way.
    auto run_short = [&](auto mode_c) {
        constexpr int NL = 8 + decltype(mode_c)::nx;
        unsigned char *p_cur = lds, *p_nxt = lds + SHORT_STAGE, *p_aft = lds + 2 * SHORT_STAGE;
#pragma unroll
        for (int st = 0; st < 3; ++st)
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (!(j & 1) || (j >> 1) < decltype(mode_c)::nx)
                    issue(lds + st * SHORT_STAGE, lds + st * SHORT_STAGE + OPB, min(st * BK, k_last), j);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NL) : "memory");
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (read_live(q)) read_one(wsA + a_base + kpos[0], wsA + OPB + b_base + kpos[0], 0, q);
#pragma unroll 1
        for (int kt = 0; kt < nk; ++kt) {
            const unsigned wcur = lds_addr(p_cur), xcur = wcur + OPB;
            const unsigned wnxt = lds_addr(p_nxt), xnxt = wnxt + OPB;
            const int k_load = min((kt + 3) * BK, k_last);
            wait_lds_reads<0>(aop[0], bop[0]);
            kstep(mode_c, 0, wcur, xcur, 1, p_cur, p_cur + OPB, k_load, k_load);
            wait_lds_reads<0>(aop[1], bop[1]);
            kstep(mode_c, 1, wcur, xcur, 2, p_cur, p_cur + OPB, k_load, k_load);
            wait_lds_reads<0>(aop[0], bop[0]);
            kstep(mode_c, 2, wcur, xcur, 3, p_cur, p_cur + OPB, k_load, k_load);
            wait_lds_reads<0>(aop[1], bop[1]);
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NL) : "memory");      // stage kt + 1 has landed; kt + 2 may be under way
            __builtin_amdgcn_s_barrier();
            kstep(mode_c, 3, wnxt, xnxt, 0, p_cur, p_cur + OPB, k_load, k_load);
            unsigned char *t = p_cur;
            p_cur = p_nxt;
            p_nxt = p_aft;
            p_aft = t;
        }
    };
    const int rows_here = row_end - row0;
    if (rows_here > SHORT_ROWS) {
        if (nsub == 8) run(TileMode<true, 0>{});
        else run(TileMode<false, 0>{});
    } else if (rows_here > 64) {
        run_short(TileMode<false, 4>{});
    } else {
        run_short(TileMode<false, 2>{});
    }
    wait_lds_reads<0>(aop[0], bop[0]);
    MOE_WAIT_VMCNT(0);

    // ---- epilogue -----------------------------------------------------------------------------------
    // Of each 32x32 accumulator tile a lane holds token lane%32 and features 8*rq + 4*(lane/32) .. +3, rq = 0..3.
    // After rounding to bf16 that is a pair of registers per rq; exchanging the upper half-wave of an even rq's pair
    // with the lower half-wave of the following odd one's leaves every lane with 8 consecutive features of its
    // token (lanes 0-31: those of the even rq, lanes 32-63: of the odd one).  Results leave as 16-byte pieces, two
    // lanes to 32 bytes of a token row, and the stores of a sub-tile complete whole 128-byte lines in L2; neither
    // LDS nor a barrier is involved.
    constexpr int NA = MODE == kBigGateUp ? 2 : 4;       // output tiles per sub-tile: silu(gate)*up, or the four tiles as they are
    // the lane index is taken afresh: a value derived from the one above would be kept alive across the main loop, where
    // no register is free for it
    const int lane_now = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    const int tok = lane_now & 31, half = lane_now >> 5;
    const int fbase = wrow0 + (GATE_UP ? ww * 64 : ww * 128) + 8 * half;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        if (b >= nb) break;
        const int row = row0 + (2 * b + wt) * 32 + tok;
#pragma unroll
        for (int a = 0; a < NA; ++a) {
            unsigned d[4][2];
#pragma unroll
            for (int rq = 0; rq < 4; ++rq)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int r = 4 * rq + 2 * j;
                    d[rq][j] = MODE == kBigGateUp ? pack_bf16x2(silu_mul_f(acc[a][b][r], acc[a + 2][b][r]),
                                                                silu_mul_f(acc[a][b][r + 1], acc[a + 2][b][r + 1]))
                                                  : pack_bf16x2(acc[a][b][r], acc[a][b][r + 1]);
                }
            // tiles 2 and 3 of the two-output form are the up products of the features of tiles 0 and 1
            bf16_t *dst = (MODE == kBigGateUpRaw && a >= 2) ? outp2 : outp;
            const int fa = MODE == kBigGateUpRaw ? (a & 1) : a;
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const u32x2 s0 = __builtin_amdgcn_permlane32_swap(d[2 * p][0], d[2 * p + 1][0], false, false);
                const u32x2 s1 = __builtin_amdgcn_permlane32_swap(d[2 * p][1], d[2 * p + 1][1], false, false);
                const u32x4 pk = {s0[0], s1[0], s0[1], s1[1]};
                const int f = fbase + fa * 32 + 16 * p;
                if (row < row_end && f < NW) *reinterpret_cast<u32x4 *>(dst + (size_t)row * NW + f) = pk;
            }
        }
    }
}

bool big_gemm_applicable(const moe_shape_t &s) {
    // whole weight tiles in both passes, whole k tiles, and enough rows per expert: measured at H = 2048, I = 768, 128
    // experts, this kernel overtakes the 64-row tiled one between 56 and 64 rows per expert on average (its 256-row tiles
    // are mostly short ones there, which cost it little more than the weights they stream)
    return s.dtype == MOE_BF16 && s.H % big::BW == 0 && s.I % (big::BW / 2) == 0 && (long)s.T * s.K >= 60L * s.E;
}

// ---- per-XCD row-tile list ---------------------------------------------------------------------------
// Two 16-byte words per row tile: list[2*(x*tiles_per_xcd + i)] = (expert, first row of the expert, end of the
// expert's rows, i) and the word after it (1, t, 0, 0), t = the tile's index inside the expert; expert = -1 past the
// end of an XCD's list.  (The first word's last field and the second word's first describe a run of consecutive row
// tiles of one expert starting at position i; the lists written here only hold runs of one tile.)
//
// Row tiles come in two kinds: long ones (more than SHORT_ROWS rows; bound by the matrix cores) and short ones (the
// tail of an expert or an expert with few rows; bound by streaming their weights).  A batch with skewed routing has
// many of both, and an XCD that works through a stretch of short tiles alone cannot pull them from memory faster
// than its own link allows while its matrix cores idle.  So each kind is dealt out evenly: XCD x gets a contiguous
// eighth of the long tiles and a contiguous eighth of the short ones (both in expert order, so that the tiles
// sharing an expert's weights still meet behind one L2), and inside an XCD's list the short tiles are spread
// evenly among the long ones, so that at any time a few CUs stream while the rest multiply.
// One block: tile counts per expert, their prefix sums, then one entry per thread and step, its expert found by
// bisection in the prefix sums.
__global__ __launch_bounds__(1024) void build_xcd_tile_list_kernel(const int32_t *__restrict__ off, int E,
                                                                   int tiles_per_xcd, i32x4 *__restrict__ list) {
    __shared__ int lfirst[kMaxExperts + 1], sfirst[kMaxExperts + 1];
    for (int e = threadIdx.x; e < E; e += 1024) {
        const int cnt = off[e + 1] - off[e], nt = (cnt + big::BT - 1) / big::BT;
        const int tail_short = cnt > 0 && cnt - (nt - 1) * big::BT <= big::SHORT_ROWS;
        lfirst[e] = nt - tail_short;
        sfirst[e] = tail_short;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int lrun = 0, srun = 0;
        for (int e = 0; e < E; ++e) {
            const int lv = lfirst[e], sv = sfirst[e];
            lfirst[e] = lrun; sfirst[e] = srun;
            lrun += lv; srun += sv;
        }
        lfirst[E] = lrun; sfirst[E] = srun;
    }
    __syncthreads();
    const int n_long = lfirst[E], n_short = sfirst[E];
    // XCD x takes a contiguous share of each kind, q = N / 8 tiles or one more.  The r = N % 8 larger shares of the long
    // tiles go to XCDs 0 .. rl - 1, those of the short tiles to the XCDs that follow (rl, rl + 1, ... round the ring), so
    // that the totals differ by one tile at most: with a handful of blocks per CU, one tile more on an XCD is one more
    // round of blocks there while the others idle (measured at 1536 tokens with a single long tile: the XCD that got
    // both extra tiles ended at 219 us, the others at 175).
    const int ql = n_long >> 3, rl = n_long & 7, qs = n_short >> 3, rs = n_short & 7;
    for (int idx = threadIdx.x; idx < 8 * tiles_per_xcd; idx += 1024) {
        const int x = idx / tiles_per_xcd, i = idx - x * tiles_per_xcd;
        int s_extra_before = 0;                                      // XCDs y < x with a larger share of the short tiles
        for (int y = 0; y < x; ++y) s_extra_before += ((y - rl) & 7) < rs;
        const int l0 = x * ql + min(x, rl), s0 = x * qs + s_extra_before;
        const int nl = ql + (x < rl), ns = qs + (((x - rl) & 7) < rs), tot = nl + ns;      // <= tiles_per_xcd by the launcher's bound
        i32x4 ea = {-1, 0, 0, 0}, eb = {1, 0, 0, 0};
        if (i < tot) {
            // position i of the XCD's list holds a short tile when the running share of short tiles steps up there
            const int s_before = (int)((long)i * ns / tot), is_short = (int)((long)(i + 1) * ns / tot) > s_before;
            const int *first = is_short ? sfirst : lfirst;
            const int t = is_short ? s0 + s_before : l0 + (i - s_before);
            int lo = 0, hi = E;                                 // last e with first[e] <= t (experts without such tiles repeat a value)
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (first[mid] <= t) lo = mid; else hi = mid;
            }
            const int n_long_e = lfirst[lo + 1] - lfirst[lo];
            ea = i32x4{lo, off[lo], off[lo + 1], i};
            eb = i32x4{1, is_short ? n_long_e : t - lfirst[lo], 0, 0};
        }
        list[2 * idx] = ea;
        list[2 * idx + 1] = eb;
    }
}

// Row tiles per XCD list: every expert ends with at most one partial tile, so there are at most T*K/BT + E row
// tiles; an eighth of the long ones and an eighth of the short ones, each rounded up.
int big_tiles_per_xcd(const moe_shape_t &s) { return (s.T * s.K / big::BT + s.E + 7) / 8 + 1; }

size_t big_tile_list_bytes(const moe_shape_t &s) { return (size_t)2 * 8 * big_tiles_per_xcd(s) * sizeof(i32x4); }

hipError_t launch_grouped_swiglu_big(const moe_shape_t &s, const bf16_t *x_rows, const int32_t *row_map,
                                     const int32_t *off, const bf16_t *wg, const bf16_t *wu, const bf16_t *wd,
                                     bf16_t *act, int32_t *tile_map, bf16_t *y_perm, hipStream_t st, Probe *probe) {
    using namespace big;
    const int tiles_per_xcd = big_tiles_per_xcd(s);
    i32x4 *list = reinterpret_cast<i32x4 *>(tile_map);
    hipLaunchKernelGGL(build_xcd_tile_list_kernel, dim3(1), dim3(1024), 0, st, off, s.E, tiles_per_xcd, list);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    probe_mark(probe);
    const int nw1 = (s.I + BW / 2 - 1) / (BW / 2), nw2 = (s.H + BW - 1) / BW;
    const int n_rows = s.T * s.K;
    hipLaunchKernelGGL(grouped_gemm_big_kernel<kBigGateUp>, dim3(8 * tiles_per_xcd * nw1), dim3(256), 0, st, x_rows, row_map,
                       s.K, list, tiles_per_xcd, wg, wu, act, (bf16_t *)nullptr, s.H, s.I, nw1, n_rows);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
    probe_mark(probe);
    hipLaunchKernelGGL(grouped_gemm_big_kernel<kBigPlain>, dim3(8 * tiles_per_xcd * nw2), dim3(256), 0, st, (const bf16_t *)act,
                       (const int32_t *)nullptr, 1, list, tiles_per_xcd, wd, wd, y_perm, (bf16_t *)nullptr, s.I, s.H, nw2, n_rows);
    return hipGetLastError();
}

// ---- both expert pre-activations of expert-sorted rows, g = W_gate[e] v and u = W_up[e] v, each to a matrix of its own --------
// (the backward pass recomputes them with this).  Needs whole k tiles and whole 128-feature weight tiles.  row_token,
// when given, names the row of `rows` that each expert-sorted row is a copy of.
bool big_pre_activations_applicable(int H, int I) { return H % big::BK == 0 && I % (big::BW / 2) == 0; }

hipError_t launch_big_tile_list(const moe_shape_t &s, const int32_t *off, void *list, hipStream_t st) {
    const int tiles_per_xcd = big_tiles_per_xcd(s);
    hipLaunchKernelGGL(build_xcd_tile_list_kernel, dim3(1), dim3(1024), 0, st, off, s.E, tiles_per_xcd, reinterpret_cast<i32x4 *>(list));
    return hipGetLastError();
}

// (row_div: expert-sorted row r is row row_token[r] / row_div of `rows`: 1 for a row -> token map, K for the forward
// pass's row -> assignment map)
hipError_t launch_big_pre_activations(const moe_shape_t &s, const bf16_t *rows, const int32_t *row_token, int row_div,
                                      const void *list, const bf16_t *wg, const bf16_t *wu, bf16_t *g, bf16_t *u, hipStream_t st) {
    const int tiles_per_xcd = big_tiles_per_xcd(s);
    const int nw = s.I / (big::BW / 2);
    hipLaunchKernelGGL(grouped_gemm_big_kernel<kBigGateUpRaw>, dim3(8 * tiles_per_xcd * nw), dim3(256), 0, st, rows, row_token,
                       row_div, reinterpret_cast<const i32x4 *>(list), tiles_per_xcd, wg, wu, g, u, s.H, s.I, nw, s.T * s.K);
    return hipGetLastError();
}

// the down pass alone, y = W_down[e] act over expert-sorted rows, with a tile list that launch_big_tile_list wrote
// (needs H a multiple of 256 and whole k tiles of I)
bool big_down_applicable(int H, int I) { return H % big::BW == 0 && I % big::BK == 0; }
hipError_t launch_big_down(const moe_shape_t &s, const bf16_t *act, const void *list, const bf16_t *wd, bf16_t *y_perm,
                           hipStream_t st) {
    const int tiles_per_xcd = big_tiles_per_xcd(s);
    const int nw2 = s.H / big::BW;
    hipLaunchKernelGGL(grouped_gemm_big_kernel<kBigPlain>, dim3(8 * tiles_per_xcd * nw2), dim3(256), 0, st, act,
                       (const int32_t *)nullptr, 1, reinterpret_cast<const i32x4 *>(list), tiles_per_xcd, wd, wd, y_perm,
                       (bf16_t *)nullptr, s.I, s.H, nw2, s.T * s.K);
    return hipGetLastError();
}

}  // namespace moe
