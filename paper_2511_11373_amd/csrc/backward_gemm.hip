// Grouped GEMMs of the backward pass (bf16 operands, float accumulation) without LDS.
//
// The backward pass multiplies by matrices along the axis they are NOT stored along: dact = dy * Wd reduces over
// the rows of Wd[e] (stored [H][I]), dWd[e] = dy^T * act reduces over the token rows of both operands.  The bf16
// MFMAs want 8 consecutive reduction indices per lane.  Instead of transposed copies in HBM or a transposing trip
// through LDS, a lane loads an 8 x 8 block (8 consecutive reduction indices x 8 consecutive rows, 16 bytes per
// reduction index, fully coalesced across the wave) and transposes it in registers; the 8 rows it then holds
// operands for become its rows in 8 different MFMAs.  That fixes which rows an MFMA tile covers:
//
//   v_mfma_f32_16x16x32_bf16: lane l = (i, q) = (l % 16, l / 16) feeds row i, reduction indices 8q .. 8q+7, of
//   both operands; result register j of the lane is D[4q + j][i].
//   Tile (ja, jb) of a wave's 128 x 128 output multiplies A rows {8 i + ja} by B rows {8 i' + jb}, i, i' = 0..15:
//   a lane's 8 result columns over jb are 8 consecutive output columns, so results leave as 32-byte pieces.
//
// A wave owns 8 x 8 such tiles (256 accumulator registers, one wave per SIMD), a block 2 x 2 waves = 256 x 256
// outputs; waves that share operand rows meet in the L1.  Operands that ARE stored along the reduction axis are
// loaded straight into the same row assignment (8 rows x 16 bytes per lane).  The next 32-wide reduction step is
// in flight in registers while the current one is multiplied.
#include "moe_internal.hpp"

namespace moe {
namespace bw {

constexpr int BT = 256;     // block tile edge (both ways); a wave owns 128 x 128

// T[c] = the 8 consecutive reduction indices of row c, from R[jj] = 8 consecutive rows at reduction index jj
__device__ __forceinline__ void transpose8x8(const u32x4 (&R)[8], u32x4 (&T)[8]) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const int w = c >> 1;
#pragma unroll
        for (int rp = 0; rp < 4; ++rp) {
            const unsigned int a = R[2 * rp][w], b = R[2 * rp + 1][w];
            T[c][rp] = (c & 1) ? ((a >> 16) | (b & 0xFFFF0000u)) : ((a & 0xFFFFu) | (b << 16));
        }
    }
}

__device__ __forceinline__ u32x4 load16(const bf16_t *p, bool ok) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (ok) v = *reinterpret_cast<const u32x4 *>(p);
    return v;
}

// One operand of a wave for one 32-wide reduction step.
//   KSLOW = false: stored [rows][ld] with the reduction index contiguous; lane (i, q) loads rows row0 + 8 i + j,
//                  j = 0..7, indices k0 + 8q .. +7.
//   KSLOW = true : stored [reduction][ld] with the rows contiguous; lane (i, q) loads reduction indices
//                  k0 + 8q + jj, jj = 0..7, rows row0 + 8 i .. +7, and transposes.
// Rows >= row_end and reduction indices >= k_end read as zero.  Addresses are plain arithmetic (gathered rows are
// copied into place beforehand), so a step's loads can be issued without waiting for anything.
template <bool KSLOW>
struct Operand {
    const bf16_t *base;
    int ld;
    __device__ __forceinline__ void fetch(u32x4 (&raw)[8], int row0, int row_end, int k0, int k_end, int i, int q) const {
        if (KSLOW) {
            const int r = row0 + 8 * i;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                const int k = k0 + 8 * q + jj;
                raw[jj] = load16(base + (size_t)k * ld + r, k < k_end && r < row_end);   // row counts are multiples of 8
            }
        } else {
            const int k = k0 + 8 * q;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int r = row0 + 8 * i + j;
                raw[j] = load16(base + (size_t)r * ld + k, r < row_end && k < k_end);    // the reduction length is a multiple of 8
            }
        }
    }
    __device__ __forceinline__ void finish(const u32x4 (&raw)[8], u32x4 (&op)[8]) const {
        if (KSLOW) transpose8x8(raw, op);
        else {
#pragma unroll
            for (int j = 0; j < 8; ++j) op[j] = raw[j];
        }
    }
};

__device__ __forceinline__ void mfma_8x8(f32x4 (&acc)[8][8], const u32x4 (&a)[8], const u32x4 (&b)[8]) {
#pragma unroll
    for (int ja = 0; ja < 8; ++ja)
#pragma unroll
        for (int jb = 0; jb < 8; ++jb)
            acc[ja][jb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[ja]), __builtin_bit_cast(bf16x8, b[jb]),
                                                                  acc[ja][jb], 0, 0, 0);
}

// acc += A[row0a.., k] * B[row0b.., k] over k in [k_begin, k_end), 32 at a time, next step prefetched.
template <bool A_KSLOW, bool B_KSLOW>
__device__ __forceinline__ void reduce_range(f32x4 (&acc)[8][8], const Operand<A_KSLOW> &A, int row0a, int enda,
                                             const Operand<B_KSLOW> &B, int row0b, int endb, int k_begin, int k_end,
                                             int i, int q) {
    if (k_begin >= k_end) return;
    u32x4 ra[8], rb[8], oa[8], ob[8];
    A.fetch(ra, row0a, enda, k_begin, k_end, i, q);
    B.fetch(rb, row0b, endb, k_begin, k_end, i, q);
    for (int k0 = k_begin; k0 < k_end; k0 += 32) {
        A.finish(ra, oa);
        B.finish(rb, ob);
        // the raw registers are free again: the next step's loads fly during the MFMAs (past k_end they are masked off)
        A.fetch(ra, row0a, enda, k0 + 32, k_end, i, q);
        B.fetch(rb, row0b, endb, k0 + 32, k_end, i, q);
        mfma_8x8(acc, oa, ob);
    }
}

__device__ __forceinline__ void store8(float *p, const float (&v)[8]) {
    *reinterpret_cast<f32x4 *>(p) = f32x4{v[0], v[1], v[2], v[3]};
    *reinterpret_cast<f32x4 *>(p + 4) = f32x4{v[4], v[5], v[6], v[7]};
}
__device__ __forceinline__ void store8(bf16_t *p, const float (&v)[8]) {
    *reinterpret_cast<u32x4 *>(p) = u32x4{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
}

// out[row][col], rows row0 + 8 (4q + j) + ja, cols col0 + 8 i + jb
template <typename OutT>
__device__ __forceinline__ void store_tile(const f32x4 (&acc)[8][8], OutT *out, size_t ld, int row0, int row_end, int col0,
                                           int col_end, int i, int q) {
    const int col = col0 + 8 * i;
    if (col >= col_end) return;                                  // column counts are multiples of 8
#pragma unroll
    for (int ja = 0; ja < 8; ++ja)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = row0 + 8 * (4 * q + j) + ja;
            if (row < row_end) {
                float v[8];
#pragma unroll
                for (int jb = 0; jb < 8; ++jb) v[jb] = acc[ja][jb][j];
                store8(out + (size_t)row * ld + col, v);
            }
        }
}

// ---- rows x weights: out[r][n] = sum over pairs p and k of A_p[r][k] * W_p[e][.], expert-sorted ragged rows ----------
//   W_KSLOW: W_p[e] is stored [KD][N] (reduce over its rows: the data-gradient products); else [N][KD] (forward form).
// Row tiles of BT rows come from the (expert, first row) list the tiled forward kernels use.
template <bool W_KSLOW, typename OutT>
__global__ __launch_bounds__(256, 1) void bw_rows_kernel(const bf16_t *__restrict__ a0, const bf16_t *__restrict__ a1,
                                                         const bf16_t *__restrict__ w0, const bf16_t *__restrict__ w1,
                                                         const int32_t *__restrict__ off, const int32_t *__restrict__ tile_map,
                                                         int max_tiles, OutT *__restrict__ out, int KD, int N) {
    if ((int)blockIdx.x >= tile_map[2 * max_tiles]) return;
    const int e = tile_map[2 * blockIdx.x], row0 = tile_map[2 * blockIdx.x + 1];
    const int row_end = off[e + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, i = lane & 15, q = lane >> 4;
    const int r0 = row0 + (wave & 1) * 128, n0 = blockIdx.y * BT + (wave >> 1) * 128;
    if (r0 >= row_end || n0 >= N) return;
    f32x4 acc[8][8];
#pragma unroll
    for (int ja = 0; ja < 8; ++ja)
#pragma unroll
        for (int jb = 0; jb < 8; ++jb) acc[ja][jb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const size_t wsz = (size_t)KD * N;
    for (int p = 0; p < (a1 ? 2 : 1); ++p) {
        const Operand<false> A{p ? a1 : a0, KD};
        const Operand<W_KSLOW> B{(p ? w1 : w0) + (size_t)e * wsz, W_KSLOW ? N : KD};
        reduce_range<false, W_KSLOW>(acc, A, r0, row_end, B, n0, N, 0, KD, i, q);
    }
    store_tile<OutT>(acc, out, (size_t)N, r0, row_end, n0, N, i, q);
}

// ---- weight gradients: out[e][m][n] = sum over the rows r of expert e of P[r][m] * Q[r][n] ---------------------------
// Both operands are stored by row r.  Experts without rows get zeros.
__global__ __launch_bounds__(256, 1) void bw_wgrad_kernel(const bf16_t *__restrict__ P, const bf16_t *__restrict__ Q,
                                                          const int32_t *__restrict__ off, float *__restrict__ out, int M, int N,
                                                          int n_tiles_n, int tiles_per_expert, int E) {
    // blocks go round-robin to the 8 XCDs: all tiles of an expert are dealt to one XCD, whose L2 then serves the
    // re-reads of the expert's rows by its other tiles
    const int slot = blockIdx.x >> 3;
    const int e = (slot / tiles_per_expert) * 8 + (blockIdx.x & 7), tile = slot % tiles_per_expert;
    if (e >= E) return;
    const int mt = tile / n_tiles_n, nt = tile - mt * n_tiles_n;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, i = lane & 15, q = lane >> 4;
    const int m0 = mt * BT + (wave & 1) * 128, n0 = nt * BT + (wave >> 1) * 128;
    if (m0 >= M || n0 >= N) return;
    f32x4 acc[8][8];
#pragma unroll
    for (int ja = 0; ja < 8; ++ja)
#pragma unroll
        for (int jb = 0; jb < 8; ++jb) acc[ja][jb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const Operand<true> A{P, M};
    const Operand<true> B{Q, N};
    reduce_range<true, true>(acc, A, m0, M, B, n0, N, off[e], off[e + 1], i, q);
    store_tile<float>(acc, out + (size_t)e * M * N, (size_t)N, m0, M, n0, N, i, q);
}

}  // namespace bw

// out[r][n] = sum_k rows[r][k] * W[e][n][k]  (W_KSLOW = false)  or  sum_k rows[r][k] * W[e][k][n]  (true), optionally the
// sum of two such products.  rows are expert-sorted (off).
template <bool W_KSLOW, typename OutT>
static hipError_t launch_rows(const bf16_t *a0, const bf16_t *a1, const bf16_t *w0, const bf16_t *w1, const int32_t *off,
                              const int32_t *tile_map, int max_tiles, OutT *out, int KD, int N, hipStream_t st) {
    dim3 grid(max_tiles, (N + bw::BT - 1) / bw::BT);
    hipLaunchKernelGGL((bw::bw_rows_kernel<W_KSLOW, OutT>), grid, dim3(256), 0, st, a0, a1, w0, w1, off, tile_map, max_tiles, out, KD, N);
    return hipGetLastError();
}

hipError_t launch_bw_rows_kfast(const bf16_t *rows, const bf16_t *w, const int32_t *off, const int32_t *tile_map, int max_tiles,
                                bf16_t *out, int KD, int N, hipStream_t st) {
    return launch_rows<false, bf16_t>(rows, nullptr, w, nullptr, off, tile_map, max_tiles, out, KD, N, st);
}
hipError_t launch_bw_rows_kslow(const bf16_t *a0, const bf16_t *a1, const bf16_t *w0, const bf16_t *w1, const int32_t *off,
                                const int32_t *tile_map, int max_tiles, bf16_t *out, int KD, int N, hipStream_t st) {
    return launch_rows<true, bf16_t>(a0, a1, w0, w1, off, tile_map, max_tiles, out, KD, N, st);
}
hipError_t launch_bw_wgrad(const bf16_t *P, const bf16_t *Q, const int32_t *off, int E, float *out, int M, int N, hipStream_t st) {
    const int tm = (M + bw::BT - 1) / bw::BT, tn = (N + bw::BT - 1) / bw::BT;
    hipLaunchKernelGGL(bw::bw_wgrad_kernel, dim3(8 * ((E + 7) / 8) * tm * tn), dim3(256), 0, st, P, Q, off, out, M, N, tn, tm * tn, E);
    return hipGetLastError();
}

}  // namespace moe
