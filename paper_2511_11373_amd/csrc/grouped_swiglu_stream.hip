// Decode-sized batches (a handful of rows per expert): the grouped SwiGLU is a 1.2 GB weight stream
// with almost no arithmetic, so the kernels here are shaped by how HBM likes to be read.  Measured on
// MI355X, 128-byte pieces of many rows give 5.2-5.4 TB/s, 1 KB pieces 5.9 TB/s and whole 4 KB rows
// 6.25 TB/s; so every wave reads whole-row pieces of 1 KB (gate/up) or a contiguous 24 KB block of 16
// rows (down) with fully coalesced 16-byte loads, keeps the next item's loads in flight in registers
// while the current one is multiplied, and transposes through a wave-private LDS buffer into the
// MFMA operand layout.  Tokens are the 16-wide N side of v_mfma_f32_16x16x32_bf16 and live in
// registers for the whole block.
//
// v_mfma_f32_16x16x32_bf16: lane l feeds row l%16, k = 8*(l/16)..+7 of both operands; result register r
// is D[4*(l/16) + r][l%16].
#include "moe_internal.hpp"

namespace moe {

namespace stream {
constexpr int NIG = 2;                // items per block, gate/up (measured best among 1, 2, 4)
constexpr int NID = 1;                // items per wave, down (measured best among 1, 2)
constexpr int GROW = 1024 + 16;       // LDS bytes per staged gate/up row piece (1 KB + pad: conflict-free reads)
constexpr int DHALF = 768 + 16;       // LDS bytes per staged half row of Wd (I = 768 only)
}  // namespace stream

__device__ __forceinline__ float silu_mul_s(float g, float u) { return g / (1.0f + __expf(-g)) * u; }
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// ---- gate/up ------------------------------------------------------------------------------------------
// Block (ib, e): NIG items of 8 features of expert e.  An item is 8 rows of Wg and the same 8 rows of Wu;
// wave w multiplies the k range [512w, 512w+512) of all 16 rows, the four partial 16x16 results meet in
// LDS and wave (item % 4) applies silu(g)*u.  MFMA row 4q+j is gate feature 2q+j (j < 2) or up feature
// 2q+j-2, so a lane ends up with g and u of the same two features of one token.
// Requires H == 2048 (4 waves x 512), I % (8*NIG) == 0, bf16 storage.  (NIG = 2, NID = 1 measured best.)
__global__ __launch_bounds__(256, 2) void stream_gate_up_kernel(
    const bf16_t *__restrict__ xrows, const int32_t *__restrict__ row_map, int K_assign,
    const int32_t *__restrict__ off, const bf16_t *__restrict__ wg, const bf16_t *__restrict__ wu,
    bf16_t *__restrict__ act, int H, int I) {
    using namespace stream;
    __shared__ __attribute__((aligned(16))) unsigned char stage[4][16 * GROW];
    __shared__ __attribute__((aligned(16))) float partial[2][4][64 * 4];
    const int e = blockIdx.y;
    const int r_begin = off[e], r_end = off[e + 1];
    if (r_begin == r_end) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, q = lane >> 4;
    const int kbase = wave * 512;
    const int feat0 = blockIdx.x * (8 * NIG);

    // this lane's piece of each of the 16 rows of an item: bytes [16*lane, +16) of the wave's 1 KB of the row
    const size_t wrow_off = ((size_t)e * I + feat0) * H + kbase + lane * 8;
    unsigned char *mine = stage[wave];
    // MFMA row (lane%16) -> staged row
    const int mrow = n, mq = mrow >> 2, mj = mrow & 3;
    const int srow = mj < 2 ? 2 * mq + mj : 8 + 2 * mq + (mj - 2);
    const unsigned char *aptr = mine + srow * GROW + q * 16;

    for (int tg = r_begin; tg < r_end; tg += 16) {
        // token operand: 16 rows x this wave's 512 k, 8 values per lane per 32-wide step
        u32x4 xop[16];
        {
            const int row = tg + n;
            const bool ok = row < r_end;
            int src = ok ? row : tg;
            if (row_map) src = row_map[src] / K_assign;
            const bf16_t *xp = xrows + (size_t)src * H + kbase + q * 8;
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (ok) v = *reinterpret_cast<const u32x4 *>(xp + s * 32);
                xop[s] = v;
            }
        }
        u32x4 wreg[16];
        auto fetch = [&](int item) {
            const bf16_t *g = wg + wrow_off + (size_t)item * 8 * H;
            const bf16_t *u = wu + wrow_off + (size_t)item * 8 * H;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                wreg[r] = load_once(g + (size_t)r * H);
                wreg[8 + r] = load_once(u + (size_t)r * H);
            }
        };
        auto work = [&](int item) {
#pragma unroll
            for (int r = 0; r < 16; ++r) *reinterpret_cast<u32x4 *>(mine + r * GROW + lane * 16) = wreg[r];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_sched_barrier(0);
            if (item + 1 < NIG) fetch(item + 1);           // in flight while this item is multiplied
            __builtin_amdgcn_sched_barrier(0);
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(aptr + s * 64);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, as_bf16x8(xop[s]), acc, 0, 0, 0);
            }
            *reinterpret_cast<f32x4 *>(&partial[item & 1][wave][lane * 4]) = acc;
            __syncthreads();                              // also: every lane is done reading this wave's stage
            if (wave == (item & 3)) {
                f32x4 t = *reinterpret_cast<const f32x4 *>(&partial[item & 1][0][lane * 4]);
#pragma unroll
                for (int w = 1; w < 4; ++w) {
                    const f32x4 p = *reinterpret_cast<const f32x4 *>(&partial[item & 1][w][lane * 4]);
                    t[0] += p[0]; t[1] += p[1]; t[2] += p[2]; t[3] += p[3];
                }
                const int row = tg + n;
                if (row < r_end) {
                    const unsigned int pk = pack_bf16x2(silu_mul_s(t[0], t[2]), silu_mul_s(t[1], t[3]));
                    *reinterpret_cast<unsigned int *>(act + (size_t)row * I + feat0 + item * 8 + 2 * q) = pk;
                }
            }
        };
        fetch(0);
#pragma unroll 1
        for (int item = 0; item < NIG; ++item) work(item);   // not unrolled: keeps one item's loads in registers
        __syncthreads();       // partial[] and stage[] are reused by the next token group
    }
}

// ---- down -----------------------------------------------------------------------------------------------
// Wave (jb, e): NID items of 16 output features, each handled as two units of 16 rows x 384 k (768 bytes per
// row, 12 KB per unit, twelve coalesced 16-byte loads per lane).  Waves are independent: no k split across
// waves, no block barrier.  Requires I == 768, H % (64*NID) == 0, bf16 weights.
template <typename SO>
__global__ __launch_bounds__(256, 2) void stream_down_kernel(
    const bf16_t *__restrict__ act, const int32_t *__restrict__ off, const bf16_t *__restrict__ wd,
    SO *__restrict__ y, int H, int I) {
    using namespace stream;
    __shared__ __attribute__((aligned(16))) unsigned char stage[4][16 * DHALF];
    const int e = blockIdx.y;
    const int r_begin = off[e], r_end = off[e + 1];
    if (r_begin == r_end) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, q = lane >> 4;
    const int j0 = (blockIdx.x * 4 + wave) * (16 * NID);
    unsigned char *mine = stage[wave];
    // piece p = c*64 + lane of a unit -> row p/48, 16-byte column p%48; three loads cover four rows
    int goff[3], soff[3];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        const int p = c * 64 + lane;
        goff[c] = (p / 48) * I + (p % 48) * 8;             // elements
        soff[c] = (p / 48) * DHALF + (p % 48) * 16;        // bytes
    }
    const bf16_t *wbase = wd + ((size_t)e * H + j0) * I;
    const unsigned char *aptr = mine + n * DHALF + q * 16;

    for (int tg = r_begin; tg < r_end; tg += 16) {
        u32x4 xop[24];
        {
            const int row = tg + n;
            const bool ok = row < r_end;
            const bf16_t *xp = act + (size_t)(ok ? row : tg) * I + q * 8;
#pragma unroll
            for (int s = 0; s < 24; ++s) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (ok) v = *reinterpret_cast<const u32x4 *>(xp + s * 32);
                xop[s] = v;
            }
        }
        u32x4 wreg[12];
        auto fetch = [&](int unit) {
            const bf16_t *p = wbase + (size_t)(unit >> 1) * 16 * I + (unit & 1) * 384;
#pragma unroll
            for (int c = 0; c < 12; ++c)
                wreg[c] = load_once(p + (size_t)(c / 3) * 4 * I + goff[c % 3]);
        };
        fetch(0);
#pragma unroll 1
        for (int item = 0; item < NID; ++item) {              // not unrolled: keeps one unit's loads in registers
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int unit = item * 2 + half;
#pragma unroll
                for (int c = 0; c < 12; ++c) *reinterpret_cast<u32x4 *>(mine + (c / 3) * 4 * DHALF + soff[c % 3]) = wreg[c];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                __builtin_amdgcn_sched_barrier(0);
                if (unit + 1 < 2 * NID) fetch(unit + 1);      // in flight while this unit is multiplied
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int s = 0; s < 12; ++s) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(aptr + s * 64);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, as_bf16x8(xop[half * 12 + s]), acc, 0, 0, 0);
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();             // every lane has read the unit before it is overwritten
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                __builtin_amdgcn_sched_barrier(0);
            }
            const int row = tg + n;
            if (row < r_end) {
                SO *dst = y + (size_t)row * H + j0 + item * 16 + 4 * q;
                if constexpr (sizeof(SO) == 2) {
                    u32x2 pk = {pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3])};
                    *reinterpret_cast<u32x2 *>(dst) = pk;
                } else {
                    *reinterpret_cast<f32x4 *>(dst) = acc;
                }
            }
        }
    }
}

bool stream_gemm_applicable(const moe_shape_t &s) {
    using namespace stream;
    return s.dtype == MOE_BF16 && s.H == 2048 && s.I == 768 && s.I % (8 * NIG) == 0 && s.H % (64 * NID) == 0 &&
           (long)s.T * s.K <= 12L * s.E;      // measured: ahead of the tiled kernel up to 12 rows per expert on average, behind it from 16
}

hipError_t launch_grouped_swiglu_stream(const moe_shape_t &s, const bf16_t *x_rows, const int32_t *row_map,
                                        const int32_t *off, const bf16_t *wg, const bf16_t *wu, const bf16_t *wd,
                                        bf16_t *act, bf16_t *y_perm, hipStream_t st, Probe *probe) {
    using namespace stream;
    hipLaunchKernelGGL(stream_gate_up_kernel, dim3(s.I / (8 * NIG), s.E), dim3(256), 0, st, x_rows, row_map, s.K, off, wg,
                       wu, act, s.H, s.I);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    probe_mark(probe);
    hipLaunchKernelGGL(stream_down_kernel<bf16_t>, dim3(s.H / (64 * NID), s.E), dim3(256), 0, st, (const bf16_t *)act, off,
                       wd, y_perm, s.H, s.I);
    return hipGetLastError();
}

}  // namespace moe
