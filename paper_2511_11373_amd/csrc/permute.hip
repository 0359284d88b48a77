// Expert-sorted permutation: a stable counting sort of the T*K assignments by
// expert id, in three steps (per-chunk LDS histograms, a scan over chunks and
// experts, a stable scatter).  Ranks come from ballots and prefix sums, never
// from the return value of an atomic, so the order inside an expert's segment
// is the assignment order and the result is unique.
#include "moe_internal.hpp"

namespace moe {

// Step 1: one wave per chunk of kPermChunk assignments; per-chunk histogram [nchunks, E].
__global__ __launch_bounds__(256) void permute_hist_kernel(const int32_t *__restrict__ idx, int n, int E,
                                                           int32_t *__restrict__ chunk_base) {
    extern __shared__ int hist_all[];   // [4][E]
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int chunk = blockIdx.x * 4 + wave;
    int *hist = hist_all + (size_t)wave * E;
    for (int e = lane; e < E; e += 64) hist[e] = 0;
    __syncthreads();
    const int a0 = chunk * kPermChunk;
    if (a0 < n) {
        const int a1 = min(a0 + kPermChunk, n);
        for (int a = a0 + lane; a < a1; a += 64) atomicAdd(&hist[min(max(idx[a], 0), E - 1)], 1);   // counts: order free
    }
    __syncthreads();
    if (a0 < n)
        for (int e = lane; e < E; e += 64) chunk_base[(size_t)chunk * E + e] = hist[e];
}

// Step 2: one block.  Turns the histograms into the first output row of every (chunk, expert) and
// writes expert_offsets.  Thread (p, e) owns the p-th slice of the chunk range of expert e; P slices per
// expert with P * E <= 1024, so one pass covers all experts.
__global__ __launch_bounds__(1024) void permute_scan_kernel(int32_t *__restrict__ chunk_base, int nchunks, int E,
                                                            int32_t *__restrict__ expert_offsets) {
    __shared__ int part[1024];       // [P][G] slice sums
    __shared__ int etotal[kMaxExperts + 1];
    int P = 1;
    while (P < 16 && P * 2 * E <= 1024 && P * 2 <= nchunks) P *= 2;
    const int G = 1024 / P;          // >= E
    const int cps = (nchunks + P - 1) / P;
    const int p = threadIdx.x / G, e = threadIdx.x % G;
    const int cb = p * cps, ce = min(cb + cps, nchunks);
    const bool mine = e < E;
    // the walks over this thread's chunks fetch 8 counts at a time so that the loads overlap
    int s = 0;
    if (mine)
        for (int c = cb; c < ce; c += 8) {
            int v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = c + j < ce ? chunk_base[(size_t)(c + j) * E + e] : 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) s += v[j];
        }
    part[threadIdx.x] = s;
    __syncthreads();
    int before = 0;                  // rows of expert e in the slices before p
    if (mine) {
        int tot = 0;
        for (int pp = 0; pp < P; ++pp) {
            const int v = part[pp * G + e];
            if (pp < p) before += v;
            tot += v;
        }
        if (p == 0) etotal[e] = tot;
    }
    __syncthreads();
    if (threadIdx.x == 0) {          // exclusive scan over experts (serial; E <= 1024)
        int run = 0;
        for (int i = 0; i < E; ++i) { const int v = etotal[i]; etotal[i] = run; run += v; }
        etotal[E] = run;
    }
    __syncthreads();
    for (int i = threadIdx.x; i <= E; i += 1024) expert_offsets[i] = etotal[i];
    if (mine) {
        int run = etotal[e] + before;
        for (int c = cb; c < ce; c += 8) {
            int v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = c + j < ce ? chunk_base[(size_t)(c + j) * E + e] : 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (c + j < ce) chunk_base[(size_t)(c + j) * E + e] = run;
                run += v[j];
            }
        }
    }
}

// Step 3: one wave per chunk.  Walks its assignments 64 at a time in order; lanes holding the same
// expert find each other with log2(E) ballots; row = running first row of that expert + number of
// lower lanes in the group.
__global__ __launch_bounds__(256) void permute_scatter_kernel(const int32_t *__restrict__ idx, int n, int E,
                                                              int ebits, const int32_t *__restrict__ chunk_base,
                                                              int32_t *__restrict__ row_to_assign,
                                                              int32_t *__restrict__ assign_to_row) {
    extern __shared__ int next_all[];   // [4][E] next free row per expert, private to a wave
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int chunk = blockIdx.x * 4 + wave;
    const int a0 = chunk * kPermChunk;
    if (a0 >= n) return;
    volatile int *next_row = next_all + (size_t)wave * E;
    for (int e = lane; e < E; e += 64) next_row[e] = chunk_base[(size_t)chunk * E + e];
    __builtin_amdgcn_wave_barrier();
    const int a1 = min(a0 + kPermChunk, n);
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int ab = a0; ab < a1; ab += 64) {
        const int a = ab + lane;
        const bool live = a < a1;
        const int e = live ? min(max(idx[a], 0), E - 1) : 0;
        unsigned long long peers = __ballot(live);
        for (int b = 0; b < ebits; ++b) {
            const unsigned long long has = __ballot((e >> b) & 1);
            peers &= ((e >> b) & 1) ? has : ~has;
        }
        if (live) {
            const int rank = __popcll(peers & below);
            const int row = next_row[e] + rank;
            row_to_assign[row] = a;
            assign_to_row[a] = row;
        }
        __builtin_amdgcn_wave_barrier();
        if (live && (peers & below) == 0ull) next_row[e] = next_row[e] + __popcll(peers);
        __builtin_amdgcn_wave_barrier();
    }
}

// ---- small batches: the whole permutation (and the GEMM's row-tile list) in one block --------------
__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(v, d, 64);
        if (lane >= d) v += o;
    }
    return v;
}
// Exclusive scan of one value per thread over a 1024-thread block; *total receives the sum.
__device__ __forceinline__ int block_exclusive_scan(int v, int *wave_sums /* [17] shared */, int *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int inc = wave_inclusive_scan(v, lane);
    __syncthreads();                       // wave_sums may still be read from a previous call
    if (lane == 63) wave_sums[wave] = inc;
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wave; ++w) before += wave_sums[w];
    if (threadIdx.x == 1023) *total = before + inc;
    return before + inc - v;
}

// n <= 16 * kPermChunk assignments.  Wave w owns chunk w of `chunk` assignments (a multiple of 64 chosen
// by the launcher so that all 16 waves have work).  Same three steps as the large path with
// the histograms kept in LDS.  With tile_rows > 0 it also writes the list of (expert, first row) row
// tiles that the grouped GEMM consumes: tile_map[2*i], tile_map[2*i+1], count at tile_map[2*max_tiles].
__global__ __launch_bounds__(1024) void permute_small_kernel(const int32_t *__restrict__ idx, int n, int chunk, int E, int ebits,
                                                             int32_t *__restrict__ expert_offsets,
                                                             int32_t *__restrict__ row_to_assign,
                                                             int32_t *__restrict__ assign_to_row, int tile_rows,
                                                             int max_tiles, int32_t *__restrict__ tile_map) {
    extern __shared__ int lds[];            // [16][E] per-wave counts, then per-wave next free row
    __shared__ int offs[kMaxExperts + 1];
    __shared__ int wave_sums[17];
    __shared__ int total;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int i = threadIdx.x; i < 16 * E; i += 1024) lds[i] = 0;
    __syncthreads();
    const int a0 = min(wave * chunk, n), a1 = min(a0 + chunk, n);
    int *mine = lds + (size_t)wave * E;
    for (int a = a0 + lane; a < a1; a += 64) atomicAdd(&mine[min(max(idx[a], 0), E - 1)], 1);
    __syncthreads();
    // per expert: running sum over the 16 waves -> rows of e in earlier chunks; total per expert
    int cnt = 0;
    if ((int)threadIdx.x < E) {
        for (int w = 0; w < 16; ++w) { const int v = lds[w * E + threadIdx.x]; lds[w * E + threadIdx.x] = cnt; cnt += v; }
    }
    const int first = block_exclusive_scan(cnt, wave_sums, &total);      // E <= 1024 = blockDim
    if ((int)threadIdx.x < E) {
        offs[threadIdx.x] = first;
        expert_offsets[threadIdx.x] = first;
        for (int w = 0; w < 16; ++w) lds[w * E + threadIdx.x] += first;
    }
    __syncthreads();
    if (threadIdx.x == 0) { offs[E] = total; expert_offsets[E] = total; }
    // row tiles
    if (tile_rows > 0) {
        const int nt = (int)threadIdx.x < E ? (cnt + tile_rows - 1) / tile_rows : 0;
        int tile_total;
        int *tt = &wave_sums[16];
        const int t0 = block_exclusive_scan(nt, wave_sums, tt);
        for (int i = 0; i < nt && t0 + i < max_tiles; ++i) {
            tile_map[2 * (t0 + i)] = threadIdx.x;
            tile_map[2 * (t0 + i) + 1] = first + i * tile_rows;
        }
        __syncthreads();
        tile_total = *tt;
        if (threadIdx.x == 0) tile_map[2 * max_tiles] = tile_total < max_tiles ? tile_total : max_tiles;
    }
    __syncthreads();
    // stable scatter, one wave per chunk
    volatile int *next_row = mine;
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int ab = a0; ab < a1; ab += 64) {
        const int a = ab + lane;
        const bool live = a < a1;
        const int e = live ? min(max(idx[a], 0), E - 1) : 0;
        unsigned long long peers = __ballot(live);
        for (int b = 0; b < ebits; ++b) {
            const unsigned long long has = __ballot((e >> b) & 1);
            peers &= ((e >> b) & 1) ? has : ~has;
        }
        if (live) {
            const int row = next_row[e] + __popcll(peers & below);
            row_to_assign[row] = a;
            assign_to_row[a] = row;
        }
        __builtin_amdgcn_wave_barrier();
        if (live && (peers & below) == 0ull) next_row[e] = next_row[e] + __popcll(peers);
        __builtin_amdgcn_wave_barrier();
    }
}

// x_perm[r,:] = x[row_to_assign[r] / K,:]; 16-byte pieces, one block per 4 rows.
__global__ __launch_bounds__(256) void gather_rows_kernel(const u32x4 *__restrict__ x, const int32_t *__restrict__ row_to_assign,
                                                          u32x4 *__restrict__ x_perm, int n, int K, int vec_per_row) {
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= n) return;
    const int t = row_to_assign[r] / K;
    for (int v = threadIdx.x & 63; v < vec_per_row; v += 64)
        x_perm[(size_t)r * vec_per_row + v] = x[(size_t)t * vec_per_row + v];
}

hipError_t launch_permute(const moe_shape_t &s, const int32_t *topk_idx, int32_t *expert_offsets,
                          int32_t *row_to_assign, int32_t *assign_to_row, int32_t *chunk_base,
                          hipStream_t st, int tile_rows, int max_tiles, int32_t *tile_map) {
    const int n = s.T * s.K;
    int ebits = 0;
    while ((1 << ebits) < s.E) ++ebits;
    if (permute_is_small(s)) {
        const int chunk = ((n + 16 * 64 - 1) / (16 * 64)) * 64;
        hipLaunchKernelGGL(permute_small_kernel, dim3(1), dim3(1024), (size_t)16 * s.E * sizeof(int), st, topk_idx, n,
                           chunk, s.E, ebits, expert_offsets, row_to_assign, assign_to_row, tile_rows, max_tiles, tile_map);
        return hipGetLastError();
    }
    const int nchunks = (n + kPermChunk - 1) / kPermChunk;
    const size_t smem = (size_t)4 * s.E * sizeof(int);
    dim3 grid((nchunks + 3) / 4);
    hipLaunchKernelGGL(permute_hist_kernel, grid, dim3(256), smem, st, topk_idx, n, s.E, chunk_base);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(permute_scan_kernel, dim3(1), dim3(1024), 0, st, chunk_base, nchunks, s.E, expert_offsets);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(permute_scatter_kernel, grid, dim3(256), smem, st, topk_idx, n, s.E, ebits, chunk_base,
                       row_to_assign, assign_to_row);
    return hipGetLastError();
}

hipError_t launch_gather_rows(const moe_shape_t &s, const void *x, const int32_t *row_to_assign,
                              void *x_perm, hipStream_t st) {
    const int n = s.T * s.K;
    const int elt = s.dtype == MOE_BF16 ? 2 : 4;
    const int vec_per_row = s.H * elt / 16;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((n + 3) / 4), dim3(256), 0, st, (const u32x4 *)x, row_to_assign,
                       (u32x4 *)x_perm, n, s.K, vec_per_row);
    return hipGetLastError();
}

}  // namespace moe
