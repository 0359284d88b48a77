// Internal declarations shared by the HIP translation units of the MoE FFN
// library (gfx950 only).  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "moe_ffn.h"

namespace moe {

typedef unsigned short bf16_t;  // raw bfloat16 bits in memory

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;   // one MFMA bf16 operand
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) double f64x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

constexpr int kWave = 64;
constexpr int kMaxExperts = 1024;      // limit of the top-k and permutation kernels
constexpr int kPermChunk = 512;        // assignments handled by one wave of the permutation kernels

__device__ __forceinline__ float bf16_bits_to_float(unsigned int b) { return __uint_as_float(b << 16); }

// float -> bf16 bits, round to nearest even (inputs are finite).
// float -> bf16, round to nearest even: gfx950 converts a pair in one instruction (v_cvt_pk_bf16_f32)
typedef __attribute__((ext_vector_type(2))) float f32x2_cvt;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_cvt;
__device__ __forceinline__ unsigned int pack_bf16x2(float lo, float hi) {
    const f32x2_cvt v = {lo, hi};
    return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, bf16x2_cvt));
}
__device__ __forceinline__ unsigned int float_to_bf16_bits(float f) { return pack_bf16x2(f, 0.f) & 0xFFFFu; }

// Data that a launch reads once, with load instructions that cover whole 128-byte lines: non-temporal loads.  Plain
// streaming reads of 8 GB reach 7.0 TB/s with them against 6.2 TB/s without.  Not for loads whose instruction covers
// part of a line and leaves the rest to a later instruction (the line may be fetched again: measured slower).
__device__ __forceinline__ u32x4 load_once(const bf16_t *p) { return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p)); }

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// Workspace carving.  Every region starts 256-byte aligned.
struct Workspace {
    double  *logit_part;     // [ksplit, T, E] partial logit sums
    int32_t *topk_idx;       // [T*K]
    float   *topk_w;         // [T*K]
    int32_t *expert_offsets; // [E+1]
    int32_t *row_to_assign;  // [T*K]
    int32_t *assign_to_row;  // [T*K]
    int32_t *chunk_base;     // [nchunks, E] per-chunk histogram, then per-chunk first row
    int32_t *tile_map;       // row-tile list of the grouped GEMM (layout is the GEMM variant's own)
    bf16_t  *act;            // [T*K, I] bf16 activations silu(g)*u
    void    *y_perm;         // [T*K, H] dtype
    size_t   total;
};

constexpr int kMaxLogitSplit = 16;
constexpr int kMinTokenTile = 16;      // smallest row tile any GEMM variant uses (bounds the tile map)

Workspace carve_workspace(const moe_shape_t &s, void *base);

// row-tile lists of the large-batch grouped GEMM (8 lists, one per XCD, of big_tiles_per_xcd entries of 32 bytes)
int big_tiles_per_xcd(const moe_shape_t &s);
size_t big_tile_list_bytes(const moe_shape_t &s);

int router_ksplit(const moe_shape_t &s);
size_t router_scratch_bytes(const moe_shape_t &s);

// Optional stage timer: when given, launchers record an event at every stage boundary.
struct Probe {
    hipEvent_t ev[MOE_NUM_STAGES + 1];
    int n = 0;
    hipStream_t st = nullptr;
    void mark() { if (n <= MOE_NUM_STAGES) (void)hipEventRecord(ev[n++], st); }
};
inline void probe_mark(Probe *p) { if (p) p->mark(); }

// Launchers (all enqueue on `st`, return the first HIP launch error).
hipError_t launch_route(const moe_shape_t &s, const void *x, const void *w_router, const float *bias,
                        double *logit_part, int32_t *topk_idx, float *topk_w, hipStream_t st,
                        Probe *probe = nullptr);
// p[t][e] = softmax over all E logits, from the partial sums launch_route left in logit_part (renormalize == 0 only)
hipError_t launch_router_probs(const moe_shape_t &s, const double *logit_part, const float *bias, float *probs, hipStream_t st);
// One-block permutation is used for batches of at most 16 chunks; it can also emit the GEMM's row-tile
// list (tile_rows > 0), which saves a launch.  Returns whether `s` takes that path.
inline bool permute_is_small(const moe_shape_t &s) { return (long)s.T * s.K <= 16L * kPermChunk; }
hipError_t launch_permute(const moe_shape_t &s, const int32_t *topk_idx, int32_t *expert_offsets,
                          int32_t *row_to_assign, int32_t *assign_to_row, int32_t *chunk_base,
                          hipStream_t st, int tile_rows = 0, int max_tiles = 0, int32_t *tile_map = nullptr);
// Row-tile geometry of the grouped GEMM that launch_grouped_swiglu will pick for `s`.
int gemm_tile_rows(const moe_shape_t &s);
int gemm_max_tiles(const moe_shape_t &s);
hipError_t launch_gather_rows(const moe_shape_t &s, const void *x, const int32_t *row_to_assign,
                              void *x_perm, hipStream_t st);
// x_rows: either x_perm (row_map == nullptr) or x with row_map = row_to_assign (row r reads x[row_map[r]/K]).
hipError_t launch_grouped_swiglu(const moe_shape_t &s, const void *x_rows, const int32_t *row_map,
                                 const int32_t *expert_offsets, const void *w_gate, const void *w_up,
                                 const void *w_down, bf16_t *act, int32_t *tile_map, void *y_perm,
                                 hipStream_t st, Probe *probe = nullptr, bool tile_map_ready = false);
hipError_t launch_combine(const moe_shape_t &s, const void *y_perm, const int32_t *assign_to_row,
                          const float *topk_w, void *out, hipStream_t st);

}  // namespace moe
