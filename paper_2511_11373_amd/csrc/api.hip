// C ABI of the MoE FFN library: argument validation (host only, before any HIP
// call), workspace carving, and the launch sequences.
#include "moe_internal.hpp"
#include <algorithm>
#include <mutex>

namespace moe {

// Scratch of moe_forward_noalloc: device memory that belongs to the loaded library itself, one copy per GPU, so that
// the call needs neither a workspace from the caller nor an allocation.  In host code the array's name is only a
// stand-in for the symbol; the device address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[MOE_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static void *scratch_ptr[kMaxDevices];      // device address of `scratch` on each GPU, nullptr until asked for

// Address of the current device's copy of `scratch` (looked up on the first call on that device).
static hipError_t static_scratch(void **out) {
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return err;
        if (!p) return hipErrorInvalidSymbol;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return hipSuccess;
}

static moe_status_t check_shape(const moe_shape_t *s) {
    if (!s) return MOE_ERR_NULL;
    if (s->dtype != MOE_BF16 && s->dtype != MOE_F32) return MOE_ERR_DTYPE;
    if (s->T < 0 || s->H < 1 || s->E < 1 || s->K < 1 || s->I < 1) return MOE_ERR_SHAPE;
    if (s->K > s->E || s->E > kMaxExperts) return MOE_ERR_SHAPE;
    if (s->H % 8 != 0 || s->I % 8 != 0) return MOE_ERR_SHAPE;
    const long long lim = 0x7FFFFFFFll;
    if ((long long)s->T * s->K > lim || (long long)s->T * s->E > lim) return MOE_ERR_SHAPE;
    return MOE_OK;
}
static bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

static size_t elt_size(const moe_shape_t &s) { return s.dtype == MOE_BF16 ? 2 : 4; }

// Addresses are carved as integers: the same code sizes a workspace from a null base, and pointer arithmetic on a null
// pointer is undefined.
template <typename P>
static void take(uintptr_t &cur, P *&field, size_t bytes) {
    field = reinterpret_cast<P *>(cur);
    cur += align256(bytes);
}

Workspace carve_workspace(const moe_shape_t &s, void *base) {
    Workspace w;
    uintptr_t cur = reinterpret_cast<uintptr_t>(base);
    const size_t n = (size_t)s.T * s.K;
    const size_t nchunks = (n + kPermChunk - 1) / kPermChunk;
    const size_t max_tiles = n / kMinTokenTile + (size_t)s.E;
    take(cur, w.logit_part, router_scratch_bytes(s));
    take(cur, w.topk_idx, sizeof(int32_t) * n);
    take(cur, w.topk_w, sizeof(float) * n);
    take(cur, w.expert_offsets, sizeof(int32_t) * ((size_t)s.E + 1));
    take(cur, w.row_to_assign, sizeof(int32_t) * n);
    take(cur, w.assign_to_row, sizeof(int32_t) * n);
    take(cur, w.chunk_base, sizeof(int32_t) * nchunks * s.E);
    // (expert, first row) pairs plus a count for the tiled kernel, or the large-batch kernel's 8 per-XCD lists
    take(cur, w.tile_map, std::max(sizeof(int32_t) * (2 * max_tiles + 4), big_tile_list_bytes(s)));
    take(cur, w.act, sizeof(bf16_t) * n * s.I);
    void *y = nullptr;
    take(cur, y, elt_size(s) * n * s.H);
    w.y_perm = y;
    w.total = (size_t)(cur - reinterpret_cast<uintptr_t>(base));
    return w;
}

static moe_status_t check_ws(const moe_shape_t &s, const void *ws, size_t ws_bytes) {
    if (!ws) return MOE_ERR_WORKSPACE;
    if (misaligned(ws)) return MOE_ERR_ALIGN;
    if (ws_bytes < carve_workspace(s, nullptr).total) return MOE_ERR_WORKSPACE;
    return MOE_OK;
}

// act = silu(g) u over whole expert-sorted rows, 8 elements per thread (the forward pass that keeps g and u)
__global__ __launch_bounds__(256) void swiglu_rows_kernel(const bf16_t *__restrict__ g, const bf16_t *__restrict__ u,
                                                          bf16_t *__restrict__ act, size_t n8) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    const u32x4 gv = *reinterpret_cast<const u32x4 *>(g + i * 8), uv = *reinterpret_cast<const u32x4 *>(u + i * 8);
    u32x4 av;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float g0 = __uint_as_float(gv[j] << 16), g1 = __uint_as_float(gv[j] & 0xFFFF0000u);
        const float u0 = __uint_as_float(uv[j] << 16), u1 = __uint_as_float(uv[j] & 0xFFFF0000u);
        av[j] = pack_bf16x2(g0 / (1.0f + __expf(-g0)) * u0, g1 / (1.0f + __expf(-g1)) * u1);
    }
    *reinterpret_cast<u32x4 *>(act + i * 8) = av;
}

bool big_pre_activations_applicable(int H, int I);
bool big_down_applicable(int H, int I);
hipError_t launch_big_tile_list(const moe_shape_t &s, const int32_t *off, void *list, hipStream_t st);
hipError_t launch_big_pre_activations(const moe_shape_t &s, const bf16_t *rows, const int32_t *row_token, int row_div,
                                      const void *list, const bf16_t *wg, const bf16_t *wu, bf16_t *g, bf16_t *u, hipStream_t st);
hipError_t launch_big_down(const moe_shape_t &s, const bf16_t *act, const void *list, const bf16_t *wd, bf16_t *y_perm,
                           hipStream_t st);

}  // namespace moe

using namespace moe;

extern "C" {

const char *moe_status_string(moe_status_t status) {
    // a C caller may pass any int: read the bits, not the enumeration (whose other values C++ leaves undefined)
    int code;
    __builtin_memcpy(&code, &status, sizeof code);
    switch (code) {
        case MOE_OK: return "ok";
        case MOE_ERR_NULL: return "a required pointer is NULL";
        case MOE_ERR_SHAPE: return "unsupported shape";
        case MOE_ERR_DTYPE: return "unknown dtype";
        case MOE_ERR_WORKSPACE: return "workspace missing or too small";
        case MOE_ERR_ALIGN: return "pointer not 16-byte aligned";
        case MOE_ERR_HIP: return "HIP launch error";
        case MOE_ERR_STATIC_LIMIT: return "shape needs more scratch than the library's static buffer holds";
    }
    return "unknown status";
}

moe_status_t moe_workspace_bytes(const moe_shape_t *shape, size_t *out_bytes) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (!out_bytes) return MOE_ERR_NULL;
    *out_bytes = carve_workspace(*shape, nullptr).total;
    return MOE_OK;
}

moe_status_t moe_route_topk(const moe_shape_t *shape, const void *x, const void *w_router,
                            const float *router_bias, int32_t *topk_idx, float *topk_w,
                            void *ws, size_t ws_bytes, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (!x || !w_router || !topk_idx || !topk_w) return MOE_ERR_NULL;
    if (misaligned(x) || misaligned(w_router) || misaligned(router_bias) || misaligned(topk_idx) || misaligned(topk_w))
        return MOE_ERR_ALIGN;
    st = check_ws(*shape, ws, ws_bytes);
    if (st != MOE_OK) return st;
    if (shape->T == 0) return MOE_OK;
    Workspace w = carve_workspace(*shape, ws);
    return launch_route(*shape, x, w_router, router_bias, w.logit_part, topk_idx, topk_w, (hipStream_t)stream) == hipSuccess
               ? MOE_OK : MOE_ERR_HIP;
}

moe_status_t moe_permute(const moe_shape_t *shape, const int32_t *topk_idx, const void *x,
                         int32_t *expert_offsets, int32_t *row_to_assign, int32_t *assign_to_row,
                         void *x_perm, void *ws, size_t ws_bytes, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (!topk_idx || !expert_offsets || !row_to_assign || !assign_to_row) return MOE_ERR_NULL;
    if (x_perm && !x) return MOE_ERR_NULL;
    if (misaligned(topk_idx) || misaligned(x) || misaligned(expert_offsets) || misaligned(row_to_assign) ||
        misaligned(assign_to_row) || misaligned(x_perm))
        return MOE_ERR_ALIGN;
    st = check_ws(*shape, ws, ws_bytes);
    if (st != MOE_OK) return st;
    if (shape->T == 0) return MOE_OK;   // nothing enqueued; expert_offsets is left untouched
    Workspace w = carve_workspace(*shape, ws);
    hipStream_t hs = (hipStream_t)stream;
    if (launch_permute(*shape, topk_idx, expert_offsets, row_to_assign, assign_to_row, w.chunk_base, hs) != hipSuccess)
        return MOE_ERR_HIP;
    if (x_perm && launch_gather_rows(*shape, x, row_to_assign, x_perm, hs) != hipSuccess) return MOE_ERR_HIP;
    return MOE_OK;
}

moe_status_t moe_grouped_swiglu(const moe_shape_t *shape, const void *x_perm, const int32_t *expert_offsets,
                                const void *w_gate, const void *w_up, const void *w_down, void *y_perm,
                                void *ws, size_t ws_bytes, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (!x_perm || !expert_offsets || !w_gate || !w_up || !w_down || !y_perm) return MOE_ERR_NULL;
    if (misaligned(x_perm) || misaligned(expert_offsets) || misaligned(w_gate) || misaligned(w_up) ||
        misaligned(w_down) || misaligned(y_perm))
        return MOE_ERR_ALIGN;
    st = check_ws(*shape, ws, ws_bytes);
    if (st != MOE_OK) return st;
    if (shape->T == 0) return MOE_OK;
    Workspace w = carve_workspace(*shape, ws);
    return launch_grouped_swiglu(*shape, x_perm, nullptr, expert_offsets, w_gate, w_up, w_down, w.act, w.tile_map,
                                 y_perm, (hipStream_t)stream) == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status_t moe_combine(const moe_shape_t *shape, const void *y_perm, const int32_t *assign_to_row,
                         const float *topk_w, void *out, void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (!y_perm || !assign_to_row || !topk_w || !out) return MOE_ERR_NULL;
    if (misaligned(y_perm) || misaligned(assign_to_row) || misaligned(topk_w) || misaligned(out)) return MOE_ERR_ALIGN;
    if (shape->T == 0) return MOE_OK;
    return launch_combine(*shape, y_perm, assign_to_row, topk_w, out, (hipStream_t)stream) == hipSuccess
               ? MOE_OK : MOE_ERR_HIP;
}

// Host-side checks of moe_forward's arguments other than the workspace (no HIP call).
static moe_status_t check_forward_args(const moe_shape_t *shape, const void *x, const void *w_router,
                                       const float *router_bias, const void *w_gate, const void *w_up,
                                       const void *w_down, const void *out, const int32_t *topk_idx_out,
                                       const float *topk_w_out) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (!x || !w_router || !w_gate || !w_up || !w_down || !out) return MOE_ERR_NULL;
    if (misaligned(x) || misaligned(w_router) || misaligned(router_bias) || misaligned(w_gate) || misaligned(w_up) ||
        misaligned(w_down) || misaligned(out) || misaligned(topk_idx_out) || misaligned(topk_w_out))
        return MOE_ERR_ALIGN;
    return MOE_OK;
}

static moe_status_t forward_impl(const moe_shape_t *shape, const void *x, const void *w_router,
                                 const float *router_bias, const void *w_gate, const void *w_up,
                                 const void *w_down, void *out, int32_t *topk_idx_out, float *topk_w_out,
                                 void *ws, size_t ws_bytes, void *stream, Probe *probe) {
    moe_status_t st = check_forward_args(shape, x, w_router, router_bias, w_gate, w_up, w_down, out, topk_idx_out, topk_w_out);
    if (st != MOE_OK) return st;
    st = check_ws(*shape, ws, ws_bytes);
    if (st != MOE_OK) return st;
    if (shape->T == 0) return MOE_OK;
    const moe_shape_t &s = *shape;
    Workspace w = carve_workspace(s, ws);
    hipStream_t hs = (hipStream_t)stream;
    int32_t *idx = topk_idx_out ? topk_idx_out : w.topk_idx;
    float *tw = topk_w_out ? topk_w_out : w.topk_w;
    if (probe) { probe->st = hs; probe->mark(); }
    if (launch_route(s, x, w_router, router_bias, w.logit_part, idx, tw, hs, probe) != hipSuccess) return MOE_ERR_HIP;
    probe_mark(probe);
    const bool fused_tiles = permute_is_small(s);
    if (launch_permute(s, idx, w.expert_offsets, w.row_to_assign, w.assign_to_row, w.chunk_base, hs,
                       fused_tiles ? gemm_tile_rows(s) : 0, gemm_max_tiles(s), w.tile_map) != hipSuccess)
        return MOE_ERR_HIP;
    probe_mark(probe);
    if (launch_grouped_swiglu(s, x, w.row_to_assign, w.expert_offsets, w_gate, w_up, w_down, w.act, w.tile_map,
                              w.y_perm, hs, probe, fused_tiles) != hipSuccess)
        return MOE_ERR_HIP;
    probe_mark(probe);
    if (launch_combine(s, w.y_perm, w.assign_to_row, tw, out, hs) != hipSuccess) return MOE_ERR_HIP;
    probe_mark(probe);
    probe_mark(probe);       // closes the empty calibration interval
    return MOE_OK;
}

moe_status_t moe_forward(const moe_shape_t *shape, const void *x, const void *w_router,
                         const float *router_bias, const void *w_gate, const void *w_up,
                         const void *w_down, void *out, int32_t *topk_idx_out, float *topk_w_out,
                         void *ws, size_t ws_bytes, void *stream) {
    return forward_impl(shape, x, w_router, router_bias, w_gate, w_up, w_down, out, topk_idx_out, topk_w_out, ws,
                        ws_bytes, stream, nullptr);
}

moe_status_t moe_forward_noalloc(const moe_shape_t *shape, const void *x, const void *w_router,
                                 const float *router_bias, const void *w_gate, const void *w_up,
                                 const void *w_down, void *out, int32_t *topk_idx_out, float *topk_w_out,
                                 void *stream) {
    // everything that can be rejected on the host is rejected before the first HIP call
    moe_status_t st = check_forward_args(shape, x, w_router, router_bias, w_gate, w_up, w_down, out, topk_idx_out, topk_w_out);
    if (st != MOE_OK) return st;
    if (carve_workspace(*shape, nullptr).total > (size_t)MOE_NOALLOC_SCRATCH_BYTES) return MOE_ERR_STATIC_LIMIT;
    if (shape->T == 0) return MOE_OK;
    void *ws = nullptr;
    if (static_scratch(&ws) != hipSuccess) return MOE_ERR_HIP;
    // No region of the workspace has to start at zero: every kernel of the forward pass writes what it later reads.
    return forward_impl(shape, x, w_router, router_bias, w_gate, w_up, w_down, out, topk_idx_out, topk_w_out, ws,
                        (size_t)MOE_NOALLOC_SCRATCH_BYTES, stream, nullptr);
}

moe_status_t moe_forward_saving(const moe_shape_t *shape, const void *x, const void *w_router, const float *router_bias,
                                const void *w_gate, const void *w_up, const void *w_down, void *out, void *g_rows,
                                void *u_rows, int32_t *topk_idx_out, float *topk_w_out, void *ws, size_t ws_bytes,
                                void *stream) {
    moe_status_t st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (shape->dtype != MOE_BF16) return MOE_ERR_DTYPE;
    if (!big_pre_activations_applicable(shape->H, shape->I) || !big_down_applicable(shape->H, shape->I)) return MOE_ERR_SHAPE;
    if (!x || !w_router || !w_gate || !w_up || !w_down || !out || !g_rows || !u_rows) return MOE_ERR_NULL;
    if (misaligned(x) || misaligned(w_router) || misaligned(router_bias) || misaligned(w_gate) || misaligned(w_up) ||
        misaligned(w_down) || misaligned(out) || misaligned(g_rows) || misaligned(u_rows) || misaligned(topk_idx_out) ||
        misaligned(topk_w_out))
        return MOE_ERR_ALIGN;
    st = check_ws(*shape, ws, ws_bytes);
    if (st != MOE_OK) return st;
    if (shape->T == 0) return MOE_OK;
    const moe_shape_t &s = *shape;
    Workspace w = carve_workspace(s, ws);
    hipStream_t hs = (hipStream_t)stream;
    int32_t *idx = topk_idx_out ? topk_idx_out : w.topk_idx;
    float *tw = topk_w_out ? topk_w_out : w.topk_w;
    if (launch_route(s, x, w_router, router_bias, w.logit_part, idx, tw, hs, nullptr) != hipSuccess) return MOE_ERR_HIP;
    if (launch_permute(s, idx, w.expert_offsets, w.row_to_assign, w.assign_to_row, w.chunk_base, hs, 0, 0, w.tile_map) != hipSuccess)
        return MOE_ERR_HIP;
    if (launch_big_tile_list(s, w.expert_offsets, w.tile_map, hs) != hipSuccess) return MOE_ERR_HIP;
    if (launch_big_pre_activations(s, (const bf16_t *)x, w.row_to_assign, s.K, w.tile_map, (const bf16_t *)w_gate,
                                   (const bf16_t *)w_up, (bf16_t *)g_rows, (bf16_t *)u_rows, hs) != hipSuccess)
        return MOE_ERR_HIP;
    const size_t n8 = (size_t)s.T * s.K * s.I / 8;
    hipLaunchKernelGGL(swiglu_rows_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, hs, (const bf16_t *)g_rows,
                       (const bf16_t *)u_rows, w.act, n8);
    if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
    if (launch_big_down(s, w.act, w.tile_map, (const bf16_t *)w_down, (bf16_t *)w.y_perm, hs) != hipSuccess) return MOE_ERR_HIP;
    if (launch_combine(s, w.y_perm, w.assign_to_row, tw, out, hs) != hipSuccess) return MOE_ERR_HIP;
    return MOE_OK;
}

moe_status_t moe_forward_stage_times(const moe_shape_t *shape, const void *x, const void *w_router,
                                     const float *router_bias, const void *w_gate, const void *w_up,
                                     const void *w_down, void *out, void *ws, size_t ws_bytes, void *stream,
                                     float *stage_ms) {
    if (!stage_ms) return MOE_ERR_NULL;
    for (int i = 0; i < MOE_NUM_STAGES; ++i) stage_ms[i] = 0.f;
    // the arguments are checked before the first HIP call, here as everywhere; the events are the one thing any
    // entry point of the library creates, and they are destroyed before it returns
    moe_status_t st = check_forward_args(shape, x, w_router, router_bias, w_gate, w_up, w_down, out, nullptr, nullptr);
    if (st != MOE_OK) return st;
    st = check_ws(*shape, ws, ws_bytes);
    if (st != MOE_OK) return st;
    if (shape->T == 0) return MOE_OK;
    Probe probe;
    for (int i = 0; i <= MOE_NUM_STAGES; ++i)
        if (hipEventCreate(&probe.ev[i]) != hipSuccess) {
            while (--i >= 0) (void)hipEventDestroy(probe.ev[i]);
            return MOE_ERR_HIP;
        }
    st = forward_impl(shape, x, w_router, router_bias, w_gate, w_up, w_down, out, nullptr, nullptr, ws,
                                   ws_bytes, stream, &probe);
    if (st == MOE_OK && probe.n == MOE_NUM_STAGES + 1) {
        if (hipEventSynchronize(probe.ev[MOE_NUM_STAGES]) != hipSuccess) st = MOE_ERR_HIP;
        for (int i = 0; i < MOE_NUM_STAGES && st == MOE_OK; ++i)
            if (hipEventElapsedTime(&stage_ms[i], probe.ev[i], probe.ev[i + 1]) != hipSuccess) st = MOE_ERR_HIP;
    }
    for (int i = 0; i <= MOE_NUM_STAGES; ++i) (void)hipEventDestroy(probe.ev[i]);
    return st;
}

}  // extern "C"
