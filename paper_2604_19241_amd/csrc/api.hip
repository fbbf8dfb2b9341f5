// extern "C" boundary: argument checks, workspace carving, launches.
// Every check happens before anything is enqueued.
#include "common.hpp"

#include <algorithm>

namespace uniep {
size_t route_workspace_bytes(const moe_shape_t& s);
int route_backward_launch(const moe_shape_t& s, const int32_t* topk_idx, const float* topk_w,
                          const float* dtopk_w, float* dlogits, hipStream_t st);
int route_launch(const moe_shape_t& s, const float* logits, const moe_routing_t& out, void* ws,
                 hipStream_t st);
int route_static_launch(const moe_shape_t& s, const float* logits, const moe_routing_t& out,
                        hipStream_t st);
int global_map_launch(const moe_shape_t& s, int W, int rank, const moe_routing_t& r,
                      const int32_t* c_all, const moe_global_map_t& out, void* ws, hipStream_t st);
size_t fwd_workspace_bytes(const moe_shape_t& s);
size_t fwd_ctrl_bytes(const moe_shape_t& s);
int fwd_launch(const moe_shape_t& s, const void* x, const void* w_gate, const void* w_up,
               const void* w_down, const moe_routing_t& r, void* y, char* gu, char* h, char* o,
               char* ws, const moe_opts_t& opts, int nw, hipStream_t st);
size_t bwd_workspace_bytes(const moe_shape_t& s, int split_rows);
bool bwd_split_ok(const moe_shape_t& s, int split_rows);
int bwd_launch(const moe_shape_t& s, const void* dy, const void* x, const void* w_gate,
               const void* w_up, const void* w_down, const moe_routing_t& r, const char* gu,
               const char* h, const char* o, void* dx, void* dw_gate, void* dw_up, void* dw_down,
               float* dtopk_w, char* ws, const moe_opts_t& opts, int nw, hipStream_t st);
}  // namespace uniep

using namespace uniep;

namespace {

int check_shape(const moe_shape_t* s) {
    if (!s) return MOE_ERR_ARG;
    if (s->T < 0 || s->d < 64 || s->I < 64 || s->E < 1 || s->k < 1) return MOE_ERR_SHAPE;
    if (s->k > kMaxTopK || s->E > kMaxExperts || s->k > s->E) return MOE_ERR_SHAPE;
    if (s->e_start < 0 || s->e_count < 1 || s->e_start + s->e_count > s->E) return MOE_ERR_SHAPE;
    if (s->d % 64 != 0 || s->I % 64 != 0) return MOE_ERR_SHAPE;
    if ((int64_t)s->T * s->k >= (1ll << 30)) return MOE_ERR_SHAPE;
    return MOE_OK;
}

bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

int check_routing(const moe_routing_t* r, int T) {
    if (!r) return MOE_ERR_ARG;
    if (!r->counts || !r->offsets) return MOE_ERR_ARG;
    if (T > 0 && (!r->topk_idx || !r->topk_w || !r->perm || !r->inv_perm)) return MOE_ERR_ARG;
    if (!aligned(r->topk_idx, 4) || !aligned(r->topk_w, 4) || !aligned(r->counts, 4) ||
        !aligned(r->offsets, 4) || !aligned(r->perm, 4) || !aligned(r->inv_perm, 4))
        return MOE_ERR_ARG;
    return MOE_OK;
}

int check_opts(const moe_opts_t* o, moe_opts_t* out) {
    moe_opts_t d = {};
    if (o) d = *o;
    if (d.schedule < 0 || d.schedule > 3 || d.workers < 0 || d.spin_limit_ms < 0) return MOE_ERR_ARG;
    if (d.tile_rows != 0 && d.tile_rows != 128 && d.tile_rows != 256) return MOE_ERR_ARG;
    if (d.skip_tail != 0 && d.skip_tail != 1) return MOE_ERR_ARG;
    if (d.dw_accumulate != 0 && d.dw_accumulate != 1) return MOE_ERR_ARG;
    if (d.dw_split_rows < 0 || d.dw_split_rows % 64 != 0 || (d.dw_split_rows != 0 && d.dw_split_rows < 256))
        return MOE_ERR_ARG;
    if (d.reserved[0] != 0) return MOE_ERR_ARG;
    *out = d;
    return MOE_OK;
}

// Waves per workgroup = row-tile height / 32.  256-row tiles (8 waves, two per
// SIMD) by default at every size: waves whose rows lie outside a tile skip the
// matrix work, and measured from 20 to 6000 rows per expert the 8-wave tiles
// are 1.3-2x faster than the 4-wave ones.
int pick_nw(const moe_shape_t&, const moe_opts_t& o) { return o.tile_rows == 128 ? 4 : 8; }

struct SavedLayout {
    size_t gu, h, o, total;
};
SavedLayout saved_layout(const moe_shape_t& s) {
    const size_t A_cap = (size_t)s.T * s.k;
    SavedLayout L;
    size_t off = 0;
    L.gu = off; off = align_up(off + A_cap * 2 * s.I * 2, 256);
    L.h = off;  off = align_up(off + A_cap * s.I * 2, 256);
    L.o = off;  off = align_up(off + A_cap * s.d * 2, 256);
    L.total = off > 0 ? off : 256;
    return L;
}

}  // namespace

// Plain streaming copy with known HBM traffic (profiler counter calibration).
__global__ void __launch_bounds__(256) calibration_copy_kernel(uniep::u32x4_t* __restrict__ dst,
                                                               const uniep::u32x4_t* __restrict__ src,
                                                               size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Dependent-free bf16 MFMA stream with non-trivial operands: what the matrix pipes sustain
// when nothing else runs (profiler and bench calibration of the matrix-core ceiling and of
// the shader clock under that load).  clk[0] = shader clocks, clk[1] = 100 MHz ticks that the
// first wave of workgroup 0 spent in the loop.
__global__ void __launch_bounds__(512) calibration_mfma_kernel(int iters, const uint32_t* __restrict__ seed,
                                                               float* __restrict__ sink, long long* clk) {
    using namespace uniep;
    u32x4_t ar, br;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        ar[i] = seed[(threadIdx.x * 4 + i) & 1023];
        br[i] = seed[(threadIdx.x * 4 + i + 512) & 1023];
    }
    const bf16x8_t a = __builtin_bit_cast(bf16x8_t, ar), b = __builtin_bit_cast(bf16x8_t, br);
    f32x16_t acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[j][v];
    if (s == 0.12345f) sink[0] = s;   // keeps the accumulators alive
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        clk[0] = c1 - c0;
        clk[1] = w1 - w0;
    }
}

__global__ void clear_status_kernel(int* ws) { ws[uniep::CTRL_STATUS] = 0; }

extern "C" {

int moe_calibration_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15) || (bytes & 15)) return MOE_ERR_ARG;
    if (bytes == 0) return MOE_OK;
    const size_t n16 = bytes / 16;
    const int grid = (int)std::min<size_t>((n16 + 255) / 256, 256 * 16);
    hipLaunchKernelGGL(calibration_copy_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream,
                       (uniep::u32x4_t*)dst, (const uniep::u32x4_t*)src, n16);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int moe_calibration_mfma(int32_t workgroups, int32_t waves, int32_t iters, const uint32_t* seed,
                         float* sink, long long* clocks, void* stream) {
    if (!seed || !sink || !clocks || ((uintptr_t)seed & 3) || ((uintptr_t)clocks & 7)) return MOE_ERR_ARG;
    if (workgroups < 1 || workgroups > 65536 || waves < 1 || waves > 8 || iters < 1) return MOE_ERR_ARG;
    hipLaunchKernelGGL(calibration_mfma_kernel, dim3(workgroups), dim3(64 * waves), 0, (hipStream_t)stream,
                       iters, seed, sink, clocks);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int moe_workspace_bytes(const moe_shape_t* shape, size_t* route_ws, size_t* fwd_ws, size_t* bwd_ws,
                        size_t* saved_bytes) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    if (route_ws) *route_ws = route_workspace_bytes(*shape);
    if (fwd_ws) *fwd_ws = fwd_workspace_bytes(*shape);
    if (bwd_ws) *bwd_ws = bwd_workspace_bytes(*shape, 0);
    if (saved_bytes) *saved_bytes = saved_layout(*shape).total;
    return MOE_OK;
}

int moe_backward_workspace_bytes(const moe_shape_t* shape, const moe_opts_t* opts, size_t* bwd_ws) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    moe_opts_t o;
    rc = check_opts(opts, &o);
    if (rc != MOE_OK) return rc;
    if (!bwd_ws || !bwd_split_ok(*shape, o.dw_split_rows)) return MOE_ERR_ARG;
    *bwd_ws = bwd_workspace_bytes(*shape, o.dw_split_rows);
    return MOE_OK;
}

int moe_saved_layout(const moe_shape_t* shape, size_t* off_gu, size_t* off_h, size_t* off_o) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    const SavedLayout L = saved_layout(*shape);
    if (off_gu) *off_gu = L.gu;
    if (off_h) *off_h = L.h;
    if (off_o) *off_o = L.o;
    return MOE_OK;
}

int moe_route(const moe_shape_t* shape, const float* logits, const moe_routing_t* out, void* ws,
              size_t ws_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    rc = check_routing(out, shape->T);
    if (rc != MOE_OK) return rc;
    if (!ws || !aligned(ws, 256)) return MOE_ERR_ARG;
    if (shape->T > 0 && (!logits || !aligned(logits, 4))) return MOE_ERR_ARG;
    if (ws_bytes < route_workspace_bytes(*shape)) return MOE_ERR_WORKSPACE;
    return route_launch(*shape, logits, *out, ws, (hipStream_t)stream);
}

int moe_route_static(const moe_shape_t* shape, const float* logits, const moe_routing_t* out,
                     void* stream) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    rc = check_routing(out, shape->T);
    if (rc != MOE_OK) return rc;
    if (shape->T > 0 && (!logits || !aligned(logits, 4))) return MOE_ERR_ARG;
    if (route_workspace_bytes(*shape) > kRouteStaticScratchBytes) return MOE_ERR_WORKSPACE;
    return route_static_launch(*shape, logits, *out, (hipStream_t)stream);
}

int moe_fused_forward(const moe_shape_t* shape, const void* x, const void* w_gate, const void* w_up,
                      const void* w_down, const moe_routing_t* routing, void* y, void* saved,
                      void* ws, size_t ws_bytes, const moe_opts_t* opts, void* stream) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    rc = check_routing(routing, shape->T);
    if (rc != MOE_OK) return rc;
    moe_opts_t o;
    rc = check_opts(opts, &o);
    if (rc != MOE_OK) return rc;
    if (!w_gate || !w_up || !w_down || !ws) return MOE_ERR_ARG;
    if (shape->T > 0 && (!x || !y)) return MOE_ERR_ARG;
    if (!aligned(x, 16) || !aligned(y, 16) || !aligned(w_gate, 16) || !aligned(w_up, 16) ||
        !aligned(w_down, 16) || !aligned(ws, 256) || !aligned(saved, 256))
        return MOE_ERR_ARG;
    if (ws_bytes < fwd_workspace_bytes(*shape)) return MOE_ERR_WORKSPACE;
    if (shape->T == 0) {   // nothing to compute: leave a clean status word for moe_device_status
        hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, (int*)ws);
        return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
    }
    char* wsb = (char*)ws;
    char *gu = nullptr, *h, *ob;
    if (saved) {
        const SavedLayout L = saved_layout(*shape);
        gu = (char*)saved + L.gu;
        h = (char*)saved + L.h;
        ob = (char*)saved + L.o;
    } else {
        const size_t A_cap = (size_t)shape->T * shape->k;
        const size_t ctrl = fwd_ctrl_bytes(*shape);
        h = wsb + ctrl;
        ob = h + align_up(A_cap * shape->I * 2, 256);
    }
    return fwd_launch(*shape, x, w_gate, w_up, w_down, *routing, y, gu, h, ob, wsb, o,
                      pick_nw(*shape, o), (hipStream_t)stream);
}

int moe_fused_backward(const moe_shape_t* shape, const void* dy, const void* x, const void* w_gate,
                       const void* w_up, const void* w_down, const moe_routing_t* routing,
                       const void* saved, void* dx, void* dw_gate, void* dw_up, void* dw_down,
                       float* dtopk_w, void* ws, size_t ws_bytes, const moe_opts_t* opts,
                       void* stream) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    rc = check_routing(routing, shape->T);
    if (rc != MOE_OK) return rc;
    moe_opts_t o;
    rc = check_opts(opts, &o);
    if (rc != MOE_OK) return rc;
    if (!w_gate || !w_up || !w_down || !ws || !saved || !dw_gate || !dw_up || !dw_down)
        return MOE_ERR_ARG;
    if (shape->T > 0 && (!x || !dy || !dx)) return MOE_ERR_ARG;
    if (!aligned(x, 16) || !aligned(dy, 16) || !aligned(dx, 16) || !aligned(w_gate, 16) ||
        !aligned(w_up, 16) || !aligned(w_down, 16) || !aligned(dw_gate, 16) ||
        !aligned(dw_up, 16) || !aligned(dw_down, 16) || !aligned(ws, 256) ||
        !aligned(saved, 256) || !aligned(dtopk_w, 4))
        return MOE_ERR_ARG;
    if (!bwd_split_ok(*shape, o.dw_split_rows)) return MOE_ERR_ARG;
    if (ws_bytes < bwd_workspace_bytes(*shape, o.dw_split_rows)) return MOE_ERR_WORKSPACE;
    const SavedLayout L = saved_layout(*shape);
    const char* sv = (const char*)saved;
    return bwd_launch(*shape, dy, x, w_gate, w_up, w_down, *routing, sv + L.gu, sv + L.h, sv + L.o,
                      dx, dw_gate, dw_up, dw_down, dtopk_w, (char*)ws, o, pick_nw(*shape, o),
                      (hipStream_t)stream);
}

int moe_route_backward(const moe_shape_t* shape, const int32_t* topk_idx, const float* topk_w,
                       const float* dtopk_w, float* dlogits, void* stream) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    if (shape->T > 0 && (!topk_idx || !topk_w || !dtopk_w || !dlogits)) return MOE_ERR_ARG;
    if (!aligned(topk_idx, 4) || !aligned(topk_w, 4) || !aligned(dtopk_w, 4) || !aligned(dlogits, 4))
        return MOE_ERR_ARG;
    return route_backward_launch(*shape, topk_idx, topk_w, dtopk_w, dlogits, (hipStream_t)stream);
}

int moe_global_map(const moe_shape_t* shape, int32_t W, int32_t rank, const moe_routing_t* routing,
                   const int32_t* c_all, const moe_global_map_t* out, void* ws, size_t ws_bytes,
                   void* stream) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    if (shape->e_start != 0 || shape->e_count != shape->E) return MOE_ERR_SHAPE;
    if (W < 1 || W > 64 || shape->E % W != 0 || rank < 0 || rank >= W) return MOE_ERR_SHAPE;
    if (!routing || !out || !c_all || !ws) return MOE_ERR_ARG;
    if (!routing->offsets || !out->recv_offsets) return MOE_ERR_ARG;
    if (shape->T > 0 && (!routing->topk_idx || !routing->inv_perm || !out->dst_rank ||
                         !out->dst_expert || !out->dst_off || !out->dst_row || !out->send ||
                         !out->n_dst_ranks))
        return MOE_ERR_ARG;
    const void* ptrs[] = {routing->topk_idx, routing->inv_perm, routing->offsets, c_all,
                          out->dst_rank, out->dst_expert, out->dst_off, out->dst_row, out->send,
                          out->n_dst_ranks, out->recv_offsets, ws};
    for (const void* q : ptrs)
        if (!aligned(q, 4)) return MOE_ERR_ARG;
    if (ws_bytes < (size_t)shape->E * 8) return MOE_ERR_WORKSPACE;
    return global_map_launch(*shape, W, rank, *routing, c_all, *out, ws, (hipStream_t)stream);
}

int moe_device_status(const void* ws, void* stream) {
    if (!ws) return MOE_ERR_ARG;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return MOE_ERR_HIP;
    int status = 0;
    if (hipMemcpy(&status, ws, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) return MOE_ERR_HIP;
    return status == 0 ? MOE_OK : MOE_ERR_DEVICE;
}

const char* moe_status_string(int code) {
    switch (code) {
        case MOE_OK: return "ok";
        case MOE_ERR_ARG: return "bad argument (null or misaligned pointer, bad option)";
        case MOE_ERR_SHAPE: return "shape outside the supported limits";
        case MOE_ERR_WORKSPACE: return "workspace too small (or the problem exceeds the static scratch of moe_route_static)";
        case MOE_ERR_HIP: return "HIP runtime call failed";
        case MOE_ERR_DEVICE: return "a kernel gave up a bounded scoreboard wait";
        default: return "unknown status";
    }
}

}  // extern "C"
