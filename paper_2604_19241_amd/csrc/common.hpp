// Shared device/host definitions of the gfx950 fused-MoE library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/uniep_moe.h"

namespace uniep {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

constexpr int kMaxTopK = 16;
constexpr int kMaxExperts = 1024;
constexpr int kWave = 64;

// ---- bf16 <-> fp32 (round-to-nearest-even; gfx950 has a native packed convert)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2_t v = {lo, hi};
    bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// ---- scoreboard primitives (agent scope: visible across all 8 XCDs' L2s)
__device__ __forceinline__ int ld_acquire(const int* p) {
    return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int ld_relaxed(const int* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void add_release(int* p, int v) {
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// Control words at the head of a forward/backward workspace.
enum CtrlWord {
    CTRL_STATUS = 0,   // 0 ok, else MOE_ERR_DEVICE
    CTRL_NRT = 1,      // number of row tiles
    CTRL_NTASK = 2,    // total tasks
    CTRL_PHASE_END = 4,  // [4..11] exclusive end task id of phase 0..7
    CTRL_CURSOR = 12,    // [12..20] cursors: [12] whole queue, [13+p] phase p
    CTRL_DONE = 24,      // [24..31] completion counters per phase
    CTRL_WORDS = 64
};

// Bounded wait for *p >= need.  Returns false (and raises the status word) if
// the bound is exceeded or another worker already raised it, so that every
// wave leaves the kernel in finite time whatever happens.
__device__ __forceinline__ bool wait_ge(const int* p, int need, int* ctrl, long long limit_ticks) {
    if (ld_acquire(p) >= need) return true;
    const long long t0 = wall_clock64();
    for (;;) {
        __builtin_amdgcn_s_sleep(8);
        if (ld_acquire(p) >= need) return true;
        if (ld_relaxed(ctrl + CTRL_STATUS) != 0) return false;
        if (wall_clock64() - t0 > limit_ticks) {
            __hip_atomic_store(ctrl + CTRL_STATUS, (int)MOE_ERR_DEVICE, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            return false;
        }
    }
}

struct RowTile {   // one row tile of one local expert
    int32_t expert;  // local expert id
    int32_t row0;    // first row (position in the expert-sorted order)
    int32_t rows;    // valid rows in this tile (1..BM)
    int32_t pad;
};

struct Task {
    int32_t rt;       // row tile (GEMM phases) or block index (combine phases)
    int32_t type_ct;  // (type << 20) | column tile
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace uniep
