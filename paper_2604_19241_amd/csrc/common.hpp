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
constexpr int kMaxDevices = 64;                           // per-device host caches are indexed by the HIP device id
constexpr size_t kRouteStaticScratchBytes = 4u << 20;     // file-scope scratch of moe_route_static

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

// Write-through stores (agent scope): the data goes past this XCD's L2 to the
// memory side, so a consumer on any XCD sees it once the store has completed
// (s_waitcnt vmcnt(0)) and the consumer has acquired.  Producers that publish a
// tile written only with these stores can signal with a relaxed atomic instead
// of a release, which would write back the whole L2 of the XCD.
__device__ __forceinline__ void store_wt8(void* p, u32x2_t v) {
    __hip_atomic_store((uint64_t*)p, __builtin_bit_cast(uint64_t, v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
// (two 8-byte stores: the compiler has no 16-byte atomic store, and a store hidden in inline
// assembly would escape its hazard handling for the data registers)
__device__ __forceinline__ void store_wt16(void* p, u32x4_t v) {
    store_wt8(p, u32x2_t{v[0], v[1]});
    store_wt8((char*)p + 8, u32x2_t{v[2], v[3]});
}
// Streaming store for outputs that are written once and not read again soon
// (o, the G|U stash, dXp, dW, y, dX): they should not displace operands in L2.
__device__ __forceinline__ void store_stream16(void* p, u32x4_t v) {
    __builtin_nontemporal_store(v, (u32x4_t*)p);
}
// All write-through stores of this wave have completed.
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" : : : "memory"); }
__device__ __forceinline__ void add_relaxed(int* p, int v) {
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- work queues -----------------------------------------------------------
// The GEMM tasks are cut into kQueues lists, one per XCD (each XCD has its own
// L2): every expert belongs to one list (see ListPlan), so the tiles that share
// an expert's weights and rows run on one XCD and meet in its L2.  Inside a list
// the experts are pipelined with a lag: the producer block of the list's
// (i+L)-th expert comes before the consumer block of its i-th, so consumers
// rarely wait.  A workgroup drains its own XCD's list first and then steals from the
// others; the token-parallel tail tasks (combine / dX) come last.  Dependencies
// point to earlier entries of the same list, and an entry is fetched only by a
// running workgroup, so the lowest unfinished entry of every list can always run.
constexpr int kQueues = 8;
// Cursor sets: 1+p = staged launch of phase p; the last set = persistent launch.  The
// persistent launches' cursors take one atomic per task from every worker and must not share
// a 128-byte line with the table (list lengths and bases) that every task fetch reads: with
// set 0, which does, the whole step was 3 % slower.
constexpr int kPasses = 7;
constexpr int kPersistentPass = kPasses - 1;

// Control words at the head of a forward/backward workspace.
enum CtrlWord {
    CTRL_STATUS = 0,   // 0 ok, else MOE_ERR_DEVICE
    CTRL_NRT = 1,      // number of row tiles
    CTRL_NTAIL = 2,    // number of tail tasks
    CTRL_NWAIT = 3,    // completions the tail tasks wait for
    CTRL_DONE = 4,     // completion counter of the last GEMM phase
    CTRL_WAIT_TICKS = 5,   // sum over workers of 10 ns ticks spent in scoreboard waits (diagnostic)
    CTRL_TAIL_WAIT_TICKS = 6,   // the same for the waits of the tail tasks
    CTRL_QLEN = 8,     // [8]  entries per list
    CTRL_QBASE = 16,   // [8]  first entry of each list in the task array
    CTRL_CURSOR = 24,  // [kPasses][kQueues + 1]  list cursors and tail cursor per pass
    CTRL_XCD_WORKERS = 24 + kPasses * (kQueues + 1) + 2,   // [8] workers that started on each XCD
    CTRL_XCD_ARRIVED = CTRL_XCD_WORKERS + kQueues,         // [8] workers of each XCD that ran out of GEMM work
    CTRL_STARTED = CTRL_XCD_ARRIVED + kQueues,             // workers that started
    CTRL_WORDS = CTRL_STARTED + 1
};

constexpr int kFetchDone = INT32_MIN;

__device__ __forceinline__ int xcc_id() {
    unsigned v;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(v));
    return (int)(v & (kQueues - 1));
}

// Called by one thread.  Returns an index into the task array (>= 0), or
// -1 - t for tail task t, or kFetchDone.  `exhausted` is the caller's bitmask of
// lists already seen empty.  use_lists / use_tail restrict a staged launch.
__device__ __forceinline__ int fetch_task(int* ctrl, int pass, int home, unsigned& exhausted,
                                          bool use_lists, bool use_tail) {
    int* cur = ctrl + CTRL_CURSOR + pass * (kQueues + 1);
    if (use_lists) {
        // (not unrolled: `home` is fixed for the kernel, and eight precomputed cursor addresses
        // would occupy registers, or scratch, across the worker's whole loop)
#pragma unroll 1
        for (int i = 0; i < kQueues; ++i) {
            const int q = (home + i) & (kQueues - 1);
            if (exhausted & (1u << q)) continue;
            const int len = ctrl[CTRL_QLEN + q];
            const int id = (len > 0) ? atomicAdd(cur + q, 1) : len;
            if (id < len) return ctrl[CTRL_QBASE + q] + id;
            exhausted |= 1u << q;
        }
    }
    if (use_tail) {
        const int t = atomicAdd(cur + kQueues, 1);
        if (t < ctrl[CTRL_NTAIL]) return -1 - t;
    }
    return kFetchDone;
}

// Split fetch, so that the round trip of the cursor atomic overlaps with the
// current task: fetch_issue() is called (by one thread) before the task runs and
// only issues the atomic on the first list not yet seen empty; fetch_finish()
// after the task turns the result into the next task, falling back to the
// blocking walk over the remaining lists and the tail.
struct PendingFetch {
    int q;     // list the atomic was issued on, -1 if none
    int id;    // value the atomic returned
};
__device__ __forceinline__ PendingFetch fetch_issue(int* ctrl, int pass, int home, unsigned exhausted,
                                                    bool use_lists) {
    PendingFetch f;
    f.q = -1;
    f.id = 0;
    // first list from `home` on (cyclically) that has not been seen empty: one computed address, so
    // that the compiler does not keep eight cursor addresses alive across the worker's whole loop
    const unsigned live = ~exhausted & ((1u << kQueues) - 1u);
    if (use_lists && live != 0) {
        const unsigned rot = ((live >> home) | (live << (kQueues - home))) & ((1u << kQueues) - 1u);
        const int q = (home + __builtin_ctz(rot)) & (kQueues - 1);
        f.q = q;
        f.id = atomicAdd(ctrl + CTRL_CURSOR + pass * (kQueues + 1) + q, 1);
    }
    return f;
}
__device__ __forceinline__ int fetch_finish(const PendingFetch f, int* ctrl, int pass, int home,
                                            unsigned& exhausted, bool use_lists, bool use_tail) {
    if (f.q >= 0) {
        if (f.id < ctrl[CTRL_QLEN + f.q]) return ctrl[CTRL_QBASE + f.q] + f.id;
        exhausted |= 1u << f.q;
    }
    return fetch_task(ctrl, pass, home, exhausted, use_lists, use_tail);
}

// Order of the nt x nct tiles (row tile j, column tile ct) of one expert inside its block of
// a list.  The CUs of an XCD take consecutive entries, and every tile they run at the same
// time streams its own A rows and its own B columns through the XCD's L2.  Entry i walks
// groups of kColGroup column tiles, inside a column group row groups of kRowGroup row tiles:
// 32 consecutive entries cover 4 row tiles x 8 column tiles (12 operand streams) where a
// row-major order covers 1 x 32 (33 streams: the weights of a 1024-row expert were fetched
// four times).  Inside a 4 x 8 group the row-tile GEMMs (forward, dH, dXp) put the row tiles
// innermost, so that the tiles that share a weight tile are fetched back to back (measured
// 1 % on the forward pass and 0.7 % on the backward pass of 512-row experts); the
// weight-gradient blocks, whose two operands are both row slabs of the expert, keep the column
// tiles innermost (the other order cost 0.5 %).
// block_pos() gives the entry of tile (j, ct); for_each_tile() hands every tile of the grid to
// the lanes of one wave, 8 row tiles x 8 column tiles per round, without a division.
constexpr int kColGroup = 8;   // 4 x 8 and 6 x 6 (rows x columns) measured within 1 % of 8 x 4
constexpr int kRowGroup = 4;
template <bool ROWS_INNERMOST>
__device__ __forceinline__ int block_pos(int j, int ct, int nt, int nct) {
    const int g = ct / kColGroup;
    const int width = min(kColGroup, nct - g * kColGroup);   // the last group may be narrower
    const int base = g * nt * kColGroup;
    if (ROWS_INNERMOST) {
        const int rg = j / kRowGroup;
        const int rows = min(kRowGroup, nt - rg * kRowGroup);   // and the last row group shorter
        return base + rg * kRowGroup * width + (ct - g * kColGroup) * rows + (j - rg * kRowGroup);
    }
    return base + j * width + (ct - g * kColGroup);
}
template <class F>
__device__ __forceinline__ void for_each_tile(int lane, int nt, int nct, F f) {
    for (int j0 = 0; j0 < nt; j0 += 8)
        for (int c0 = 0; c0 < nct; c0 += 8) {
            const int j = j0 + (lane >> 3), ct = c0 + (lane & 7);
            if (j < nt && ct < nct) f(j, ct);
        }
}

// Which expert goes to which list.  The lists should end at the same time:
// work that one XCD steals from another list has lost the L2 sharing between
// the tiles of a row tile and of an expert, and runs about half as fast.  So the
// experts are sorted by cost (rows, descending; ties by id) and dealt to the
// lists in boustrophedon order (ranks 0..7 to lists 0..7, ranks 8..15 to lists
// 7..0, ...).  Big experts come first in every list, small ones fill the end.
// The plan depends only on the counts, so it is the same on every run.
struct ListPlan {
    int32_t cost[kMaxExperts];              // in: cost of every local expert (0 beyond e_count)
    uint16_t order[kMaxExperts];            // experts by descending cost
    uint16_t member[kQueues][kMaxExperts];  // member[q][i] = i-th expert of list q
    uint16_t list_of[kMaxExperts];
    uint16_t slot_of[kMaxExperts];
    int32_t size[kQueues];                  // experts per list
};

// Called by all 1024 threads of the prologue workgroup after plan.cost is written
// (and a barrier).  Ends with a barrier.
__device__ __forceinline__ void plan_lists(ListPlan& plan, int ec) {
    const int e = threadIdx.x;
    if (e < ec) {
        const int32_t mine = plan.cost[e];
        int r = 0;
        for (int j = 0; j < ec; ++j) {
            const int32_t c = plan.cost[j];
            r += (c > mine || (c == mine && j < e)) ? 1 : 0;
        }
        plan.order[r] = (uint16_t)e;
    }
    __syncthreads();
    if (e < ec) {
        const int x = plan.order[e];
        const int i = e / kQueues, c = e % kQueues;
        const int q = (i & 1) ? kQueues - 1 - c : c;
        plan.member[q][i] = (uint16_t)x;
        plan.list_of[x] = (uint16_t)q;
        plan.slot_of[x] = (uint16_t)i;
    }
    if (e < kQueues) {
        int n = 0;
        for (int i = 0; i * kQueues < ec; ++i) {
            const int c = (i & 1) ? kQueues - 1 - e : e;
            n += (i * kQueues + c < ec) ? 1 : 0;
        }
        plan.size[e] = n;
    }
    __syncthreads();
}

// Position of expert e's producer block (pos_a) and consumer block (pos_b)
// inside its list, given the block sizes ga[], gb[] of all experts (shared
// memory) and the lag L >= 1: the consumer block of the list's i-th expert
// follows the producer block of its (i+L)-th.  List order for L = 1:
// A0, A1, B0, A2, B1, ..., A(n-1), B(n-2), B(n-1).
__device__ __forceinline__ void queue_positions(const ListPlan& plan, const int* ga, const int* gb, int e,
                                                int lag, int& pos_a, int& pos_b) {
    const int q = plan.list_of[e], i = plan.slot_of[e];
    const int nq = plan.size[q];
    int sa_i = 0, sb_i = 0, sb_lag = 0, sa_n = 0;
    const int lim = min(i + lag + 1, nq);
    for (int j = 0; j < lim; ++j) {
        const int ej = plan.member[q][j];
        if (j < i) {
            sa_i += ga[ej];
            sb_i += gb[ej];
            if (j < i - lag) sb_lag += gb[ej];
        }
        sa_n += ga[ej];
    }
    pos_a = sa_i + sb_lag;
    pos_b = sa_n + sb_i;
}

// Lag (in experts) between an expert's producer and consumer blocks: enough
// producer tasks in between (about four rounds of one XCD's workgroups) that a
// consumer's inputs are complete when it is fetched, also near the end of the
// lists, where stealing workgroups drain the consumer blocks quickly.
__device__ __forceinline__ int queue_lag(int total_producer_tasks, int ec) {
    const int per = max(1, total_producer_tasks / max(1, ec));
    return min(16, max(1, (128 + per - 1) / per));
}

// Bounded wait for *p >= need.  Returns false (and raises the status word) if
// the bound is exceeded or another worker already raised it, so that every
// wave leaves the kernel in finite time whatever happens.
__device__ __forceinline__ void fence_acquire() {
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}
// The polls are relaxed loads; the one acquire fence follows the successful
// poll.  An acquire per poll would invalidate this XCD's L2 at the polling
// rate and slow down every tile still running on it.
__device__ __forceinline__ bool wait_ge(const int* p, int need, int* ctrl, long long limit_ticks,
                                        int stat_word = CTRL_WAIT_TICKS) {
    if (ld_relaxed(p) >= need) {
        fence_acquire();
        return true;
    }
    const long long t0 = wall_clock64();
    // Back off to one poll per ~3 us: a few hundred waiting workgroups polling one address at full
    // rate saturate its memory channel and slow down the tiles that are still running.
    for (int round = 0;; ++round) {
        if (round < 4) __builtin_amdgcn_s_sleep(16);
        else if (round < 8) __builtin_amdgcn_s_sleep(48);
        else __builtin_amdgcn_s_sleep(127);
        if (ld_relaxed(p) >= need) {
            fence_acquire();
            atomicAdd(ctrl + stat_word, (int)(wall_clock64() - t0));
            return true;
        }
        if (ld_relaxed(ctrl + CTRL_STATUS) != 0) return false;
        if (wall_clock64() - t0 > limit_ticks) {
            __hip_atomic_store(ctrl + CTRL_STATUS, (int)MOE_ERR_DEVICE, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            return false;
        }
    }
}

// Publication of the rows a persistent worker wrote with ordinary (write-back)
// stores, for consumers that wait for ALL workers (the tail tasks).  A release
// writes back the whole L2 of the XCD, which stalls the tiles still running on
// it, so only the last worker of each XCD to run out of GEMM work releases, on
// behalf of the XCD: the others only count themselves in after their own stores
// have completed, which orders those stores before the releasing worker's
// write-back.  worker_started() is called once at kernel start, worker_arrived()
// once when the worker has no GEMM work left (both by one thread, the second
// after s_waitcnt vmcnt(0) and a workgroup barrier).
__device__ __forceinline__ void worker_started(int* ctrl, int xcd) {
    add_relaxed(ctrl + CTRL_XCD_WORKERS + xcd, 1);
    add_relaxed(ctrl + CTRL_STARTED, 1);
}
__device__ __forceinline__ void worker_arrived(int* ctrl, int xcd, int workers, long long limit_ticks) {
    if (!wait_ge(ctrl + CTRL_STARTED, workers, ctrl, limit_ticks)) return;   // every worker is registered
    const int on_xcd = ld_relaxed(ctrl + CTRL_XCD_WORKERS + xcd);
    const int before = __hip_atomic_fetch_add(ctrl + CTRL_XCD_ARRIVED + xcd, 1, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT);
    if (before + 1 == on_xcd) add_release(ctrl + CTRL_DONE, on_xcd);
}

struct RowTile {   // one row tile of one local expert
    int32_t expert;  // local expert id
    int32_t row0;    // first row (position in the expert-sorted order)
    int32_t rows;    // valid rows in this tile (1..BM)
};

// One GEMM task, self-contained so that a worker needs a single 16-byte load
// before it can start: no second trip to a row-tile table or to the offsets.
struct Task {
    int32_t idx;      // row-tile tasks: row tile index (its scoreboard flag); weight-gradient tasks: row-tile of the output (m index)
    int32_t code;     // (type << 28) | (local expert << 16) | column tile
    int32_t row0;     // row-tile tasks: first row of the tile; weight-gradient tasks: first row of the expert
    int32_t rows;     // row-tile tasks: rows in the tile; weight-gradient tasks: rows of the expert (the reduction length)
};
__host__ __device__ __forceinline__ int32_t task_code(int type, int expert, int ct) {
    return (int32_t)(((uint32_t)type << 28) | ((uint32_t)expert << 16) | (uint32_t)ct);
}
__device__ __forceinline__ int task_type(const Task& t) { return (int)((uint32_t)t.code >> 28); }
__device__ __forceinline__ int task_expert(const Task& t) { return (t.code >> 16) & 0xfff; }
__device__ __forceinline__ int task_ct(const Task& t) { return t.code & 0xffff; }
__device__ __forceinline__ RowTile task_row_tile(const Task& t) { return RowTile{task_expert(t), t.row0, t.rows}; }

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace uniep
