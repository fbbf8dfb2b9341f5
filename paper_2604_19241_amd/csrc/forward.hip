// Forward MegaKernel: dispatch(gather) + grouped GEMM gate/up + SwiGLU +
// grouped GEMM down + combine, as one persistent work-queue kernel.
//
// Paper: Section 3.1 (persistent workers, scoreboard, dynamic scheduling),
// Section 3.2 (GroupGEMM+Combine, top-k accumulation constraint), Section 4.3
// (producers and consumers walk the experts in the same ascending order),
// Listing 1 (the fetch loop).  On one GPU the "dispatch" of a token to its
// expert is a gather: the GEMM1 tile reads the rows of x through the
// permutation while it stages them into LDS, so the dispatched copy is never
// written to HBM; the scoreboard that remains orders GEMM1 -> GEMM2 per row
// tile and GEMM2 -> combine.  SwiGLU runs in the GEMM1 epilogue on the fp32
// accumulators.
#include "mma.hpp"

#include <mutex>

namespace uniep {

enum TaskType { TASK_GEMM1 = 0, TASK_GEMM2 = 1, TASK_COMBINE = 2 };

// Where GEMM1 stages its A operand (the gathered rows of x): 1 = straight into registers,
// 0 = through LDS with 128-byte coalesced row pieces.

constexpr int kCombineTokens = 16;   // tokens per combine task (4 per wave)

struct FwdParams {
    moe_shape_t s;
    const char* x;
    const char* w_gate;
    const char* w_up;
    const char* w_down;
    const float* topk_w;
    const int32_t* offsets;
    const int32_t* perm;
    const int32_t* inv_perm;
    char* y;
    char* gu;   // saved G|U [A,2I] or null
    char* h;    // [A,I]
    char* o;    // [A,d]
    int* ctrl;
    int* flag1;   // per row tile: GEMM1 column tiles finished
    Task* tasks;
    int nct1, nct2;   // column tiles of GEMM1 (128 h-columns each) and GEMM2 (256 each)
    int max_rt;
    int workers;   // workgroups of the worker launch (the tail waits for all of them)
    long long spin_ticks;
};

// ------------------------------------------------------------- prologue
// One workgroup: row-tile table from the expert offsets, the per-XCD task lists
// (GEMM1 block of expert i+1 ahead of the GEMM2 block of expert i) and a
// cleared scoreboard.
template <int BM>
__global__ void __launch_bounds__(1024) fwd_prologue_kernel(FwdParams p) {
    __shared__ int32_t s_scan[kMaxExperts];
    __shared__ int32_t s_g1[kMaxExperts];
    __shared__ int32_t s_g2[kMaxExperts];
    __shared__ int32_t s_nt[kMaxExperts];
    __shared__ int32_t s_qbase[kQueues + 1];
    __shared__ int32_t s_qlen[kQueues];
    __shared__ int32_t s_lag;
    __shared__ ListPlan s_plan;
    const int e = threadIdx.x;
    const int ec = p.s.e_count;
    int cnt = 0, nt = 0;
    if (e < ec) {
        cnt = p.offsets[e + 1] - p.offsets[e];
        nt = (cnt + BM - 1) / BM;
    }
    s_plan.cost[e] = cnt;
    s_scan[e] = nt;
    s_nt[e] = nt;
    s_g1[e] = nt * p.nct1;
    s_g2[e] = nt * p.nct2;
    __syncthreads();
    for (int off = 1; off < kMaxExperts; off <<= 1) {
        const int32_t add = (e >= off) ? s_scan[e - off] : 0;
        __syncthreads();
        s_scan[e] += add;
        __syncthreads();
    }
    const int nrt = s_scan[kMaxExperts - 1];
    plan_lists(s_plan, ec);
    if (e < kQueues) {   // length of list e
        int len = 0;
        for (int j = 0; j < s_plan.size[e]; ++j) {
            const int x = s_plan.member[e][j];
            len += s_g1[x] + s_g2[x];
        }
        s_qlen[e] = len;
    }
    __syncthreads();
    if (e == 0) {
        int base = 0;
        for (int q = 0; q < kQueues; ++q) {
            s_qbase[q] = base;
            base += s_qlen[q];
        }
        s_qbase[kQueues] = base;
        s_lag = queue_lag(nrt * p.nct1, ec);
    }
    __syncthreads();
    __shared__ int32_t s_rt0[kMaxExperts];
    __shared__ int32_t s_r0[kMaxExperts];
    __shared__ int32_t s_t1[kMaxExperts];
    __shared__ int32_t s_t2[kMaxExperts];
    if (e < ec) {
        const int rt0 = s_scan[e] - nt;
        s_r0[e] = p.offsets[e];
        for (int i = 0; i < nt; ++i) p.flag1[rt0 + i] = 0;
        int pos1, pos2;
        queue_positions(s_plan, s_g1, s_g2, e, s_lag, pos1, pos2);
        s_rt0[e] = rt0;
        s_t1[e] = s_qbase[s_plan.list_of[e]] + pos1;
        s_t2[e] = s_qbase[s_plan.list_of[e]] + pos2;
    }
    __syncthreads();
    for (int x = e >> 6; x < ec; x += 16) {   // one wave writes the two blocks of an expert
        const int rt0 = s_rt0[x], lane = e & 63;
        Task* t1 = p.tasks + s_t1[x];
        Task* t2 = p.tasks + s_t2[x];
        const int r0 = s_r0[x], rows_x = s_plan.cost[x];
        const int nt_x = s_nt[x];
        for_each_tile(lane, nt_x, p.nct1, [&](int j, int ct) {
            t1[block_pos<true>(j, ct, nt_x, p.nct1)] =
                Task{rt0 + j, task_code(TASK_GEMM1, x, ct), r0 + j * BM, min(BM, rows_x - j * BM)};
        });
        for_each_tile(lane, nt_x, p.nct2, [&](int j, int ct) {
            t2[block_pos<true>(j, ct, nt_x, p.nct2)] =
                Task{rt0 + j, task_code(TASK_GEMM2, x, ct), r0 + j * BM, min(BM, rows_x - j * BM)};
        });
    }
    if (e < CTRL_WORDS) {
        int v = 0;
        if (e == CTRL_NRT) v = nrt;
        if (e == CTRL_NTAIL) v = (p.s.T + kCombineTokens - 1) / kCombineTokens;
        if (e == CTRL_NWAIT) v = p.workers;
        if (e >= CTRL_QLEN && e < CTRL_QLEN + kQueues) v = s_qbase[e - CTRL_QLEN + 1] - s_qbase[e - CTRL_QLEN];
        if (e >= CTRL_QBASE && e < CTRL_QBASE + kQueues) v = s_qbase[e - CTRL_QBASE];
        p.ctrl[e] = v;
    }
}

// ------------------------------------------------------------- GEMM1 task
// h[row0.., ct*128 .. +128) = silu(x_e W_gate) * (x_e W_up) for one row tile.
// Tile rows = the tile's tokens (their rows of x fetched through the permutation: the dispatch);
// tile columns = 128 gate columns and the same 128 up columns, arranged so that column fragment
// 0 of a wave holds gate columns and fragment 1 the same up columns: G and U of one h element
// sit in the same lane and accumulator element.
template <class Hook>
__device__ __forceinline__ void gemm1_task(const FwdParams& p, const RowTile rt, int ct,
                                           char* smem, Hook after_mainloop) {
    const int d = p.s.d, I = p.s.I, k = p.s.k;
    const int n0h = ct * (BN / 2);
    const Lane ln;
    FragAddr fa;
    frag_addresses<true, false>(fa, lds_addr(smem), ln);
    KcLoader lb;
    KsLoader la;
    lb.n = KcLoader::blocks_for(ln, rt.rows);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = min(KcGeom::row(ln, i), rt.rows - 1);   // rows past the tile alias its last row
        const int tok = p.perm[rt.row0 + m] / k;
        lb.p[i] = p.x + ((size_t)tok * d + KcGeom::chunk(ln, i) * 8) * 2;
        const int c = KsGeom::chunk(ln, i);                    // tile column chunk: (wave column, gate|up, 8-column piece)
        const int hc = min(n0h + 32 * (c >> 3) + 8 * (c & 3), I - 8);   // chunks past I alias the last chunk
        const char* w = ((c >> 2) & 1) ? p.w_up : p.w_gate;
        la.p[i] = w + (((size_t)rt.expert * d + KsGeom::krow(ln, i)) * I + hc) * 2;
    }
    la.step = (long long)BK * I * 2;
    f32x16_t acc[4][2];
    mma_tile<true, false>(lb, la, d / BK, rt.rows, smem, fa, acc);
    after_mainloop();

    // epilogue.  The wave's sub-tile is 128 rows x (32 gate columns | the same 32 up columns).
    // First the G|U stash, through the wave's LDS region so that 4 neighbouring lanes store 64
    // contiguous bytes; then h = silu(G) * U on the accumulators, out the same way in 8-byte
    // write-through pieces (8 lanes per 64-byte row segment): GEMM2 tiles on any XCD read it.
    const Lane le;
    const int l31 = le.l31, hf = le.hf;
    const int wm = le.wm, wn = le.wn;
    const int hc0 = n0h + 32 * wn;        // first h column of this wave
    const int rows_w = rt.rows - 128 * wm; // rows of the tile inside this wave's 128
    if (p.gu) {
        WaveRepack<8> rp(smem, le);
#pragma unroll
        for (int tf = 0; tf < 4; ++tf)
#pragma unroll
            for (int af = 0; af < 2; ++af)
#pragma unroll
                for (int vg = 0; vg < 2; ++vg) rp.put(32 * tf + l31, 4 * af + 2 * vg + hf, pack8(acc[tf][af], vg));
        const int pc = rp.get_piece();                       // 0..3: G pieces, 4..7: U pieces
        const int col = hc0 + 8 * (pc & 3);
        char* gbase = p.gu + ((size_t)(rt.row0 + 128 * wm) * 2 * I + ((pc & 4) ? I : 0) + col) * 2;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int row = rp.get_row(j);
            const u32x4_t v = rp.get(j);
            if (row < rows_w && col < I) store_stream16(gbase + (size_t)row * 2 * I * 2, v);
        }
    }
    {
        WaveRepack<4> rp(smem, le);
#pragma unroll
        for (int tf = 0; tf < 4; ++tf)
#pragma unroll
            for (int vg = 0; vg < 2; ++vg) {
                float hv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float g = acc[tf][0][8 * vg + e], u = acc[tf][1][8 * vg + e];
                    hv[e] = g * sigmoid_f(g) * u;
                }
                rp.put(32 * tf + l31, 2 * vg + hf,
                       u32x4_t{pack_bf16x2(hv[0], hv[1]), pack_bf16x2(hv[2], hv[3]), pack_bf16x2(hv[4], hv[5]),
                               pack_bf16x2(hv[6], hv[7])});
            }
        const int col = hc0 + 4 * rp.get8_piece();   // 8-byte pieces: 4 columns each
        char* hbase = p.h + ((size_t)(rt.row0 + 128 * wm) * I + col) * 2;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int row = rp.get8_row(j);
            const u32x2_t v = rp.get8(j);
            if (row < rows_w && col < I) store_wt8(hbase + (size_t)row * I * 2, v);
        }
    }
}

// ------------------------------------------------------------- GEMM2 task
// o[row0.., ct*256 .. +256) = h_e W_down[e] for one row tile.
template <class Hook>
__device__ __forceinline__ void gemm2_task(const FwdParams& p, const RowTile rt, int ct,
                                           char* smem, Hook after_mainloop) {
    const int d = p.s.d, I = p.s.I;
    const int n0 = ct * BN;
    const Lane ln;
    FragAddr fa;
    frag_addresses<true, false>(fa, lds_addr(smem), ln);
    KcLoader lb;
    KsLoader la;
    lb.n = KcLoader::blocks_for(ln, rt.rows);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = min(KcGeom::row(ln, i), rt.rows - 1);
        lb.p[i] = p.h + ((size_t)(rt.row0 + m) * I + KcGeom::chunk(ln, i) * 8) * 2;
        const int c = min(n0 + KsGeom::chunk(ln, i) * 8, d - 8);
        la.p[i] = p.w_down + (((size_t)rt.expert * I + KsGeom::krow(ln, i)) * d + c) * 2;
    }
    la.step = (long long)BK * d * 2;
    f32x16_t acc[4][2];
    mma_tile<true, false>(lb, la, I / BK, rt.rows, smem, fa, acc);
    after_mainloop();
    char* obase = p.o + ((size_t)rt.row0 * d + n0) * 2;
    store_subtile_bf16(acc, smem, rt.rows, d - n0, [&](int row, int col, u32x4_t v) {
        store_stream16(obase + ((size_t)row * d + col) * 2, v);
    });
}

// ------------------------------------------------------------- combine task
// y[t] = sum_j w[t,j] * o[row(t,j)], slot order, fp32; one wave per token, 16
// bytes per lane, no LDS (Section 5.2 "Relay & Reduce Workers").
// KM = compile-time bound on k (8 or kMaxTopK): the row loads of all KM slots are in flight
// at once, so the smaller bound halves the registers and doubles the waves per SIMD.
template <int NW, int KM = kMaxTopK>
__device__ __forceinline__ void combine_task(const FwdParams& p, int block) {
    const int d = p.s.d, k = p.s.k, T = p.s.T;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int tt = wave; tt < kCombineTokens; tt += NW) {
        const int t = block * kCombineTokens + tt;
        if (t >= T) break;
        int rows[KM];
        float w[KM];
#pragma unroll
        for (int j = 0; j < KM; ++j) {
            rows[j] = (j < k) ? p.inv_perm[(size_t)t * k + j] : -1;
            w[j] = (j < k) ? p.topk_w[(size_t)t * k + j] : 0.f;
        }
        // two 16-byte column pieces per lane and round: all 2k row loads are issued before the
        // first is used, so a wave keeps up to 2k KB in flight
        for (int c0 = lane * 8; c0 < d; c0 += 2 * 64 * 8) {
            const int c1 = c0 + 64 * 8;
            const bool two = c1 < d;
            u32x4_t v0[KM], v1[KM];
#pragma unroll
            for (int j = 0; j < KM; ++j) {
                v0[j] = zero4();
                v1[j] = zero4();
                if (j < k && rows[j] >= 0) {
                    const char* src = p.o + (size_t)rows[j] * d * 2;
                    v0[j] = *(const u32x4_t*)(src + (size_t)c0 * 2);
                    if (two) v1[j] = *(const u32x4_t*)(src + (size_t)c1 * 2);
                }
            }
            float a0[8], a1[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) a0[q] = a1[q] = 0.f;
#pragma unroll
            for (int j = 0; j < KM; ++j) {
                if (j < k && rows[j] >= 0) {   // slot order, local slots only
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        a0[2 * q] += w[j] * bf16_lo(v0[j][q]);
                        a0[2 * q + 1] += w[j] * bf16_hi(v0[j][q]);
                        a1[2 * q] += w[j] * bf16_lo(v1[j][q]);
                        a1[2 * q + 1] += w[j] * bf16_hi(v1[j][q]);
                    }
                }
            }
            u32x4_t y0, y1;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                y0[q] = pack_bf16x2(a0[2 * q], a0[2 * q + 1]);
                y1[q] = pack_bf16x2(a1[2 * q], a1[2 * q + 1]);
            }
            store_stream16(p.y + ((size_t)t * d + c0) * 2, y0);
            if (two) store_stream16(p.y + ((size_t)t * d + c1) * 2, y1);
        }
    }
}

// ------------------------------------------------------------- the worker loop
// phase = -1: all tasks with scoreboard waits (persistent MegaKernel).
// phase = -2: every GEMM task with scoreboard waits, no tail tasks: the workers leave
// when the lists are empty and the combine runs as a launch of its own (fwd_tail_kernel).
// phase >= 0: only that phase's tasks (staged schedule; the waits are already
// satisfied by stream order).
__global__ void __launch_bounds__(kMmaThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
fwd_worker_kernel(FwdParams p, int phase) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __shared__ int s_task;
    __shared__ int s_ok;
    int* ctrl = p.ctrl;
    const int pass = phase < 0 ? kPersistentPass : 1 + phase;
    const int home = xcc_id();
    const bool use_lists = phase != TASK_COMBINE;
    const bool use_tail = phase == -1 || phase == TASK_COMBINE;
    // this launch runs GEMM2 tiles: its workers publish their o rows once, when they run out of
    // GEMM work, instead of once per tile
    const bool publishes = phase == -1 || phase == TASK_GEMM2;
    bool arrived = false;
    unsigned exhausted = 0;
    if (threadIdx.x == 0) {
        if (phase == -1) worker_started(ctrl, home);
        s_task = fetch_task(ctrl, pass, home, exhausted, use_lists, use_tail);
    }
    __syncthreads();
    for (;;) {
        const int id = s_task;
        if (id == kFetchDone) break;
        // The cursor atomic of the next task is issued behind the main loop of this one: vector
        // memory results return in order, so an atomic issued ahead of a tile would hold back
        // the first loads of its wave by the atomic's round trip.
        PendingFetch pf;
        pf.q = -1;
        pf.id = 0;
        bool issued = false;
        auto issue = [&]() {
            if (!issued && threadIdx.x == 0) pf = fetch_issue(ctrl, pass, home, exhausted, use_lists);
            issued = true;
        };
        if (id >= 0) {
            // the task is the same for every lane: keep its fields in scalar registers
            Task task = p.tasks[id];
            task.idx = rfl(task.idx);
            task.code = rfl(task.code);
            task.row0 = rfl(task.row0);
            task.rows = rfl(task.rows);
            const int type = task_type(task), ct = task_ct(task);
            if (phase >= 0 && type != phase) {
                // staged launch: another phase's task, nothing to do
            } else if (type == TASK_GEMM1) {
                const RowTile rt = task_row_tile(task);
                gemm1_task(p, rt, ct, smem, issue);
                wait_stores();
                __syncthreads();   // the write-through h stores of every wave have completed
                if (threadIdx.x == 0) add_relaxed(p.flag1 + task.idx, 1);
            } else {
                if (threadIdx.x == 0) s_ok = wait_ge(p.flag1 + task.idx, p.nct1, ctrl, p.spin_ticks);
                __syncthreads();
                if (s_ok) {
                    const RowTile rt = task_row_tile(task);
                    gemm2_task(p, rt, ct, smem, issue);
                }
            }
        } else {
            if (publishes && !arrived) {   // first tail task: all of this worker's o rows are written
                arrived = true;
                wait_stores();
                __syncthreads();
                if (threadIdx.x == 0) {
                    if (phase < 0) worker_arrived(ctrl, home, ctrl[CTRL_NWAIT], p.spin_ticks);
                    else add_release(ctrl + CTRL_DONE, 1);
                }
            }
            if (threadIdx.x == 0)
                s_ok = wait_ge(ctrl + CTRL_DONE, ctrl[CTRL_NWAIT], ctrl, p.spin_ticks, CTRL_TAIL_WAIT_TICKS);
            __syncthreads();
            if (s_ok) combine_task<8>(p, -1 - id);
        }
        issue();           // tasks without a main loop (tail, skipped, given up)
        __syncthreads();   // every thread has read s_task / s_ok of this round
        if (threadIdx.x == 0) s_task = fetch_finish(pf, ctrl, pass, home, exhausted, use_lists, use_tail);
        __syncthreads();
    }
    if (phase == -2) return;   // the kernel boundary publishes the rows
    if (publishes && !arrived) {   // ran out of work without seeing a tail task
        wait_stores();
        __syncthreads();
        if (threadIdx.x == 0) {
            if (phase < 0) worker_arrived(ctrl, home, ctrl[CTRL_NWAIT], p.spin_ticks);
            else add_release(ctrl + CTRL_DONE, 1);
        }
    }
}

// The combine as a plain grid launch, one workgroup per block of kCombineTokens tokens, for
// the default schedule: it follows the GEMM MegaKernel in stream order, so it needs no
// scoreboard wait, no task cursor and no LDS, and as many workgroups as fit share a CU.
template <int NW, int KM>
__global__ void __launch_bounds__(64 * NW) fwd_tail_kernel(FwdParams p) {
    combine_task<NW, KM>(p, blockIdx.x);
}

// ------------------------------------------------------------------ host side

struct FwdLayout {
    size_t ctrl, flag1, tasks, h, o, total;
    int max_rt, nct1, nct2;
    size_t max_tasks;
};

FwdLayout fwd_layout(const moe_shape_t& s, bool with_ho) {
    FwdLayout L;
    const size_t A_cap = (size_t)s.T * s.k;
    L.max_rt = (int)((A_cap + 127) / 128) + s.e_count;
    L.nct1 = (s.I + BN / 2 - 1) / (BN / 2);
    L.nct2 = (s.d + BN - 1) / BN;
    L.max_tasks = (size_t)L.max_rt * (L.nct1 + L.nct2) + (s.T + kCombineTokens - 1) / kCombineTokens;
    size_t off = 0;
    L.ctrl = off;  off = align_up(off + CTRL_WORDS * sizeof(int), 256);
    L.flag1 = off; off = align_up(off + (size_t)L.max_rt * sizeof(int), 256);
    L.tasks = off; off = align_up(off + L.max_tasks * sizeof(Task), 256);
    L.h = off;     if (with_ho) off = align_up(off + A_cap * s.I * 2, 256);
    L.o = off;     if (with_ho) off = align_up(off + A_cap * s.d * 2, 256);
    L.total = off;
    return L;
}

size_t fwd_workspace_bytes(const moe_shape_t& s) { return fwd_layout(s, true).total; }
size_t fwd_ctrl_bytes(const moe_shape_t& s) { return fwd_layout(s, false).total; }

// Resident worker slots per device: the one piece of process-wide state, filled on first use
// under a lock and constant afterwards.
static std::mutex g_workers_mu;
static int g_workers[kMaxDevices];

static int resident_workers(int* out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOE_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_workers_mu);
    if (g_workers[dev] == 0) {
        if (hipFuncSetAttribute((const void*)fwd_worker_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                kMmaSmem) != hipSuccess)
            return MOE_ERR_HIP;
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fwd_worker_kernel, kMmaThreads,
                                                         kMmaSmem) != hipSuccess)
            return MOE_ERR_HIP;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return MOE_ERR_HIP;
        if (per_cu < 1 || cus < 1) return MOE_ERR_HIP;
        g_workers[dev] = per_cu * cus;
    }
    *out = g_workers[dev];
    return MOE_OK;
}

// BM = rows per row tile: 256, or 128 (every tile then leaves the upper half of the workgroup's
// rows empty; kept as an option because results must not depend on it).
template <int BM>
static int fwd_launch_bm(FwdParams& p, const moe_opts_t& opts, hipStream_t st) {
    int resident = 0;
    int rc = resident_workers(&resident);
    if (rc != MOE_OK) return rc;
    int workers = opts.workers > 0 ? min(opts.workers, resident) : resident;
    p.workers = workers;
    hipLaunchKernelGGL(fwd_prologue_kernel<BM>, dim3(1), dim3(1024), 0, st, p);
    if (opts.schedule == 2) {
        for (int phase = 0; phase < 3; ++phase)
            hipLaunchKernelGGL(fwd_worker_kernel, dim3(workers), dim3(kMmaThreads), kMmaSmem, st, p, phase);
    } else if (opts.schedule != 1) {   // 0 (default) and 3: GEMM MegaKernel, then the tail tasks
        hipLaunchKernelGGL(fwd_worker_kernel, dim3(workers), dim3(kMmaThreads), kMmaSmem, st, p, -2);
        const int n_tail = (p.s.T + kCombineTokens - 1) / kCombineTokens;
        if (n_tail > 0 && !opts.skip_tail) {
            if (p.s.k <= 8)
                hipLaunchKernelGGL((fwd_tail_kernel<8, 8>), dim3(n_tail), dim3(kMmaThreads), 0, st, p);
            else
                hipLaunchKernelGGL((fwd_tail_kernel<8, kMaxTopK>), dim3(n_tail), dim3(kMmaThreads), 0, st, p);
        }
    } else {
        hipLaunchKernelGGL(fwd_worker_kernel, dim3(workers), dim3(kMmaThreads), kMmaSmem, st, p, -1);
    }
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int fwd_launch(const moe_shape_t& s, const void* x, const void* w_gate, const void* w_up,
               const void* w_down, const moe_routing_t& r, void* y, char* gu, char* h, char* o,
               char* ws, const moe_opts_t& opts, int nw, hipStream_t st) {
    const FwdLayout L = fwd_layout(s, false);
    FwdParams p;
    p.s = s;
    p.x = (const char*)x;
    p.w_gate = (const char*)w_gate;
    p.w_up = (const char*)w_up;
    p.w_down = (const char*)w_down;
    p.topk_w = r.topk_w;
    p.offsets = r.offsets;
    p.perm = r.perm;
    p.inv_perm = r.inv_perm;
    p.y = (char*)y;
    p.gu = gu;
    p.h = h;
    p.o = o;
    p.ctrl = (int*)(ws + L.ctrl);
    p.flag1 = (int*)(ws + L.flag1);
    p.tasks = (Task*)(ws + L.tasks);
    p.nct1 = L.nct1;
    p.nct2 = L.nct2;
    p.max_rt = L.max_rt;
    const int ms = opts.spin_limit_ms > 0 ? opts.spin_limit_ms : 2000;
    p.spin_ticks = (long long)ms * 100000ll;   // wall_clock64 ticks at 100 MHz
    return nw == 4 ? fwd_launch_bm<128>(p, opts, st) : fwd_launch_bm<256>(p, opts, st);
}



}  // namespace uniep
