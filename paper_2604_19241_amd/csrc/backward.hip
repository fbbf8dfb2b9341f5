// Backward MegaKernel of the fused MoE layer.
//
// Paper: Section 2.1 "Backward Propagation and Numerical Stability": the
// gradient of the output is dispatched to the experts with the same token
// mapping, input gradients are grouped GEMMs over the row tiles, and the weight
// gradients are "transposed" grouped GEMMs that reduce over an expert's rows.
// Because the rows of an expert sit in the deterministic order of Algorithm 1
// and every tile walks them front to back in one workgroup, the accumulation
// order of every dW element is fixed: bitwise reproducible, no float atomics,
// no split of the reduction.  Scheduling follows Section 3.1 (one work queue,
// scoreboard, producers before consumers).
//
// Phases (task ids ascending; a task only ever waits on lower ids):
//   0  dH = dO W_down^T per row tile, dO = gate*dY gathered on the fly;
//      SwiGLU backward in the epilogue -> dG|dU                       (MFMA)
//   1  dW_down[e] = h_e^T dO_e            (no dependency: fills the queue)
//   2  dXp = dG W_gate^T + dU W_up^T per row tile (one GEMM over k = 2I)
//   3  dW_gate[e], dW_up[e] = x_e^T dG_e, x_e^T dU_e
//   4  dX[t] = sum_j dXp[row(t,j)] in slot order; dtopk_w = <dY[t], o[row]>
#include "mma.hpp"

#include <algorithm>
#include <mutex>

namespace uniep {

enum BwdTask { B_DH = 0, B_DWD = 1, B_DXP = 2, B_DWGU = 3, B_DX = 4 };
constexpr int kDxTokens = 16;

struct BwdParams {
    moe_shape_t s;
    const char* dy;
    const char* x;
    const char* w_gate;
    const char* w_up;
    const char* w_down;
    const float* topk_w;
    const int32_t* offsets;
    const int32_t* perm;
    const int32_t* inv_perm;
    const char* gu;   // saved G|U [A,2I]
    const char* h;    // saved h [A,I]
    const char* o;    // saved o [A,d]
    char* dx;
    char* dw_gate;
    char* dw_up;
    char* dw_down;
    float* dtopk_w;
    int* ctrl;
    int* flag_rt;   // per row tile: dH column tiles finished
    int* flag_e;    // per expert: dH tiles finished
    Task* tasks;
    int32_t* row_tok;
    float* row_w;
    char* dgu;   // [A,2I]
    char* dxp;   // [A,d]
    char* hw;    // [A,I]  gate * h, the row operand of dW_down (dO = gate * dY, with the gate moved to the other factor)
    float* dots; // [4 * nct_dh][T*k] per dH column tile and wave column: sum over its 64 columns of (dY W_down^T)[r][i] * h[r][i]
    int nct_dh, nct_dxp;        // column tiles of phase 0 (256 of I) and phase 2 (256 of d)
    int mt_dwd, nt_dwd;         // dW_down tiles per expert: ceil(I/256) x ceil(d/256)
    int mt_dwgu, nt_dwgu;       // dW_gate/up tiles per expert: ceil(d/256) x ceil(I/128)
    int split_rows;             // 0, or the fixed split distance of the weight-gradient reductions (multiple of 64)
    int32_t* split_base;        // [e_count]  first partial-tile slot of expert e (split experts only)
    int32_t* split_cnt;         // [split tiles]  partial tiles written so far, per output tile of a split expert
    int32_t* split_tile0;       // [e_count]  first entry of expert e in split_cnt
    char* split_buf;            // [slots][256 KB]  fp32 partial tiles in accumulator layout
    int n_dots;                 // partial sums per routed row: 4 * nct_dh
    int bm;                     // rows per row tile (256, or 128)
    int workers;                // workgroups of the worker launch (the tail waits for all of them)
    long long spin_ticks;
};

// Weight-gradient tasks carry (output row tile, part, parts) in Task.idx.
__host__ __device__ __forceinline__ int wgrad_idx(int mt, int part, int parts) { return mt | (part << 8) | (parts << 20); }
__device__ __forceinline__ int wgrad_mt(int idx) { return idx & 0xff; }
__device__ __forceinline__ int wgrad_part(int idx) { return (idx >> 8) & 0xfff; }
__device__ __forceinline__ int wgrad_parts(int idx) { return (idx >> 20) & 0xfff; }
constexpr int kMaxSplitParts = 0xfff;
constexpr size_t kPartialTileBytes = (size_t)BMAX * BN * sizeof(float);

// ------------------------------------------------------------- row metadata
// row_tok[r] = token of expert row r, row_w[r] = its gate (the backward
// "dispatch" of dY is a gather through these).
__global__ void __launch_bounds__(256) row_meta_kernel(BwdParams p) {
    const int A = p.offsets[p.s.e_count];
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r < A) {
        const int f = p.perm[r];
        p.row_tok[r] = f / p.s.k;
        p.row_w[r] = p.topk_w[f];
    }
}

// One workgroup: row tiles, per-XCD task lists, cleared scoreboard.  List order
// per XCD (experts i = 0..n-1 of that list): [dH_0], [dH_1], [dXp_0, dWgu_0, dWdown_0],
// [dH_2], [dXp_1, dWgu_1, dWdown_1], ...: the consumers of expert i sit `lag` experts
// behind its producers.  All three consumer kinds read what the dH tiles wrote
// (dG|dU, and gate * h for dW_down).
template <int BM>
__global__ void __launch_bounds__(1024) bwd_prologue_kernel(BwdParams p) {
    __shared__ int32_t s_scan[kMaxExperts];
    __shared__ int32_t s_ga[kMaxExperts];
    __shared__ int32_t s_gb[kMaxExperts];
    __shared__ int32_t s_rt0[kMaxExperts];
    __shared__ int32_t s_r0[kMaxExperts];
    __shared__ int32_t s_ta[kMaxExperts];
    __shared__ int32_t s_tb[kMaxExperts];
    __shared__ int32_t s_qbase[kQueues + 1];
    __shared__ int32_t s_qlen[kQueues];
    __shared__ int32_t s_lag;
    __shared__ ListPlan s_plan;
    const int e = threadIdx.x;
    const int ec = p.s.e_count;
    const int per_dwd = p.mt_dwd * p.nt_dwd, per_dwgu = p.mt_dwgu * p.nt_dwgu;
    int cnt = 0, nt = 0;
    if (e < ec) {
        cnt = p.offsets[e + 1] - p.offsets[e];
        nt = (cnt + BM - 1) / BM;
    }
    // Section 6.3 prices bitwise reproducibility in the backward pass: the order of the
    // weight-gradient reduction is fixed.  An expert with more than split_rows rows has that
    // reduction cut at the fixed points r0 + j * split_rows (a function of the counts only) into
    // `parts` tasks per output tile; their fp32 partial tiles are added in the order of j.
    const int parts = (p.split_rows > 0 && cnt > p.split_rows) ? (cnt + p.split_rows - 1) / p.split_rows : 1;
    __shared__ int32_t s_parts[kMaxExperts];
    s_parts[e] = parts;
    s_plan.cost[e] = cnt;
    s_scan[e] = nt;
    s_ga[e] = (e < ec) ? nt * p.nct_dh : 0;
    s_gb[e] = (e < ec) ? nt * p.nct_dxp + (per_dwgu + per_dwd) * parts : 0;
    __syncthreads();
    for (int off = 1; off < kMaxExperts; off <<= 1) {
        const int32_t add = (e >= off) ? s_scan[e - off] : 0;
        __syncthreads();
        s_scan[e] += add;
        __syncthreads();
    }
    const int nrt = s_scan[kMaxExperts - 1];
    if (p.split_rows > 0) {   // slots of the split experts: output tiles, and partial tiles
        __shared__ int32_t s_st[kMaxExperts];
        __shared__ int32_t s_sp[kMaxExperts];
        const int tiles = (e < ec && parts > 1) ? per_dwgu + per_dwd : 0;
        s_st[e] = tiles;
        s_sp[e] = tiles * parts;
        __syncthreads();
        for (int off = 1; off < kMaxExperts; off <<= 1) {
            const int32_t a0 = (e >= off) ? s_st[e - off] : 0, a1 = (e >= off) ? s_sp[e - off] : 0;
            __syncthreads();
            s_st[e] += a0;
            s_sp[e] += a1;
            __syncthreads();
        }
        if (e < ec) {
            p.split_tile0[e] = s_st[e] - tiles;
            p.split_base[e] = s_sp[e] - tiles * parts;
            for (int i = 0; i < tiles; ++i) p.split_cnt[s_st[e] - tiles + i] = 0;
        }
    }
    plan_lists(s_plan, ec);
    if (e < kQueues) {   // length of list e
        int len = 0;
        for (int j = 0; j < s_plan.size[e]; ++j) {
            const int x = s_plan.member[e][j];
            len += s_ga[x] + s_gb[x];
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
        s_lag = queue_lag(nrt * p.nct_dh, ec);
    }
    __syncthreads();
    if (e < ec) {
        const int rt0 = s_scan[e] - nt;
        s_r0[e] = p.offsets[e];
        for (int i = 0; i < nt; ++i) p.flag_rt[rt0 + i] = 0;
        p.flag_e[e] = 0;
        int pa, pb;
        queue_positions(s_plan, s_ga, s_gb, e, s_lag, pa, pb);
        s_rt0[e] = rt0;
        s_ta[e] = s_qbase[s_plan.list_of[e]] + pa;
        s_tb[e] = s_qbase[s_plan.list_of[e]] + pb;
    }
    __syncthreads();
    for (int x = e >> 6; x < ec; x += 16) {   // one wave writes the two blocks of an expert
        const int rt0 = s_rt0[x], lane = e & 63;
        const int parts_x = s_parts[x];
        const int n_dxp = s_gb[x] - (per_dwgu + per_dwd) * parts_x;
        Task* ta = p.tasks + s_ta[x];
        Task* tb = p.tasks + s_tb[x];
        const int r0 = s_r0[x], rows_x = s_plan.cost[x];
        // every block in the grouped order of block_pos(): row-tile GEMMs over (row tile, column
        // tile), weight-gradient GEMMs over (output row tile, output column tile)
        const int nt_x = (rows_x + BM - 1) / BM;
        for_each_tile(lane, nt_x, p.nct_dh, [&](int j, int ct) {
            ta[block_pos<true>(j, ct, nt_x, p.nct_dh)] =
                Task{rt0 + j, task_code(B_DH, x, ct), r0 + j * BM, min(BM, rows_x - j * BM)};
        });
        for_each_tile(lane, nt_x, p.nct_dxp, [&](int j, int ct) {
            tb[block_pos<true>(j, ct, nt_x, p.nct_dxp)] =
                Task{rt0 + j, task_code(B_DXP, x, ct), r0 + j * BM, min(BM, rows_x - j * BM)};
        });
        // weight-gradient tasks: idx = output row tile | part << 8 | parts << 20; row0 / rows = the part's rows
        for_each_tile(lane, p.mt_dwgu, p.nt_dwgu, [&](int mt, int nt) {
            for (int j = 0; j < parts_x; ++j) {
                const int first = (parts_x > 1) ? j * p.split_rows : 0;
                const int len = (parts_x > 1) ? min(p.split_rows, rows_x - first) : rows_x;
                tb[n_dxp + block_pos<false>(mt, nt, p.mt_dwgu, p.nt_dwgu) * parts_x + j] =
                    Task{wgrad_idx(mt, j, parts_x), task_code(B_DWGU, x, nt), r0 + first, len};
            }
        });
        for_each_tile(lane, p.mt_dwd, p.nt_dwd, [&](int mt, int nt) {
            for (int j = 0; j < parts_x; ++j) {
                const int first = (parts_x > 1) ? j * p.split_rows : 0;
                const int len = (parts_x > 1) ? min(p.split_rows, rows_x - first) : rows_x;
                tb[n_dxp + per_dwgu * parts_x + block_pos<false>(mt, nt, p.mt_dwd, p.nt_dwd) * parts_x + j] =
                    Task{wgrad_idx(mt, j, parts_x), task_code(B_DWD, x, nt), r0 + first, len};
            }
        });
    }
    if (e < CTRL_WORDS) {
        int v = 0;
        if (e == CTRL_NRT) v = nrt;
        if (e == CTRL_NTAIL) v = (p.s.T + kDxTokens - 1) / kDxTokens;
        if (e == CTRL_NWAIT) v = p.workers;
        if (e >= CTRL_QLEN && e < CTRL_QLEN + kQueues) v = s_qbase[e - CTRL_QLEN + 1] - s_qbase[e - CTRL_QLEN];
        if (e >= CTRL_QBASE && e < CTRL_QBASE + kQueues) v = s_qbase[e - CTRL_QBASE];
        p.ctrl[e] = v;
    }
}

// ------------------------------------------------------------- phase 0: dH
// dH = dO W_down^T for one row tile and 256 columns of I, dO = gate * dY gathered on the fly:
// the GEMM runs on the raw dY rows and the gate multiplies the fp32 accumulators, because the
// unscaled product is also what dtopk_w needs: <dY[t], o[r]> = sum_i (dY[t] W_down^T)[i] h[r][i].
// Epilogue: SwiGLU backward with the stashed G, U -> dG|dU; gate * h -> hw (dW_down's operand);
// the partial dot products.
template <class Hook>
__device__ __forceinline__ void dh_task(const BwdParams& p, const RowTile rt, int ct, char* smem,
                                        Hook after_mainloop) {
    const int d = p.s.d, I = p.s.I;
    const int n0 = ct * BN;
    const Lane ln;
    FragAddr fa;
    frag_addresses<false, false>(fa, lds_addr(smem), ln);
    KcLoader lb, la;
    lb.n = KcLoader::blocks_for(ln, rt.rows);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = rt.row0 + min(KcGeom::row(ln, i), rt.rows - 1);   // rows past the tile alias its last row
        lb.p[i] = p.dy + ((size_t)p.row_tok[row] * d + KcGeom::chunk(ln, i) * 8) * 2;
        const int col = min(n0 + KcGeom::row(ln, i), I - 1);              // columns past I alias the last one
        la.p[i] = p.w_down + (((size_t)rt.expert * I + col) * d + KcGeom::chunk(ln, i) * 8) * 2;
    }
    f32x16_t acc[4][2];
    mma_tile<false, false>(lb, la, d / BK, rt.rows, smem, fa, acc);
    after_mainloop();
    // epilogue, one row fragment (32 rows x the wave's 64 columns) at a time: the three outputs
    // pass through three 4 KB pieces of the wave's LDS region and leave as 8-byte write-through
    // stores, 16 neighbouring lanes on one 128-byte row segment
    const Lane le;
    const int lane = le.l, wn = le.wn;
    const bool want_dots = p.dtopk_w != nullptr;
    WaveRepack<8> rg(smem, le), ru(smem + 4096, le), rh(smem + 8192, le);
    const int rows_w = rt.rows - 128 * le.wm;      // rows of the tile inside this wave's 128
    const int ocol = n0 + 64 * wn + 4 * rg.get8_piece();   // first of this lane's 4 columns on the way out
#pragma unroll
    for (int tf = 0; tf < 4; ++tf) {
        const int m = acc_row(le, tf);
        const float gt = p.row_w[rt.row0 + min(m, rt.rows - 1)];
        float dot = 0.f;
        const size_t row = (size_t)(rt.row0 + min(m, rt.rows - 1));
#pragma unroll
        for (int af = 0; af < 2; ++af)
#pragma unroll
            for (int vg = 0; vg < 2; ++vg) {
                const int col = min(n0 + acc_col8(le, af, vg), I - 8);   // pieces past I alias a valid one, never stored
                const size_t base = (row * 2 * I + col) * 2;
                const u32x4_t gv = *(const u32x4_t*)(p.gu + base);
                const u32x4_t uv = *(const u32x4_t*)(p.gu + base + (size_t)I * 2);
                // the h that GEMM2 multiplied (bf16), not silu(g) * u of the rounded g, u
                const u32x4_t hv = *(const u32x4_t*)(p.h + (row * I + col) * 2);
                const bool live = m < rt.rows && n0 + acc_col8(le, af, vg) < I;
                float dg[8], du[8], hs[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float g = (e & 1) ? bf16_hi(gv[e >> 1]) : bf16_lo(gv[e >> 1]);
                    const float u = (e & 1) ? bf16_hi(uv[e >> 1]) : bf16_lo(uv[e >> 1]);
                    const float hh = (e & 1) ? bf16_hi(hv[e >> 1]) : bf16_lo(hv[e >> 1]);
                    const float raw = acc[tf][af][8 * vg + e];
                    const float dh = gt * raw;
                    const float sg = sigmoid_f(g);
                    if (live) dot += raw * hh;
                    hs[e] = gt * hh;
                    du[e] = dh * (g * sg);
                    dg[e] = dh * u * (sg * (1.f + g * (1.f - sg)));
                }
                u32x4_t dgp, dup, hwp;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    dgp[q] = pack_bf16x2(dg[2 * q], dg[2 * q + 1]);
                    dup[q] = pack_bf16x2(du[2 * q], du[2 * q + 1]);
                    hwp[q] = pack_bf16x2(hs[2 * q], hs[2 * q + 1]);
                }
                const int pi = 4 * af + 2 * vg + le.hf;
                rg.put(le.l31, pi, dgp);
                ru.put(le.l31, pi, dup);
                rh.put(le.l31, pi, hwp);
            }
        // consumed by dXp / dW tiles on any XCD
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = 32 * tf + rg.get8_row(j);
            if (r < rows_w && ocol < I) {
                const size_t orow = (size_t)(rt.row0 + 128 * le.wm + r);
                store_wt8(p.dgu + (orow * 2 * I + ocol) * 2, rg.get8(j));
                store_wt8(p.dgu + (orow * 2 * I + I + ocol) * 2, ru.get8(j));
                store_wt8(p.hw + (orow * I + ocol) * 2, rh.get8(j));
            }
        }
        if (want_dots) {
            // the two lane halves hold the wave's 64 columns of row m between them
            dot += __shfl_xor(dot, 32);
            if (lane < 32 && m < rt.rows)
                p.dots[(size_t)(ct * 4 + wn) * ((size_t)p.s.T * p.s.k) + rt.row0 + m] = dot;
        }
    }
}

// ------------------------------------------------------------- phase 2: dXp
// dXp = dG W_gate^T + dU W_up^T for one row tile and 256 columns of d: one GEMM over k = 2I whose
// column operand switches from the rows of W_gate to the rows of W_up half way.
template <class Hook>
__device__ __forceinline__ void dxp_task(const BwdParams& p, const RowTile rt, int ct, char* smem,
                                        Hook after_mainloop) {
    const int d = p.s.d, I = p.s.I;
    const int n0 = ct * BN;
    const Lane ln;
    FragAddr fa;
    frag_addresses<false, false>(fa, lds_addr(smem), ln);
    KcLoader lb;
    KcSplitLoader la;
    lb.n = KcLoader::blocks_for(ln, rt.rows);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = rt.row0 + min(KcGeom::row(ln, i), rt.rows - 1);
        lb.p[i] = p.dgu + ((size_t)row * 2 * I + KcGeom::chunk(ln, i) * 8) * 2;
        const int c = min(n0 + KcGeom::row(ln, i), d - 1);
        la.p[i] = p.w_gate + (((size_t)rt.expert * d + c) * I + KcGeom::chunk(ln, i) * 8) * 2;
    }
    la.left = I / BK;
    la.delta = (long long)(p.w_up - p.w_gate) - (long long)I * 2;
    f32x16_t acc[4][2];
    mma_tile<false, false>(lb, la, 2 * I / BK, rt.rows, smem, fa, acc);
    after_mainloop();
    char* obase = p.dxp + ((size_t)rt.row0 * d + n0) * 2;
    store_subtile_bf16(acc, smem, rt.rows, d - n0, [&](int row, int col, u32x4_t v) {
        store_stream16(obase + ((size_t)row * d + col) * 2, v);
    });
}

// Weight gradients added to an fp32 gradient buffer (a training loop's main gradient) instead
// of written as bf16: q[0..8) += the lane's 8 consecutive columns 8 vg .. 8 vg + 7.
// Every element belongs to exactly one tile, so the read-modify-write needs no atomic and the
// sum does not depend on the schedule.
__device__ __forceinline__ void accumulate8(float* q, const f32x16_t& a, int vg) {
    typedef __attribute__((ext_vector_type(4))) float f32x4_t;
    f32x4_t lo = ((const f32x4_t*)q)[0], hi = ((const f32x4_t*)q)[1];
    lo += f32x4_t{a[8 * vg], a[8 * vg + 1], a[8 * vg + 2], a[8 * vg + 3]};
    hi += f32x4_t{a[8 * vg + 4], a[8 * vg + 5], a[8 * vg + 6], a[8 * vg + 7]};
    __builtin_nontemporal_store(lo, (f32x4_t*)q);
    __builtin_nontemporal_store(hi, (f32x4_t*)q + 1);
}

// ------------------------------------------------------------- split weight-gradient reductions
// One part of a split reduction ends here: the fp32 accumulators go to the part's slot in
// accumulator layout (every store instruction writes 512 consecutive bytes), the tile's
// counter is advanced, and the workgroup that finds all other parts already counted adds the
// `parts` partial tiles in the order of the part index, starting from zero: the sum does not
// depend on which workgroup adds, nor on the order in which the parts were computed.
// Returns whether acc now holds the complete sum (the caller then stores the tile).
__device__ __forceinline__ bool finish_part(const BwdParams& p, int e, int tile, int part, int parts,
                                            f32x16_t (&acc)[4][2], int* s_flag) {
    if (parts <= 1) return true;
    const Lane ln;
    // 8-byte write-through stores: the two halves of a register quad go to separate 512-byte runs,
    // so that every store instruction of a wave writes consecutive bytes
    const size_t lane_off = (size_t)ln.w * 32768 + (size_t)ln.l * 8;
    char* slots = p.split_buf + ((size_t)p.split_base[e] + (size_t)tile * parts) * kPartialTileBytes;
    char* mine = slots + (size_t)part * kPartialTileBytes + lane_off;
#pragma unroll
    for (int tf = 0; tf < 4; ++tf)
#pragma unroll
        for (int af = 0; af < 2; ++af)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x2_t lo = {acc[tf][af][4 * q], acc[tf][af][4 * q + 1]};
                const f32x2_t hi = {acc[tf][af][4 * q + 2], acc[tf][af][4 * q + 3]};
                char* dst = mine + ((tf * 2 + af) * 4 + q) * 1024;
                store_wt8(dst, __builtin_bit_cast(u32x2_t, lo));
                store_wt8(dst + 512, __builtin_bit_cast(u32x2_t, hi));
            }
    wait_stores();
    __syncthreads();   // the partial tile of every wave has reached memory
    if (threadIdx.x == 0) {
        const int before = __hip_atomic_fetch_add(p.split_cnt + p.split_tile0[e] + tile, 1, __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_AGENT);
        if (before == parts - 1) fence_acquire();
        *s_flag = before;
    }
    __syncthreads();
    if (*s_flag != parts - 1) return false;
#pragma unroll
    for (int tf = 0; tf < 4; ++tf)
#pragma unroll
        for (int af = 0; af < 2; ++af)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tf][af][v] = 0.f;
    for (int j = 0; j < parts; ++j) {
        const char* src = slots + (size_t)j * kPartialTileBytes + lane_off;
#pragma unroll
        for (int tf = 0; tf < 4; ++tf)
#pragma unroll
            for (int af = 0; af < 2; ++af)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const char* blk = src + ((tf * 2 + af) * 4 + q) * 1024;
                    const f32x2_t lo = *(const f32x2_t*)blk, hi = *(const f32x2_t*)(blk + 512);
                    acc[tf][af][4 * q] += lo[0];
                    acc[tf][af][4 * q + 1] += lo[1];
                    acc[tf][af][4 * q + 2] += hi[0];
                    acc[tf][af][4 * q + 3] += hi[1];
                }
    }
    return true;
}

// ------------------------------------------------------------- phase 1: dW_down
// dW_down[e][i][c] = sum over the expert's rows r (ascending) of (gate_r h[r][i]) * dY[tok_r][c].
// Output tile: 256 rows of I by 256 columns of d; both operands have k = r as their memory row.
template <bool ACC, bool SPLIT, class Hook>
__device__ __forceinline__ void dwd_task(const BwdParams& p, int e, int idx, int nt, int r0, int cnt,
                                         char* smem, int* s_flag, Hook after_mainloop) {
    const int mt = wgrad_mt(idx);
    const int d = p.s.d, I = p.s.I;
    const int m0 = mt * BMAX, n0 = nt * BN;
    const Lane ln;
    FragAddr fa;
    frag_addresses<true, true>(fa, lds_addr(smem), ln);
    KsTailLoader lb;
    KsGatherLoader la;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        lb.p[i] = p.hw + (((size_t)r0 + KsGeom::krow(ln, i)) * I + min(m0 + KsGeom::chunk(ln, i) * 8, I - 8)) * 2;
        la.coloff[i] = (uint32_t)min(n0 + KsGeom::chunk(ln, i) * 8, d - 8) * 2u;
    }
    lb.k0 = KsGeom::krow(ln, 0);
    lb.ld_bytes = (long long)I * 2;
    lb.K = cnt;
    la.init(ln, p.dy, (long long)d * 2, p.row_tok + r0, cnt);
    f32x16_t acc[4][2];
    mma_tile<true, true>(lb, la, (cnt + BK - 1) / BK, min(BMAX, I - m0), smem, fa, acc);
    after_mainloop();
    if (SPLIT && !finish_part(p, e, p.mt_dwgu * p.nt_dwgu + mt * p.nt_dwd + nt, wgrad_part(idx), wgrad_parts(idx), acc, s_flag)) return;
    if (ACC) {
        const Lane le;
#pragma unroll
        for (int tf = 0; tf < 4; ++tf) {
            const int m = m0 + acc_row(le, tf);
            if (m < I && cnt > 0) {
#pragma unroll
                for (int af = 0; af < 2; ++af)
#pragma unroll
                    for (int vg = 0; vg < 2; ++vg) {
                        const int col = n0 + acc_col8(le, af, vg);
                        if (col < d) accumulate8((float*)p.dw_down + ((size_t)e * I + m) * d + col, acc[tf][af], vg);
                    }
            }
        }
    } else {
        char* obase = p.dw_down + (((size_t)e * I + m0) * d + n0) * 2;
        store_subtile_bf16(acc, smem, I - m0, d - n0, [&](int row, int col, u32x4_t v) {
            store_stream16(obase + ((size_t)row * d + col) * 2, v);
        });
    }
}

// ------------------------------------------------------------- phase 3: dW_gate, dW_up
// dW_gate[e][c][i] = sum_r x[tok(r)][c] * dG[r][i]; dW_up likewise with dU.
// Output tile: 256 rows of d by 128 columns of I, for both matrices at once: column fragment 0
// of a wave holds dG columns, fragment 1 the same dU columns.
template <bool ACC, bool SPLIT, class Hook>
__device__ __forceinline__ void dwgu_task(const BwdParams& p, int e, int idx, int nt, int r0, int cnt,
                                          char* smem, int* s_flag, Hook after_mainloop) {
    const int mt = wgrad_mt(idx);
    const int d = p.s.d, I = p.s.I;
    const int m0 = mt * BMAX, n0i = nt * (BN / 2);
    const Lane ln;
    FragAddr fa;
    frag_addresses<true, true>(fa, lds_addr(smem), ln);
    KsGatherLoader lb;
    KsTailLoader la;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        lb.coloff[i] = (uint32_t)min(m0 + KsGeom::chunk(ln, i) * 8, d - 8) * 2u;
        const int c = KsGeom::chunk(ln, i);
        const int icol = min(n0i + 32 * (c >> 3) + 8 * (c & 3), I - 8);
        la.p[i] = p.dgu + (((size_t)r0 + KsGeom::krow(ln, i)) * 2 * I + (((c >> 2) & 1) ? I : 0) + icol) * 2;
    }
    la.k0 = KsGeom::krow(ln, 0);
    la.ld_bytes = (long long)2 * I * 2;
    la.K = cnt;
    lb.init(ln, p.x, (long long)d * 2, p.row_tok + r0, cnt);
    f32x16_t acc[4][2];
    mma_tile<true, true>(lb, la, (cnt + BK - 1) / BK, min(BMAX, d - m0), smem, fa, acc);
    after_mainloop();
    if (SPLIT && !finish_part(p, e, mt * p.nt_dwgu + nt, wgrad_part(idx), wgrad_parts(idx), acc, s_flag)) return;
    if (ACC) {
        const Lane le;
#pragma unroll
        for (int tf = 0; tf < 4; ++tf) {
            const int m = m0 + acc_row(le, tf);
            if (m < d && cnt > 0) {
#pragma unroll
                for (int af = 0; af < 2; ++af)
#pragma unroll
                    for (int vg = 0; vg < 2; ++vg) {
                        const int icol = n0i + 32 * le.wn + 16 * vg + 8 * le.hf;
                        if (icol < I)
                            accumulate8((float*)(af ? p.dw_up : p.dw_gate) + ((size_t)e * d + m) * I + icol, acc[tf][af], vg);
                    }
            }
        }
    } else {
        // the wave's 64 columns are 32 columns of dW_gate and the same 32 of dW_up: pieces 0..3 | 4..7
        const size_t ebase = ((size_t)e * d + m0) * I;
        store_subtile_bf16(acc, smem, d - m0, BN, [&](int row, int col, u32x4_t v) {
            const int pc = (col >> 3) & 7;
            const int icol = n0i + 32 * (col >> 6) + 8 * (pc & 3);
            if (icol < I) store_stream16(((pc & 4) ? p.dw_up : p.dw_gate) + (ebase + (size_t)row * I + icol) * 2, v);
        });
    }
}

// ------------------------------------------------------------- phase 4: dX, dtopk_w
// KM = compile-time bound on k (8 or kMaxTopK).
template <int NW, int KM = kMaxTopK>
__device__ __forceinline__ void dx_task(const BwdParams& p, int block) {
    const int d = p.s.d, k = p.s.k, T = p.s.T;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool want_dots = p.dtopk_w != nullptr;
    for (int tt = wave; tt < kDxTokens; tt += NW) {
        const int t = block * kDxTokens + tt;
        if (t >= T) break;
        int rows[KM];
#pragma unroll
        for (int j = 0; j < KM; ++j) rows[j] = (j < k) ? p.inv_perm[(size_t)t * k + j] : -1;
        // two 16-byte column pieces per lane and round, as in the forward combine: all 2k row
        // loads are issued before the first is used
        for (int c0 = lane * 8; c0 < d; c0 += 2 * 64 * 8) {
            const int c1 = c0 + 64 * 8;
            const bool two = c1 < d;
            u32x4_t v0[KM], v1[KM];
#pragma unroll
            for (int j = 0; j < KM; ++j) {
                v0[j] = zero4();
                v1[j] = zero4();
                if (j < k && rows[j] >= 0) {
                    const char* src = p.dxp + (size_t)rows[j] * d * 2;
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
                        a0[2 * q] += bf16_lo(v0[j][q]);
                        a0[2 * q + 1] += bf16_hi(v0[j][q]);
                        a1[2 * q] += bf16_lo(v1[j][q]);
                        a1[2 * q + 1] += bf16_hi(v1[j][q]);
                    }
                }
            }
            u32x4_t o0, o1;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                o0[q] = pack_bf16x2(a0[2 * q], a0[2 * q + 1]);
                o1[q] = pack_bf16x2(a1[2 * q], a1[2 * q + 1]);
            }
            store_stream16(p.dx + ((size_t)t * d + c0) * 2, o0);
            if (two) store_stream16(p.dx + ((size_t)t * d + c1) * 2, o1);
        }
        if (want_dots && lane < k) {
            // dtopk_w[t][j] = <dY[t], o[row]>: the partial sums of the row's dH column tiles (four
            // per tile, one per wave column), added in column order; 0 for a slot whose expert is not local
            const int r = p.inv_perm[(size_t)t * k + lane];
            float s = 0.f;
            if (r >= 0)
                for (int ct = 0; ct < p.n_dots; ++ct) s += p.dots[(size_t)ct * ((size_t)T * k) + r];
            p.dtopk_w[(size_t)t * k + lane] = s;
        }
    }
}


// ------------------------------------------------------------- worker loop
// ACC: the weight gradients are added to fp32 buffers (moe_opts_t.dw_accumulate).
// SPLIT: weight-gradient tasks may be parts of a split reduction (moe_opts_t.dw_split_rows > 0); the
// default kernel carries none of that code.
template <bool ACC, bool SPLIT>
__device__ __forceinline__ void bwd_worker_body(const BwdParams& p, int phase, char* smem) {
    __shared__ int s_task;
    __shared__ int s_ok;
    int* ctrl = p.ctrl;
    const int pass = phase < 0 ? kPersistentPass : 1 + phase;
    const int home = xcc_id();
    const bool use_lists = phase != B_DX;
    const bool use_tail = phase == -1 || phase == B_DX;
    // this launch runs dXp tiles: its workers publish their rows once, when they run out of GEMM work
    const bool publishes = phase == -1 || phase == B_DXP;
    bool arrived = false;
    unsigned exhausted = 0;
    int seen_e = -1;   // the expert whose dH tiles this worker last found complete
    if (threadIdx.x == 0) {
        if (phase == -1) worker_started(ctrl, home);
        s_task = fetch_task(ctrl, pass, home, exhausted, use_lists, use_tail);
    }
    __syncthreads();
    for (;;) {
        const int id = s_task;
        if (id == kFetchDone) break;
        // issued behind the main loop of the task (see the forward worker)
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
                // staged launch: another phase's task
            } else if (type == B_DH) {
                const RowTile rt = task_row_tile(task);
                dh_task(p, rt, ct, smem, issue);
                wait_stores();
                __syncthreads();   // the write-through dG|dU stores of every wave have completed
                if (threadIdx.x == 0) {
                    add_relaxed(p.flag_rt + task.idx, 1);
                    add_relaxed(p.flag_e + rt.expert, 1);
                }
            } else if (type == B_DXP) {
                if (threadIdx.x == 0) s_ok = wait_ge(p.flag_rt + task.idx, p.nct_dh, ctrl, p.spin_ticks);
                __syncthreads();
                if (s_ok) {
                    const RowTile rt = task_row_tile(task);
                    dxp_task(p, rt, ct, smem, issue);
                }
            } else {
                // weight-gradient tiles read what ALL dH tiles of the expert wrote (dG|dU, gate * h):
                // its row tiles times the dH column tiles
                const int e = task_expert(task);
                // rows of the whole expert (a part of a split reduction carries only its own share)
                const int rows_e = SPLIT ? p.offsets[e + 1] - p.offsets[e] : task.rows;
                const int need = (rows_e + p.bm - 1) / p.bm * p.nct_dh;
                // a worker takes several of an expert's 72 output tiles in a row: the expert it has
                // already seen complete (and acquired) needs no second look at the flag
                if (e != seen_e) {
                    if (threadIdx.x == 0) s_ok = wait_ge(p.flag_e + e, need, ctrl, p.spin_ticks);
                    __syncthreads();
                    if (s_ok) seen_e = e;
                }
                if (e == seen_e) {
                    if (type == B_DWD) dwd_task<ACC, SPLIT>(p, e, task.idx, ct, task.row0, task.rows, smem, &s_ok, issue);
                    else dwgu_task<ACC, SPLIT>(p, e, task.idx, ct, task.row0, task.rows, smem, &s_ok, issue);
                }
            }
        } else {
            if (publishes && !arrived) {
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
            if (s_ok) dx_task<8>(p, -1 - id);
        }
        issue();           // tasks without a main loop (tail, skipped, given up)
        __syncthreads();
        if (threadIdx.x == 0) s_task = fetch_finish(pf, ctrl, pass, home, exhausted, use_lists, use_tail);
        __syncthreads();
    }
    if (phase == -2) return;   // GEMM tasks only: the kernel boundary publishes the rows
    if (publishes && !arrived) {
        wait_stores();
        __syncthreads();
        if (threadIdx.x == 0) {
            if (phase < 0) worker_arrived(ctrl, home, ctrl[CTRL_NWAIT], p.spin_ticks);
            else add_release(ctrl + CTRL_DONE, 1);
        }
    }
}

#define UNIEP_BWD_WORKER(name, ACC, SPLIT)                                                         \
    __global__ void __launch_bounds__(kMmaThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))       \
    name(BwdParams p, int phase) {                                                                  \
        extern __shared__ __attribute__((aligned(16))) char smem[];                                 \
        bwd_worker_body<ACC, SPLIT>(p, phase, smem);                                                \
    }
UNIEP_BWD_WORKER(bwd_worker_kernel, false, false)
UNIEP_BWD_WORKER(bwd_worker_acc_kernel, true, false)
UNIEP_BWD_WORKER(bwd_worker_split_kernel, false, true)
UNIEP_BWD_WORKER(bwd_worker_acc_split_kernel, true, true)
#undef UNIEP_BWD_WORKER
typedef void (*BwdWorkerFn)(BwdParams, int);
static BwdWorkerFn bwd_worker_fn(bool acc, bool split) {
    return split ? (acc ? bwd_worker_acc_split_kernel : bwd_worker_split_kernel)
                 : (acc ? bwd_worker_acc_kernel : bwd_worker_kernel);
}

// dX (and dtopk_w) as a plain grid launch behind the GEMM MegaKernel, one workgroup per block
// of kDxTokens tokens: no scoreboard wait, no task cursor, no LDS.
template <int NW, int KM>
__global__ void __launch_bounds__(64 * NW) bwd_tail_kernel(BwdParams p) {
    dx_task<NW, KM>(p, blockIdx.x);
}

// ------------------------------------------------------------------ host side

struct BwdLayout {
    size_t ctrl, flag_rt, flag_e, tasks, row_tok, row_w, dgu, dxp, hw, dots, split_base, split_tile0, split_cnt, split_buf, total;
    int max_rt, nct_dh, nct_dxp, mt_dwd, nt_dwd, mt_dwgu, nt_dwgu;
};

static BwdLayout bwd_layout(const moe_shape_t& s, int split_rows) {
    BwdLayout L;
    const size_t A_cap = (size_t)s.T * s.k;
    L.max_rt = (int)((A_cap + 127) / 128) + s.e_count;   // 128-row tiles need the most entries
    L.nct_dh = (s.I + BN - 1) / BN;
    L.nct_dxp = (s.d + BN - 1) / BN;
    L.mt_dwd = (s.I + BMAX - 1) / BMAX;
    L.nt_dwd = (s.d + BN - 1) / BN;
    L.mt_dwgu = (s.d + BMAX - 1) / BMAX;
    L.nt_dwgu = (s.I + BN / 2 - 1) / (BN / 2);
    // split reductions: at most A_cap / split_rows experts have more than split_rows rows, and their
    // parts number at most A_cap / split_rows more than that
    const size_t tiles_pe = (size_t)L.mt_dwd * L.nt_dwd + (size_t)L.mt_dwgu * L.nt_dwgu;
    const size_t split_experts = split_rows > 0 ? std::min(A_cap / split_rows, (size_t)s.e_count) : 0;
    const size_t split_parts = split_rows > 0 ? A_cap / split_rows + split_experts : 0;
    const size_t max_tasks = (size_t)L.max_rt * (L.nct_dh + L.nct_dxp) +
                             (size_t)s.e_count * tiles_pe + split_parts * tiles_pe +
                             (s.T + kDxTokens - 1) / kDxTokens;
    size_t off = 0;
    L.ctrl = off;    off = align_up(off + CTRL_WORDS * sizeof(int), 256);
    L.flag_rt = off; off = align_up(off + (size_t)L.max_rt * sizeof(int), 256);
    L.flag_e = off;  off = align_up(off + (size_t)s.e_count * sizeof(int), 256);
    L.tasks = off;   off = align_up(off + max_tasks * sizeof(Task), 256);
    L.row_tok = off; off = align_up(off + A_cap * sizeof(int32_t), 256);
    L.row_w = off;   off = align_up(off + A_cap * sizeof(float), 256);
    L.dgu = off;     off = align_up(off + A_cap * 2 * s.I * 2, 256);
    L.dxp = off;     off = align_up(off + A_cap * s.d * 2, 256);
    L.hw = off;      off = align_up(off + A_cap * s.I * 2, 256);
    L.dots = off;    off = align_up(off + (size_t)4 * L.nct_dh * A_cap * sizeof(float), 256);
    L.split_base = off;  off = align_up(off + (size_t)s.e_count * sizeof(int32_t), 256);
    L.split_tile0 = off; off = align_up(off + (size_t)s.e_count * sizeof(int32_t), 256);
    L.split_cnt = off;   off = align_up(off + split_experts * tiles_pe * sizeof(int32_t), 256);
    L.split_buf = off;   off = align_up(off + split_parts * tiles_pe * kPartialTileBytes, 256);
    L.total = off;
    return L;
}

size_t bwd_workspace_bytes(const moe_shape_t& s, int split_rows) { return bwd_layout(s, split_rows).total; }
// parts per expert and output row tiles per expert must fit the fields of a weight-gradient task
bool bwd_split_ok(const moe_shape_t& s, int split_rows) {
    if (split_rows == 0) return true;
    const BwdLayout L = bwd_layout(s, split_rows);
    return (size_t)s.T * s.k / split_rows + 1 < (size_t)kMaxSplitParts && L.mt_dwd < 256 && L.mt_dwgu < 256;
}

static std::mutex g_bwd_workers_mu;
static int g_bwd_workers[kMaxDevices * 4];   // per device and kernel variant; filled on first use under the lock, constant afterwards

static int bwd_resident_workers(bool acc, bool split, int* out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOE_ERR_HIP;
    const int slot = dev * 4 + (acc ? 1 : 0) + (split ? 2 : 0);
    std::lock_guard<std::mutex> lock(g_bwd_workers_mu);
    if (g_bwd_workers[slot] == 0) {
        const BwdWorkerFn fn = bwd_worker_fn(acc, split);
        if (hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, kMmaSmem) != hipSuccess)
            return MOE_ERR_HIP;
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kMmaThreads, kMmaSmem) != hipSuccess)
            return MOE_ERR_HIP;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return MOE_ERR_HIP;
        if (per_cu < 1 || cus < 1) return MOE_ERR_HIP;
        g_bwd_workers[slot] = per_cu * cus;
    }
    *out = g_bwd_workers[slot];
    return MOE_OK;
}

static void launch_worker(bool acc, bool split, const BwdParams& p, int workers, int phase, hipStream_t st) {
    hipLaunchKernelGGL(bwd_worker_fn(acc, split), dim3(workers), dim3(kMmaThreads), kMmaSmem, st, p, phase);
}

template <int BM>
static int bwd_launch_bm(BwdParams& p, const moe_opts_t& opts, hipStream_t st) {
    const bool acc = opts.dw_accumulate != 0, split = opts.dw_split_rows > 0;
    int resident = 0;
    int rc = bwd_resident_workers(acc, split, &resident);
    if (rc != MOE_OK) return rc;
    const int workers = opts.workers > 0 ? min(opts.workers, resident) : resident;
    p.workers = workers;
    p.bm = BM;
    const int A_cap = p.s.T * p.s.k;
    if (A_cap > 0)
        hipLaunchKernelGGL(row_meta_kernel, dim3((A_cap + 255) / 256), dim3(256), 0, st, p);
    hipLaunchKernelGGL(bwd_prologue_kernel<BM>, dim3(1), dim3(1024), 0, st, p);
    if (opts.schedule == 2) {
        for (int phase = 0; phase < 5; ++phase) launch_worker(acc, split, p, workers, phase, st);
    } else if (opts.schedule != 1) {   // 0 (default) and 3: GEMM MegaKernel, then the tail tasks
        launch_worker(acc, split, p, workers, -2, st);
        const int n_tail = (p.s.T + kDxTokens - 1) / kDxTokens;
        if (n_tail > 0 && !opts.skip_tail) {
            if (p.s.k <= 8)
                hipLaunchKernelGGL((bwd_tail_kernel<8, 8>), dim3(n_tail), dim3(kMmaThreads), 0, st, p);
            else
                hipLaunchKernelGGL((bwd_tail_kernel<8, kMaxTopK>), dim3(n_tail), dim3(kMmaThreads), 0, st, p);
        }
    } else {
        launch_worker(acc, split, p, workers, -1, st);
    }
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int bwd_launch(const moe_shape_t& s, const void* dy, const void* x, const void* w_gate,
               const void* w_up, const void* w_down, const moe_routing_t& r, const char* gu,
               const char* h, const char* o, void* dx, void* dw_gate, void* dw_up, void* dw_down,
               float* dtopk_w, char* ws, const moe_opts_t& opts, int nw, hipStream_t st) {
    const BwdLayout L = bwd_layout(s, opts.dw_split_rows);
    BwdParams p;
    p.s = s;
    p.dy = (const char*)dy;
    p.x = (const char*)x;
    p.w_gate = (const char*)w_gate;
    p.w_up = (const char*)w_up;
    p.w_down = (const char*)w_down;
    p.topk_w = r.topk_w;
    p.offsets = r.offsets;
    p.perm = r.perm;
    p.inv_perm = r.inv_perm;
    p.gu = gu;
    p.h = h;
    p.o = o;
    p.dx = (char*)dx;
    p.dw_gate = (char*)dw_gate;
    p.dw_up = (char*)dw_up;
    p.dw_down = (char*)dw_down;
    p.dtopk_w = dtopk_w;
    p.ctrl = (int*)(ws + L.ctrl);
    p.flag_rt = (int*)(ws + L.flag_rt);
    p.flag_e = (int*)(ws + L.flag_e);
    p.tasks = (Task*)(ws + L.tasks);
    p.row_tok = (int32_t*)(ws + L.row_tok);
    p.row_w = (float*)(ws + L.row_w);
    p.dgu = ws + L.dgu;
    p.dxp = ws + L.dxp;
    p.hw = ws + L.hw;
    p.dots = (float*)(ws + L.dots);
    p.split_rows = opts.dw_split_rows;
    p.split_base = (int32_t*)(ws + L.split_base);
    p.split_tile0 = (int32_t*)(ws + L.split_tile0);
    p.split_cnt = (int32_t*)(ws + L.split_cnt);
    p.split_buf = ws + L.split_buf;
    p.n_dots = 4 * L.nct_dh;
    p.nct_dh = L.nct_dh;
    p.nct_dxp = L.nct_dxp;
    p.mt_dwd = L.mt_dwd;
    p.nt_dwd = L.nt_dwd;
    p.mt_dwgu = L.mt_dwgu;
    p.nt_dwgu = L.nt_dwgu;
    const int ms = opts.spin_limit_ms > 0 ? opts.spin_limit_ms : 2000;
    p.spin_ticks = (long long)ms * 100000ll;
    return nw == 4 ? bwd_launch_bm<128>(p, opts, st) : bwd_launch_bm<256>(p, opts, st);
}

}  // namespace uniep
