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
#include "tiles.hpp"

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
    float* dots; // [nct_dh][T*k] per dH column tile: sum over its columns of (dY W_down^T)[r][i] * h[r][i]
    int nct_dh, nct_dxp;        // column tiles of phase 0 (256 of I) and phase 2 (256 of d)
    int mt_dwd, nt_dwd;         // dW_down tiles per expert: ceil(I/256) x ceil(d/256)
    int mt_dwgu, nt_dwgu;       // dW_gate/up tiles per expert: ceil(d/256) x ceil(I/128)
    int workers;                // workgroups of the worker launch (the tail waits for all of them)
    long long spin_ticks;
};

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
// per XCD (experts i = 0..n-1 of that list): [dH_0, dWdown_0], [dH_1, dWdown_1],
// [dXp_0, dWgu_0], [dH_2, dWdown_2], [dXp_1, dWgu_1], ...: the consumers of
// expert i sit one expert behind its producers.
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
    s_plan.cost[e] = cnt;
    s_scan[e] = nt;
    s_ga[e] = (e < ec) ? nt * p.nct_dh + per_dwd : 0;
    s_gb[e] = (e < ec) ? nt * p.nct_dxp + per_dwgu : 0;
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
        s_lag = queue_lag(nrt * p.nct_dh + ec * per_dwd, ec);
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
        const int n_dh = s_ga[x] - per_dwd, n_dxp = s_gb[x] - per_dwgu;
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
        for_each_tile(lane, p.mt_dwd, p.nt_dwd, [&](int mt, int nt) {
            ta[n_dh + block_pos<false>(mt, nt, p.mt_dwd, p.nt_dwd)] = Task{mt, task_code(B_DWD, x, nt), r0, rows_x};
        });
        for_each_tile(lane, nt_x, p.nct_dxp, [&](int j, int ct) {
            tb[block_pos<true>(j, ct, nt_x, p.nct_dxp)] =
                Task{rt0 + j, task_code(B_DXP, x, ct), r0 + j * BM, min(BM, rows_x - j * BM)};
        });
        for_each_tile(lane, p.mt_dwgu, p.nt_dwgu, [&](int mt, int nt) {
            tb[n_dxp + block_pos<false>(mt, nt, p.mt_dwgu, p.nt_dwgu)] = Task{mt, task_code(B_DWGU, x, nt), r0, rows_x};
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
template <int NW, class Hook>
__device__ __forceinline__ void dh_task(const BwdParams& p, const RowTile rt, int ct, char* smem,
                                        Hook after_mainloop) {
    typedef Geom<NW> G;
    const int d = p.s.d, I = p.s.I;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kc = tid & 7;
    // A = dY gathered; the gate multiplies the fp32 accumulators in the epilogue, which also
    // needs the unscaled product: <dY[t], o[r]> = sum_i (dY[t] W_down^T)[i] * h[r][i].
    DirectRowLoader<false> al;
    float gate;   // of tile row wave*32 + lane%32
    {
        const int row = rt.row0 + min(wave * 32 + (lane & 31), rt.rows - 1);
        al.rp = p.dy + ((size_t)p.row_tok[row] * d + (lane >> 5) * 32) * 2;
        gate = p.row_w[row];
    }
    typedef RowLoader<G::NT, BN, false> BL;   // B rows are rows of W_down[e]: k (= d) contiguous
    BL bl;
    bl.init();
    const int n0 = ct * BN;
#pragma unroll
    for (int q = 0; q < BL::NP; ++q) {
        const int rho = BL::row(q);                       // LDS row j*32 + nb <-> column nb*8 + j
        const int c = min(n0 + (rho & 31) * 8, I - 8) + (rho >> 5);
        bl.rp[q] = p.w_down + (((size_t)rt.expert * I + c) * d + kc * 8) * 2;
    }
    f32x16_t acc[8];
    mma_mainloop_direct<NW>(al, bl, d / BK, smem, wave * 32 < rt.rows, acc);
    after_mainloop();
    // epilogue: SwiGLU backward with the saved G, U of the same rows and columns
    const int col = n0 + (lane & 31) * 8;
    const bool want_dots = p.dtopk_w != nullptr;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int m = wave * 32 + frag_row(v, lane);
        const float gt = __shfl(gate, frag_row(v, lane));
        float dot = 0.f;
        if (col < I && m < rt.rows) {
            const size_t base = ((size_t)(rt.row0 + m) * 2 * I + col) * 2;
            const u32x4_t gv = *(const u32x4_t*)(p.gu + base);
            const u32x4_t uv = *(const u32x4_t*)(p.gu + base + (size_t)I * 2);
            u32x4_t hv = zero4();   // the h that GEMM2 multiplied (bf16), not silu(g) * u of the rounded g, u
            if (want_dots) hv = *(const u32x4_t*)(p.h + ((size_t)(rt.row0 + m) * I + col) * 2);
            float dg[8], du[8];
#pragma unroll
            for (int f = 0; f < 8; ++f) {
                const float g = (f & 1) ? bf16_hi(gv[f >> 1]) : bf16_lo(gv[f >> 1]);
                const float u = (f & 1) ? bf16_hi(uv[f >> 1]) : bf16_lo(uv[f >> 1]);
                const float raw = acc[f][v];
                const float dh = gt * raw;
                const float sg = sigmoid_f(g);
                const float silu = g * sg;
                dot += raw * ((f & 1) ? bf16_hi(hv[f >> 1]) : bf16_lo(hv[f >> 1]));
                du[f] = dh * silu;
                dg[f] = dh * u * (sg * (1.f + g * (1.f - sg)));
            }
            u32x4_t dgp, dup;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                dgp[q] = pack_bf16x2(dg[2 * q], dg[2 * q + 1]);
                dup[q] = pack_bf16x2(du[2 * q], du[2 * q + 1]);
            }
            // consumed by dXp / dW_gate / dW_up tiles on any XCD
            store_wt16(p.dgu + base, dgp);
            store_wt16(p.dgu + base + (size_t)I * 2, dup);
        }
        if (want_dots) {
            // the 32 lanes of a half hold the 256 columns of row m: fixed butterfly order
#pragma unroll
            for (int off = 16; off >= 1; off >>= 1) dot += __shfl_xor(dot, off);
            if ((lane & 31) == 0 && m < rt.rows)
                p.dots[(size_t)ct * ((size_t)p.s.T * p.s.k) + rt.row0 + m] = dot;
        }
    }
}

// ------------------------------------------------------------- phase 2: dXp
template <int NW, class Hook>
__device__ __forceinline__ void dxp_task(const BwdParams& p, const RowTile rt, int ct, char* smem,
                                        Hook after_mainloop) {
    typedef Geom<NW> G;
    const int d = p.s.d, I = p.s.I;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kc = tid & 7;
    DirectRowLoader<false> al;
    {
        const int row = rt.row0 + min(wave * 32 + (lane & 31), rt.rows - 1);
        al.rp = p.dgu + ((size_t)row * 2 * I + (lane >> 5) * 32) * 2;
    }
    typedef SplitRowLoader<G::NT, BN> BL;   // k < I: row of W_gate[e][c], k >= I: row of W_up[e][c]
    BL bl;
    bl.init();
    const int n0 = ct * BN;
#pragma unroll
    for (int q = 0; q < BL::NP; ++q) {
        const int rho = BL::row(q);
        const int c = min(n0 + (rho & 31) * 8, d - 8) + (rho >> 5);
        bl.rp[q] = p.w_gate + (((size_t)rt.expert * d + c) * I + kc * 8) * 2;
    }
    bl.delta = (long long)(p.w_up - p.w_gate);
    bl.switch_stage = I / BK;
    f32x16_t acc[8];
    mma_mainloop_direct<NW>(al, bl, 2 * I / BK, smem, wave * 32 < rt.rows, acc);
    after_mainloop();
    const int col = n0 + (lane & 31) * 8;
    if (col < d) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = wave * 32 + frag_row(v, lane);
            if (m < rt.rows)
                store_stream16(p.dxp + ((size_t)(rt.row0 + m) * d + col) * 2, pack_row8(acc, v));
        }
    }
}

// Weight gradients added to an fp32 gradient buffer (a training loop's main gradient) instead
// of written as bf16: q[0..8) += the lane's 8 consecutive columns of accumulator element v.
// Every element belongs to exactly one tile, so the read-modify-write needs no atomic and the
// sum does not depend on the schedule.
__device__ __forceinline__ void accumulate_row8(float* q, const f32x16_t (&acc)[8], int v) {
    typedef __attribute__((ext_vector_type(4))) float f32x4_t;
    f32x4_t a = ((const f32x4_t*)q)[0], b = ((const f32x4_t*)q)[1];
    a += f32x4_t{acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
    b += f32x4_t{acc[4][v], acc[5][v], acc[6][v], acc[7][v]};
    __builtin_nontemporal_store(a, (f32x4_t*)q);
    __builtin_nontemporal_store(b, (f32x4_t*)q + 1);
}

// ------------------------------------------------------------- phase 1: dW_down
// dW_down[e][i][c] = sum over the expert's rows r (ascending) of h[r][i] * dO[r][c].
// Output tile: 32*NW rows of I by 256 columns of d.
template <int NW, bool ACC, class Hook>
__device__ __forceinline__ void dwd_task(const BwdParams& p, int e, int mt, int nt, int r0, int cnt,
                                         char* smem, Hook after_mainloop) {
    typedef Geom<NW> G;
    const int d = p.s.d, I = p.s.I;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    typedef StridedLoaderK<G::NT, 4 * NW> AL;
    AL al;
    al.init();
    al.ld_bytes = (size_t)I * 2;
    al.K = cnt;
    al.bp = p.h + ((size_t)r0 * I + min(mt * G::BM + AL::TG::chunk() * 8, I - 8)) * 2;
    typedef GatherStridedLoader<G::NT, 32, true> BL;
    BL bl;
    bl.init();
    bl.ld_bytes = (size_t)d * 2;
    bl.row_tok = p.row_tok;
    bl.row_w = p.row_w;
    bl.row0 = r0;
    bl.K = cnt;
    bl.ring = smem + G::SMEM;
    bl.src = p.dy + (size_t)min(nt * BN + BL::TG::chunk() * 8, d - 8) * 2;
    f32x16_t acc[8];
    mma_mainloop<NW>(al, bl, (cnt + BK - 1) / BK, smem, true, acc);
    after_mainloop();
    const int col = nt * BN + (lane & 31) * 8;
    if (col < d) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = mt * G::BM + tr_tile_row<NW>(wave * 32 + frag_row(v, lane));
            if (m < I) {
                if (ACC) {
                    if (cnt > 0) accumulate_row8((float*)p.dw_down + ((size_t)e * I + m) * d + col, acc, v);
                } else {
                    store_stream16(p.dw_down + (((size_t)e * I + m) * d + col) * 2, pack_row8(acc, v));
                }
            }
        }
    }
}

// ------------------------------------------------------------- phase 3: dW_gate, dW_up
// dW_gate[e][c][i] = sum_r x[tok(r)][c] * dG[r][i]; dW_up likewise with dU.
// Output tile: 32*NW rows of d by 128 columns of I, for both matrices at once.
// B-tile chunk nb: even -> 8 columns of dG, odd -> the same 8 columns of dU.
template <int NW, bool ACC, class Hook>
__device__ __forceinline__ void dwgu_task(const BwdParams& p, int e, int mt, int nt, int r0, int cnt,
                                          char* smem, Hook after_mainloop) {
    typedef Geom<NW> G;
    const int d = p.s.d, I = p.s.I;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    typedef GatherStridedLoader<G::NT, 4 * NW, false> AL;
    AL al;
    al.init();
    al.ld_bytes = (size_t)d * 2;
    al.row_tok = p.row_tok;
    al.row_w = p.row_w;
    al.row0 = r0;
    al.K = cnt;
    al.ring = smem + G::SMEM;
    al.src = p.x + (size_t)min(mt * G::BM + AL::TG::chunk() * 8, d - 8) * 2;
    typedef StridedLoaderK<G::NT, 32> BL;
    BL bl;
    bl.init();
    bl.ld_bytes = (size_t)I * 4;
    bl.K = cnt;
    {
        const int cb = BL::TG::chunk();
        bl.bp = p.dgu + ((size_t)r0 * 2 * I + ((cb & 1) ? I : 0) + min(nt * 128 + (cb >> 1) * 8, I - 8)) * 2;
    }
    f32x16_t acc[8];
    mma_mainloop<NW>(al, bl, (cnt + BK - 1) / BK, smem, true, acc);
    after_mainloop();
    const int nb = lane & 31;
    const int icol = nt * 128 + (nb >> 1) * 8;
    char* dst = (nb & 1) ? p.dw_up : p.dw_gate;
    if (icol < I) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = mt * G::BM + tr_tile_row<NW>(wave * 32 + frag_row(v, lane));
            if (m < d) {
                if (ACC) {
                    if (cnt > 0) accumulate_row8((float*)dst + ((size_t)e * d + m) * I + icol, acc, v);
                } else {
                    store_stream16(dst + (((size_t)e * d + m) * I + icol) * 2, pack_row8(acc, v));
                }
            }
        }
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
            // dtopk_w[t][j] = <dY[t], o[row]>: the partial sums of the row's dH column tiles,
            // added in column-tile order; 0 for a slot whose expert is not local
            const int r = p.inv_perm[(size_t)t * k + lane];
            float s = 0.f;
            if (r >= 0)
                for (int ct = 0; ct < p.nct_dh; ++ct) s += p.dots[(size_t)ct * ((size_t)T * k) + r];
            p.dtopk_w[(size_t)t * k + lane] = s;
        }
    }
}


// ------------------------------------------------------------- worker loop
// ACC: the weight gradients are added to fp32 buffers (moe_opts_t.dw_accumulate).
template <int NW, bool ACC>
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
            const Task task = p.tasks[id];
            const int type = task_type(task), ct = task_ct(task);
            if (phase >= 0 && type != phase) {
                // staged launch: another phase's task
            } else if (type == B_DH) {
                const RowTile rt = task_row_tile(task);
                dh_task<NW>(p, rt, ct, smem, issue);
                wait_stores();
                __syncthreads();   // the write-through dG|dU stores of every wave have completed
                if (threadIdx.x == 0) {
                    add_relaxed(p.flag_rt + task.idx, 1);
                    add_relaxed(p.flag_e + rt.expert, 1);
                }
            } else if (type == B_DWD) {
                dwd_task<NW, ACC>(p, task_expert(task), task.idx, ct, task.row0, task.rows, smem, issue);
            } else if (type == B_DXP) {
                if (threadIdx.x == 0) s_ok = wait_ge(p.flag_rt + task.idx, p.nct_dh, ctrl, p.spin_ticks);
                __syncthreads();
                if (s_ok) {
                    const RowTile rt = task_row_tile(task);
                    dxp_task<NW>(p, rt, ct, smem, issue);
                }
            } else {
                const int e = task_expert(task);
                // all dH tiles of the expert: its row tiles times the dH column tiles
                const int need = (task.rows + Geom<NW>::BM - 1) / Geom<NW>::BM * p.nct_dh;
                if (threadIdx.x == 0) s_ok = wait_ge(p.flag_e + e, need, ctrl, p.spin_ticks);
                __syncthreads();
                if (s_ok) dwgu_task<NW, ACC>(p, e, task.idx, ct, task.row0, task.rows, smem, issue);
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
            if (s_ok) dx_task<NW>(p, -1 - id);
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

template <int NW>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2)))
bwd_worker_kernel(BwdParams p, int phase) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bwd_worker_body<NW, false>(p, phase, smem);
}
template <int NW>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2)))
bwd_worker_acc_kernel(BwdParams p, int phase) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bwd_worker_body<NW, true>(p, phase, smem);
}

// dX (and dtopk_w) as a plain grid launch behind the GEMM MegaKernel, one workgroup per block
// of kDxTokens tokens: no scoreboard wait, no task cursor, no LDS.
template <int NW, int KM>
__global__ void __launch_bounds__(64 * NW) bwd_tail_kernel(BwdParams p) {
    dx_task<NW, KM>(p, blockIdx.x);
}

// ------------------------------------------------------------------ host side

struct BwdLayout {
    size_t ctrl, flag_rt, flag_e, tasks, row_tok, row_w, dgu, dxp, dots, total;
    int max_rt, nct_dh, nct_dxp, mt_dwd, nt_dwd, mt_dwgu, nt_dwgu;
};

static BwdLayout bwd_layout(const moe_shape_t& s, int bm) {
    BwdLayout L;
    const size_t A_cap = (size_t)s.T * s.k;
    L.max_rt = (int)((A_cap + 127) / 128) + s.e_count;
    L.nct_dh = (s.I + BN - 1) / BN;
    L.nct_dxp = (s.d + BN - 1) / BN;
    L.mt_dwd = (s.I + bm - 1) / bm;
    L.nt_dwd = (s.d + 255) / 256;
    L.mt_dwgu = (s.d + bm - 1) / bm;
    L.nt_dwgu = (s.I + 127) / 128;
    const size_t max_tasks = (size_t)L.max_rt * (L.nct_dh + L.nct_dxp) +
                             (size_t)s.e_count * (L.mt_dwd * L.nt_dwd + L.mt_dwgu * L.nt_dwgu) +
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
    L.dots = off;    off = align_up(off + (size_t)L.nct_dh * A_cap * sizeof(float), 256);
    L.total = off;
    return L;
}

size_t bwd_workspace_bytes(const moe_shape_t& s) { return bwd_layout(s, 128).total; }   // 128-row tiles need the most tasks

static std::mutex g_bwd_workers_mu;
static int g_bwd_workers[kMaxDevices * 4];   // filled on first use under the lock, constant afterwards

template <int NW, bool ACC>
static int bwd_resident_workers(int* out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOE_ERR_HIP;
    const int slot = (dev * 2 + (NW == 8 ? 1 : 0)) * 2 + (ACC ? 1 : 0);
    std::lock_guard<std::mutex> lock(g_bwd_workers_mu);
    if (g_bwd_workers[slot] == 0) {
        const void* fn = ACC ? (const void*)bwd_worker_acc_kernel<NW> : (const void*)bwd_worker_kernel<NW>;
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize,
                                Geom<NW>::SMEM + kIdxRingBytes) != hipSuccess)
            return MOE_ERR_HIP;
        int per_cu = 0, cus = 0;
        const hipError_t occ = ACC
            ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, bwd_worker_acc_kernel<NW>, Geom<NW>::NT,
                                                           Geom<NW>::SMEM + kIdxRingBytes)
            : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, bwd_worker_kernel<NW>, Geom<NW>::NT,
                                                           Geom<NW>::SMEM + kIdxRingBytes);
        if (occ != hipSuccess) return MOE_ERR_HIP;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return MOE_ERR_HIP;
        if (per_cu < 1 || cus < 1) return MOE_ERR_HIP;
        g_bwd_workers[slot] = per_cu * cus;
    }
    *out = g_bwd_workers[slot];
    return MOE_OK;
}

template <int NW, bool ACC>
static void launch_worker(const BwdParams& p, int workers, int phase, hipStream_t st) {
    if (ACC)
        hipLaunchKernelGGL(bwd_worker_acc_kernel<NW>, dim3(workers), dim3(Geom<NW>::NT),
                           Geom<NW>::SMEM + kIdxRingBytes, st, p, phase);
    else
        hipLaunchKernelGGL(bwd_worker_kernel<NW>, dim3(workers), dim3(Geom<NW>::NT),
                           Geom<NW>::SMEM + kIdxRingBytes, st, p, phase);
}

template <int NW, bool ACC>
static int bwd_launch_nw(BwdParams& p, const moe_opts_t& opts, hipStream_t st) {
    int resident = 0;
    int rc = bwd_resident_workers<NW, ACC>(&resident);
    if (rc != MOE_OK) return rc;
    const int workers = opts.workers > 0 ? min(opts.workers, resident) : resident;
    p.workers = workers;
    const int A_cap = p.s.T * p.s.k;
    if (A_cap > 0)
        hipLaunchKernelGGL(row_meta_kernel, dim3((A_cap + 255) / 256), dim3(256), 0, st, p);
    hipLaunchKernelGGL(bwd_prologue_kernel<Geom<NW>::BM>, dim3(1), dim3(1024), 0, st, p);
    if (opts.schedule == 2) {
        for (int phase = 0; phase < 5; ++phase) launch_worker<NW, ACC>(p, workers, phase, st);
    } else if (opts.schedule != 1) {   // 0 (default) and 3: GEMM MegaKernel, then the tail tasks
        launch_worker<NW, ACC>(p, workers, -2, st);
        const int n_tail = (p.s.T + kDxTokens - 1) / kDxTokens;
        if (n_tail > 0 && !opts.skip_tail) {
            if (p.s.k <= 8)
                hipLaunchKernelGGL((bwd_tail_kernel<NW, 8>), dim3(n_tail), dim3(Geom<NW>::NT), 0, st, p);
            else
                hipLaunchKernelGGL((bwd_tail_kernel<NW, kMaxTopK>), dim3(n_tail), dim3(Geom<NW>::NT), 0, st, p);
        }
    } else {
        launch_worker<NW, ACC>(p, workers, -1, st);
    }
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int bwd_launch(const moe_shape_t& s, const void* dy, const void* x, const void* w_gate,
               const void* w_up, const void* w_down, const moe_routing_t& r, const char* gu,
               const char* h, const char* o, void* dx, void* dw_gate, void* dw_up, void* dw_down,
               float* dtopk_w, char* ws, const moe_opts_t& opts, int nw, hipStream_t st) {
    const BwdLayout L = bwd_layout(s, 32 * nw);
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
    p.dots = (float*)(ws + L.dots);
    p.nct_dh = L.nct_dh;
    p.nct_dxp = L.nct_dxp;
    p.mt_dwd = L.mt_dwd;
    p.nt_dwd = L.nt_dwd;
    p.mt_dwgu = L.mt_dwgu;
    p.nt_dwgu = L.nt_dwgu;
    const int ms = opts.spin_limit_ms > 0 ? opts.spin_limit_ms : 2000;
    p.spin_ticks = (long long)ms * 100000ll;
    if (opts.dw_accumulate)
        return nw == 4 ? bwd_launch_nw<4, true>(p, opts, st) : bwd_launch_nw<8, true>(p, opts, st);
    return nw == 4 ? bwd_launch_nw<4, false>(p, opts, st) : bwd_launch_nw<8, false>(p, opts, st);
}

}  // namespace uniep
