// Routing and deterministic token mapping on one GPU.
//
// Paper: Section 2.1 (gating, top-k), Section 3.1 "Deterministic Token Mapping",
// Algorithm 1 lines 1-2 (BinCount, CumSum) and the local stable order M_loc; with
// one rank the global offset base is zero, so the destination row of a
// (token, slot) pair is  offsets[e] + rank of the pair among the pairs of e.
//
// No position is ever handed out by an atomic: the flat slots are cut into
// fixed chunks, each chunk counts its experts, a scan over chunks gives every
// chunk its starting row per expert, and inside a chunk ranks come from wave
// ballots in lane order.  The result is therefore the same on every run.
#include "common.hpp"

#include <mutex>

namespace uniep {

constexpr int kChunk = 256;        // flat slots per wave-chunk (4 wave iterations)
constexpr int kRouteThreads = 256; // 4 waves per workgroup

// ---------------------------------------------------------------- top-k + gates
// One wave per token.  Lane l holds experts l, l+64, ...  k rounds of arg-max
// under the order (value desc, expert id asc); gates from the k selected logits
// (the softmax denominator over all E cancels in the renormalisation).
template <int EPL>
__global__ void __launch_bounds__(kRouteThreads)
topk_gate_kernel(const float* __restrict__ logits, int T, int E, int k,
                 int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * (kRouteThreads / 64) + (threadIdx.x >> 6);
    if (t >= T) return;
    const float* row = logits + (size_t)t * E;
    float v[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        const int e = lane + 64 * i;
        v[i] = (e < E) ? row[e] : -INFINITY;
    }
    uint32_t taken = 0;
#pragma unroll
    for (int i = 0; i < EPL; ++i)
        if (lane + 64 * i >= E) taken |= 1u << i;   // padding lanes never win
    float my_val = 0.f;
    int my_idx = 0;
    float top1 = 0.f;
    for (int j = 0; j < k; ++j) {
        float bv = -INFINITY;
        int be = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            const int e = lane + 64 * i;
            const bool free_ = !((taken >> i) & 1u);
            if (free_ && (v[i] > bv || (v[i] == bv && e < be))) { bv = v[i]; be = e; }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(bv, off);
            const int oe = __shfl_xor(be, off);
            if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
        }
        // every lane now agrees on (bv, be); the owner retires it
        if ((be & 63) == lane) taken |= 1u << (be >> 6);
        if (j == 0) top1 = bv;
        if (lane == j) { my_val = bv; my_idx = be; }
    }
    float p = (lane < k) ? __expf(my_val - top1) : 0.f;
    float s = p;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
    if (lane < k) {
        topk_idx[(size_t)t * k + lane] = my_idx;
        topk_w[(size_t)t * k + lane] = p / s;
    }
}

// ------------------------------------------------------- per-chunk BinCount
// chunk_cnt[c][e] = number of slots of chunk c routed to local expert e.
// Also pre-fills perm with -1 (rows at and beyond A keep it).
__global__ void __launch_bounds__(kRouteThreads)
chunk_count_kernel(const int32_t* __restrict__ topk_idx, int F, int e_start, int e_count,
                   int32_t* __restrict__ chunk_cnt, int32_t* __restrict__ perm) {
    extern __shared__ int32_t s_cnt[];   // [4][e_count]
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int chunk = blockIdx.x * (kRouteThreads / 64) + wave;
    int32_t* cnt = s_cnt + wave * e_count;
    for (int e = lane; e < e_count; e += 64) cnt[e] = 0;
    __syncthreads();
    const int f0 = chunk * kChunk;
    for (int it = 0; it < kChunk / 64; ++it) {
        const int f = f0 + it * 64 + lane;
        if (f < F) {
            perm[f] = -1;
            const int el = topk_idx[f] - e_start;
            if (el >= 0 && el < e_count) atomicAdd(&cnt[el], 1);   // integer sum: order-free
        }
    }
    __syncthreads();
    if (f0 < F)
        for (int e = lane; e < e_count; e += 64) chunk_cnt[(size_t)chunk * e_count + e] = cnt[e];
}

// ------------------------------------------- scan over chunks, then over experts
// One workgroup.  In place: chunk_cnt[c][e] becomes the number of e-slots in
// chunks before c.  counts[e] = total, offsets = exclusive CumSum(counts).
// The chunks are cut into G = 1024 / e_pad contiguous groups (e_pad = e_count
// rounded up to a power of two); thread (g, e) first sums its group, the group
// sums are scanned over g, then the thread rewrites its chunks with the running value.
__global__ void __launch_bounds__(1024)
scan_kernel(int32_t* __restrict__ chunk_cnt, int n_chunks, int e_count,
            int32_t* __restrict__ counts, int32_t* __restrict__ offsets) {
    __shared__ int32_t s_tot[kMaxExperts];
    __shared__ int32_t s_grp[kMaxExperts];   // [G][e_pad]
    const int tid = threadIdx.x;
    int e_pad = 1;
    while (e_pad < e_count) e_pad <<= 1;
    const int G = kMaxExperts / e_pad;
    const int e = tid & (e_pad - 1), g = tid / e_pad;
    const int per = (n_chunks + G - 1) / G;
    const int c0 = min(g * per, n_chunks), c1 = min(c0 + per, n_chunks);
    int32_t sum = 0;
    if (e < e_count) {
        int c = c0;
        for (; c + 8 <= c1; c += 8) {
            int32_t tmp[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) tmp[u] = chunk_cnt[(size_t)(c + u) * e_count + e];
#pragma unroll
            for (int u = 0; u < 8; ++u) sum += tmp[u];
        }
        for (; c < c1; ++c) sum += chunk_cnt[(size_t)c * e_count + e];
    }
    s_grp[tid] = sum;
    __syncthreads();
    int32_t run = 0, total = 0;
    for (int j = 0; j < G; ++j) {
        const int32_t v = s_grp[j * e_pad + e];
        if (j < g) run += v;
        total += v;
    }
    if (e < e_count) {
        int c = c0;
        for (; c + 8 <= c1; c += 8) {
            int32_t tmp[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) tmp[u] = chunk_cnt[(size_t)(c + u) * e_count + e];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                chunk_cnt[(size_t)(c + u) * e_count + e] = run;
                run += tmp[u];
            }
        }
        for (; c < c1; ++c) {
            const int32_t tmp = chunk_cnt[(size_t)c * e_count + e];
            chunk_cnt[(size_t)c * e_count + e] = run;
            run += tmp;
        }
        if (g == 0) counts[e] = total;
    }
    __syncthreads();
    s_tot[tid] = (g == 0 && e < e_count) ? total : 0;   // g == 0: tid == e
    __syncthreads();
    // inclusive Hillis-Steele scan over 1024 entries
    for (int off = 1; off < kMaxExperts; off <<= 1) {
        const int32_t add = (tid >= off) ? s_tot[tid - off] : 0;
        __syncthreads();
        s_tot[tid] += add;
        __syncthreads();
    }
    if (tid < e_count) offsets[tid + 1] = s_tot[tid];
    if (tid == 0) offsets[0] = 0;
}

// ------------------------------------------------------------ stable positions
// Each wave walks its chunk 64 slots at a time.  cur[e] = next free row of
// expert e for this chunk; lanes that share an expert take consecutive rows in
// lane order (= flat-slot order): the set of such lanes is the intersection of
// the ballots of the expert id's bits, a lane's rank the set bits below it.
__global__ void __launch_bounds__(kRouteThreads)
position_kernel(const int32_t* __restrict__ topk_idx, int F, int e_start, int e_count,
                const int32_t* __restrict__ chunk_base, const int32_t* __restrict__ offsets,
                int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
    extern __shared__ int32_t s_cur_all[];   // [4][e_count]
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int chunk = blockIdx.x * (kRouteThreads / 64) + wave;
    volatile int32_t* cur = s_cur_all + wave * e_count;
    const int f0 = chunk * kChunk;
    if (f0 >= F) return;   // whole wave leaves together; no workgroup barrier below
    for (int e = lane; e < e_count; e += 64)
        cur[e] = offsets[e] + chunk_base[(size_t)chunk * e_count + e];
    __builtin_amdgcn_wave_barrier();
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    for (int it = 0; it < kChunk / 64; ++it) {
        const int f = f0 + it * 64 + lane;
        int el = -1;
        if (f < F) {
            el = topk_idx[f] - e_start;
            if (el < 0 || el >= e_count) el = -1;
        }
        // lanes with the same expert: intersect the ballots of the expert id's bits
        uint64_t m = __ballot(el >= 0);
        for (int b = 0; (1 << b) < e_count; ++b) {
            const uint64_t bb = __ballot((el >> b) & 1);
            m &= ((el >> b) & 1) ? bb : ~bb;
        }
        int row = -1;
        if (el >= 0) {
            row = cur[el] + __popcll(m & lt_mask);
        }
        __builtin_amdgcn_wave_barrier();
        if (el >= 0 && (m >> lane) <= 1ull) cur[el] = row + 1;   // the group's last lane moves the cursor
        __builtin_amdgcn_wave_barrier();
        if (f < F) {
            inv_perm[f] = row;
            if (row >= 0) perm[row] = f;
        }
    }
}

// ------------------------------------------------------------ router gradient
// One wave per token.  Lanes j < k hold slot j; s = sum_j w_j g_j by a wave
// reduction; then every lane writes its experts of the row: the value of the
// slot that selected the expert, or zero.
__global__ void __launch_bounds__(kRouteThreads)
route_backward_kernel(const int32_t* __restrict__ topk_idx, const float* __restrict__ topk_w,
                      const float* __restrict__ dtopk_w, int T, int E, int k,
                      float* __restrict__ dlogits) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * (kRouteThreads / 64) + (threadIdx.x >> 6);
    if (t >= T) return;
    int idx = -1;
    float w = 0.f, g = 0.f;
    if (lane < k) {
        idx = topk_idx[(size_t)t * k + lane];
        w = topk_w[(size_t)t * k + lane];
        g = dtopk_w[(size_t)t * k + lane];
    }
    float s = w * g;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
    const float mine = w * (g - s);
    for (int e = lane; e < E; e += 64) {
        float v = 0.f;
        for (int j = 0; j < k; ++j) {
            const int ej = __shfl(idx, j);
            const float vj = __shfl(mine, j);
            if (ej == e) v = vj;
        }
        dlogits[(size_t)t * E + e] = v;
    }
}

// ------------------------------------------------------------------ global mapping, W > 1
// Algorithm 1 for one rank of W (Section 3.1).  The AllGather of the per-rank
// histograms is the caller's; c_all [W, E] is its result.

// One workgroup of 1024 threads, thread e per expert.  Eq. 1 along the rank axis,
// the total rows every expert receives, and the start of every expert's segment
// in its destination rank's buffer (exclusive scan inside each group of n_epr
// experts).  Writes off_base[e] = O_all[rank, e] - O_exp[e] and row_base[e] =
// segment start + off_base[e], so that the mapping kernel only adds M_loc, and
// this rank's own segment table recv_offsets [n_epr + 1].
__global__ void __launch_bounds__(1024)
global_offsets_kernel(const int32_t* __restrict__ c_all, const int32_t* __restrict__ o_exp, int E,
                      int W, int rank, int n_epr, int32_t* __restrict__ off_base,
                      int32_t* __restrict__ row_base, int32_t* __restrict__ recv_offsets) {
    __shared__ int32_t s_scan[1024];
    const int e = threadIdx.x;
    int total = 0, before = 0;
    if (e < E) {
        for (int r = 0; r < W; ++r) {
            const int c = c_all[(size_t)r * E + e];
            if (r < rank) before += c;
            total += c;
        }
    }
    s_scan[e] = total;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {       // inclusive scan over all experts
        const int add = (e >= off) ? s_scan[e - off] : 0;
        __syncthreads();
        s_scan[e] += add;
        __syncthreads();
    }
    if (e < E) {
        const int g0 = (e / n_epr) * n_epr;              // first expert of e's rank
        const int start = (s_scan[e] - total) - (g0 > 0 ? s_scan[g0 - 1] : 0);
        const int ob = before - o_exp[e];
        off_base[e] = ob;
        row_base[e] = start + ob;
        if (e / n_epr == rank) {
            recv_offsets[e - g0] = start;
            if (e - g0 == n_epr - 1) recv_offsets[n_epr] = start + total;
        }
    }
}

// One thread per token: destination (rank, local expert, offset inside the expert's
// segment, row of the destination buffer) of each of its k slots; `send` marks the first
// slot, in slot order, that targets a rank (the copy that crosses the link; the relay
// worker of Section 3.2 replicates it for the token's other experts on that rank).
__global__ void __launch_bounds__(kRouteThreads)
global_map_kernel(const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ m_loc, int T,
                  int k, int n_epr, const int32_t* __restrict__ off_base,
                  const int32_t* __restrict__ row_base, int32_t* __restrict__ dst_rank,
                  int32_t* __restrict__ dst_expert, int32_t* __restrict__ dst_off,
                  int32_t* __restrict__ dst_row, int32_t* __restrict__ send,
                  int32_t* __restrict__ n_dst_ranks) {
    const int t = blockIdx.x * kRouteThreads + threadIdx.x;
    if (t >= T) return;
    unsigned long long seen = 0ull;
    for (int j = 0; j < k; ++j) {
        const size_t f = (size_t)t * k + j;
        const int e = topk_idx[f];
        const int r_tgt = e / n_epr;
        const int loc = m_loc[f];
        dst_rank[f] = r_tgt;
        dst_expert[f] = e - r_tgt * n_epr;
        dst_off[f] = loc + off_base[e];
        dst_row[f] = loc + row_base[e];
        const unsigned long long bit = 1ull << r_tgt;
        send[f] = (seen & bit) ? 0 : 1;
        seen |= bit;
    }
    n_dst_ranks[t] = __popcll(seen);
}

// ------------------------------------------------------------------ host side

int global_map_launch(const moe_shape_t& s, int W, int rank, const moe_routing_t& r,
                      const int32_t* c_all, const moe_global_map_t& out, void* ws, hipStream_t st) {
    int32_t* off_base = (int32_t*)ws;
    int32_t* row_base = off_base + s.E;
    const int n_epr = s.E / W;
    hipLaunchKernelGGL(global_offsets_kernel, dim3(1), dim3(1024), 0, st, c_all, r.offsets, s.E, W,
                       rank, n_epr, off_base, row_base, out.recv_offsets);
    if (s.T > 0)
        hipLaunchKernelGGL(global_map_kernel, dim3((s.T + kRouteThreads - 1) / kRouteThreads),
                           dim3(kRouteThreads), 0, st, r.topk_idx, r.inv_perm, s.T, s.k, n_epr,
                           off_base, row_base, out.dst_rank, out.dst_expert, out.dst_off,
                           out.dst_row, out.send, out.n_dst_ranks);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}


int route_backward_launch(const moe_shape_t& s, const int32_t* topk_idx, const float* topk_w,
                          const float* dtopk_w, float* dlogits, hipStream_t st) {
    if (s.T == 0) return MOE_OK;
    const int per = kRouteThreads / 64;
    hipLaunchKernelGGL(route_backward_kernel, dim3((s.T + per - 1) / per), dim3(kRouteThreads), 0, st,
                       topk_idx, topk_w, dtopk_w, s.T, s.E, s.k, dlogits);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

size_t route_workspace_bytes(const moe_shape_t& s) {
    const size_t F = (size_t)s.T * s.k;
    const size_t n_chunks = (F + kChunk - 1) / kChunk;
    return align_up(n_chunks * (size_t)s.e_count * sizeof(int32_t) + 256, 256);
}

template <int EPL>
static void launch_topk(const moe_shape_t& s, const float* logits, int32_t* idx, float* w,
                        hipStream_t st) {
    const int per = kRouteThreads / 64;
    hipLaunchKernelGGL(topk_gate_kernel<EPL>, dim3((s.T + per - 1) / per), dim3(kRouteThreads), 0,
                       st, logits, s.T, s.E, s.k, idx, w);
}

int route_launch(const moe_shape_t& s, const float* logits, const moe_routing_t& out, void* ws,
                 hipStream_t st) {
    int32_t* chunk_cnt = (int32_t*)ws;
    const int F = s.T * s.k;
    const int n_chunks = (F + kChunk - 1) / kChunk;
    if (s.T > 0) {
        const int epl = (s.E + 63) / 64;
        if (epl <= 1) launch_topk<1>(s, logits, (int32_t*)out.topk_idx, (float*)out.topk_w, st);
        else if (epl <= 2) launch_topk<2>(s, logits, (int32_t*)out.topk_idx, (float*)out.topk_w, st);
        else if (epl <= 4) launch_topk<4>(s, logits, (int32_t*)out.topk_idx, (float*)out.topk_w, st);
        else if (epl <= 8) launch_topk<8>(s, logits, (int32_t*)out.topk_idx, (float*)out.topk_w, st);
        else launch_topk<16>(s, logits, (int32_t*)out.topk_idx, (float*)out.topk_w, st);
        const int per = kRouteThreads / 64;
        const size_t sm = (size_t)per * s.e_count * sizeof(int32_t);
        hipLaunchKernelGGL(chunk_count_kernel, dim3((n_chunks + per - 1) / per),
                           dim3(kRouteThreads), sm, st, out.topk_idx, F, s.e_start, s.e_count,
                           chunk_cnt, (int32_t*)out.perm);
    }
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, st, chunk_cnt, n_chunks, s.e_count,
                       (int32_t*)out.counts, (int32_t*)out.offsets);
    if (s.T > 0) {
        const int per = kRouteThreads / 64;
        const size_t sm = (size_t)per * s.e_count * sizeof(int32_t);
        hipLaunchKernelGGL(position_kernel, dim3((n_chunks + per - 1) / per), dim3(kRouteThreads),
                           sm, st, out.topk_idx, F, s.e_start, s.e_count, chunk_cnt, out.offsets,
                           (int32_t*)out.perm, (int32_t*)out.inv_perm);
    }
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// ------------------------------------------------ routing without a caller workspace
// For callers that may not allocate (code under graph capture, tight serving loops): the
// per-chunk histogram lives in a file-scope device array instead of a workspace argument.
// Each device holds its own copy of the array at its own address, looked up once per
// device (with that device current) and kept; host code never uses the array's name as an
// address.  Every entry the kernels read is written earlier in the same call, so nothing
// has to be cleared; calls that overlap on one device share the array and race.
static __device__ __align__(256) unsigned char scratch[kRouteStaticScratchBytes];

static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices];

int route_static_launch(const moe_shape_t& s, const float* logits, const moe_routing_t& out,
                        hipStream_t st) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOE_ERR_HIP;
    void* ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mu);
        ptr = g_scratch_ptr[dev];
        if (!ptr) {
            if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MOE_ERR_HIP;
            g_scratch_ptr[dev] = ptr;
        }
    }
    return route_launch(s, logits, out, ptr, st);
}

}  // namespace uniep
