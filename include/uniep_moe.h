/*
 * uniep_moe.h -- C ABI of the MI355X (gfx950) fused MoE layer.
 *
 * One GPU's share of the expert-parallel MoE hot path described in the UniEP
 * paper: deterministic token mapping (Section 3.1, Algorithm 1), then
 * dispatch -> grouped GEMM (gate/up) -> SwiGLU -> grouped GEMM (down) ->
 * weighted combine (Section 2.1 "Forward Propagation", Sections 3.1-3.2), run
 * as one persistent work-queue kernel with a global-memory scoreboard
 * (Section 3.1 "Scoreboard-based Synchronization", "Dynamic Scheduling";
 * Listing 1), and the matching backward pass (Section 2.1 "Backward
 * Propagation": input gradients and the transposed grouped GEMM for weight
 * gradients, reduced in the order the token mapping fixes).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers (HIP global memory) unless a
 *     parameter is marked "host".  moe_shape_t / moe_routing_t / moe_opts_t
 *     structs themselves live in host memory.
 *   - The caller owns every buffer.  The library allocates nothing and keeps no
 *     data between calls (the only process-wide state is a per-device cache of
 *     how many worker workgroups fit on the device, filled on first use under a
 *     lock and never changed afterwards, and the file-scope scratch array of
 *     moe_route_static).  All work is enqueued on `stream` (a hipStream_t passed
 *     as void*; NULL = the default stream) and no call synchronises with the
 *     host: the number of routed rows and all tile tables stay on the device.
 *   - Arrays are dense row-major.  bf16 tensors are passed as void*.
 *   - Outputs are overwritten, never accumulated into, with one exception the
 *     caller asks for: moe_opts_t.dw_accumulate = 1 adds the weight gradients
 *     to fp32 buffers.
 *   - Return value: MOE_OK or a negative error code.  All argument, shape and
 *     workspace checks happen before anything is enqueued, so a failed call
 *     has no effect.
 *   - Base pointers of bf16 tensors and of the workspace must be 16-byte
 *     aligned (256-byte for workspaces).
 *   - Two calls that share a workspace must be ordered on the stream.
 *
 * Shape limits (MOE_ERR_SHAPE otherwise): 1 <= k <= 16, k <= E <= 1024,
 * 0 <= e_start, 1 <= e_count, e_start + e_count <= E, d and I multiples of 64,
 * T >= 0 (T == 0 is a no-op apart from zeroed counts/offsets), T*k < 2^30
 * (byte offsets inside the kernels are 64-bit).
 */
#ifndef UNIEP_MOE_H
#define UNIEP_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_OK 0
#define MOE_ERR_ARG (-1)       /* NULL or misaligned pointer */
#define MOE_ERR_SHAPE (-2)     /* shape outside the limits above */
#define MOE_ERR_WORKSPACE (-3) /* ws_bytes too small (the size of `saved` is not passed and cannot be checked) */
#define MOE_ERR_HIP (-4)       /* a HIP runtime call failed (launch, attribute) */
#define MOE_ERR_DEVICE (-5)    /* reported by moe_device_status: a kernel gave up a bounded wait */

/* Problem shape; all sizes in elements.  Local experts are
 * [e_start, e_start + e_count): with N_epr experts per rank this is rank
 * r_tgt = e / N_epr, local id e_loc = e % N_epr of Algorithm 1 (lines 5-6). */
typedef struct {
    int32_t T;       /* tokens resident on this GPU (N_tok) */
    int32_t d;       /* hidden size (H_dim) */
    int32_t E;       /* experts the router ranks (N_exp) */
    int32_t k;       /* top-k */
    int32_t I;       /* expert intermediate size (H_inter) */
    int32_t e_start; /* first local expert */
    int32_t e_count; /* number of local experts */
} moe_shape_t;

/* Output of moe_route / input of forward and backward (device pointers).
 * A = offsets[e_count] is the number of (token, slot) assignments that land on
 * local experts; "row" r in [0, A) is a position in the expert-sorted order. */
typedef struct {
    const int32_t* topk_idx; /* [T,k]  expert id of slot j (descending logit; ties: lower id) */
    const float* topk_w;     /* [T,k]  gate: softmax renormalised over the k selected */
    const int32_t* counts;   /* [e_count]    C_exp: rows per local expert */
    const int32_t* offsets;  /* [e_count+1]  O_exp: exclusive prefix sum of counts */
    const int32_t* perm;     /* [T*k]  row -> flat slot t*k+j; entries >= A are -1 */
    const int32_t* inv_perm; /* [T,k]  flat slot -> row, or -1 if the expert is not local */
} moe_routing_t;

/* Launch options (host struct; NULL = all defaults). */
typedef struct {
    int32_t schedule; /* 0 = default (= 3), 1 = one persistent work-queue MegaKernel for every
                         task, 2 = staged: one launch per phase (same tile code; for profiling),
                         3 = one persistent MegaKernel for all GEMM tasks with scoreboard
                         waits, then a plain grid kernel for the tail tasks (combine / dX:
                         fwd_tail_kernel / bwd_tail_kernel, one workgroup per 16 tokens),
                         which may only start once every GEMM task is done.
                         Schedule 1 makes the tail tasks wait inside the kernel until EVERY
                         worker has started and run out of GEMM work, so it needs all
                         `workers` workgroups co-resident: the occupancy query that bounds
                         `workers` cannot see kernels of other streams or processes, and if
                         some worker never becomes resident the waits end at spin_limit_ms
                         with MOE_ERR_DEVICE and partly written y / dx.  Schedules 0, 2, 3
                         have no such precondition. */
    int32_t workers;  /* persistent workgroups; 0 = one per resident slot (never more than
                         can be co-resident: the deadlock-freedom condition of Section 3.1) */
    int32_t spin_limit_ms; /* bound on every scoreboard wait; 0 = 2000 ms.  A wait that
                              exceeds it sets MOE_ERR_DEVICE in the workspace and drains */
    int32_t tile_rows;     /* rows per GEMM row tile: 0 = default (256), or 128 / 256 */
    int32_t skip_tail;     /* measurement aid, 0 or 1: with the default schedule, 1 leaves out the
                              tail kernel (combine / dX), so that y / dx and dtopk_w are not
                              written and a timer around the call sees the GEMM MegaKernel and
                              its prologue alone */
    int32_t dw_accumulate; /* moe_fused_backward only, 0 or 1.  1: dw_gate, dw_up, dw_down are fp32
                              buffers of the same shapes (16-byte aligned) and the weight
                              gradients are ADDED to them in fp32, straight from the
                              accumulators (no bf16 rounding): the gradient-accumulation buffer
                              of a mixed-precision training loop.  Experts without rows are left
                              untouched.  Every element is updated by exactly one tile, so the
                              result is as reproducible as with 0. */
    int32_t dw_split_rows; /* moe_fused_backward only.  0 = every weight-gradient element is one sum over
                              the expert's rows in ascending order.  S > 0 (a multiple of 64, at least
                              256): the reduction of an expert with more than S rows is cut at the fixed
                              points S, 2S, ... (a function of the expert's row count only) into parts
                              that run as tasks of their own; the fp32 partial tiles are added in the
                              order of the parts.  More parallelism for a few very large experts
                              (skewed routing), at the price Section 6.3 discusses: the result is still
                              bitwise identical from run to run, across schedules and worker counts, but
                              not to the S = 0 result (another association of the same sum).  Needs the
                              larger workspace that moe_backward_workspace_bytes reports. */
    int32_t reserved[1];   /* must be 0 */
} moe_opts_t;

/* Bytes each call needs (host outputs; any may be NULL).  `saved_bytes` is the
 * size of the optional activation stash forward fills for backward. */
int moe_workspace_bytes(const moe_shape_t* shape, size_t* route_ws, size_t* fwd_ws,
                        size_t* bwd_ws, size_t* saved_bytes);

/* Workspace bytes of moe_fused_backward with these options (host output).  Equal to bwd_ws of
 * moe_workspace_bytes unless opts->dw_split_rows > 0: the partial tiles of the split
 * weight-gradient reductions (Section 6.3, the cost of a fixed reduction order) are sized for
 * the worst routing, 2 * T * k / dw_split_rows parts of every output tile of an expert.
 * MOE_ERR_ARG for options moe_fused_backward would reject. */
int moe_backward_workspace_bytes(const moe_shape_t* shape, const moe_opts_t* opts, size_t* bwd_ws);

/* Byte offsets inside the `saved` stash (host outputs), for a given shape:
 *   gu  [A_cap, 2*I] bf16  per row: G (I values) then U (I values), A_cap = T*k
 *   h   [A_cap, I]   bf16  silu(G)*U
 *   o   [A_cap, d]   bf16  expert outputs before the combine
 * Rows at and beyond A are unspecified. */
int moe_saved_layout(const moe_shape_t* shape, size_t* off_gu, size_t* off_h, size_t* off_o);

/* Routing and deterministic token mapping (Section 2.1 gating; Algorithm 1,
 * lines 1-2 and the local stable order M_loc, with one rank: base_off = 0).
 *   logits   [T,E] fp32, finite.  Selection is on the raw logits: larger
 *            first, equal values -> lower expert id first; slot j is the j-th
 *            in that order.  Gate = softmax over all E renormalised over the k
 *            selected.
 * Writes the six arrays of moe_routing_t (the struct's pointers are used as
 * outputs here).  Row of flat slot f = t*k+j with local expert e:
 *   offsets[e - e_start] + #{f' < f : topk_idx[f'] == e}
 * i.e. a stable sort of the flat slots by expert, computed without atomics on
 * positions, so it is identical on every run. */
int moe_route(const moe_shape_t* shape, const float* logits, const moe_routing_t* out,
              void* ws, size_t ws_bytes, void* stream);

/* moe_route for callers that cannot allocate or bring a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same inputs, outputs
 * and results as moe_route, but the per-chunk histogram lives in a file-scope device
 * array of MOE_ROUTE_STATIC_SCRATCH_BYTES that every device the library runs on holds
 * until the process ends.  The call allocates nothing and calls no allocating routine.
 * Problems whose moe_workspace_bytes(...).route_ws exceeds that size return
 * MOE_ERR_WORKSPACE before anything is enqueued.  Every call on a device shares that
 * device's array: calls that overlap on one device (different streams, different host
 * threads) race; calls ordered on one stream are safe.  Nothing in the array has to
 * survive between calls, and every entry a call reads it has written itself. */
#define MOE_ROUTE_STATIC_SCRATCH_BYTES (4u << 20)
int moe_route_static(const moe_shape_t* shape, const float* logits, const moe_routing_t* out,
                     void* stream);

/* Forward: y[t] = sum_j topk_w[t,j] * o[row(t,j)] over the local slots of t in
 * slot order, fp32 accumulate, where for row r of local expert e holding token
 * t:  h = silu(x[t] W_gate[e]) * (x[t] W_up[e]),  o[r] = h W_down[e]
 * (Section 2.1; combine only after all k contributions exist and in one fixed
 * order, Section 3.2).  bf16 in, fp32 accumulate, h / o / y rounded to bf16.
 *   x       [T,d] bf16
 *   w_gate  [e_count,d,I] bf16,  w_up [e_count,d,I] bf16,  w_down [e_count,I,d] bf16
 *   y       [T,d] bf16 (tokens with no local slot get zeros)
 *   saved   NULL, or saved_bytes of device memory that receives G,U,h,o for backward
 *   ws      fwd_ws bytes */
int moe_fused_forward(const moe_shape_t* shape, const void* x, const void* w_gate,
                      const void* w_up, const void* w_down, const moe_routing_t* routing,
                      void* y, void* saved, void* ws, size_t ws_bytes, const moe_opts_t* opts,
                      void* stream);

/* Backward of the above given dy [T,d] bf16 (Section 2.1 "Backward
 * Propagation"): dO[r] = topk_w * dy[t];  dH = dO W_down^T;  SwiGLU backward;
 * dXp = dG W_gate^T + dU W_up^T;  dx[t] = sum_j dXp[row(t,j)] in slot order;
 * dW_down[e] = h_e^T dO_e, dW_gate[e] = x_e^T dG_e, dW_up[e] = x_e^T dU_e, each
 * reduced over the expert's rows in row order (fixed by the token mapping, so
 * bitwise reproducible).  Experts with no rows get exact zeros.
 *   saved    the stash a forward call with the same inputs filled.  REQUIRED:
 *            NULL returns MOE_ERR_ARG.  A backward pass that recomputes G, U and h
 *            instead is not built: it would repeat two thirds of the forward
 *            GEMM work inside the backward kernel to save a stash that costs
 *            6 % of the forward pass's traffic to write.
 *   dx       [T,d] bf16;  dw_gate, dw_up [e_count,d,I] bf16;  dw_down [e_count,I,d] bf16
 *            (overwritten; with opts->dw_accumulate = 1: fp32, added to)
 *   dtopk_w  [T,k] fp32 = <dy[t], o[row(t,j)]> (0 for non-local slots), or NULL.
 *            Evaluated as sum_i (dy[t] W_down[e]^T)[i] * h[r][i] from the fp32
 *            accumulators of the dH tiles and the stashed h, column tiles added
 *            in ascending order: the same number without the bf16 rounding of
 *            o, and the stashed o is not read.
 *   ws       bwd_ws bytes */
int moe_fused_backward(const moe_shape_t* shape, const void* dy, const void* x,
                       const void* w_gate, const void* w_up, const void* w_down,
                       const moe_routing_t* routing, const void* saved, void* dx, void* dw_gate,
                       void* dw_up, void* dw_down, float* dtopk_w, void* ws, size_t ws_bytes,
                       const moe_opts_t* opts, void* stream);

/* Gradient of the gates with respect to the router logits, for the selection
 * that moe_route made (Section 2.1: the gating scores weight the expert
 * outputs; with dtopk_w from moe_fused_backward this makes the layer trainable
 * end to end).  For token t and its slots i:  dlogits[t, topk_idx[t,i]] =
 * topk_w[t,i] * (dtopk_w[t,i] - sum_j topk_w[t,j] * dtopk_w[t,j]);  all other
 * entries of the row are zero (the softmax denominator over all experts cancels
 * in the renormalised gates, so unselected logits do not move them).
 *   topk_idx [T,k] int32, topk_w [T,k] fp32, dtopk_w [T,k] fp32 (device, read)
 *   dlogits  [T,E] fp32 (device, every element written)
 * No workspace.  Returns MOE_ERR_ARG for NULL pointers when T > 0. */
int moe_route_backward(const moe_shape_t* shape, const int32_t* topk_idx, const float* topk_w,
                       const float* dtopk_w, float* dlogits, void* stream);

/* Outputs of moe_global_map (device pointers, all written by the call). */
typedef struct {
    int32_t* dst_rank;     /* [T,k]  r_tgt = e / N_epr */
    int32_t* dst_expert;   /* [T,k]  e_loc = e % N_epr */
    int32_t* dst_off;      /* [T,k]  final_idx: position inside the expert's segment */
    int32_t* dst_row;      /* [T,k]  row of the destination rank's buffer: segment start + final_idx */
    int32_t* send;         /* [T,k]  1 = first slot of its token for that rank (the copy that
                                     crosses the link), 0 = replicated at the destination */
    int32_t* n_dst_ranks;  /* [T]    distinct destination ranks of the token */
    int32_t* recv_offsets; /* [E/W + 1]  this rank as destination: start of each local expert's
                                     segment, and the total rows it receives */
} moe_global_map_t;

/* Deterministic global token mapping for one rank of W (Section 3.1, Algorithm 1
 * lines 3-14 and Eq. 1), the part of the W > 1 index stage that runs on one
 * GPU; the AllGather of the histograms is the caller's and arrives as c_all.
 * With N_epr = E / W experts per rank, slot (t,j) with expert e goes to rank
 * e / N_epr, local expert e % N_epr, at
 *   final_idx = M_loc[t,j] - O_exp[e] + sum_{r' < rank} c_all[r', e]
 * inside that expert's segment; segments of a rank's experts follow each other
 * without padding, each as long as the column sum of c_all, so
 *   dst_row = sum_{e' in the rank, e' < e} sum_r c_all[r, e'] + final_idx.
 * Rows of one expert end up ordered by (source rank, token, slot): the stable
 * sort of the rank-concatenated tokens, with no atomics.
 *   shape    T, E, k are used; e_start must be 0 and e_count = E (the routing
 *            must rank all experts: M_loc = routing->inv_perm, O_exp =
 *            routing->offsets); E % W == 0, 1 <= W <= 64, 0 <= rank < W
 *            (MOE_ERR_SHAPE otherwise)
 *   routing  what moe_route wrote for this rank's tokens (topk_idx, inv_perm,
 *            offsets are read)
 *   c_all    [W,E] int32, device: row r = rank r's counts; row `rank` must equal
 *            routing->counts (not checked)
 *   ws       8*E bytes of device scratch */
int moe_global_map(const moe_shape_t* shape, int32_t W, int32_t rank, const moe_routing_t* routing,
                   const int32_t* c_all, const moe_global_map_t* out, void* ws, size_t ws_bytes,
                   void* stream);

/* Synchronises `stream`, reads the status word a forward/backward call left in
 * its workspace and returns MOE_OK or MOE_ERR_DEVICE (test and debug aid; the
 * hot path never calls it). */
int moe_device_status(const void* ws, void* stream);

/* ---- Analytical performance model and configuration search (host only) -------
 * Section 4.2, Algorithm 2 and its equations; search space of Section 6.2.  The
 * model predicts the latency of one expert-parallel MoE pass (dispatch + up GEMM,
 * SwiGLU, down GEMM + combine) for a split of the chip's workers between
 * communication, relay, reduce and GEMM work, and the search returns the split
 * with the smallest predicted latency.  Nothing here touches a GPU: all pointers
 * are host pointers, the calls are synchronous and allocate only host memory.
 *
 * Hardware H: n_sm workers (SMs / CUs, 2..1024), p_peak FLOP/s, beta_hbm and beta_link
 * (one direction) in bytes/s, w_sat = warps (waves) that saturate a bandwidth,
 * tau_sync seconds per tile for its scoreboard traffic, mu[i] = GEMM utilisation
 * with 8, 16, 32 warps per worker (the paper: 0.7, 0.65, 0.6; w_sat 1024; 2 us).
 * Problem P: n_tok tokens per rank, h_dim, h_inter, n_exp experts over `world`
 * ranks (n_exp % world == 0), top_k, GEMM block b_m x b_n, elem_bytes per element.
 * What the paper leaves open is read as follows: balanced routing; X = W (1 -
 * (1 - 1/W)^k) destination ranks per token; V_nvl = n_tok X S_tok for dispatch
 * and combine; the relay copies V_hbm = n_tok (k - X) S_tok; the reduce reads
 * V_hbm_total = n_tok k S_tok; S_tok = h_dim elem_bytes; per rank n_tok k rows
 * over n_exp / world experts, ceil(rows / b_m) row tiles each, ceil(2 h_inter /
 * b_n) column tiles in the up GEMM and ceil(h_dim / b_n) in the down GEMM.
 * Configuration C: n_disp, n_relay, n_comb, n_red workers and `warps` in
 * {8, 16, 32}; valid iff 1 <= n_disp < n_sm, 1 <= n_comb < n_sm, n_relay >= 1,
 * 1 <= n_red <= n_sm and n_disp + n_relay < n_sm (Section 4.1). */
typedef struct {
    int32_t n_sm, w_sat;
    double p_peak, beta_hbm, beta_link, tau_sync;
    double mu[3];
} moe_perf_hw_t;
typedef struct {
    int32_t n_tok, h_dim, h_inter, n_exp, top_k, world, b_m, b_n, elem_bytes;
} moe_perf_problem_t;
typedef struct {
    int32_t n_disp, n_relay, n_comb, n_red, warps;
} moe_perf_config_t;
typedef struct {   /* every intermediate of Algorithm 2's loop body, seconds */
    double t_up, t_down, l_swiglu, l_disp, l_up, l_s1, l_comb, t_red, l_down, l_s2, l_total;
} moe_perf_latency_t;

/* Algorithm 2's loop body for one configuration.  MOE_ERR_ARG for a NULL pointer,
 * MOE_ERR_SHAPE for values outside the ranges above or an invalid configuration. */
int moe_perf_model_eval(const moe_perf_hw_t* hw, const moe_perf_problem_t* problem,
                        const moe_perf_config_t* config, moe_perf_latency_t* out);

/* Algorithm 2 over the space of Section 6.2: n_disp, n_comb in {4, 8, ..,
 * 4 floor(n_sm / 4)}; n_relay in {1, 5, 9, ..} up to n_disp / 2; n_red in {1, 17,
 * 33, ..} up to n_sm with n_sm itself appended when the steps miss it; warps in
 * {8, 16, 32}.  Invalid configurations are counted in *n_enumerated and skipped.
 * Ties keep the configuration met first in the nested order n_disp, n_relay,
 * n_comb, n_red, warps.  *best_latency receives the winner's intermediates;
 * n_enumerated and n_valid may be NULL.  MOE_ERR_SHAPE if no configuration is
 * valid (n_sm < 6) or hw / problem are out of range. */
int moe_perf_model_search(const moe_perf_hw_t* hw, const moe_perf_problem_t* problem,
                          moe_perf_config_t* best, moe_perf_latency_t* best_latency,
                          int64_t* n_enumerated, int64_t* n_valid);

/* Static string for a return code. */
const char* moe_status_string(int code);

/* Measurement aid, not part of the MoE path: copies `bytes` (a multiple of 16)
 * from src to dst (device pointers, 16-byte aligned, not overlapping) with one
 * plain streaming kernel, `calibration_copy_kernel`.  Its known traffic (bytes
 * read, bytes written) is what the HBM byte counters of a profiler run are
 * scaled by.  Returns MOE_ERR_ARG for a NULL/misaligned pointer or size. */
int moe_calibration_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Measurement aid, not part of the MoE path: `workgroups` workgroups of `waves` waves
 * (1..8) each run `iters` rounds of 8 dependent-free v_mfma_f32_32x32x16_bf16 on operands
 * taken from seed[0..1023] (device, any bit patterns of finite bf16 pairs).  What this
 * reaches is the matrix-core ceiling under the power limit, the denominator the roofline
 * fractions are compared with besides the published peak.
 *   sink    device, 1 float (never written in practice)
 *   clocks  device, 2 x int64: [0] shader clocks, [1] 100 MHz ticks that the first wave
 *           of workgroup 0 spent in the loop: their ratio is the shader clock under load. */
int moe_calibration_mfma(int32_t workgroups, int32_t waves, int32_t iters, const uint32_t* seed,
                         float* sink, long long* clocks, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* UNIEP_MOE_H */
