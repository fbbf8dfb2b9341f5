// Analytical performance model of the expert-parallel MegaKernel and the
// exhaustive configuration search over it (Section 4.2, Algorithm 2 and its
// equations; search space of Section 6.2).  Host code only: the tuner runs once
// per (hardware, problem) on the CPU and its result is cached by the caller.
//
// The latency separates into  L_S1(N_disp, N_relay, w) + L_S2(N_comb, N_red, w) +
// L_swiglu, so the search evaluates each stage once per (stage configuration, w)
// (about a thousand stage evaluations instead of one per configuration) and then
// compares the sums of all pairs in the enumeration order of Algorithm 2's loop.
// All arithmetic is fp64 in the order the equations are printed.
#include "../../include/uniep_moe.h"

#include <cmath>
#include <cstdint>
#include <limits>
#include <vector>

namespace {

constexpr int kWarps[3] = {8, 16, 32};

int warp_slot(int w) {
    for (int i = 0; i < 3; ++i)
        if (kWarps[i] == w) return i;
    return -1;
}

bool hw_ok(const moe_perf_hw_t& h) {
    if (h.n_sm < 2 || h.n_sm > 1024 || h.w_sat < 1) return false;   // the pair walk is O(n_sm^4 / 4096)
    if (!(h.p_peak > 0) || !(h.beta_hbm > 0) || !(h.beta_link > 0) || !(h.tau_sync >= 0)) return false;
    for (int i = 0; i < 3; ++i)
        if (!(h.mu[i] > 0)) return false;
    return true;
}

bool problem_ok(const moe_perf_problem_t& p) {
    return p.n_tok >= 1 && p.h_dim >= 1 && p.h_inter >= 1 && p.n_exp >= 1 && p.top_k >= 1 &&
           p.world >= 1 && p.n_exp % p.world == 0 && p.top_k <= p.n_exp && p.b_m >= 1 && p.b_n >= 1 &&
           p.elem_bytes >= 1;
}

bool config_ok(const moe_perf_hw_t& h, const moe_perf_config_t& c) {
    return warp_slot(c.warps) >= 0 && c.n_disp >= 1 && c.n_disp < h.n_sm && c.n_comb >= 1 &&
           c.n_comb < h.n_sm && c.n_relay >= 1 && c.n_red >= 1 && c.n_red <= h.n_sm &&
           c.n_disp + c.n_relay < h.n_sm;
}

// Volumes and tile counts of a problem (the paper leaves them to the reader): balanced routing,
// X = W (1 - (1 - 1/W)^k) destination ranks per token.
struct Derived {
    double s_tok, v_nvl, v_hbm_disp, v_hbm_total;
    int64_t tiles_up, tiles_down;
};

Derived derive(const moe_perf_problem_t& p) {
    Derived d;
    const double x = p.world * (1.0 - std::pow(1.0 - 1.0 / p.world, p.top_k));
    d.s_tok = (double)((int64_t)p.h_dim * p.elem_bytes);
    d.v_nvl = p.n_tok * x * d.s_tok;
    d.v_hbm_disp = p.n_tok * (p.top_k - x) * d.s_tok;
    d.v_hbm_total = (double)((int64_t)p.n_tok * p.top_k) * d.s_tok;
    const int64_t e_loc = p.n_exp / p.world;
    const int64_t rows = (int64_t)p.n_tok * p.top_k;
    const int64_t per_expert = (rows + e_loc - 1) / e_loc;
    const int64_t row_tiles = e_loc * ((per_expert + p.b_m - 1) / p.b_m);
    d.tiles_up = row_tiles * ((2 * (int64_t)p.h_inter + p.b_n - 1) / p.b_n);
    d.tiles_down = row_tiles * (((int64_t)p.h_dim + p.b_n - 1) / p.b_n);
    return d;
}

// ---- the model, as two kinds of table entry ------------------------------------------------
// The latency of a configuration is (entry of stage 1) + (entry of stage 2) + a constant.  A
// stage-1 entry depends on (N_disp, N_relay, w), a stage-2 entry on (N_comb, N_red, w), and
// nothing couples the two.  Both moe_perf_model_eval and the search are built on the entry
// constructors below: eval makes the two entries of its configuration, the search makes every
// entry once and walks the pairs.  Each constructor states the scheduling picture the
// equations of Section 4.2 describe; the fp64 expressions keep the printed association so that
// both agree with a term-by-term evaluation to the last bit.

// Copy rate that n workers of w warps reach on a path of rate beta: linear in the warps in
// flight until w_sat of them saturate it.
double copy_rate(int n, double beta, int w, int w_sat) { return std::fmin(n * (double)w * beta / w_sat, beta); }

// One tile of b_m x b_n over a reduction of k_dim on one worker's share of the matrix rate
// (scaled by the efficiency mu of that warp count), plus the per-tile synchronisation.
double tile_time(const moe_perf_hw_t& h, const moe_perf_problem_t& p, int k_dim, int w) {
    const double mu = h.mu[warp_slot(w)];
    return 2.0 * p.b_m * p.b_n * k_dim / (h.p_peak * (mu / h.n_sm)) + h.tau_sync;
}

// `tiles` tiles in waves over n workers.
double tiles_on(int64_t tiles, double per_tile, int n) { return (double)((tiles + n - 1) / n) * per_tile; }

struct Stage1Entry {   // tokens arrive (link copy + relay copies) while the up GEMM consumes them
    double arrive, gemm, total;
};
Stage1Entry stage1_entry(const moe_perf_hw_t& h, const Derived& d, int n_disp, int n_relay, int w, double up_tile) {
    Stage1Entry e;
    const int gemm_workers = h.n_sm - n_disp;
    e.arrive = d.v_nvl / copy_rate(n_disp, h.beta_link, w, h.w_sat) +
               d.v_hbm_disp / copy_rate(n_relay, h.beta_hbm, w, h.w_sat);
    e.gemm = tiles_on(d.tiles_up, up_tile, gemm_workers);
    // GEMM outlasts the copies: what is left of it when they end continues on every worker.
    // Copies outlast the GEMM: one more tile after the last token.
    e.total = (e.gemm > e.arrive) ? e.arrive + (e.gemm - e.arrive) * h.n_sm / gemm_workers : e.arrive + up_tile;
    return e;
}

struct Stage2Entry {   // down GEMM next to the combine copies; the reduce fills idle worker time
    double leave, one_reducer, gemm, total;
};
Stage2Entry stage2_entry(const moe_perf_hw_t& h, const Derived& d, int n_comb, int n_red, int w, double down_tile) {
    Stage2Entry e;
    const int gemm_workers = h.n_sm - n_comb;
    e.leave = d.v_nvl / copy_rate(n_comb, h.beta_link, w, h.w_sat);
    e.one_reducer = d.v_hbm_total / copy_rate(1, h.beta_hbm, w, h.w_sat);
    e.gemm = tiles_on(d.tiles_down, down_tile, gemm_workers);
    // Whichever of the two ends first leaves its workers idle for the difference; reduce work
    // beyond that idle worker-time is spread over all workers.
    const double idle_worker_time = std::fabs(e.gemm - e.leave) * gemm_workers;
    const double reduce_work = n_red * e.one_reducer;
    e.total = std::fmax(e.gemm, e.leave) + std::fmax(0.0, reduce_work - idle_worker_time) / h.n_sm;
    return e;
}

// The part no configuration changes: SwiGLU as a pass over the routed activations.
double swiglu_pass(const moe_perf_hw_t& h, const moe_perf_problem_t& p, const Derived& d) {
    return 2.0 * p.n_tok * d.s_tok / h.beta_hbm;
}

void evaluate(const moe_perf_hw_t& h, const moe_perf_problem_t& p, const Derived& d,
              const moe_perf_config_t& c, moe_perf_latency_t* out) {
    out->t_up = tile_time(h, p, p.h_dim, c.warps);
    out->t_down = tile_time(h, p, p.h_inter, c.warps);
    const Stage1Entry a = stage1_entry(h, d, c.n_disp, c.n_relay, c.warps, out->t_up);
    const Stage2Entry b = stage2_entry(h, d, c.n_comb, c.n_red, c.warps, out->t_down);
    out->l_swiglu = swiglu_pass(h, p, d);
    out->l_disp = a.arrive;
    out->l_up = a.gemm;
    out->l_s1 = a.total;
    out->l_comb = b.leave;
    out->t_red = b.one_reducer;
    out->l_down = b.gemm;
    out->l_s2 = b.total;
    out->l_total = out->l_s1 + out->l_s2 + out->l_swiglu;
}

std::vector<int> comm_choices(int n_sm) {
    std::vector<int> v;
    for (int n = 4; n <= 4 * (n_sm / 4); n += 4) v.push_back(n);
    return v;
}
std::vector<int> relay_choices(int n_disp) {
    std::vector<int> v;
    for (int n = 1; n <= n_disp / 2; n += 4) v.push_back(n);
    return v;
}
std::vector<int> reduce_choices(int n_sm) {
    std::vector<int> v;
    for (int n = 1; n <= n_sm; n += 16) v.push_back(n);
    if (v.back() != n_sm) v.push_back(n_sm);
    return v;
}

}  // namespace

extern "C" int moe_perf_model_eval(const moe_perf_hw_t* hw, const moe_perf_problem_t* problem,
                                   const moe_perf_config_t* config, moe_perf_latency_t* out) {
    if (!hw || !problem || !config || !out) return MOE_ERR_ARG;
    if (!hw_ok(*hw) || !problem_ok(*problem) || !config_ok(*hw, *config)) return MOE_ERR_SHAPE;
    const Derived d = derive(*problem);
    evaluate(*hw, *problem, d, *config, out);
    return MOE_OK;
}

extern "C" int moe_perf_model_search(const moe_perf_hw_t* hw, const moe_perf_problem_t* problem,
                                     moe_perf_config_t* best, moe_perf_latency_t* best_latency,
                                     int64_t* n_enumerated, int64_t* n_valid) {
    if (!hw || !problem || !best || !best_latency) return MOE_ERR_ARG;
    if (!hw_ok(*hw) || !problem_ok(*problem)) return MOE_ERR_SHAPE;
    const moe_perf_hw_t& h = *hw;
    const moe_perf_problem_t& p = *problem;
    const Derived d = derive(p);
    const std::vector<int> comm = comm_choices(h.n_sm), red = reduce_choices(h.n_sm);

    // The two tables: every stage entry per warp count, each in the order the nested enumeration
    // (N_disp, N_relay, N_comb, N_red, w) meets them.
    struct S1 { int n_disp, n_relay; double l[3]; };
    struct S2 { int n_comb, n_red; double l[3]; };
    std::vector<S1> s1;
    std::vector<S2> s2;
    int64_t enum1 = 0, enum2 = 0;
    double t_up[3], t_down[3];
    for (int wi = 0; wi < 3; ++wi) {
        t_up[wi] = tile_time(h, p, p.h_dim, kWarps[wi]);
        t_down[wi] = tile_time(h, p, p.h_inter, kWarps[wi]);
    }
    for (int n_disp : comm)
        for (int n_relay : relay_choices(n_disp)) {
            ++enum1;
            if (!(n_disp < h.n_sm && n_disp + n_relay < h.n_sm)) continue;
            S1 c{n_disp, n_relay, {0, 0, 0}};
            for (int wi = 0; wi < 3; ++wi) c.l[wi] = stage1_entry(h, d, n_disp, n_relay, kWarps[wi], t_up[wi]).total;
            s1.push_back(c);
        }
    for (int n_comb : comm)
        for (int n_red : red) {
            ++enum2;
            if (!(n_comb < h.n_sm)) continue;
            S2 c{n_comb, n_red, {0, 0, 0}};
            for (int wi = 0; wi < 3; ++wi) c.l[wi] = stage2_entry(h, d, n_comb, n_red, kWarps[wi], t_down[wi]).total;
            s2.push_back(c);
        }
    if (n_enumerated) *n_enumerated = enum1 * enum2 * 3;
    if (n_valid) *n_valid = (int64_t)s1.size() * (int64_t)s2.size() * 3;
    if (s1.empty() || s2.empty()) return MOE_ERR_SHAPE;   // no configuration leaves compute workers

    // L_total(c) = (L_S1 + L_S2) + L_swiglu in exactly this association, as evaluate() adds it, so
    // the minimum over the product space is taken on the same fp64 values a term-by-term walk
    // would compare.  The space is small enough (about 1e5 sums) to compare every pair, which
    // keeps the tie rule of Algorithm 2 (first strictly smaller total in enumeration order)
    // without any argument about rounding: walk the pairs in enumeration order.
    const double l_sw = swiglu_pass(h, p, d);
    double l_min = std::numeric_limits<double>::infinity();
    size_t bi = 0, bj = 0;
    int bw = 0;
    for (size_t i = 0; i < s1.size(); ++i)
        for (size_t j = 0; j < s2.size(); ++j)
            for (int wi = 0; wi < 3; ++wi) {
                const double l = s1[i].l[wi] + s2[j].l[wi] + l_sw;
                if (l < l_min) {
                    l_min = l;
                    bi = i;
                    bj = j;
                    bw = wi;
                }
            }
    best->n_disp = s1[bi].n_disp;
    best->n_relay = s1[bi].n_relay;
    best->n_comb = s2[bj].n_comb;
    best->n_red = s2[bj].n_red;
    best->warps = kWarps[bw];
    evaluate(h, p, d, *best, best_latency);
    return MOE_OK;
}
