/*
 * CPU ORACLE for the fused MoE layer  --  TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code, header, table or helper with the HIP
 * library, and nothing here is tuned: every function is the plain definition
 * written as loops, so it can be checked against the paper by eye.
 *
 * What it computes (UniEP paper, Section 2.1 "MoE Training Workflow" and
 * Section 3.1 "Deterministic Token Mapping", Algorithm 1 with one rank):
 *
 *   route     top-k experts per token on raw fp32 logits (larger first, equal
 *             values -> lower expert id first), gate = softmax over all
 *             experts renormalised over the k selected; BinCount, exclusive
 *             CumSum, and the stable (token, slot) order: row of flat slot
 *             f = t*k+j is  offsets[e] + #{same-expert slots f' < f}.
 *   forward   per row r (expert e, token t):  G = x[t] W_gate[e],
 *             U = x[t] W_up[e], h = silu(G)*U, o[r] = h W_down[e];
 *             y[t] = sum_j w[t,j] o[row(t,j)]  with j ascending, local slots only
 *             (the top-k accumulation constraint of Section 3.2: all k
 *             contributions, one fixed order, no partial pre-reduction).
 *   backward  the calculus of the above; weight gradients reduce over an
 *             expert's rows in row order (the "Transposed GroupGEMM" of
 *             Section 2.1, whose accumulation order the token mapping fixes).
 *   route_backward  gradient of the gates with respect to the logits for the
 *             fixed selection, chain rule through renormalisation and softmax.
 *
 * Precision: the accumulate type is ACC_T (this file is built twice, as
 * double and as float).  With round_bf16 != 0 every value the pipeline hands
 * from one stage to the next (h, o, y, dO, dG, dU, dXp, dX, dW) is rounded to
 * bf16, round-to-nearest-even, in one rounding from ACC_T; with 0 nothing is
 * rounded (used by the finite-difference and brute-force pins).
 *
 * Inputs x, dy and the weights come either as bf16 bit patterns (in_dtype 0)
 * or as float64 (in_dtype 1, for the pins that need unquantised inputs).
 * All floating outputs are float64 arrays.  Optional outputs may be NULL.
 *
 * Parity pins: tests/test_oracle_route.py, tests/test_oracle_forward.py,
 * tests/test_oracle_backward.py (brute force, library routines, closed forms,
 * finite differences, autograd).  The paper prints no worked numeric example
 * of y or of a gradient, so absolute values are pinned by those means only.
 */
#ifdef _OPENMP
#include <omp.h>
#endif
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ACC_T
#define ACC_T double
#endif
#ifndef SFX
#define SFX f64
#endif
#define CAT_(a, b) a##_##b
#define CAT(a, b) CAT_(a, b)
#define FN(name) CAT(name, SFX)

typedef ACC_T acc_t;

enum { SH_T = 0, SH_D, SH_E, SH_K, SH_I, SH_ESTART, SH_ECOUNT };

/* ------------------------------------------------------------------ bf16 */

static double bf16_bits_to_double(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* One rounding of v to the nearest bf16 value (8 significant bits, float32's
 * exponent range), ties to even; returned in the accumulate type. */
static acc_t round_to_bf16(acc_t v) {
    double x = (double)v;
    if (x == 0.0 || isnan(x) || isinf(x)) return v;
    int e = ilogb(x);                 /* floor(log2|x|) */
    if (e < -126) e = -126;           /* subnormal range: fixed spacing */
    double q = ldexp(1.0, e - 7);     /* spacing of bf16 values in this binade */
    double r = nearbyint(x / q) * q;  /* default rounding mode = nearest even */
    if (fabs(r) >= ldexp(1.0, 128)) r = (x > 0) ? INFINITY : -INFINITY;
    return (acc_t)r;
}

static inline acc_t maybe_round(acc_t v, int round_bf16) {
    return round_bf16 ? round_to_bf16(v) : v;
}

static void load_slab(const void* src, int in_dtype, size_t off, size_t n, acc_t* dst) {
    if (in_dtype == 0) {
        const uint16_t* p = (const uint16_t*)src + off;
        for (size_t i = 0; i < n; ++i) dst[i] = (acc_t)bf16_bits_to_double(p[i]);
    } else {
        const double* p = (const double*)src + off;
        for (size_t i = 0; i < n; ++i) dst[i] = (acc_t)p[i];
    }
}

/* ----------------------------------------------------------------- route */

/* Section 2.1 (gating) + Algorithm 1 lines 1-2 and the local stable order.
 * perm has T*k entries; entries at and beyond A = offsets[e_count] are -1. */
int FN(oracle_route)(const int32_t* sh, const float* logits, int32_t* topk_idx, float* topk_w,
                     int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm) {
    const int T = sh[SH_T], E = sh[SH_E], k = sh[SH_K];
    const int e_start = sh[SH_ESTART], e_count = sh[SH_ECOUNT];
    if (k > E || k < 1 || e_start < 0 || e_count < 1 || e_start + e_count > E) return -1;
    char* taken = (char*)malloc((size_t)E);
    acc_t* p = (acc_t*)malloc(sizeof(acc_t) * (size_t)E);
    for (int t = 0; t < T; ++t) {
        const float* row = logits + (size_t)t * E;
        /* k rounds of arg-max; strict '>' keeps the lowest index among equals */
        memset(taken, 0, (size_t)E);
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || row[e] > row[best]) best = e;
            }
            taken[best] = 1;
            topk_idx[(size_t)t * k + j] = best;
        }
        /* softmax over all experts, then renormalise the selected k */
        acc_t mx = (acc_t)row[0];
        for (int e = 1; e < E; ++e)
            if ((acc_t)row[e] > mx) mx = (acc_t)row[e];
        acc_t den = 0;
        for (int e = 0; e < E; ++e) {
            p[e] = (acc_t)exp((double)((acc_t)row[e] - mx));
            den += p[e];
        }
        for (int e = 0; e < E; ++e) p[e] = p[e] / den;
        acc_t sel = 0;
        for (int j = 0; j < k; ++j) sel += p[topk_idx[(size_t)t * k + j]];
        for (int j = 0; j < k; ++j)
            topk_w[(size_t)t * k + j] = (float)(p[topk_idx[(size_t)t * k + j]] / sel);
    }
    free(taken);
    free(p);

    /* BinCount over local experts, exclusive CumSum */
    for (int e = 0; e < e_count; ++e) counts[e] = 0;
    const size_t F = (size_t)T * k;
    for (size_t f = 0; f < F; ++f) {
        int el = topk_idx[f] - e_start;
        if (el >= 0 && el < e_count) counts[el]++;
    }
    offsets[0] = 0;
    for (int e = 0; e < e_count; ++e) offsets[e + 1] = offsets[e] + counts[e];
    /* walking the flat slots in increasing f is a stable sort by expert */
    int32_t* cursor = (int32_t*)calloc((size_t)e_count, sizeof(int32_t));
    for (size_t f = 0; f < F; ++f) perm[f] = -1;
    for (size_t f = 0; f < F; ++f) {
        int el = topk_idx[f] - e_start;
        if (el >= 0 && el < e_count) {
            int32_t r = offsets[el] + cursor[el]++;
            inv_perm[f] = r;
            perm[r] = (int32_t)f;
        } else {
            inv_perm[f] = -1;
        }
    }
    free(cursor);
    return 0;
}

/* ------------------------------------------------------- one expert's math */

typedef struct {
    int d, I;
    acc_t *wg, *wu, *wd; /* [d,I], [d,I], [I,d] in the accumulate type */
} expert_w;

static void expert_alloc(expert_w* w, int d, int I) {
    w->d = d;
    w->I = I;
    w->wg = (acc_t*)malloc(sizeof(acc_t) * (size_t)d * I);
    w->wu = (acc_t*)malloc(sizeof(acc_t) * (size_t)d * I);
    w->wd = (acc_t*)malloc(sizeof(acc_t) * (size_t)d * I);
}
static void expert_free(expert_w* w) {
    free(w->wg);
    free(w->wu);
    free(w->wd);
}
static void expert_load(expert_w* w, int in_dtype, const void* wg, const void* wu, const void* wd,
                        int el) {
    size_t n = (size_t)w->d * w->I;
    load_slab(wg, in_dtype, (size_t)el * n, n, w->wg);
    load_slab(wu, in_dtype, (size_t)el * n, n, w->wu);
    load_slab(wd, in_dtype, (size_t)el * n, n, w->wd);
}

static acc_t sigmoid_acc(acc_t z) { return (acc_t)(1.0 / (1.0 + exp(-(double)z))); }

/* G = x W_gate, U = x W_up, h = silu(G)*U, o = h W_down  (one row) */
static void row_forward(const expert_w* w, const acc_t* x, int round_bf16, acc_t* G, acc_t* U,
                        acc_t* h, acc_t* o) {
    const int d = w->d, I = w->I;
    for (int n = 0; n < I; ++n) G[n] = U[n] = 0;
    for (int c = 0; c < d; ++c) {
        const acc_t xv = x[c];
        const acc_t* g = w->wg + (size_t)c * I;
        const acc_t* u = w->wu + (size_t)c * I;
        for (int n = 0; n < I; ++n) {
            G[n] += xv * g[n];
            U[n] += xv * u[n];
        }
    }
    for (int n = 0; n < I; ++n) {
        acc_t silu = G[n] * sigmoid_acc(G[n]); /* z / (1 + e^-z) */
        h[n] = maybe_round(silu * U[n], round_bf16);
    }
    for (int c = 0; c < d; ++c) o[c] = 0;
    for (int n = 0; n < I; ++n) {
        const acc_t hv = h[n];
        const acc_t* wd = w->wd + (size_t)n * d;
        for (int c = 0; c < d; ++c) o[c] += hv * wd[c];
    }
    for (int c = 0; c < d; ++c) o[c] = maybe_round(o[c], round_bf16);
}

/* Given G, U (unrounded) of the row:  dO = gate*dY,  dH = dO W_down^T,
 * dU = dH*silu(G),  dG = dH*U*s*(1+G(1-s)) with s = sigmoid(G),
 * dXp = dG W_gate^T + dU W_up^T. */
static void row_backward(const expert_w* w, const acc_t* dy, acc_t gate, int round_bf16,
                         const acc_t* G, const acc_t* U, acc_t* dO, acc_t* dH, acc_t* dG,
                         acc_t* dU, acc_t* dXp) {
    const int d = w->d, I = w->I;
    for (int c = 0; c < d; ++c) dO[c] = maybe_round(gate * dy[c], round_bf16);
    for (int n = 0; n < I; ++n) {
        const acc_t* wd = w->wd + (size_t)n * d;
        acc_t s = 0;
        for (int c = 0; c < d; ++c) s += dO[c] * wd[c];
        dH[n] = s;
    }
    for (int n = 0; n < I; ++n) {
        acc_t s = sigmoid_acc(G[n]);
        dU[n] = maybe_round(dH[n] * (G[n] * s), round_bf16);
        dG[n] = maybe_round(dH[n] * U[n] * (s * (1 + G[n] * (1 - s))), round_bf16);
    }
    for (int c = 0; c < d; ++c) {
        const acc_t* g = w->wg + (size_t)c * I;
        const acc_t* u = w->wu + (size_t)c * I;
        acc_t sg = 0, su = 0;
        for (int n = 0; n < I; ++n) sg += dG[n] * g[n];
        for (int n = 0; n < I; ++n) su += dU[n] * u[n];
        dXp[c] = maybe_round(sg + su, round_bf16);
    }
}

/* --------------------------------------------------------------- forward */

/* Whole layer.  Optional per-row outputs (NULL to skip): G,U,h [A,I]; o [A,d]. */
int FN(oracle_forward)(const int32_t* sh, int in_dtype, const void* x, const void* wg,
                       const void* wu, const void* wd, const float* topk_w,
                       const int32_t* offsets, const int32_t* perm, const int32_t* inv_perm,
                       int round_bf16, double* y, double* G_out, double* U_out, double* h_out,
                       double* o_out) {
    const int T = sh[SH_T], d = sh[SH_D], k = sh[SH_K], I = sh[SH_I], e_count = sh[SH_ECOUNT];
    const int A = offsets[e_count];
    acc_t* o_all = (acc_t*)malloc(sizeof(acc_t) * (size_t)(A > 0 ? A : 1) * d);
    expert_w w;
    expert_alloc(&w, d, I);
    for (int el = 0; el < e_count; ++el) {
        const int r0 = offsets[el], r1 = offsets[el + 1];
        if (r0 == r1) continue;
        expert_load(&w, in_dtype, wg, wu, wd, el);
#pragma omp parallel
        {
            acc_t* xr = (acc_t*)malloc(sizeof(acc_t) * (size_t)d);
            acc_t* G = (acc_t*)malloc(sizeof(acc_t) * (size_t)I * 3);
            acc_t *U = G + I, *h = G + 2 * (size_t)I;
#pragma omp for schedule(static)
            for (int r = r0; r < r1; ++r) {
                const int t = perm[r] / k;
                load_slab(x, in_dtype, (size_t)t * d, (size_t)d, xr);
                acc_t* o = o_all + (size_t)r * d;
                row_forward(&w, xr, round_bf16, G, U, h, o);
                for (int n = 0; n < I; ++n) {
                    if (G_out) G_out[(size_t)r * I + n] = (double)G[n];
                    if (U_out) U_out[(size_t)r * I + n] = (double)U[n];
                    if (h_out) h_out[(size_t)r * I + n] = (double)h[n];
                }
                if (o_out)
                    for (int c = 0; c < d; ++c) o_out[(size_t)r * d + c] = (double)o[c];
            }
            free(xr);
            free(G);
        }
    }
    expert_free(&w);
    /* combine: all k contributions of a token, slot order, accumulate type */
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int c = 0; c < d; ++c) {
            acc_t acc = 0;
            for (int j = 0; j < k; ++j) {
                const int r = inv_perm[(size_t)t * k + j];
                if (r < 0) continue;
                acc += (acc_t)topk_w[(size_t)t * k + j] * o_all[(size_t)r * d + c];
            }
            y[(size_t)t * d + c] = (double)maybe_round(acc, round_bf16);
        }
    }
    free(o_all);
    return 0;
}

/* The same definition for a list of tokens only (full-size sampled parity).
 * y_rows [n_tok,d]; o_rows [n_tok,k,d] (zeros for non-local slots) or NULL. */
int FN(oracle_forward_tokens)(const int32_t* sh, int in_dtype, const void* x, const void* wg,
                              const void* wu, const void* wd, const int32_t* topk_idx,
                              const float* topk_w, int round_bf16, int n_tok,
                              const int32_t* tok_list, double* y_rows, double* o_rows) {
    const int d = sh[SH_D], k = sh[SH_K], I = sh[SH_I];
    const int e_start = sh[SH_ESTART], e_count = sh[SH_ECOUNT];
#pragma omp parallel
    {
        expert_w w;
        expert_alloc(&w, d, I);
        acc_t* xr = (acc_t*)malloc(sizeof(acc_t) * (size_t)d);
        acc_t* G = (acc_t*)malloc(sizeof(acc_t) * (size_t)I * 3);
        acc_t *U = G + I, *h = G + 2 * (size_t)I;
        acc_t* o = (acc_t*)malloc(sizeof(acc_t) * (size_t)d * k);
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < n_tok; ++i) {
            const int t = tok_list[i];
            load_slab(x, in_dtype, (size_t)t * d, (size_t)d, xr);
            for (int j = 0; j < k; ++j) {
                const int el = topk_idx[(size_t)t * k + j] - e_start;
                acc_t* oj = o + (size_t)j * d;
                if (el < 0 || el >= e_count) {
                    for (int c = 0; c < d; ++c) oj[c] = 0;
                    continue;
                }
                expert_load(&w, in_dtype, wg, wu, wd, el);
                row_forward(&w, xr, round_bf16, G, U, h, oj);
            }
            for (int c = 0; c < d; ++c) {
                acc_t acc = 0;
                for (int j = 0; j < k; ++j) {
                    const int el = topk_idx[(size_t)t * k + j] - e_start;
                    if (el < 0 || el >= e_count) continue;
                    acc += (acc_t)topk_w[(size_t)t * k + j] * o[(size_t)j * d + c];
                }
                y_rows[(size_t)i * d + c] = (double)maybe_round(acc, round_bf16);
            }
            if (o_rows)
                for (size_t q = 0; q < (size_t)k * d; ++q)
                    o_rows[(size_t)i * k * d + q] = (double)o[q];
        }
        free(o);
        free(G);
        free(xr);
        expert_free(&w);
    }
    return 0;
}

/* -------------------------------------------------------------- backward */

/* Rows of one local expert: forward recompute (G,U unrounded, h, o), then the
 * row gradients; weight gradients reduce over the rows in row order. */
typedef struct {
    acc_t *G, *U, *h, *o, *dO, *dH, *dG, *dU, *dXp, *xr;
} rows_buf;

static void rows_alloc(rows_buf* b, int n, int d, int I) {
    size_t nI = (size_t)(n > 0 ? n : 1) * I, nd = (size_t)(n > 0 ? n : 1) * d;
    b->G = (acc_t*)malloc(sizeof(acc_t) * nI);
    b->U = (acc_t*)malloc(sizeof(acc_t) * nI);
    b->h = (acc_t*)malloc(sizeof(acc_t) * nI);
    b->dH = (acc_t*)malloc(sizeof(acc_t) * nI);
    b->dG = (acc_t*)malloc(sizeof(acc_t) * nI);
    b->dU = (acc_t*)malloc(sizeof(acc_t) * nI);
    b->o = (acc_t*)malloc(sizeof(acc_t) * nd);
    b->dO = (acc_t*)malloc(sizeof(acc_t) * nd);
    b->dXp = (acc_t*)malloc(sizeof(acc_t) * nd);
    b->xr = (acc_t*)malloc(sizeof(acc_t) * nd);
}
static void rows_free(rows_buf* b) {
    free(b->G); free(b->U); free(b->h); free(b->dH); free(b->dG); free(b->dU);
    free(b->o); free(b->dO); free(b->dXp); free(b->xr);
}

static void expert_rows_backward(const expert_w* w, int in_dtype, const void* x, const void* dy,
                                 const float* topk_w, const int32_t* perm, int k, int r0, int r1,
                                 int round_bf16, rows_buf* b) {
    const int d = w->d, I = w->I;
#pragma omp parallel
    {
        acc_t* dyr = (acc_t*)malloc(sizeof(acc_t) * (size_t)d);
#pragma omp for schedule(static)
        for (int r = r0; r < r1; ++r) {
            const size_t i = (size_t)(r - r0);
            const int f = perm[r];
            const int t = f / k;
            load_slab(x, in_dtype, (size_t)t * d, (size_t)d, b->xr + i * d);
            load_slab(dy, in_dtype, (size_t)t * d, (size_t)d, dyr);
            row_forward(w, b->xr + i * d, round_bf16, b->G + i * I, b->U + i * I, b->h + i * I,
                        b->o + i * d);
            row_backward(w, dyr, (acc_t)topk_w[f], round_bf16, b->G + i * I, b->U + i * I,
                         b->dO + i * d, b->dH + i * I, b->dG + i * I, b->dU + i * I,
                         b->dXp + i * d);
        }
        free(dyr);
    }
}

/* dW_gate[c][n] = sum_r x[r][c] dG[r][n], dW_up likewise, dW_down[n][c] =
 * sum_r h[r][n] dO[r][c]; r ascending (row order) for every element. */
static void expert_weight_grads(int d, int I, int nrows, const rows_buf* b, int round_bf16,
                                double* dwg, double* dwu, double* dwd) {
#pragma omp parallel for schedule(static)
    for (int c = 0; c < d; ++c) {
        acc_t* ag = (acc_t*)calloc((size_t)I * 2, sizeof(acc_t));
        acc_t* au = ag + I;
        for (int r = 0; r < nrows; ++r) {
            const acc_t xv = b->xr[(size_t)r * d + c];
            const acc_t* dG = b->dG + (size_t)r * I;
            const acc_t* dU = b->dU + (size_t)r * I;
            for (int n = 0; n < I; ++n) {
                ag[n] += xv * dG[n];
                au[n] += xv * dU[n];
            }
        }
        for (int n = 0; n < I; ++n) {
            dwg[(size_t)c * I + n] = (double)maybe_round(ag[n], round_bf16);
            dwu[(size_t)c * I + n] = (double)maybe_round(au[n], round_bf16);
        }
        free(ag);
    }
#pragma omp parallel for schedule(static)
    for (int n = 0; n < I; ++n) {
        acc_t* a = (acc_t*)calloc((size_t)d, sizeof(acc_t));
        for (int r = 0; r < nrows; ++r) {
            const acc_t hv = b->h[(size_t)r * I + n];
            const acc_t* dO = b->dO + (size_t)r * d;
            for (int c = 0; c < d; ++c) a[c] += hv * dO[c];
        }
        for (int c = 0; c < d; ++c) dwd[(size_t)n * d + c] = (double)maybe_round(a[c], round_bf16);
        free(a);
    }
}

/* Whole backward.  dx [T,d]; dwg,dwu [e_count,d,I]; dwd [e_count,I,d];
 * dtopk_w [T,k] (0 for non-local slots); optional per-row dG,dU [A,I], dXp,dO [A,d]. */
int FN(oracle_backward)(const int32_t* sh, int in_dtype, const void* x, const void* dy,
                        const void* wg, const void* wu, const void* wd, const float* topk_w,
                        const int32_t* offsets, const int32_t* perm, const int32_t* inv_perm,
                        int round_bf16, double* dx, double* dwg, double* dwu, double* dwd,
                        double* dtopk_w, double* dG_out, double* dU_out, double* dXp_out,
                        double* dO_out) {
    const int T = sh[SH_T], d = sh[SH_D], k = sh[SH_K], I = sh[SH_I], e_count = sh[SH_ECOUNT];
    const int A = offsets[e_count];
    const size_t wsz = (size_t)d * I;
    acc_t* dxp_all = (acc_t*)malloc(sizeof(acc_t) * (size_t)(A > 0 ? A : 1) * d);
    if (dtopk_w)
        for (size_t f = 0; f < (size_t)T * k; ++f) dtopk_w[f] = 0.0;
    expert_w w;
    expert_alloc(&w, d, I);
    for (int el = 0; el < e_count; ++el) {
        const int r0 = offsets[el], r1 = offsets[el + 1], n = r1 - r0;
        if (n == 0) { /* an expert that received nothing has exactly zero gradient */
            for (size_t q = 0; q < wsz; ++q) dwg[el * wsz + q] = dwu[el * wsz + q] = dwd[el * wsz + q] = 0.0;
            continue;
        }
        expert_load(&w, in_dtype, wg, wu, wd, el);
        rows_buf b;
        rows_alloc(&b, n, d, I);
        expert_rows_backward(&w, in_dtype, x, dy, topk_w, perm, k, r0, r1, round_bf16, &b);
        expert_weight_grads(d, I, n, &b, round_bf16, dwg + el * wsz, dwu + el * wsz, dwd + el * wsz);
        acc_t* dyr = (acc_t*)malloc(sizeof(acc_t) * (size_t)d);
        for (int r = r0; r < r1; ++r) {
            const size_t i = (size_t)(r - r0);
            memcpy(dxp_all + (size_t)r * d, b.dXp + i * d, sizeof(acc_t) * (size_t)d);
            if (dtopk_w) { /* <dY[t], o[r]> */
                const int f = perm[r];
                load_slab(dy, in_dtype, (size_t)(f / k) * d, (size_t)d, dyr);
                acc_t s = 0;
                for (int c = 0; c < d; ++c) s += dyr[c] * b.o[i * d + c];
                dtopk_w[f] = (double)s;
            }
            for (int q = 0; q < I; ++q) {
                if (dG_out) dG_out[(size_t)r * I + q] = (double)b.dG[i * I + q];
                if (dU_out) dU_out[(size_t)r * I + q] = (double)b.dU[i * I + q];
            }
            for (int c = 0; c < d; ++c) {
                if (dXp_out) dXp_out[(size_t)r * d + c] = (double)b.dXp[i * d + c];
                if (dO_out) dO_out[(size_t)r * d + c] = (double)b.dO[i * d + c];
            }
        }
        free(dyr);
        rows_free(&b);
    }
    expert_free(&w);
    /* dX[t] = sum_j dXp[row(t,j)], slot order, local slots only */
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int c = 0; c < d; ++c) {
            acc_t acc = 0;
            for (int j = 0; j < k; ++j) {
                const int r = inv_perm[(size_t)t * k + j];
                if (r < 0) continue;
                acc += dxp_all[(size_t)r * d + c];
            }
            dx[(size_t)t * d + c] = (double)maybe_round(acc, round_bf16);
        }
    }
    free(dxp_all);
    return 0;
}

/* Weight gradients of a list of local experts only (full-size sampled parity).
 * Outputs are packed in list order: dwg,dwu [n_exp,d,I], dwd [n_exp,I,d]. */
int FN(oracle_backward_experts)(const int32_t* sh, int in_dtype, const void* x, const void* dy,
                                const void* wg, const void* wu, const void* wd,
                                const float* topk_w, const int32_t* offsets, const int32_t* perm,
                                int round_bf16, int n_exp, const int32_t* exp_list, double* dwg,
                                double* dwu, double* dwd) {
    const int d = sh[SH_D], k = sh[SH_K], I = sh[SH_I];
    const size_t wsz = (size_t)d * I;
    expert_w w;
    expert_alloc(&w, d, I);
    for (int i = 0; i < n_exp; ++i) {
        const int el = exp_list[i];
        const int r0 = offsets[el], r1 = offsets[el + 1], n = r1 - r0;
        if (n == 0) {
            for (size_t q = 0; q < wsz; ++q) dwg[i * wsz + q] = dwu[i * wsz + q] = dwd[i * wsz + q] = 0.0;
            continue;
        }
        expert_load(&w, in_dtype, wg, wu, wd, el);
        rows_buf b;
        rows_alloc(&b, n, d, I);
        expert_rows_backward(&w, in_dtype, x, dy, topk_w, perm, k, r0, r1, round_bf16, &b);
        expert_weight_grads(d, I, n, &b, round_bf16, dwg + i * wsz, dwu + i * wsz, dwd + i * wsz);
        rows_free(&b);
    }
    expert_free(&w);
    return 0;
}

/* dX rows and dtopk_w rows of a list of tokens only.  dx_rows [n_tok,d],
 * dtopk_w_rows [n_tok,k] (0 for non-local slots). */
int FN(oracle_backward_tokens)(const int32_t* sh, int in_dtype, const void* x, const void* dy,
                               const void* wg, const void* wu, const void* wd,
                               const int32_t* topk_idx, const float* topk_w, int round_bf16,
                               int n_tok, const int32_t* tok_list, double* dx_rows,
                               double* dtopk_w_rows) {
    const int d = sh[SH_D], k = sh[SH_K], I = sh[SH_I];
    const int e_start = sh[SH_ESTART], e_count = sh[SH_ECOUNT];
#pragma omp parallel
    {
        expert_w w;
        expert_alloc(&w, d, I);
        acc_t* xr = (acc_t*)malloc(sizeof(acc_t) * (size_t)d * 4);
        acc_t *dyr = xr + d, *o = xr + 2 * (size_t)d, *dO = xr + 3 * (size_t)d;
        acc_t* G = (acc_t*)malloc(sizeof(acc_t) * (size_t)I * 6);
        acc_t *U = G + I, *h = G + 2 * (size_t)I, *dH = G + 3 * (size_t)I, *dG = G + 4 * (size_t)I,
              *dU = G + 5 * (size_t)I;
        acc_t* dXp = (acc_t*)malloc(sizeof(acc_t) * (size_t)d * k);
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < n_tok; ++i) {
            const int t = tok_list[i];
            load_slab(x, in_dtype, (size_t)t * d, (size_t)d, xr);
            load_slab(dy, in_dtype, (size_t)t * d, (size_t)d, dyr);
            for (int j = 0; j < k; ++j) {
                const size_t f = (size_t)t * k + j;
                const int el = topk_idx[f] - e_start;
                acc_t* dxj = dXp + (size_t)j * d;
                if (el < 0 || el >= e_count) {
                    for (int c = 0; c < d; ++c) dxj[c] = 0;
                    if (dtopk_w_rows) dtopk_w_rows[(size_t)i * k + j] = 0.0;
                    continue;
                }
                expert_load(&w, in_dtype, wg, wu, wd, el);
                row_forward(&w, xr, round_bf16, G, U, h, o);
                row_backward(&w, dyr, (acc_t)topk_w[f], round_bf16, G, U, dO, dH, dG, dU, dxj);
                if (dtopk_w_rows) {
                    acc_t s = 0;
                    for (int c = 0; c < d; ++c) s += dyr[c] * o[c];
                    dtopk_w_rows[(size_t)i * k + j] = (double)s;
                }
            }
            for (int c = 0; c < d; ++c) {
                acc_t acc = 0;
                for (int j = 0; j < k; ++j) {
                    const int el = topk_idx[(size_t)t * k + j] - e_start;
                    if (el < 0 || el >= e_count) continue;
                    acc += dXp[(size_t)j * d + c];
                }
                dx_rows[(size_t)i * d + c] = (double)maybe_round(acc, round_bf16);
            }
        }
        free(dXp);
        free(G);
        free(xr);
        expert_free(&w);
    }
    return 0;
}

/* ---------------------------------------------------------- router gradient
 * Gradient of the gates with respect to the logits, for a fixed selection
 * (Section 2.1: gating scores; the selection itself is piecewise constant).
 * The gate of slot j is  w_j = p_{e_j} / S,  p = softmax(logits[t, :]) over all
 * E experts,  S = sum of p over the k selected experts.  Chain rule, written
 * out without simplification: first the gradient with respect to p, then
 * through the softmax.  dlogits is [T,E] in double. */
int FN(oracle_route_backward)(const int32_t* sh, const float* logits, const int32_t* topk_idx,
                              const float* dtopk_w, double* dlogits) {
    const int T = sh[SH_T], E = sh[SH_E], k = sh[SH_K];
    acc_t* p = (acc_t*)malloc(sizeof(acc_t) * (size_t)E);
    acc_t* dp = (acc_t*)malloc(sizeof(acc_t) * (size_t)E);
    for (int t = 0; t < T; ++t) {
        const float* row = logits + (size_t)t * E;
        const int32_t* sel = topk_idx + (size_t)t * k;
        const float* g = dtopk_w + (size_t)t * k;
        acc_t mx = (acc_t)row[0];
        for (int e = 1; e < E; ++e)
            if ((acc_t)row[e] > mx) mx = (acc_t)row[e];
        acc_t den = 0;
        for (int e = 0; e < E; ++e) {
            p[e] = (acc_t)exp((double)((acc_t)row[e] - mx));
            den += p[e];
        }
        for (int e = 0; e < E; ++e) p[e] = p[e] / den;
        acc_t S = 0;
        for (int j = 0; j < k; ++j) S += p[sel[j]];
        /* d loss / d p_a : w_j = p_{e_j} / S */
        acc_t cross = 0;
        for (int j = 0; j < k; ++j) cross += (acc_t)g[j] * p[sel[j]];
        for (int e = 0; e < E; ++e) dp[e] = 0;
        for (int j = 0; j < k; ++j) dp[sel[j]] = (acc_t)g[j] / S - cross / (S * S);
        /* through the softmax: d p_a / d l_e = p_a (delta_ae - p_e) */
        acc_t dot = 0;
        for (int a = 0; a < E; ++a) dot += dp[a] * p[a];
        for (int e = 0; e < E; ++e) dlogits[(size_t)t * E + e] = (double)(p[e] * (dp[e] - dot));
    }
    free(p);
    free(dp);
    return 0;
}

/* The rounding rule on its own, so a test can pin it against a library cast. */
void FN(oracle_round_bf16)(const double* in, double* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = (double)round_to_bf16((acc_t)in[i]);
}

/* Threads the parallel loops above run on (what omp_get_max_threads() reports in this
 * process): a benchmark that times the oracle states it beside the timing. */
int FN(oracle_max_threads)(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
