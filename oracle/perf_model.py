"""CPU oracle of the analytical performance model and the exhaustive configuration
search (Section 4.2, Algorithm 2 and its six equations; search space of
Section 6.2 "Optimization Space Size").

TEST INFRASTRUCTURE, NOT A PRODUCT PATH (same rule as the rest of oracle/).
Plain Python floats (fp64), one function per equation, in the algorithm's order
and notation; nothing is hoisted out of the search loop or vectorised.

Readings of the paper taken here (it does not define the volumes, the tile
counts or the exact ranges):
  * One warp count w per configuration (the five-tuple of Section 6.2), used
    both in the effective bandwidth and in mu(w).
  * X = W * (1 - (1 - 1/W)^k), the expected number of distinct destination
    ranks of a token (5.25 for top-8 on 8 ranks, Section 4.1).
  * V_nvl = N_tok * X * S_tok for dispatch and for combine (Section 4.1).
  * V_hbm of the dispatch = N_tok * (k - X) * S_tok: the copies the relay
    workers make for the slots that did not cross the link.
  * V_hbm_total of the reduce = N_tok * k * S_tok: the k replicas of every token.
  * S_tok = H_dim * bytes per element.
  * Tiles: balanced routing, every rank receives N_tok * k rows spread evenly
    over its N_exp / W experts; rows per expert rounded up, then
    ceil(rows / B_M) row tiles per expert, times ceil(2 H_inter / B_N) column
    tiles for the up GEMM (gate and up side by side) and ceil(H_dim / B_N) for
    the down GEMM.
  * N_disp, N_comb in {4, 8, ..., 4 floor(N_SM / 4)}; N_relay in {1, 5, 9, ...}
    up to N_disp / 2; N_red in {1, 17, 33, ...} up to N_SM, with N_SM itself
    appended when the steps do not reach it (the paper's tuned configurations
    all use N_red = N_SM); w in {8, 16, 32}.
  * A configuration is valid only if it leaves compute workers in both stages
    (N_disp < N_SM, N_comb < N_SM) and N_disp + N_relay < N_SM (the deadlock
    constraint of Section 4.1); invalid ones are enumerated and skipped.
  * Ties keep the configuration met first, in the nested order
    N_disp, N_relay, N_comb, N_red, w (ascending each); Algorithm 2 replaces the
    incumbent only on a strictly smaller latency.
  * w_red = N_red * t_red is taken as printed, although with it a larger N_red
    can only lengthen stage 2, which is at odds with the tuned configurations
    the paper reports.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

WARP_CHOICES = (8, 16, 32)


@dataclass(frozen=True)
class Hardware:
    n_sm: int
    p_peak: float        # FLOP/s
    beta_hbm: float      # B/s
    beta_link: float     # B/s, one direction
    w_sat: int = 1024
    tau_sync: float = 2e-6
    mu: tuple = (0.7, 0.65, 0.6)   # GEMM FLOPs utilisation at w = 8, 16, 32


@dataclass(frozen=True)
class Problem:
    n_tok: int
    h_dim: int
    h_inter: int
    n_exp: int
    top_k: int
    world: int
    b_m: int = 128
    b_n: int = 128
    elem_bytes: int = 2


@dataclass(frozen=True)
class Config:
    n_disp: int
    n_relay: int
    n_comb: int
    n_red: int
    warps: int


def expected_destinations(world: int, top_k: int) -> float:
    return world * (1.0 - (1.0 - 1.0 / world) ** top_k)


def s_tok(p: Problem) -> float:
    return float(p.h_dim * p.elem_bytes)


def v_nvl(p: Problem) -> float:
    return p.n_tok * expected_destinations(p.world, p.top_k) * s_tok(p)


def v_hbm_dispatch(p: Problem) -> float:
    return p.n_tok * (p.top_k - expected_destinations(p.world, p.top_k)) * s_tok(p)


def v_hbm_total(p: Problem) -> float:
    return p.n_tok * p.top_k * s_tok(p)


def row_tiles(p: Problem) -> int:
    e_loc = p.n_exp // p.world
    rows = p.n_tok * p.top_k
    per_expert = -(-rows // e_loc)
    return e_loc * (-(-per_expert // p.b_m))


def n_tiles_up(p: Problem) -> int:
    return row_tiles(p) * (-(-(2 * p.h_inter) // p.b_n))


def n_tiles_down(p: Problem) -> int:
    return row_tiles(p) * (-(-p.h_dim // p.b_n))


def effective_bandwidth(n: int, beta: float, w: int, w_sat: int) -> float:
    """B(n, beta) = min(n w beta / w_sat, beta)  (paragraph "Effective Bandwidth")."""
    return min(n * w * beta / w_sat, beta)


def t_gemm(h: Hardware, p: Problem, k_dim: int, w: int) -> float:
    """One B_M x B_N tile over reduction length K (paragraph "GEMM Block Latency")."""
    mu = h.mu[WARP_CHOICES.index(w)]
    return 2.0 * p.b_m * p.b_n * k_dim / (h.p_peak * (mu / h.n_sm)) + h.tau_sync


def l_swiglu(h: Hardware, p: Problem) -> float:
    return 2.0 * p.n_tok * s_tok(p) / h.beta_hbm


def l_disp(h: Hardware, p: Problem, c: Config) -> float:
    return (v_nvl(p) / effective_bandwidth(c.n_disp, h.beta_link, c.warps, h.w_sat)
            + v_hbm_dispatch(p) / effective_bandwidth(c.n_relay, h.beta_hbm, c.warps, h.w_sat))


def l_comp(n_tiles: int, t_block: float, n_comp: int) -> float:
    return math.ceil(n_tiles / n_comp) * t_block


def l_comb_and_t_red(h: Hardware, p: Problem, c: Config):
    l_comb = v_nvl(p) / effective_bandwidth(c.n_comb, h.beta_link, c.warps, h.w_sat)
    t_red = v_hbm_total(p) / effective_bandwidth(1, h.beta_hbm, c.warps, h.w_sat)
    return l_comb, t_red


def is_valid(h: Hardware, c: Config) -> bool:
    return (c.warps in WARP_CHOICES and 1 <= c.n_disp < h.n_sm and 1 <= c.n_comb < h.n_sm
            and c.n_relay >= 1 and c.n_red >= 1 and c.n_red <= h.n_sm
            and c.n_disp + c.n_relay < h.n_sm)


def evaluate(h: Hardware, p: Problem, c: Config) -> dict:
    """The body of Algorithm 2's loop for one configuration; every intermediate is returned."""
    assert is_valid(h, c)
    # 1. basic operation latencies
    t_up = t_gemm(h, p, p.h_dim, c.warps)
    t_down = t_gemm(h, p, p.h_inter, c.warps)
    l_sw = l_swiglu(h, p)
    # 2. stage 1: dispatch + up GEMM
    n_comp1 = h.n_sm - c.n_disp
    l_d = l_disp(h, p, c)
    l_up = l_comp(n_tiles_up(p), t_up, n_comp1)
    if l_up > l_d:
        l_s1 = l_d + (l_up - l_d) * h.n_sm / n_comp1
    else:
        l_s1 = l_d + t_up
    # 3. stage 2: down GEMM + combine, the reduce fills the gap between the two
    n_comp2 = h.n_sm - c.n_comb
    l_c, t_red = l_comb_and_t_red(h, p, c)
    l_down = l_comp(n_tiles_down(p), t_down, n_comp2)
    l_base = max(l_down, l_c)
    w_gap = abs(l_down - l_c) * n_comp2
    w_red = c.n_red * t_red
    w_rem = max(0.0, w_red - w_gap)
    l_s2 = l_base + w_rem / h.n_sm
    # 4. total
    return {"t_up": t_up, "t_down": t_down, "l_swiglu": l_sw, "l_disp": l_d, "l_up": l_up,
            "l_s1": l_s1, "l_comb": l_c, "t_red": t_red, "l_down": l_down, "l_s2": l_s2,
            "l_total": l_s1 + l_s2 + l_sw}


def comm_choices(n_sm: int):
    return list(range(4, 4 * (n_sm // 4) + 1, 4))


def relay_choices(n_disp: int):
    return list(range(1, n_disp // 2 + 1, 4))


def reduce_choices(n_sm: int):
    r = list(range(1, n_sm + 1, 16))
    if r[-1] != n_sm:
        r.append(n_sm)
    return r


def search_space(h: Hardware):
    """Every configuration of Section 6.2's space, valid or not, in enumeration order."""
    for n_disp in comm_choices(h.n_sm):
        for n_relay in relay_choices(n_disp):
            for n_comb in comm_choices(h.n_sm):
                for n_red in reduce_choices(h.n_sm):
                    for w in WARP_CHOICES:
                        yield Config(n_disp, n_relay, n_comb, n_red, w)


def search(h: Hardware, p: Problem):
    """Algorithm 2: (best configuration, its latency, configurations enumerated, valid ones)."""
    l_min, best = math.inf, None
    n_enum = n_valid = 0
    for c in search_space(h):
        n_enum += 1
        if not is_valid(h, c):
            continue
        n_valid += 1
        l_total = evaluate(h, p, c)["l_total"]
        if l_total < l_min:
            l_min, best = l_total, c
    return best, l_min, n_enum, n_valid
