"""CPU oracle of the deterministic global token mapping for W > 1 ranks
(Section 3.1, Algorithm 1 and Eq. 1), written out for all ranks at once.

TEST INFRASTRUCTURE, NOT A PRODUCT PATH (same rule as the rest of oracle/).
Plain numpy and Python loops, in the algorithm's order and notation; integer
work only, so every output has exactly one correct value.

Readings of the paper taken here:
  * CumSum is the exclusive prefix sum (the start offset of each expert;
    `loc_idx - O_exp[e]` must be 0 for an expert's first token).
  * O_all is written with three indices in Algorithm 1 and two in Eq. 1; it is
    one table, O_all[r, e] with e = r_tgt * N_epr + e_loc.
  * The segment of expert e_loc in the destination rank's buffer starts at the
    exclusive scan, over that rank's local experts in ascending order, of the
    total rows each receives (contiguous, padding-free storage).
  * A token copy crosses the link once per distinct destination rank
    (Section 3.2, relay multicast): the first slot, in slot order, that targets
    a rank is the one that is sent; later slots for the same rank are local
    copies at the destination.
"""
from __future__ import annotations

import numpy as np


def local_stable_sort_index(e_sel: np.ndarray, n_exp: int):
    """C_exp, exclusive O_exp and M_loc of one rank (Algorithm 1, lines 1-2 and its second
    input): M_loc[t, j] is the position of slot (t, j) in the stable sort of the rank's flat
    slots by expert."""
    flat = np.asarray(e_sel, dtype=np.int64).reshape(-1)
    c_exp = np.zeros(n_exp, dtype=np.int64)
    for e in flat:
        c_exp[e] += 1
    o_exp = np.zeros(n_exp + 1, dtype=np.int64)
    for e in range(n_exp):
        o_exp[e + 1] = o_exp[e] + c_exp[e]
    cursor = o_exp[:-1].copy()
    m_loc = np.empty(flat.shape[0], dtype=np.int64)
    for f, e in enumerate(flat):          # flat slot order f = t * k + j
        m_loc[f] = cursor[e]
        cursor[e] += 1
    return c_exp, o_exp, m_loc.reshape(np.asarray(e_sel).shape)


def global_map(e_sel_per_rank, n_exp: int) -> dict:
    """Algorithm 1 for every rank r of W = len(e_sel_per_rank).

    e_sel_per_rank[r] is rank r's [N_tok_r, k] array of selected experts (token counts may
    differ between ranks).  Returns C_all [W, N_exp], O_all [W, N_exp], recv_offsets
    [W, N_epr + 1] (expert segments of every destination rank) and, per source rank, the arrays
    dst_rank, dst_expert (e_loc), dst_off (final_idx inside the expert's segment), dst_row
    (row of the destination rank's buffer), send (1 = this slot's copy crosses the link) and
    n_dst_ranks [N_tok_r]."""
    W = len(e_sel_per_rank)
    assert n_exp % W == 0
    n_epr = n_exp // W
    local = [local_stable_sort_index(e, n_exp) for e in e_sel_per_rank]
    c_all = np.stack([c for c, _, _ in local])                     # AllGather(C_exp): [W, N_exp]
    o_all = np.zeros((W, n_exp), dtype=np.int64)                   # Eq. 1
    for r in range(1, W):
        o_all[r] = o_all[r - 1] + c_all[r - 1]
    total = c_all.sum(axis=0)
    recv_offsets = np.zeros((W, n_epr + 1), dtype=np.int64)
    for rt in range(W):
        for el in range(n_epr):
            recv_offsets[rt, el + 1] = recv_offsets[rt, el] + total[rt * n_epr + el]
    ranks = []
    for r in range(W):
        e_sel = np.asarray(e_sel_per_rank[r], dtype=np.int64)
        _, o_exp, m_loc = local[r]
        n_tok, k = e_sel.shape
        out = {key: np.zeros((n_tok, k), dtype=np.int32)
               for key in ("dst_rank", "dst_expert", "dst_off", "dst_row", "send")}
        n_dst = np.zeros(n_tok, dtype=np.int32)
        for t in range(n_tok):
            seen = set()
            for j in range(k):
                e_id = int(e_sel[t, j])
                r_tgt, e_loc = e_id // n_epr, e_id % n_epr
                base_off = o_all[r, e_id]
                final_idx = m_loc[t, j] - o_exp[e_id] + base_off
                out["dst_rank"][t, j] = r_tgt
                out["dst_expert"][t, j] = e_loc
                out["dst_off"][t, j] = final_idx
                out["dst_row"][t, j] = recv_offsets[r_tgt, e_loc] + final_idx
                out["send"][t, j] = 0 if r_tgt in seen else 1
                seen.add(r_tgt)
            n_dst[t] = len(seen)
        out["n_dst_ranks"] = n_dst
        out["counts"] = local[r][0].astype(np.int32)
        out["offsets"] = o_exp.astype(np.int32)
        out["m_loc"] = m_loc.astype(np.int32)
        ranks.append(out)
    return {"c_all": c_all.astype(np.int32), "o_all": o_all.astype(np.int32),
            "recv_offsets": recv_offsets.astype(np.int32), "ranks": ranks}
