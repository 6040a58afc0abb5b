"""Diagnostics on the oracle's runs: the attention row that each method implies, and its
Hellinger distance (Eq. 7) from the full-attention row.

TEST INFRASTRUCTURE ONLY, like the rest of this package; plain numpy over the oracle's state.

At a generation step the full model spreads probability softmax(q K^T / sqrt(D)) over every token
seen so far.  A sparse policy alone gives the discarded tokens nothing; LESS gives discarded
token j the weight phi(q) psi(k_j)^T of Eq. 3 (H is the sum of psi(k_j)^T v_j, Eq. 6, so that
is v_j's coefficient in the output).  Normalised by Eq. 3's denominator these weights are the
row of the attention matrix the method stands for (Sec. 3.1), and row @ V is its output.

Baseline+ (Sec. 4, "Setup"): the sparse policy alone with 4 more slots, the storage that H
takes at rank 8.
"""
from __future__ import annotations

import numpy as np

from . import less_oracle as lo


def full_row(q, keys):
    """softmax(q K^T / sqrt(D)) over all keys [n,D]."""
    s = keys @ q / np.sqrt(q.shape[0])
    e = np.exp(s - s.max())
    return e / e.sum()


def implied_row(q, keys, cached, f_phi=None, psi_all=None):
    """The row over all n tokens that Eq. 3 stands for.

    keys [n,D] every key seen so far, the current one last; cached: bool [n], True for the pairs
    in K' (the sparse cache and the current token).  f_phi [R] = phi(q) and psi_all [n,R] = psi
    of every key give the discarded tokens their low-rank weight; without them they get 0
    (the sparse policy alone).
    """
    s = keys @ q / np.sqrt(q.shape[0])
    shift = s[cached].max()
    w = np.where(cached, np.exp(np.minimum(s - shift, 0.0)), 0.0)
    if f_phi is not None:
        low = (psi_all @ f_phi) * np.exp(-shift)
        w = np.where(cached, w, low)
    return w / w.sum()


def unit_diagnostics(D, n_heavy, n_recent, rank, hidden, W, inp, flags=0, extra_slots=4):
    """Runs one unit through the oracle three ways and compares the implied rows of every
    generation step with the full-attention row.

    W: the unit's weights Wq1 [D,R'], Wq2 [R',R], Wk1, Wk2, Wk3 [R,R]; inp: Q, K, V [P,D] and
    q, k, v [T,D].  Returns dict of arrays [T]: hellinger_less, hellinger_sparse,
    hellinger_sparse_plus (the policy alone with n_heavy + n_recent + extra_slots slots, split
    evenly), and output_gap [T]: max |row @ V - out| of the LESS run, which ties the rows to the
    oracle's own Eq. 3 output.
    """
    Ws = {k: np.asarray(v, dtype=np.float64)[None] for k, v in W.items()}
    zero = {k: np.zeros_like(v) for k, v in Ws.items()}
    half = extra_slots // 2
    runs = {
        "less": lo.OracleState(1, 1, D, n_heavy, n_recent, rank, hidden, Ws, flags=flags),
        "sparse": lo.OracleState(1, 1, D, n_heavy, n_recent, rank, hidden, zero, flags=flags),
        "sparse_plus": lo.OracleState(1, 1, D, n_heavy + half, n_recent + extra_slots - half, rank, hidden,
                                      zero, flags=flags),
    }
    Q, K, V, q, k, v = (np.asarray(inp[n], dtype=np.float64) for n in ("Q", "K", "V", "q", "k", "v"))
    P, T = K.shape[0], q.shape[0]
    if P:
        for st in runs.values():
            st.prefill(Q[None], K[None], V[None], want_out=False)
    keys = np.concatenate([K, k]); vals = np.concatenate([V, v])
    psi_all = np.stack([lo.psi(kk, Ws["Wk1"][0], Ws["Wk2"][0], Ws["Wk3"][0]) for kk in keys])
    res = {n: np.empty(T) for n in ("hellinger_less", "hellinger_sparse", "hellinger_sparse_plus", "output_gap")}
    for t in range(T):
        n = P + t + 1
        ref = full_row(q[t], keys[:n])
        rows = {}
        for name, st in runs.items():
            cached = np.zeros(n, dtype=bool)
            pos = st.pos[0]
            cached[pos[pos >= 0]] = True
            cached[n - 1] = True
            if name == "less":
                f = lo.phi(q[t], Ws["Wq1"][0], Ws["Wq2"][0])
                rows[name] = implied_row(q[t], keys[:n], cached, f, psi_all[:n])
            else:
                rows[name] = implied_row(q[t], keys[:n], cached)
        outs = {name: st.step(q[t][None], k[t][None], v[t][None])["out"][0] for name, st in runs.items()}
        res["output_gap"][t] = np.abs(rows["less"] @ vals[:n] - outs["less"]).max()
        res["hellinger_less"][t] = lo.hellinger(ref, rows["less"])
        res["hellinger_sparse"][t] = lo.hellinger(ref, rows["sparse"])
        res["hellinger_sparse_plus"][t] = lo.hellinger(ref, rows["sparse_plus"])
    return res
