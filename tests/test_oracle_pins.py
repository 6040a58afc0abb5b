"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of it.

None of these tests touches the HIP library.  Each one names the passage it
rests on.  Sizes are tiny; the whole file runs in seconds.
"""
import os

import numpy as np
import pytest
import torch
from scipy.stats import norm

from oracle import less_oracle as lo
from oracle.less_bruteforce import BruteForceUnit, phi as bf_phi, psi as bf_psi

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as fh:
        return [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]


def make_weights(rng, heads, D, Rp, R, scale=1.0):
    def mat(a, b):
        return rng.standard_normal((heads, a, b)) / np.sqrt(a) * scale
    return {"Wq1": mat(D, Rp), "Wq2": mat(Rp, R), "Wk1": mat(D, Rp), "Wk2": mat(Rp, R),
            "Wk3": mat(R, R)}


def head_w(W, h):
    return {k: v[h] for k, v in W.items()}


def sdpa_last_row(q, K, V):
    """Textbook softmax attention of one query over K, V through torch's SDPA (fp64)."""
    tq = torch.from_numpy(np.asarray(q, dtype=np.float64))[None, None, None, :]
    tk = torch.from_numpy(np.asarray(K, dtype=np.float64))[None, None]
    tv = torch.from_numpy(np.asarray(V, dtype=np.float64))[None, None]
    return torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, 0, 0].numpy()


# ---------------------------------------------------------------- Table 1, Sec. 4
def test_budget_rule_matches_table1():
    for _model, max_len, pct, tokens in _rows("table1_token_counts.txt"):
        assert lo.budget_tokens(float(pct), int(max_len)) == int(tokens)


def test_state_size_equals_four_tokens_at_rank8():
    (R, extra), = _rows("state_size.txt")
    D = 128
    st = lo.OracleState(1, 1, D, 2, 2, int(R), 16,
                        make_weights(np.random.default_rng(0), 1, D, 16, int(R)))
    assert st.H[0].size == int(extra) * 2 * D          # R x D numbers = 4 (key row + value row)


def test_per_head_weights_stay_below_two_percent_of_13b():
    (layers, heads, D, Rp, R, params, frac), = _rows("param_overhead.txt")
    layers, heads, D, Rp, R = map(int, (layers, heads, D, Rp, R))
    W = make_weights(np.random.default_rng(0), 1, D, Rp, R)
    per_head = sum(v[0].size for v in W.values())       # shapes of Eq. 1 / Eq. 2
    total = per_head * heads * layers
    assert total < float(frac) * float(params)
    assert total > 0.01 * float(params)                 # shared-across-heads would be 40x smaller


# ---------------------------------------------------------------- GELU (Sec. 3.2)
def test_gelu_against_normal_cdf_and_identities():
    xs = np.array([-6.0, -3.0, -1.0, -0.25, 0.0, 0.5, 1.0, 2.5, 7.0])
    for x in xs:
        assert lo.gelu(x) == pytest.approx(x * norm.cdf(x), rel=1e-13, abs=1e-300)
        assert lo.gelu(x) - lo.gelu(-x) == pytest.approx(x, rel=1e-14, abs=1e-15)
    assert lo.gelu(1.0) == pytest.approx(0.8413447460685429, rel=1e-14)
    assert lo.gelu(-1.0) == pytest.approx(-0.15865525393145707, rel=1e-13)
    assert lo.gelu(0.0) == 0.0


# ---------------------------------------------------------------- Eq. 1, Eq. 2
def test_feature_maps_scalar_case_by_hand():
    # D = R' = R = 1: phi(q) = |g(g(q a) b)|, psi(k) = |g(g(k a) b) c|
    g = lambda x: x * norm.cdf(x)
    q, a, b, c = 0.7, -1.3, 2.1, -0.6
    f = lo.phi([q], [[a]], [[b]])
    assert f[0] == pytest.approx(abs(g(g(q * a) * b)), rel=1e-13)
    p = lo.psi([q], [[a]], [[b]], [[c]])
    assert p[0] == pytest.approx(abs(g(g(q * a) * b) * c), rel=1e-13)


def test_feature_maps_against_numpy_twin_nonsquare():
    rng = np.random.default_rng(3)
    D, Rp, R = 6, 10, 3                                   # all different: catches transposes
    W = head_w(make_weights(rng, 1, D, Rp, R), 0)
    x = rng.standard_normal(D)
    np.testing.assert_allclose(lo.phi(x, W["Wq1"], W["Wq2"]),
                               bf_phi(x, W["Wq1"], W["Wq2"]), rtol=1e-12)
    np.testing.assert_allclose(lo.psi(x, W["Wk1"], W["Wk2"], W["Wk3"]),
                               bf_psi(x, W["Wk1"], W["Wk2"], W["Wk3"]), rtol=1e-12)
    assert (lo.phi(x, W["Wq1"], W["Wq2"]) >= 0).all()
    assert (lo.psi(x, W["Wk1"], W["Wk2"], W["Wk3"]) >= 0).all()


def test_psi_without_third_matrix_is_abs_of_second_activation():
    # Eq. 2 has no activation after W3; with W3 = I, psi = |g(g(k W1) W2)| = phi with psi's weights
    rng = np.random.default_rng(4)
    D, Rp, R = 5, 7, 4
    W = head_w(make_weights(rng, 1, D, Rp, R), 0)
    x = rng.standard_normal(D)
    np.testing.assert_allclose(lo.psi(x, W["Wk1"], W["Wk2"], np.eye(R)),
                               lo.phi(x, W["Wk1"], W["Wk2"]), rtol=1e-13)
    # and a permutation W3 permutes the outputs (rows of W3 index the input side)
    perm = np.eye(R)[[2, 0, 3, 1]]
    np.testing.assert_allclose(lo.psi(x, W["Wk1"], W["Wk2"], perm),
                               lo.phi(x, W["Wk1"], W["Wk2"]) @ perm, rtol=1e-13)


# ---------------------------------------------------------------- remark after Eq. 3
def _run_prefill_decode(st, Q, K, V, q, k, v):
    pre = st.prefill(Q, K, V)
    outs, evs, shares = [], [], []
    for t in range(q.shape[0]):
        r = st.step(q[t], k[t], v[t])
        outs.append(r["out"]); evs.append(r["evicted"]); shares.append(r["share"])
    return pre, np.array(outs), np.array(evs), np.array(shares)


def test_unbounded_budget_is_full_attention():
    # budget >= P + T: nothing is ever discarded, H = z = 0, so Eq. 3 is softmax attention
    rng = np.random.default_rng(5)
    U, heads, D, Rp, R, P, T = 3, 2, 8, 12, 3, 9, 7
    W = make_weights(rng, heads, D, Rp, R)
    st = lo.OracleState(U, heads, D, 10, 10, R, Rp, W)
    Q, K, V = (rng.standard_normal((U, P, D)) * 1.5 for _ in range(3))
    q, k, v = (rng.standard_normal((T, U, D)) * 1.5 for _ in range(3))
    pre, outs, evs, shares = _run_prefill_decode(st, Q, K, V, q, k, v)
    assert (evs == -1).all() and (shares == 0).all()
    assert pre["kept"].all()
    for u in range(U):
        # prompt phase: causal attention through the library routine
        tq, tk, tv = (torch.from_numpy(a[u])[None, None] for a in (Q, K, V))
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
        np.testing.assert_allclose(pre["out"][u], ref[0, 0].numpy(), rtol=1e-11, atol=1e-13)
        for t in range(T):
            Kall = np.concatenate([K[u], k[:t + 1, u]]); Vall = np.concatenate([V[u], v[:t + 1, u]])
            np.testing.assert_allclose(outs[t, u], sdpa_last_row(q[t, u], Kall, Vall),
                                       rtol=1e-11, atol=1e-13)


def test_prompt_column_sums_are_attention_mass():
    # every causal row is a probability vector: column sums add up to P, and the
    # last token's column sum is its own diagonal entry
    rng = np.random.default_rng(6)
    U, D, P = 2, 4, 11
    W = make_weights(rng, 1, D, 6, 2)
    st = lo.OracleState(U, 1, D, 2, 2, 2, 6, W)
    Q, K, V = (rng.standard_normal((U, P, D)) for _ in range(3))
    pre = st.prefill(Q, K, V)
    np.testing.assert_allclose(pre["colsum"].sum(axis=1), P, rtol=1e-13)
    for u in range(U):
        S = Q[u] @ K[u].T / np.sqrt(D)
        last = np.exp(S[P - 1] - np.logaddexp.reduce(S[P - 1]))
        assert pre["colsum"][u, P - 1] == pytest.approx(last[P - 1], rel=1e-12)
        assert pre["colsum"][u, 0] >= 1.0                # first row attends only to token 0


def test_zero_feature_maps_is_pure_h2o():
    # f = 0 removes both low-rank terms of Eq. 3: softmax over the retained pairs + the new one
    rng = np.random.default_rng(7)
    U, heads, D, Rp, R, P, T = 2, 2, 8, 8, 2, 20, 12
    W = make_weights(rng, heads, D, Rp, R)
    W["Wq2"] = np.zeros_like(W["Wq2"])
    st = lo.OracleState(U, heads, D, 3, 3, R, Rp, W)
    Q, K, V = (rng.standard_normal((U, P, D)) for _ in range(3))
    q, k, v = (rng.standard_normal((T, U, D)) for _ in range(3))
    st.prefill(Q, K, V)
    for t in range(T):
        Kc, Vc, live = st.Kc.copy(), st.Vc.copy(), st.pos >= 0
        r = st.step(q[t], k[t], v[t])
        assert (r["share"] == 0).all()
        for u in range(U):
            Kp = np.concatenate([Kc[u][live[u]], k[t, u][None]])
            Vp = np.concatenate([Vc[u][live[u]], v[t, u][None]])
            np.testing.assert_allclose(r["out"][u], sdpa_last_row(q[t, u], Kp, Vp), rtol=1e-11)
    assert (st.z > 0).any()                              # the state still accumulates (psi != 0)


# ---------------------------------------------------------------- Eq. 4-6, Alg. 1
@pytest.mark.parametrize("Nh,Nr,P,T,flags,seed", [
    (3, 3, 17, 25, 0, 0), (3, 3, 17, 25, 1, 1), (4, 0, 9, 14, 0, 2), (0, 5, 12, 14, 0, 3),
    (2, 6, 0, 30, 0, 4), (5, 2, 4, 20, 1, 5), (1, 1, 30, 10, 0, 6), (8, 8, 64, 24, 0, 7),
    # Lambda-masking (flag bit 1), alone and with the sparse-denominator reading
    (4, 6, 21, 25, 2, 8), (4, 6, 0, 30, 2, 9), (3, 0, 9, 12, 2, 10), (0, 5, 12, 14, 2, 11),
    (2, 3, 4, 20, 3, 12),
])
def test_against_set_based_twin(Nh, Nr, P, T, flags, seed):
    """Outputs, eviction log, kept set and state equal the brute-force simulator's."""
    rng = np.random.default_rng(100 + seed)
    U, heads, D, Rp, R = 3, 2, 6, 9, 3
    W = make_weights(rng, heads, D, Rp, R)
    st = lo.OracleState(U, heads, D, Nh, Nr, R, Rp, W, flags=flags)
    Q, K, V = (rng.standard_normal((U, P, D)) for _ in range(3))
    q, k, v = (rng.standard_normal((T, U, D)) for _ in range(3))
    twins = [BruteForceUnit(D, Nh, Nr, head_w(W, u % heads), sparse_denominator=bool(flags & 1),
                            policy="lambda" if flags & 2 else "h2o")
             for u in range(U)]
    if P:
        pre = st.prefill(Q, K, V)
        for u, tw in enumerate(twins):
            np.testing.assert_allclose(pre["out"][u], tw.prefill(Q[u], K[u], V[u]), rtol=1e-10)
            assert set(np.flatnonzero(pre["kept"][u])) == tw.alive
    else:
        st.reset()
    for t in range(T):
        r = st.step(q[t], k[t], v[t])
        for u, tw in enumerate(twins):
            o, ev = tw.step(q[t, u], k[t, u], v[t, u])
            assert r["evicted"][u] == ev, (t, u)
            np.testing.assert_allclose(r["out"][u], o, rtol=1e-9, atol=1e-12)
            assert set(st.pos[u][st.pos[u] >= 0]) == tw.alive
            Hc, zc = tw.state()                           # Eq. 6, rebuilt from the whole history
            np.testing.assert_allclose(st.H[u], Hc, rtol=1e-10, atol=1e-13)
            np.testing.assert_allclose(st.z[u], zc, rtol=1e-10, atol=1e-13)
            for j in np.flatnonzero(st.pos[u] >= 0):
                assert st.acc[u, j] == pytest.approx(tw.score[int(st.pos[u, j])], rel=1e-10)


@pytest.mark.parametrize("P", [0, 5, 40])
def test_lambda_masking_keeps_the_first_and_the_latest_tokens(P):
    """Sec. 4, "Setup": under Lambda-masking the cache is the first tokens plus the most
    recent ones.  That fixes everything about the policy in closed form: after n tokens the
    cache is {0..Nh-1} and {n-Nr..n-1}, token n-Nr leaves when token n arrives, and H, z
    are Eq. 6 over positions Nh..n-Nr-1; the output is Eq. 3 written out over those sets."""
    rng = np.random.default_rng(21 + P)
    U, heads, D, Rp, R, Nh, Nr, T = 2, 2, 6, 10, 3, 4, 7, 30
    W = make_weights(rng, heads, D, Rp, R)
    st = lo.OracleState(U, heads, D, Nh, Nr, R, Rp, W, flags=2)
    Q, K, V = (rng.standard_normal((U, P, D)) for _ in range(3))
    q, k, v = (rng.standard_normal((T, U, D)) for _ in range(3))
    if P:
        pre = st.prefill(Q, K, V)
        want = np.zeros(P, bool); want[:Nh] = True; want[max(P - Nr, 0):] = True
        if P <= Nh + Nr:
            want[:] = True
        assert (pre["kept"] == want).all()
    else:
        st.reset()
    keys = [[K[u, i] for i in range(P)] for u in range(U)]
    vals = [[V[u, i] for i in range(P)] for u in range(U)]
    for t in range(T):
        n = P + t
        r = st.step(q[t], k[t], v[t])
        for u in range(U):
            Wh = head_w(W, u % heads)
            cached = sorted(set(range(min(Nh, n))) | set(range(max(n - Nr, 0), n)))
            if n <= Nh + Nr:
                cached = list(range(n))
            gone = [p for p in range(n) if p not in cached]
            keys[u].append(k[t, u]); vals[u].append(v[t, u])
            g = [bf_psi(keys[u][p], Wh["Wk1"], Wh["Wk2"], Wh["Wk3"]) for p in gone]
            H = sum((np.outer(gp, vals[u][p]) for gp, p in zip(g, gone)), np.zeros((R, D)))
            z = sum(g, np.zeros(R))
            f = bf_phi(q[t, u], Wh["Wq1"], Wh["Wq2"])
            w = np.array([np.exp(q[t, u] @ keys[u][p] / np.sqrt(D)) for p in cached + [n]])
            num = f @ H + w @ np.array([vals[u][p] for p in cached + [n]])
            np.testing.assert_allclose(r["out"][u], num / (f @ z + w.sum()), rtol=1e-9, atol=1e-12)
            assert r["evicted"][u] == (n - Nr if n >= Nh + Nr else -1)
    n = P + T
    for u in range(U):
        assert sorted(st.pos[u]) == list(range(Nh)) + list(range(n - Nr, n))


@pytest.mark.parametrize("flags", [4, 6])
def test_stepwise_prompt_is_the_generation_loop(flags):
    """Sec. 4.1's setting: the sparse policy acts from the first token on.  The prompt phase
    is then nothing but Algorithm 1 applied to every prompt token: same outputs, evictions and
    state as the set-based twin stepping through the prompt from an empty cache."""
    rng = np.random.default_rng(31 + flags)
    U, heads, D, Rp, R, Nh, Nr, P, T = 3, 2, 6, 9, 3, 3, 4, 25, 6
    W = make_weights(rng, heads, D, Rp, R)
    st = lo.OracleState(U, heads, D, Nh, Nr, R, Rp, W, flags=flags)
    Q, K, V = (rng.standard_normal((U, P, D)) for _ in range(3))
    q, k, v = (rng.standard_normal((T, U, D)) for _ in range(3))
    pre = st.prefill(Q, K, V)
    twins = [BruteForceUnit(D, Nh, Nr, head_w(W, u % heads), policy="lambda" if flags & 2 else "h2o")
             for u in range(U)]
    for u, tw in enumerate(twins):
        for t in range(P):
            o, _ = tw.step(Q[u, t], K[u, t], V[u, t])
            np.testing.assert_allclose(pre["out"][u, t], o, rtol=1e-9, atol=1e-12)
        assert set(st.pos[u][st.pos[u] >= 0]) == tw.alive and st.n[u] == P
        Hc, zc = tw.state()
        np.testing.assert_allclose(st.H[u], Hc, rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(st.z[u], zc, rtol=1e-10, atol=1e-13)
    for t in range(T):                                    # and generation carries on from there
        r = st.step(q[t], k[t], v[t])
        for u, tw in enumerate(twins):
            o, ev = tw.step(q[t, u], k[t, u], v[t, u])
            assert r["evicted"][u] == ev
            np.testing.assert_allclose(r["out"][u], o, rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("Nh,Nr,flags", [(3, 4, 6), (0, 5, 6), (4, 0, 6), (2, 6, 7)])
def test_lambda_masking_through_the_prompt_is_a_masked_attention_matrix(Nh, Nr, flags):
    """Under Lambda-masking the cache token t meets is known beforehand (tokens 0..Nh-1 and
    t-Nr..t-1), so the token-by-token walk equals one masked matrix (Sec. 3.2 builds it for
    training): e^{q_t k_j / sqrt(D)} where pair j is cached or is t itself, phi(q_t) psi(k_j)^T
    where it was discarded; out = row V / row 1.  Accumulated scores are the column sums of the
    cached entries over the normalisation of the flags' reading; slots follow in-place replacement."""
    rng = np.random.default_rng(77 + Nh + Nr)
    U, heads, D, Rp, R, P = 2, 2, 6, 9, 3, 23
    W = make_weights(rng, heads, D, Rp, R)
    st = lo.OracleState(U, heads, D, Nh, Nr, R, Rp, W, flags=flags)
    Q, K, V = (rng.standard_normal((U, P, D)) for _ in range(3))
    pre = st.prefill(Q, K, V)
    t_idx, j_idx = np.arange(P)[:, None], np.arange(P)[None, :]
    causal = j_idx <= t_idx
    cached = causal & ((j_idx < Nh) | (j_idx >= t_idx - Nr))
    for u in range(U):
        w = head_w(W, u % heads)
        F = np.stack([bf_phi(Q[u, t], w["Wq1"], w["Wq2"]) for t in range(P)])
        G = np.stack([bf_psi(K[u, j], w["Wk1"], w["Wk2"], w["Wk3"]) for j in range(P)])
        E = np.where(cached, np.exp(Q[u] @ K[u].T / np.sqrt(D)), 0.0)
        Lr = np.where(causal & ~cached, F @ G.T, 0.0)
        A = E + Lr
        np.testing.assert_allclose(pre["out"][u], (A @ V[u]) / A.sum(1, keepdims=True), rtol=1e-9, atol=1e-12)
        den = E.sum(1) if flags & 1 else A.sum(1)
        col = (E / den[:, None]).sum(0)
        for s_ in np.flatnonzero(st.pos[u] >= 0):
            j = int(st.pos[u, s_])
            assert st.acc[u, s_] == pytest.approx(col[j], rel=1e-10)
            assert s_ == (j if j < Nh else Nh + (j - Nh) % Nr)
        kept = sorted(st.pos[u][st.pos[u] >= 0])
        assert kept == list(range(Nh)) + list(range(P - Nr, P))
        gone = [j for j in range(Nh, P - Nr)]
        np.testing.assert_allclose(st.H[u], G[gone].T @ V[u][gone], rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(st.z[u], G[gone].sum(0), rtol=1e-10, atol=1e-13)


# ---------------------------------------------------------------- several query heads per KV head
def make_weights_gqa(rng, heads, G, D, Rp, R):
    W = make_weights(rng, heads, D, Rp, R)
    Wq = make_weights(rng, heads * G, D, Rp, R)
    W["Wq1"], W["Wq2"] = Wq["Wq1"], Wq["Wq2"]
    return W


@pytest.mark.parametrize("G,Nh,Nr,P,T,flags,seed", [
    (2, 3, 3, 17, 20, 0, 0), (3, 4, 0, 9, 14, 1, 1), (4, 2, 5, 0, 25, 0, 2), (2, 4, 6, 21, 12, 2, 3),
    (3, 3, 4, 19, 8, 4, 4),
])
def test_query_groups_against_set_based_twin(G, Nh, Nr, P, T, flags, seed):
    """Sec. 3.2: with several query heads per key/value head the sparse policy sees the attention
    mass of all of them.  Outputs per query head, evictions and state equal the twin's."""
    rng = np.random.default_rng(300 + seed)
    U, heads, D, Rp, R = 3, 2, 6, 9, 3
    W = make_weights_gqa(rng, heads, G, D, Rp, R)
    st = lo.OracleState(U, heads, D, Nh, Nr, R, Rp, W, flags=flags, q_per_kv=G)
    Q = rng.standard_normal((U, G, P, D)); K, V = (rng.standard_normal((U, P, D)) for _ in range(2))
    q = rng.standard_normal((T, U, G, D)); k, v = (rng.standard_normal((T, U, D)) for _ in range(2))
    def twin_w(u):
        h = u % heads
        w = head_w(W, h)
        w["Wq1"], w["Wq2"] = W["Wq1"][h * G:(h + 1) * G], W["Wq2"][h * G:(h + 1) * G]
        return w
    twins = [BruteForceUnit(D, Nh, Nr, twin_w(u), sparse_denominator=bool(flags & 1),
                            policy="lambda" if flags & 2 else "h2o", q_per_kv=G) for u in range(U)]
    if P:
        pre = st.prefill(Q, K, V)
        for u, tw in enumerate(twins):
            if flags & 4:                                    # the policy runs through the prompt
                for t in range(P):
                    o, _ = tw.step(Q[u, :, t], K[u, t], V[u, t])
                    np.testing.assert_allclose(pre["out"][u, :, t], o, rtol=1e-9, atol=1e-12)
            else:
                np.testing.assert_allclose(pre["out"][u], tw.prefill(Q[u], K[u], V[u]), rtol=1e-10)
            assert set(st.pos[u][st.pos[u] >= 0]) == tw.alive
    else:
        st.reset()
    for t in range(T):
        r = st.step(q[t], k[t], v[t])
        for u, tw in enumerate(twins):
            o, ev = tw.step(q[t, u], k[t, u], v[t, u])
            assert r["evicted"][u] == ev, (t, u)
            np.testing.assert_allclose(r["out"][u], o, rtol=1e-9, atol=1e-12)
            Hc, zc = tw.state()
            np.testing.assert_allclose(st.H[u], Hc, rtol=1e-10, atol=1e-13)
            np.testing.assert_allclose(st.z[u], zc, rtol=1e-10, atol=1e-13)
            for j in np.flatnonzero(st.pos[u] >= 0):
                assert st.acc[u, j] == pytest.approx(tw.score[int(st.pos[u, j])], rel=1e-10)


def test_identical_query_heads_behave_as_one():
    """Two query heads with the same query and the same phi see the same probabilities, so
    every accumulated score is twice the single-head one: same outputs, same evictions,
    same state as the single-head run."""
    rng = np.random.default_rng(41)
    U, heads, D, Rp, R, Nh, Nr, P, T = 2, 2, 6, 8, 3, 3, 3, 15, 20
    W1 = make_weights(rng, heads, D, Rp, R)
    W2 = dict(W1); W2["Wq1"] = np.repeat(W1["Wq1"], 2, axis=0); W2["Wq2"] = np.repeat(W1["Wq2"], 2, axis=0)
    one = lo.OracleState(U, heads, D, Nh, Nr, R, Rp, W1)
    two = lo.OracleState(U, heads, D, Nh, Nr, R, Rp, W2, q_per_kv=2)
    Q, K, V = (rng.standard_normal((U, P, D)) for _ in range(3))
    q, k, v = (rng.standard_normal((T, U, D)) for _ in range(3))
    p1 = one.prefill(Q, K, V); p2 = two.prefill(np.stack([Q, Q], axis=1), K, V)
    assert (p1["kept"] == p2["kept"]).all()
    np.testing.assert_array_equal(p2["out"][:, 0], p1["out"]); np.testing.assert_array_equal(p2["out"][:, 1], p1["out"])
    for t in range(T):
        r1 = one.step(q[t], k[t], v[t]); r2 = two.step(np.stack([q[t], q[t]], axis=1), k[t], v[t])
        assert (r1["evicted"] == r2["evicted"]).all()
        np.testing.assert_array_equal(r2["out"][:, 0], r1["out"]); np.testing.assert_array_equal(r2["out"][:, 1], r1["out"])
        np.testing.assert_allclose(two.acc, 2.0 * one.acc, rtol=1e-14)
        np.testing.assert_array_equal(two.H, one.H); np.testing.assert_array_equal(two.z, one.z)


def test_query_groups_with_unbounded_budget_are_full_attention_per_head():
    rng = np.random.default_rng(42)
    U, heads, G, D, Rp, R, P, T = 2, 1, 3, 8, 8, 2, 9, 5
    W = make_weights_gqa(rng, heads, G, D, Rp, R)
    st = lo.OracleState(U, heads, D, 40, 40, R, Rp, W, q_per_kv=G)
    Q = rng.standard_normal((U, G, P, D)); K, V = (rng.standard_normal((U, P, D)) for _ in range(2))
    q = rng.standard_normal((T, U, G, D)); k, v = (rng.standard_normal((T, U, D)) for _ in range(2))
    pre = st.prefill(Q, K, V)
    for u in range(U):
        for g in range(G):
            for i in range(P):
                np.testing.assert_allclose(pre["out"][u, g, i], sdpa_last_row(Q[u, g, i], K[u, :i + 1], V[u, :i + 1]),
                                           rtol=1e-11)
    Ks, Vs = K.copy(), V.copy()
    for t in range(T):
        r = st.step(q[t], k[t], v[t])
        Ks = np.concatenate([Ks, k[t][:, None]], axis=1); Vs = np.concatenate([Vs, v[t][:, None]], axis=1)
        for u in range(U):
            for g in range(G):
                np.testing.assert_allclose(r["out"][u, g], sdpa_last_row(q[t, u, g], Ks[u], Vs[u]), rtol=1e-11)


def test_policy_invariants_and_convexity():
    rng = np.random.default_rng(11)
    U, heads, D, Rp, R, Nh, Nr, P, T = 4, 2, 8, 16, 4, 4, 4, 30, 40
    W = make_weights(rng, heads, D, Rp, R)
    st = lo.OracleState(U, heads, D, Nh, Nr, R, Rp, W)
    Q, K, V = (rng.standard_normal((U, P, D)) for _ in range(3))
    q, k, v = (rng.standard_normal((T, U, D)) for _ in range(3))
    pre = st.prefill(Q, K, V)
    evicted = [set(np.flatnonzero(~pre["kept"][u])) for u in range(U)]
    vmin, vmax = V.min(axis=1), V.max(axis=1)
    for t in range(T):
        n = P + t
        r = st.step(q[t], k[t], v[t])
        vmin = np.minimum(vmin, v[t]); vmax = np.maximum(vmax, v[t])
        # a-hat is a convex combination of every value seen so far (nonnegative weights)
        assert (r["out"] >= vmin - 1e-12).all() and (r["out"] <= vmax + 1e-12).all()
        assert ((r["share"] > 0) & (r["share"] < 1)).all()
        for u in range(U):
            assert r["evicted"][u] >= 0                   # full cache: exactly one pair leaves
            assert r["evicted"][u] <= n - Nr              # never a recent token
            evicted[u].add(int(r["evicted"][u]))
            kept = set(st.pos[u][st.pos[u] >= 0])
            assert len(kept) == Nh + Nr
            assert kept.isdisjoint(evicted[u]) and kept | evicted[u] == set(range(n + 1))
            assert set(range(n - Nr + 1, n + 1)) <= kept  # the Nr most recent are cached
            assert st.n[u] == n + 1


def test_probabilities_of_a_step_sum_to_one():
    # while the cache is filling nothing is overwritten, so the step's increments of the
    # accumulated scores are the sparse probabilities; with the low-rank share they sum to 1
    rng = np.random.default_rng(12)
    U, D, Rp, R = 2, 6, 8, 3
    W = make_weights(rng, 1, D, Rp, R)
    st = lo.OracleState(U, 1, D, 20, 20, R, Rp, W)
    st.reset()
    # give the state something: pretend a few pairs were discarded earlier
    st.z[:] = rng.random((U, R)) * 5; st.H[:] = rng.standard_normal((U, R, D))
    for t in range(6):
        before = st.acc.sum(axis=1)
        r = st.step(*(rng.standard_normal((U, D)) for _ in range(3)))
        np.testing.assert_allclose(st.acc.sum(axis=1) - before + r["share"], 1.0, rtol=1e-12)
    st.flags = lo.FLAG_SPARSE_DENOM                      # other reading: sparse part sums to 1
    before = st.acc.sum(axis=1)
    st.step(*(rng.standard_normal((U, D)) for _ in range(3)))
    np.testing.assert_allclose(st.acc.sum(axis=1) - before, 1.0, rtol=1e-12)


def test_low_rank_term_by_hand():
    # one cached pair, D = 1, R = 1: a-hat = (f H + e^{q k0} v0 + e^{q k1} v1) / (f z + e^{q k0} + e^{q k1})
    g = lambda x: x * norm.cdf(x)
    W = {"Wq1": [[[1.5]]], "Wq2": [[[-0.8]]], "Wk1": [[[1.0]]], "Wk2": [[[1.0]]], "Wk3": [[[1.0]]]}
    st = lo.OracleState(1, 1, 1, 1, 1, 1, 1, W)
    st.reset()
    st.step([[0.3]], [[0.9]], [[2.0]])                    # caches (k0, v0) = (0.9, 2.0)
    st.H[0, 0, 0] = 0.75; st.z[0, 0] = 0.4                # a state as if something was discarded
    q, k1, v1 = -1.1, 0.2, -3.0
    r = st.step([[q]], [[k1]], [[v1]])
    f = abs(g(g(q * 1.5) * -0.8))
    e0, e1 = np.exp(q * 0.9), np.exp(q * k1)
    assert r["out"][0, 0] == pytest.approx((f * 0.75 + e0 * 2.0 + e1 * v1) / (f * 0.4 + e0 + e1),
                                           rel=1e-13)
    assert r["share"][0] == pytest.approx(f * 0.4 / (f * 0.4 + e0 + e1), rel=1e-13)


def test_large_scores_do_not_overflow():
    # Eq. 3 is printed unshifted; the oracle's common shift must give the same ratio
    rng = np.random.default_rng(13)
    U, D, Rp, R, P, T = 1, 8, 8, 2, 12, 5
    W = make_weights(rng, 1, D, Rp, R)
    st = lo.OracleState(U, 1, D, 20, 20, R, Rp, W)
    Q, K, V = (rng.standard_normal((U, P, D)) * 40 for _ in range(3))
    q, k, v = (rng.standard_normal((T, U, D)) * 40 for _ in range(3))
    pre, outs, _, _ = _run_prefill_decode(st, Q, K, V, q, k, v)
    assert np.isfinite(outs).all() and np.isfinite(pre["out"]).all()
    for t in range(T):
        Kall = np.concatenate([K[0], k[:t + 1, 0]]); Vall = np.concatenate([V[0], v[:t + 1, 0]])
        np.testing.assert_allclose(outs[t, 0], sdpa_last_row(q[t, 0], Kall, Vall), rtol=1e-10)
    # very negative scores with a live state: the low-rank term must dominate, not vanish
    st2 = lo.OracleState(1, 1, D, 2, 2, R, Rp, W)
    st2.reset(); st2.z[:] = 1.0; st2.H[:] = 3.0
    qq = np.full((1, D), 50.0); kk = np.full((1, D), -50.0)
    r = st2.step(qq, kk, np.zeros((1, D)))
    assert np.isfinite(r["out"]).all() and r["share"][0] == pytest.approx(1.0)
    np.testing.assert_allclose(r["out"][0], 3.0, rtol=1e-12)   # f H / f z = 3


def test_forced_eviction_protocol():
    rng = np.random.default_rng(14)
    U, D, Rp, R, Nh, Nr, P = 2, 4, 6, 2, 3, 2, 10
    W = make_weights(rng, 1, D, Rp, R)
    a = lo.OracleState(U, 1, D, Nh, Nr, R, Rp, W); b = lo.OracleState(U, 1, D, Nh, Nr, R, Rp, W)
    Q, K, V = (rng.standard_normal((U, P, D)) for _ in range(3))
    a.prefill(Q, K, V); b.prefill(Q, K, V)
    x = [rng.standard_normal((U, D)) for _ in range(3)]
    ra = a.step(*x)
    second = ra["dec"][:, 3].astype(np.int64)
    assert (ra["dec"][:, 1] == ra["evicted"]).all()
    assert (ra["dec"][:, 0] <= ra["dec"][:, 2]).all()
    rb = b.step(*x, force=second)                         # take the runner-up instead
    assert (rb["evicted"] == second).all()
    np.testing.assert_array_equal(ra["out"], rb["out"])   # the output precedes the cache update
    for u in range(U):
        assert second[u] not in b.pos[u] and ra["evicted"][u] in b.pos[u]
    with pytest.raises(ValueError):
        b.step(*x, force=np.array([P + 1, -1]))           # a recent token is no candidate


def test_tie_evicts_the_older_token():
    # identical keys get identical probabilities; with equal scores the older one goes
    D, Rp, R = 4, 4, 2
    W = make_weights(np.random.default_rng(15), 1, D, Rp, R)
    st = lo.OracleState(1, 1, D, 2, 1, R, Rp, W)
    st.reset()
    kk = np.ones((1, D)); vv = np.ones((1, D))
    for _ in range(3):
        st.step(np.zeros((1, D)), kk, vv)                 # q = 0: uniform attention
    st.acc[0, :2] = 0.5; st.acc[0, 2] = 5.0               # exact tie between positions 0 and 1
    r = st.step(np.zeros((1, D)), kk, vv)
    assert r["evicted"][0] == 0 and r["dec"][0, 0] == r["dec"][0, 2]


# ---------------------------------------------------------------- Eq. 7
def test_hellinger_distance():
    assert lo.hellinger([0.2, 0.3, 0.5], [0.2, 0.3, 0.5]) == 0.0
    assert lo.hellinger([1.0, 0.0], [0.0, 1.0]) == pytest.approx(1.0)
    # H^2 = 1 - sum sqrt(p q)  (Bhattacharyya coefficient)
    p = np.array([0.1, 0.6, 0.3]); q = np.array([0.5, 0.25, 0.25])
    assert lo.hellinger(p, q) ** 2 == pytest.approx(1.0 - np.sqrt(p * q).sum(), rel=1e-12)
    assert lo.hellinger(p, q) == pytest.approx(lo.hellinger(q, p))
