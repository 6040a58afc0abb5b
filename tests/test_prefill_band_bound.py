"""The selection band of the prompt phase (H2O scores of the prompt, Sec. 2.1: column sums of the
causal attention matrix).  With fp16 storage the library first sums every column cheaply (fp16
matrix products with fp32 accumulation, fp32 log-sums, fp32 exponential, fp32 running sums) and
computes exact fp64 sums only for tokens whose cheap sum lies within a relative band of the
selection boundary.  That is sound if every cheap sum is within the band of the exact one.  Here
the cheap path is emulated in numpy fp32 arithmetic on the workloads whose column sums lie close
together and on heavy-tailed keys, and compared with the oracle's fp64 column sums: the error
must stay inside the bound the kernel derives (lessdec_prefill.hip, prefill_band_kernel), and the
bound inside half the band the kernel then uses."""
import numpy as np
import pytest

from paper_2402_09398_amd import workloads as wl
from tests import harness as hz

K_BAND = 1.0 / 256.0
U32 = 2.0 ** -24


def error_bound(M, D, P, G):
    """eps of prefill_band_kernel's comment: relative error bound of a cheap column sum."""
    return U32 * ((D + 6) * M + 3 * np.log(P) + G * P / 16 + 6)


def cheap_column_sums(Q, K, lse):
    """fp32 emulation of the cheap pass for one unit: Q [G,P,D], K [P,D] fp16, lse [G,P] fp64."""
    G, P, D = Q.shape
    scale = np.float32(1.0 / np.sqrt(D))
    cs = np.zeros(P, dtype=np.float32)
    K32 = K.astype(np.float32)
    causal = np.tril(np.ones((P, P), dtype=bool))
    for g in range(G):
        acc = (Q[g].astype(np.float32) @ K32.T).astype(np.float32)           # fp32 accumulation of exact products
        x = (acc * scale).astype(np.float32) - lse[g].astype(np.float32)[:, None]
        with np.errstate(over="ignore"):                                    # entries above the diagonal are masked out
            a = np.where(causal, np.exp(x.astype(np.float32)), np.float32(0)).astype(np.float32)
        # a lane's running sum over its share of the rows, then the lanes: sequential fp32 sums
        cs = (cs + np.cumsum(a, axis=0, dtype=np.float32)[-1]).astype(np.float32)
    return cs


CASES = [
    wl.WORKLOADS[1].scaled(name="close-column-sums-f16", dtype="f16", head_dim=128, batch=1, heads=3,
                           prompt=900, steps=0, n_heavy=300, n_recent=20, rank=8, hidden=128),
    wl.WORKLOADS[1].scaled(name="close-column-sums-f16-d64", dtype="f16", head_dim=64, batch=1, heads=2,
                           prompt=333, steps=0, n_heavy=40, n_recent=7, rank=4, hidden=64),
    wl.WORKLOADS[4].scaled(name="heavy-tailed-keys", batch=2, heads=8, prompt=768, steps=0, n_heavy=30,
                           n_recent=30, hidden=128),
    wl.WORKLOADS[3].scaled(name="peaked-heads", batch=1, heads=8, prompt=1024, steps=0, hidden=128),
    wl.WORKLOADS[3].scaled(name="two-query-heads", batch=1, heads=4, prompt=400, steps=0, hidden=128, q_per_kv=2),
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_cheap_column_sums_stay_inside_the_band(w):
    inp = wl.all_inputs(w)
    units = list(range(w.units))
    st = hz.make_oracle(w, units)
    pre = st.prefill(inp["Q"], inp["K"], inp["V"], want_out=False)
    G, P, D = w.q_per_kv, w.prompt, w.head_dim
    worst, worst_bound = 0.0, 0.0
    for u in units:
        Qu = inp["Q"][u].reshape(G, P, D)
        Ku = inp["K"][u]
        s = np.einsum("gpd,jd->gpj", Qu.astype(np.float64), Ku.astype(np.float64)) / np.sqrt(D)
        s = np.where(np.tril(np.ones((P, P), dtype=bool))[None], s, -np.inf)
        m = s.max(axis=2, keepdims=True)
        lse = (m + np.log(np.exp(s - m).sum(axis=2, keepdims=True)))[..., 0]
        exact = pre["colsum"][u]
        # the oracle's own column sums are these rows normalised and summed: a pin of the emulation's reference
        ref = np.exp(s - lse[..., None]).sum(axis=(0, 1))
        np.testing.assert_allclose(ref, exact, rtol=1e-11)
        cheap = cheap_column_sums(Qu, Ku, lse).astype(np.float64)
        err = np.abs(cheap - exact) / exact
        M = np.linalg.norm(Qu.astype(np.float64), axis=-1).max() * np.linalg.norm(Ku.astype(np.float64), axis=-1).max() / np.sqrt(D)
        eps = error_bound(M, D, P, G)
        worst, worst_bound = max(worst, err.max()), max(worst_bound, eps)
        assert err.max() <= eps, (u, err.max(), eps)
    print(f"\n{w.name}: largest relative error {worst:.2e}, largest bound {worst_bound:.2e}, band {K_BAND:.2e}")
    assert 2 * worst_bound <= K_BAND      # at these shapes the fixed band is the one in force


def test_the_band_grows_with_the_scores():
    """Keys sixteen times larger: the derived bound passes the fixed band, and the kernel's band
    (twice the bound) still covers the emulated error."""
    w = wl.WORKLOADS[3].scaled(name="huge-keys", batch=1, heads=4, prompt=256, steps=0, hidden=128)
    inp = wl.all_inputs(w)
    inp["K"] = (inp["K"].astype(np.float32) * 16).astype(np.float16)
    st = hz.make_oracle(w, list(range(w.units)))
    pre = st.prefill(inp["Q"], inp["K"], inp["V"], want_out=False)
    P, D = w.prompt, w.head_dim
    grew = False
    for u in range(w.units):
        Qu, Ku = inp["Q"][u][None], inp["K"][u]
        s = (Qu[0].astype(np.float64) @ Ku.astype(np.float64).T) / np.sqrt(D)
        s = np.where(np.tril(np.ones((P, P), dtype=bool)), s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        lse = (m + np.log(np.exp(s - m).sum(axis=1, keepdims=True)))[None, :, 0]
        cheap = cheap_column_sums(Qu, Ku, lse).astype(np.float64)
        exact = pre["colsum"][u]
        M = np.linalg.norm(Qu.astype(np.float64), axis=-1).max() * np.linalg.norm(Ku.astype(np.float64), axis=-1).max() / np.sqrt(D)
        eps = error_bound(M, D, P, 1)
        grew = grew or 2 * eps > K_BAND
        ok = exact > 1e-30
        assert (np.abs(cheap - exact)[ok] / exact[ok]).max() <= eps
    assert grew
