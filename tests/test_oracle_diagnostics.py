"""The diagnostics built on the oracle (implied attention rows, Eq. 7's Hellinger distance):
pinned by closed forms and by the oracle's own Eq. 3 output.  CPU only."""
import numpy as np
import pytest

from oracle import less_diagnostics as ld
from paper_2402_09398_amd import workloads as wl


def _unit(**kw):
    d = dict(name="diag", batch=1, heads=1, head_dim=64, prompt=30, steps=20, n_heavy=4, n_recent=4,
             rank=4, hidden=64, dtype="f32")
    d.update(kw)
    w = wl.WORKLOADS[2].scaled(**d)
    hp = wl.head_params(w, 0)
    W = {k: hp[k] for k in ("Wq1", "Wq2", "Wk1", "Wk2", "Wk3")}
    return w, W, wl.unit_inputs(w, 0)


def test_implied_row_by_hand():
    # D = 1, sqrt(D) = 1: scores are q * k
    q = np.array([1.0]); keys = np.array([[0.0], [np.log(2.0)], [np.log(3.0)]])
    cached = np.array([True, False, True])
    row = ld.implied_row(q, keys, cached)                      # the policy alone: weights 1, 0, 3
    assert row == pytest.approx([0.25, 0.0, 0.75])
    f = np.array([2.0, 1.0]); psi = np.array([[9.0, 9.0], [0.5, 1.0], [9.0, 9.0]])
    row = ld.implied_row(q, keys, cached, f, psi)              # discarded token: phi psi^T = 2
    assert row == pytest.approx([1 / 6, 2 / 6, 3 / 6])
    assert ld.full_row(q, keys) == pytest.approx([1 / 6, 2 / 6, 3 / 6])


def test_rows_reproduce_the_oracle_output_and_are_distributions():
    w, W, inp = _unit()
    r = ld.unit_diagnostics(w.head_dim, w.n_heavy, w.n_recent, w.rank, w.hidden, W, inp)
    assert r["output_gap"].max() < 1e-10                       # row @ V is Eq. 3's output
    for n in ("hellinger_less", "hellinger_sparse", "hellinger_sparse_plus"):
        assert np.all(r[n] >= 0.0) and np.all(r[n] <= 1.0)
    assert r["hellinger_sparse"].min() > 0.0                   # tokens were discarded: mass is missing


def test_unbounded_budget_has_no_distance():
    w, W, inp = _unit(n_heavy=40, n_recent=40)
    r = ld.unit_diagnostics(w.head_dim, w.n_heavy, w.n_recent, w.rank, w.hidden, W, inp)
    for n in ("hellinger_less", "hellinger_sparse", "hellinger_sparse_plus"):
        assert r[n].max() < 1e-7
    assert r["output_gap"].max() < 1e-10


def test_zero_feature_maps_are_the_policy_alone():
    w, W, inp = _unit()
    Z = {k: np.zeros_like(v) for k, v in W.items()}
    r = ld.unit_diagnostics(w.head_dim, w.n_heavy, w.n_recent, w.rank, w.hidden, Z, inp)
    assert np.array_equal(r["hellinger_less"], r["hellinger_sparse"])


def test_lambda_masking_rows():
    w, W, inp = _unit(n_heavy=4, n_recent=8)
    r = ld.unit_diagnostics(w.head_dim, w.n_heavy, w.n_recent, w.rank, w.hidden, W, inp, flags=2)
    assert r["output_gap"].max() < 1e-10
    # the policy alone keeps tokens 0..3 and the last 8: its distance is the closed form from the
    # full row's mass on the kept tokens, H^2 = 1 - sqrt(kept mass)
    K = np.concatenate([inp["K"], inp["k"]]).astype(np.float64)
    for t in (0, 7, 19):
        n = w.prompt + t + 1
        ref = ld.full_row(inp["q"][t].astype(np.float64), K[:n])
        kept = np.r_[0:4, n - 9:n]
        assert r["hellinger_sparse"][t] ** 2 == pytest.approx(1.0 - np.sqrt(ref[kept].sum()), abs=1e-12)
