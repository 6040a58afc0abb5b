"""Host logic of the parity protocol, on the CPU: the oracle plays both sides, with mistakes
planted in the side that stands for the GPU, so that every branch of tests/harness.py (exact,
exempt near-tie, failure, per-unit invariants) is known to do what the GPU tests rely on."""
import numpy as np
import pytest

from paper_2402_09398_amd import workloads as wl
from tests import harness as hz

W = wl.WORKLOADS[2].scaled(name="host", batch=2, heads=3, prompt=48, steps=16, n_heavy=6, n_recent=6,
                           hidden=64)


def stand_in_run(w, inp, flags=0, state_edit=None, force_at=None):
    """A run in the shape gpu_run() returns, produced by a second oracle instance.
    state_edit(st) rewrites the state after the prompt; force_at = {step: forced positions}."""
    units = list(range(w.units))
    st = hz.make_oracle(w, units, flags=flags)
    pre = st.prefill(inp["Q"], inp["K"], inp["V"], want_out=True)
    if state_edit:
        state_edit(st)

    def snap():
        return dict(k_cache=st.Kc.copy(), v_cache=st.Vc.copy(), acc=st.acc.copy(), pos=st.pos.copy(),
                    psi=np.zeros((w.units, w.capacity, w.rank)), H=st.H.copy(), z=st.z.copy(),
                    n_seen=st.n.copy())
    res = {"prefill_out": pre["out"], "after_prefill": snap()}
    outs, ev = [], []
    for t in range(w.steps):
        r = st.step(inp["q"][t], inp["k"][t], inp["v"][t], force=(force_at or {}).get(t))
        outs.append(r["out"]); ev.append(r["evicted"])
    res["outs"] = np.array(outs); res["evicted"] = np.array(ev); res["final"] = snap()
    return res


def test_a_faithful_run_passes():
    inp = wl.all_inputs(W)
    res = stand_in_run(W, inp)
    rep = hz.check_against_oracle(W, inp, list(range(W.units)), res)
    assert rep.ok() and rep.exact == rep.decisions == W.units * W.steps and rep.exempt == 0
    assert hz.check_every_unit(W, res) == []


def test_exact_tie_is_planted_and_the_older_pair_leaves():
    inp = wl.all_inputs(W)
    slots = {}
    res = stand_in_run(W, inp, state_edit=lambda st: slots.update(ab=hz.plant_score_tie(st)))
    a, b = slots["ab"]
    older = res["after_prefill"]["pos"][:, b]
    assert (res["evicted"][0] == older).all()           # the older token sits in the higher slot
    st = hz.make_oracle(W, list(range(W.units)))
    st.prefill(inp["Q"], inp["K"], inp["V"], want_out=False)
    hz.plant_score_tie(st)
    rep = hz.check_against_oracle(W, inp, list(range(W.units)), res, oracle_state=st)
    assert rep.ok() and rep.min_gap == 0.0 and rep.exempt == 0


def _near_tie(st, rel):
    a, b = hz.plant_score_tie(st)
    st.acc[:, a] *= 1.0 + rel                           # the newer token now scores a little more
    return a, b


def test_runner_up_inside_the_gap_is_exempt_and_the_run_goes_on():
    inp = wl.all_inputs(W)
    probe = hz.make_oracle(W, list(range(W.units)))
    probe.prefill(inp["Q"], inp["K"], inp["V"], want_out=False)
    a, b = _near_tie(probe, 1e-7)
    newer = probe.pos[:, a].copy()
    # the stand-in discards the runner-up (the newer token) at the first step
    res = stand_in_run(W, inp, state_edit=lambda st: _near_tie(st, 1e-7), force_at={0: newer})
    st = hz.make_oracle(W, list(range(W.units)))
    st.prefill(inp["Q"], inp["K"], inp["V"], want_out=False)
    _near_tie(st, 1e-7)
    rep = hz.check_against_oracle(W, inp, list(range(W.units)), res, oracle_state=st)
    assert rep.ok(), rep.failures[:3]
    assert rep.exempt == W.units and rep.exact == rep.decisions - W.units
    assert hz.check_every_unit(W, res) == []


def test_runner_up_outside_the_gap_fails():
    inp = wl.all_inputs(W)
    probe = hz.make_oracle(W, list(range(W.units)))
    probe.prefill(inp["Q"], inp["K"], inp["V"], want_out=False)
    a, b = _near_tie(probe, 1e-4)
    newer = probe.pos[:, a].copy()
    res = stand_in_run(W, inp, state_edit=lambda st: _near_tie(st, 1e-4), force_at={0: newer})
    st = hz.make_oracle(W, list(range(W.units)))
    st.prefill(inp["Q"], inp["K"], inp["V"], want_out=False)
    _near_tie(st, 1e-4)
    rep = hz.check_against_oracle(W, inp, list(range(W.units)), res, oracle_state=st)
    assert not rep.ok() and rep.exempt == 0


def test_a_derailed_unit_does_not_hide_the_others():
    """State is compared per unit: one failing unit must not switch the comparison off."""
    inp = wl.all_inputs(W)
    res = stand_in_run(W, inp)
    res["final"]["H"][W.units - 1] *= 1.01               # a wrong state in the last unit only
    res["evicted"][3, 0] = res["evicted"][2, 0]          # and an impossible eviction in the first
    rep = hz.check_against_oracle(W, inp, list(range(W.units)), res)
    assert any("unit 0" in f for f in rep.failures)
    assert any(f"unit {W.units - 1} H off" in f for f in rep.failures)


@pytest.mark.parametrize("plant", ["nan-out", "n-seen", "dup-pos", "evict-recent", "evict-twice", "no-evict",
                                   "lost-token"])
def test_invariants_catch_planted_faults(plant):
    inp = wl.all_inputs(W)
    res = stand_in_run(W, inp)
    u = W.units - 1
    if plant == "nan-out":
        res["outs"][5, u, 3] = np.nan
    elif plant == "n-seen":
        res["final"]["n_seen"][u] -= 1
    elif plant == "dup-pos":
        res["final"]["pos"][u, 0] = res["final"]["pos"][u, 1]
    elif plant == "evict-recent":
        res["evicted"][4, u] = W.prompt + 4 - 1
    elif plant == "evict-twice":
        res["evicted"][5, u] = res["evicted"][4, u]
    elif plant == "no-evict":
        res["evicted"][5, u] = -1
    elif plant == "lost-token":
        res["final"]["pos"][u, 0] = -1
    assert hz.check_every_unit(W, res) != []


@pytest.mark.parametrize("dtype,supers,nh", [("f16", (), 1), ("f32", (5, 9), 3)])
def test_prompt_tie_is_planted_and_the_later_token_is_kept(dtype, supers, nh):
    w = W.scaled(name="prompt-tie", dtype=dtype, n_heavy=nh, prompt=80)
    inp = wl.all_inputs(w)
    j1, j2 = hz.plant_prompt_tie(w, inp, 19, supers)
    st = hz.make_oracle(w, list(range(w.units)))
    pre = st.prefill(inp["Q"], inp["K"], inp["V"], want_out=False)
    assert (pre["colsum"][:, j1] == pre["colsum"][:, j2]).all()
    assert (pre["dec"][:, 0] == pre["dec"][:, 2]).all()              # the boundary pair is the tie
    assert pre["kept"][:, j2].all() and not pre["kept"][:, j1].any()
    for s in supers:
        assert pre["kept"][:, s].all()
