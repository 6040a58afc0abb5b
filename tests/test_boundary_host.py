"""Host-side checks of the C-ABI library: it loads, exports what the header declares,
and rejects bad descriptors before anything is launched.  No GPU needed."""
import ctypes as C
import os
import re

import pytest

from oracle import less_oracle as lo
from paper_2402_09398_amd import binding, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    src = open(os.path.join(ROOT, "include", "lessdec.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return set(re.findall(r"\b(lessdec_[a-z_]+)\s*\(", src))


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    names = header_functions()
    assert names == set(binding.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_descriptor_layout_matches_header():
    # 9 int32 fields (padded to 8 bytes), 17 pointers, 1 size_t on LP64
    assert C.sizeof(binding.Desc) == 10 * 4 + 17 * 8 + 8
    assert binding.Desc.k_cache.offset == 40


def test_budget_helper_matches_table1_and_workloads():
    for pct, L_, tok in [(2, 4096, 80), (5, 4096, 204), (10, 4096, 408),
                         (2, 2048, 40), (5, 2048, 102), (10, 2048, 204)]:
        assert binding.lessdec_budget_tokens(pct, L_) == tok
    # slot counts of the workloads (their percentages are taken of the prompt length)
    for cfg, pct in [(2, 10), (3, 10), (4, 8), (5, 4)]:
        w = wl.WORKLOADS[cfg]
        assert binding.lessdec_budget_tokens(pct, w.prompt) == w.capacity
        assert lo.budget_tokens(pct, w.prompt) == w.capacity
        assert w.n_heavy == w.n_recent == w.capacity // 2
    assert wl.WORKLOADS[5].prompt - wl.WORKLOADS[5].capacity == 7866


def _desc(**kw):
    d = binding.Desc()
    d.batch, d.heads, d.head_dim = 2, 2, 128
    d.n_heavy, d.n_recent, d.rank, d.hidden, d.dtype = 4, 4, 8, 64, binding.DTYPE_F16
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def _workload_desc(w, **kw):
    d = binding.Desc()
    d.batch, d.heads, d.head_dim = w.batch, w.heads, w.head_dim
    d.n_heavy, d.n_recent, d.rank, d.hidden = w.n_heavy, w.n_recent, w.rank, w.hidden
    d.dtype = binding.DTYPE_F16 if w.dtype == "f16" else binding.DTYPE_F32
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def test_launches_per_step_of_the_workloads():
    """Which form of the step a shape takes is decided on the host: the four fp16 workloads run it
    as one launch (feature-map jobs in front of the attention waves), four or eight query heads per
    unit too; the other shapes keep a launch of their own for the feature maps."""
    got = {c: binding.lessdec_step_launches(_workload_desc(wl.WORKLOADS[c])) for c in range(1, 6)}
    assert got == {1: 3, 2: 1, 3: 1, 4: 1, 5: 1}
    w3 = wl.WORKLOADS[3]
    for g, n in [(2, 2), (4, 1), (8, 1), (16, 3)]:
        assert binding.lessdec_step_launches(_workload_desc(w3, heads=w3.heads // g, q_per_kv=g)) == n
    assert binding.lessdec_step_launches(_workload_desc(w3, rank=20)) == 3       # any-shape kernels
    assert binding.lessdec_step_launches(_workload_desc(w3, hidden=1024)) == 2   # more parts than a wave keeps
    assert binding.lessdec_step_launches(_workload_desc(w3, head_dim=64)) == 2
    assert binding.lessdec_step_launches(_workload_desc(w3, batch=-1)) == 0      # invalid shape


def test_workspace_bytes_and_shape_validation():
    assert binding.lessdec_workspace_bytes(_desc(), 0) > 0
    assert binding.lessdec_workspace_bytes(_desc(), 512) > binding.lessdec_workspace_bytes(_desc(), 0)
    # Lambda-masking through the prompt also holds phi of every prompt query
    assert binding.lessdec_workspace_bytes(_desc(flags=6), 512) > binding.lessdec_workspace_bytes(_desc(flags=2), 512)
    assert binding.lessdec_workspace_bytes(_desc(flags=4), 512) == binding.lessdec_workspace_bytes(_desc(), 512)
    for bad in (dict(head_dim=96), dict(rank=0), dict(rank=65), dict(hidden=0), dict(hidden=4096),
                dict(n_heavy=0, n_recent=0), dict(n_heavy=4000, n_recent=4000), dict(dtype=7),
                dict(batch=0), dict(flags=8), dict(n_heavy=-1), dict(q_per_kv=-1), dict(q_per_kv=129),
                dict(q_per_kv=2, n_heavy=1024, n_recent=1024)):
        assert binding.lessdec_workspace_bytes(_desc(**bad), 0) == 0, bad


def test_calls_reject_bad_descriptors_on_the_host():
    L = binding.lib()
    d = _desc()                                             # all pointers NULL
    assert L.lessdec_state_reset(C.byref(d), None) == binding.EINVAL
    assert L.lessdec_state_sync(C.byref(d), None) == binding.EINVAL
    assert L.lessdec_step(C.byref(d), None, None, None, None, None, None) == binding.EINVAL
    assert L.lessdec_step_features(C.byref(d), None, None, None) == binding.EINVAL
    assert L.lessdec_step_attend(C.byref(d), None, None, None, None, None, None) == binding.EINVAL
    assert L.lessdec_prefill(C.byref(d), None, None, None, 16, None, None) == binding.EINVAL
    # plausible pointers but no workspace -> workspace error; misaligned cache -> invalid
    for f in ("k_cache", "v_cache", "acc", "pos", "psi", "H", "z", "n_seen",
              "pend_slot", "pend_v", "pend_psi", "Wq1", "Wq2", "Wk1", "Wk2", "Wk3"):
        setattr(d, f, 0x10000)
    assert L.lessdec_state_reset(C.byref(d), None) == binding.EWORKSPACE
    d.workspace = 0x20000; d.workspace_bytes = 16
    assert L.lessdec_state_reset(C.byref(d), None) == binding.EWORKSPACE
    d.workspace_bytes = 1 << 30
    d.k_cache = 0x10002
    assert L.lessdec_state_reset(C.byref(d), None) == binding.EINVAL
    d.k_cache = 0x10000
    assert L.lessdec_prefill(C.byref(d), 0x30000, 0x30000, 0x30000, 0, None, None) == binding.EINVAL
    assert L.lessdec_step(C.byref(d), 0x30000, 0x30000, 0x30004, 0x30000, None, None) == binding.EINVAL
    assert L.lessdec_step_features(C.byref(d), 0x30000, 0x30008, None) == binding.EINVAL
    assert L.lessdec_step_attend(C.byref(d), 0x30000, 0x30000, 0x30000, None, None, None) == binding.EINVAL
    assert b"workspace" in L.lessdec_strerror(binding.EWORKSPACE)
    assert L.lessdec_strerror(12345) is not None


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2402_09398_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "less_oracle" not in text and "import oracle" not in text and "from oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2402_09398_amd" not in text and "lessdec" not in text, f


def test_workload_generator_shapes_and_determinism():
    import numpy as np
    w = wl.WORKLOADS[4].scaled(batch=1, heads=3, prompt=40, steps=5)
    a = wl.unit_inputs(w, 1); b = wl.unit_inputs(w, 1)
    for k in a:
        assert np.array_equal(a[k], b[k])
    assert a["Q"].shape == (40, 128) and a["q"].shape == (5, 128) and a["K"].dtype == np.float16
    assert not np.array_equal(a["K"], wl.unit_inputs(w, 2)["K"])
    hp = wl.head_params(w, 1)
    assert len(hp["outlier_channels"]) == 4 and 0.5 <= hp["sigma"] <= 2.0
    assert hp["Wk3"].shape == (16, 16) and hp["Wq1"].shape == (128, 512)
    allw = wl.head_weights(w)
    assert allw["Wq2"].shape == (3, 512, 16)
    full = wl.all_inputs(w, units=[0, 2])
    assert full["Q"].shape == (2, 40, 128) and full["q"].shape == (5, 2, 128)
    assert np.array_equal(full["k"][:, 1], wl.unit_inputs(w, 2)["k"])
    w1 = wl.WORKLOADS[1]
    assert wl.unit_inputs(w1, 0)["Q"].dtype == np.float32
    # several query heads per unit: an extra axis on the queries and on phi's weights only;
    # the first query head and everything else are the single-head draws
    wg = w.scaled(q_per_kv=3)
    g = wl.unit_inputs(wg, 1)
    assert g["Q"].shape == (3, 40, 128) and g["q"].shape == (5, 3, 128) and g["K"].shape == (40, 128)
    assert np.array_equal(g["Q"][0], a["Q"]) and np.array_equal(g["q"][:, 0], a["q"]) and np.array_equal(g["v"], a["v"])
    gw = wl.head_weights(wg)
    assert gw["Wq1"].shape == (9, 128, 512) and gw["Wk1"].shape == (3, 128, 512)
    assert np.array_equal(gw["Wq1"][3], allw["Wq1"][1]) and np.array_equal(gw["Wk2"], allw["Wk2"])
    fullg = wl.all_inputs(wg, units=[0, 2])
    assert fullg["Q"].shape == (2, 3, 40, 128) and fullg["q"].shape == (5, 2, 3, 128)


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr
