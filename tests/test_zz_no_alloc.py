"""lessdec_step_static (the step for callers that cannot allocate: its scratch is a buffer built
into the library) against lessdec_step, through the C ABI: two runs in a row on one GPU, the
second on a smaller shape, so that the second finds the first one's leftovers in the shared
buffer.  Same kernels, so the bar is bit-equality of outputs, eviction log and every state
buffer; the descriptor handed to the static call carries no workspace at all."""
import ctypes as C

import numpy as np
import pytest

from paper_2402_09398_amd import binding, workloads as wl
from tests import harness as hz

pytestmark = pytest.mark.gpu

BASE = wl.WORKLOADS[2]


def _run_both(w, steps):
    import torch
    inp = wl.all_inputs(w)
    q, k, v = (torch.from_numpy(inp[n]).cuda() for n in ("q", "k", "v"))
    Q, K, V = (torch.from_numpy(inp[n]).cuda() for n in ("Q", "K", "V"))
    ref = hz.make_gpu(w)
    ref.prefill(Q, K, V)
    got = hz.make_gpu(w)
    for n in got.STATE:
        getattr(got, n).copy_(getattr(ref, n))
    bare = binding.Desc()
    C.memmove(C.byref(bare), C.byref(got.desc), C.sizeof(binding.Desc))
    bare.workspace = None
    bare.workspace_bytes = 0
    out_r = torch.empty_like(q[:steps]); out_g = torch.empty_like(q[:steps])
    ev_r = torch.full((steps, w.units), -7, dtype=torch.int32, device="cuda"); ev_g = ev_r.clone()
    for t in range(steps):
        ref.step(q[t], k[t], v[t], out_r[t], ev_r[t])
        binding.lessdec_step_static(bare, q[t], k[t], v[t], out_g[t], ev_g[t])
    torch.cuda.synchronize()
    assert torch.equal(out_r, out_g), "outputs differ"
    assert torch.equal(ev_r, ev_g), "eviction logs differ"
    assert int((ev_r >= 0).sum()) > 0
    for n in got.STATE:
        assert torch.equal(getattr(ref, n), getattr(got, n)), n
    assert np.isfinite(out_g.float().cpu().numpy()).all()


@pytest.mark.parametrize("kind", ["streaming", "multi-head", "general"])
def test_static_scratch_step_matches_step_twice_in_a_row(kind):
    kw = {"multi-head": dict(q_per_kv=4), "general": dict(rank=20), "streaming": {}}[kind]
    d = dict(head_dim=128, n_heavy=6, n_recent=6, rank=8, hidden=128, dtype="f16", prompt=40)
    d.update(kw)
    big = BASE.scaled(name=f"static-{kind}-big", batch=64, heads=16, steps=12, **d)
    little = BASE.scaled(name=f"static-{kind}-small", batch=2, heads=3, steps=12, **d)
    _run_both(big, 12)
    _run_both(little, 12)


def test_static_scratch_refuses_a_shape_beyond_its_buffer():
    """Refused on the host before any launch, with the error code of its own."""
    w = BASE.scaled(name="static-too-big", batch=512, heads=32, head_dim=128, n_heavy=6, n_recent=6,
                    rank=8, hidden=512, dtype="f16", prompt=0, steps=1)
    d = binding.Desc()
    d.batch, d.heads, d.head_dim = w.batch, w.heads, w.head_dim
    d.n_heavy, d.n_recent, d.rank, d.hidden = w.n_heavy, w.n_recent, w.rank, w.hidden
    d.dtype, d.flags, d.q_per_kv = binding.DTYPE_F16, 0, 1
    assert binding.lessdec_workspace_bytes(d, 0) > binding.STATIC_SCRATCH_BYTES
    rc = binding.lib().lessdec_step_static(C.byref(d), None, None, None, None, None, None)
    assert rc == binding.ESCRATCH
