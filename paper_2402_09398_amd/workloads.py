"""Seeded synthetic workloads for the LESS decode path.

This module only draws random numbers and rounds them to the storage type.  It
holds none of the method's arithmetic (no attention, no feature maps, no
eviction rule), so both the CPU oracle's tests and the HIP path's tests can
take their inputs from it without sharing any computation.

The paper's efficiency runs use synthetic prompts padded to one length and
batched (Sec. 4.3); the five workloads below have the attention shapes of
Llama 2 7B / 13B (Table 6 names the models) and stand in for those runs.
Every unit (batch row, head) has its own random stream, so a test may
generate a handful of units of a large workload without generating the rest.

Recipe
------
* cfg 1: q, k, v ~ N(0, 1)/sqrt(64), stored in fp32.
* cfg 2, 3, 5: per head sigma_h ~ U[0.5, 2]; q, k ~ N(0, sigma_h^2) per
  element, v ~ N(0, 1); rounded once to fp16.
* cfg 4: as above, and per head 4 of the 128 key channels (fixed over tokens)
  draw sigma_h * Student-t(nu=3) instead; clamped to +-6e4 before the fp16
  cast.
* feature-map weights: every matrix ~ N(0, 1/fan_in), per head, rounded to the
  storage type.
"""
from __future__ import annotations

from dataclasses import dataclass
from concurrent.futures import ThreadPoolExecutor

import numpy as np

BASE_SEED = 24020939

_KIND_HEAD = 1
_KIND_UNIT = 2


@dataclass(frozen=True)
class Workload:
    cfg: int
    name: str
    batch: int
    heads: int
    head_dim: int
    prompt: int
    steps: int
    n_heavy: int
    n_recent: int
    rank: int
    hidden: int
    dtype: str            # "f32" or "f16": storage type of q/k/v, the cache, the weights, out
    outlier_channels: int = 0
    q_per_kv: int = 1     # query heads per key/value head; > 1: q, Q and Wq1, Wq2 get an axis G

    @property
    def units(self) -> int:
        return self.batch * self.heads

    @property
    def capacity(self) -> int:
        return self.n_heavy + self.n_recent

    @property
    def np_dtype(self):
        return np.float32 if self.dtype == "f32" else np.float16

    def scaled(self, **kw) -> "Workload":
        """A copy with some fields replaced (smaller batch, fewer steps...)."""
        d = dict(self.__dict__)
        d.update(kw)
        return Workload(**d)


# Slot counts are literal here; the budget rule that produces them from a
# percentage lives with the code that owns it (the oracle has one, the library
# binding has one) and the tests check both against these numbers.
WORKLOADS = {
    1: Workload(1, "tiny", 1, 2, 64, 128, 64, 8, 8, 4, 64, "f32"),
    2: Workload(2, "llama2-7b-b8", 8, 32, 128, 1024, 256, 51, 51, 8, 512, "f16"),
    3: Workload(3, "llama2-7b-b64", 64, 32, 128, 1024, 512, 51, 51, 8, 512, "f16"),
    4: Workload(4, "llama2-13b-b32", 32, 40, 128, 2048, 512, 81, 81, 16, 512, "f16",
                outlier_channels=4),
    5: Workload(5, "long-context", 4, 32, 128, 8192, 1024, 163, 163, 8, 512, "f16"),
}


def _rng(w: Workload, kind: int, index: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(
        np.random.SeedSequence([BASE_SEED, w.cfg, kind, index])))


def head_params(w: Workload, h: int) -> dict:
    """Per-head scale, outlier channels and feature-map weights (storage dtype)."""
    g = _rng(w, _KIND_HEAD, h)
    D, Rp, R = w.head_dim, w.hidden, w.rank
    sigma = 1.0 if w.cfg == 1 else float(g.uniform(0.5, 2.0))
    outl = np.sort(g.choice(D, size=w.outlier_channels, replace=False)) \
        if w.outlier_channels else np.zeros(0, dtype=np.int64)

    def mat(rows, cols):
        m = g.standard_normal((rows, cols)) / np.sqrt(rows)
        return m.astype(np.float32).astype(w.np_dtype)

    p = {
        "sigma": sigma,
        "outlier_channels": outl,
        "Wq1": mat(D, Rp), "Wq2": mat(Rp, R),
        "Wk1": mat(D, Rp), "Wk2": mat(Rp, R), "Wk3": mat(R, R),
    }
    if w.q_per_kv > 1:          # the head's further query heads, drawn after everything else
        p["Wq1"] = np.stack([p["Wq1"]] + [mat(D, Rp) for _ in range(w.q_per_kv - 1)])
        p["Wq2"] = np.stack([p["Wq2"]] + [mat(Rp, R) for _ in range(w.q_per_kv - 1)])
    return p


def head_weights(w: Workload) -> dict:
    """All heads' weights stacked: Wq1 [Hh,D,R'], Wq2 [Hh,R',R], Wk1, Wk2, Wk3 [Hh,R,R]."""
    hp = [head_params(w, h) for h in range(w.heads)]
    W = {k: np.stack([p[k] for p in hp]) for k in ("Wq1", "Wq2", "Wk1", "Wk2", "Wk3")}
    if w.q_per_kv > 1:          # [Hh,G,..] -> [Hh*G,..]: head h's query heads in a row
        W["Wq1"] = W["Wq1"].reshape((-1,) + W["Wq1"].shape[2:])
        W["Wq2"] = W["Wq2"].reshape((-1,) + W["Wq2"].shape[2:])
    return W


def unit_inputs(w: Workload, u: int, prompt: int | None = None, steps: int | None = None) -> dict:
    """Prompt Q,K,V [P,D] and decode q,k,v [T,D] of unit u = b*heads + h, storage dtype.

    The prompt is drawn first, then the decode tokens, so a shorter prompt or
    fewer steps is a prefix of the full draw only for the prompt part; tests
    that shrink a workload use `scaled()` and compare both sides on the same
    shrunken draw.
    """
    P = w.prompt if prompt is None else prompt
    T = w.steps if steps is None else steps
    h = u % w.heads
    hp = head_params(w, h)
    g = _rng(w, _KIND_UNIT, u)
    D = w.head_dim

    def draw_qk(rows, is_key):
        if w.cfg == 1:
            x = g.standard_normal((rows, D)) / 8.0
        else:
            x = g.standard_normal((rows, D)) * hp["sigma"]
            if is_key and w.outlier_channels:
                t = g.standard_t(3.0, size=(rows, w.outlier_channels)) * hp["sigma"]
                x[:, hp["outlier_channels"]] = t
        return x

    def draw_v(rows):
        x = g.standard_normal((rows, D))
        return x / 8.0 if w.cfg == 1 else x

    def store(x):
        x = x.astype(np.float32)
        if w.dtype == "f16":
            x = np.clip(x, -6.0e4, 6.0e4)
        return x.astype(w.np_dtype)

    Q = store(draw_qk(P, False)); K = store(draw_qk(P, True)); V = store(draw_v(P))
    q = store(draw_qk(T, False)); k = store(draw_qk(T, True)); v = store(draw_v(T))
    if w.q_per_kv > 1:          # further query heads, drawn after everything else: Q [G,P,D], q [T,G,D]
        Q = np.stack([Q] + [store(draw_qk(P, False)) for _ in range(w.q_per_kv - 1)])
        q = np.stack([q] + [store(draw_qk(T, False)) for _ in range(w.q_per_kv - 1)], axis=1)
    return {"Q": Q, "K": K, "V": V, "q": q, "k": k, "v": v}


def all_inputs(w: Workload, units=None, workers: int = 8) -> dict:
    """Stacked inputs for the given units (default: all): Q,K,V [U,P,D]; q,k,v [T,U,D]
    (Q [U,G,P,D] and q [T,U,G,D] with several query heads per unit)."""
    units = list(range(w.units)) if units is None else list(units)
    with ThreadPoolExecutor(max_workers=workers) as ex:
        per = list(ex.map(lambda u: unit_inputs(w, u), units))
    out = {k: np.stack([p[k] for p in per]) for k in ("Q", "K", "V")}
    for k in ("q", "k", "v"):
        out[k] = np.ascontiguousarray(np.stack([p[k] for p in per], axis=1))
    return out
