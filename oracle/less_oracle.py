"""ctypes front end of the CPU oracle (oracle/less_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg.  It imports nothing from the HIP package.

The C file is compiled on first use with gcc (-O2, OpenMP over units, no
fast-math) into libless_oracle.so next to this file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "less_oracle.c"
_LIB = _HERE / "libless_oracle.so"
_lib = None

FLAG_SPARSE_DENOM = 1
FLAG_LAMBDA = 2          # Lambda-masking instead of H2O (Sec. 4, setup)
FLAG_PROMPT_STEPWISE = 4 # the policy runs from the first prompt token (Sec. 4.1 setting)


def build(force: bool = False) -> Path:
    """Compile the oracle; returns the library path."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", str(tmp), str(_SRC), "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _State(C.Structure):
    _fields_ = [
        ("U", C.c_int32), ("heads", C.c_int32), ("D", C.c_int32),
        ("n_heavy", C.c_int32), ("n_recent", C.c_int32), ("R", C.c_int32), ("Rp", C.c_int32),
        ("flags", C.c_uint32), ("G", C.c_int32),
        ("head", C.c_void_p),
        ("Wq1", C.c_void_p), ("Wq2", C.c_void_p),
        ("Wk1", C.c_void_p), ("Wk2", C.c_void_p), ("Wk3", C.c_void_p),
        ("Kc", C.c_void_p), ("Vc", C.c_void_p), ("acc", C.c_void_p), ("pos", C.c_void_p),
        ("H", C.c_void_p), ("z", C.c_void_p), ("n", C.c_void_p),
    ]


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(str(build()))
        _lib.less_oracle_budget_tokens.restype = C.c_int64
        _lib.less_oracle_budget_tokens.argtypes = [C.c_double, C.c_int64]
        _lib.less_oracle_gelu.restype = C.c_double
        _lib.less_oracle_gelu.argtypes = [C.c_double]
        _lib.less_oracle_hellinger.restype = C.c_double
        _lib.less_oracle_hellinger.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        _lib.less_oracle_phi.restype = None
        _lib.less_oracle_phi.argtypes = [C.c_void_p] * 3 + [C.c_int] * 3 + [C.c_void_p]
        _lib.less_oracle_psi.restype = None
        _lib.less_oracle_psi.argtypes = [C.c_void_p] * 4 + [C.c_int] * 3 + [C.c_void_p]
        _lib.less_oracle_reset.restype = None
        _lib.less_oracle_reset.argtypes = [C.POINTER(_State)]
        _lib.less_oracle_step.restype = C.c_int
        _lib.less_oracle_step.argtypes = [C.POINTER(_State)] + [C.c_void_p] * 8
        _lib.less_oracle_prefill.restype = None
        _lib.less_oracle_prefill.argtypes = ([C.POINTER(_State)] + [C.c_void_p] * 3 +
                                             [C.c_int64] + [C.c_void_p] * 4)
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def budget_tokens(percent: float, max_len: int) -> int:
    """Table 1: tokens cached at `percent` of the model's maximum length."""
    return int(lib().less_oracle_budget_tokens(float(percent), int(max_len)))


def gelu(x: float) -> float:
    return float(lib().less_oracle_gelu(float(x)))


def hellinger(p, q) -> float:
    p = _f64(p); q = _f64(q)
    assert p.shape == q.shape and p.ndim == 1
    return float(lib().less_oracle_hellinger(_ptr(p), _ptr(q), p.size))


def phi(q, W1, W2):
    q = _f64(q); W1 = _f64(W1); W2 = _f64(W2)
    D, Rp = W1.shape; R = W2.shape[1]
    assert q.shape == (D,) and W2.shape == (Rp, R) and R <= 64
    f = np.empty(R)
    lib().less_oracle_phi(_ptr(q), _ptr(W1), _ptr(W2), D, Rp, R, _ptr(f))
    return f


def psi(k, W1, W2, W3):
    k = _f64(k); W1 = _f64(W1); W2 = _f64(W2); W3 = _f64(W3)
    D, Rp = W1.shape; R = W2.shape[1]
    assert k.shape == (D,) and W2.shape == (Rp, R) and W3.shape == (R, R) and R <= 64
    g = np.empty(R)
    lib().less_oracle_psi(_ptr(k), _ptr(W1), _ptr(W2), _ptr(W3), D, Rp, R, _ptr(g))
    return g


class OracleState:
    """State of U independent (batch, head) units, all fp64 on the host.

    weights: dict Wq1 [Hh*G,D,R'], Wq2 [Hh*G,R',R] (per query head, head h's G query heads in
    a row), Wk1 [Hh,D,R'], Wk2 [Hh,R',R], Wk3 [Hh,R,R] (any float dtype; the values are taken
    exactly and widened to fp64).
    head_of_unit: (KV) head index of every unit (default u % heads).
    q_per_kv: G, query heads that share a unit's keys, values, cache and state (multi-query /
    grouped-query attention); with G > 1 queries and outputs carry an extra axis: q [U,G,D],
    Q [U,G,P,D].
    """

    def __init__(self, units, heads, head_dim, n_heavy, n_recent, rank, hidden, weights,
                 flags=0, head_of_unit=None, q_per_kv=1):
        self.G = int(q_per_kv)
        assert self.G >= 1
        self.U, self.heads, self.D = int(units), int(heads), int(head_dim)
        self.Nh, self.Nr = int(n_heavy), int(n_recent)
        self.C = self.Nh + self.Nr
        self.R, self.Rp = int(rank), int(hidden)
        assert self.R <= 64
        self.flags = int(flags)
        self.head = np.ascontiguousarray(
            np.arange(self.U) % self.heads if head_of_unit is None else head_of_unit,
            dtype=np.int32)
        assert self.head.shape == (self.U,) and self.head.max(initial=0) < self.heads
        self.W = {k: _f64(weights[k]) for k in ("Wq1", "Wq2", "Wk1", "Wk2", "Wk3")}
        assert self.W["Wq1"].shape == (self.heads * self.G, self.D, self.Rp)
        assert self.W["Wq2"].shape == (self.heads * self.G, self.Rp, self.R)
        assert self.W["Wk1"].shape == (self.heads, self.D, self.Rp)
        assert self.W["Wk2"].shape == (self.heads, self.Rp, self.R)
        assert self.W["Wk3"].shape == (self.heads, self.R, self.R)
        U, Cc, D, R = self.U, self.C, self.D, self.R
        self.Kc = np.zeros((U, Cc, D)); self.Vc = np.zeros((U, Cc, D))
        self.acc = np.zeros((U, Cc)); self.pos = np.full((U, Cc), -1, dtype=np.int64)
        self.H = np.zeros((U, R, D)); self.z = np.zeros((U, R))
        self.n = np.zeros(U, dtype=np.int64)

    def _struct(self):
        s = _State()
        s.U, s.heads, s.D = self.U, self.heads, self.D
        s.n_heavy, s.n_recent, s.R, s.Rp, s.flags = self.Nh, self.Nr, self.R, self.Rp, self.flags
        s.G = self.G
        s.head = self.head.ctypes.data
        for k in ("Wq1", "Wq2", "Wk1", "Wk2", "Wk3"):
            setattr(s, k, self.W[k].ctypes.data)
        s.Kc, s.Vc = self.Kc.ctypes.data, self.Vc.ctypes.data
        s.acc, s.pos = self.acc.ctypes.data, self.pos.ctypes.data
        s.H, s.z, s.n = self.H.ctypes.data, self.z.ctypes.data, self.n.ctypes.data
        return s

    def reset(self):
        lib().less_oracle_reset(C.byref(self._struct()))

    def step(self, q, k, v, force=None, strict=True):
        """One generation step for all units. q,k,v [U,D].

        Returns dict(out [U,D], evicted [U], dec [U,4], share [U]).
        force: None or int array [U]; entries >= 0 override the policy's choice.  A forced
        position that is not an eviction candidate is an error (strict) or leaves that unit
        on the policy's own choice, which `evicted` then shows (not strict).
        """
        q = _f64(q); k = _f64(k); v = _f64(v)
        qshape = (self.U, self.D) if self.G == 1 else (self.U, self.G, self.D)
        assert q.shape == qshape and k.shape == v.shape == (self.U, self.D)
        out = np.empty(qshape); ev = np.empty(self.U, dtype=np.int64)
        dec = np.empty((self.U, 4)); share = np.empty(self.U)
        fo = None if force is None else np.ascontiguousarray(force, dtype=np.int64)
        bad = lib().less_oracle_step(C.byref(self._struct()), _ptr(q), _ptr(k), _ptr(v),
                                     _ptr(fo), _ptr(out), _ptr(ev), _ptr(dec), _ptr(share))
        if bad and strict:
            raise ValueError(f"{bad} unit(s): forced position is not an eviction candidate")
        return {"out": out, "evicted": ev, "dec": dec, "share": share}

    def prefill(self, Q, K, V, want_out=True):
        """Prompt phase for all units. Q,K,V [U,P,D].

        Returns dict(out [U,P,D] or None, colsum [U,P], kept [U,P] bool, dec [U,4]).
        """
        Q = _f64(Q); K = _f64(K); V = _f64(V)
        assert K.shape == V.shape and K.shape[0] == self.U and K.shape[2] == self.D
        P = K.shape[1]
        assert Q.shape == (K.shape if self.G == 1 else (self.U, self.G, P, self.D))
        out = np.empty(Q.shape) if want_out else None
        colsum = np.zeros((self.U, P)); kept = np.ones((self.U, P), dtype=np.int8)
        dec = np.full((self.U, 4), np.inf); dec[:, 1::2] = -1
        lib().less_oracle_prefill(C.byref(self._struct()), _ptr(Q), _ptr(K), _ptr(V), P,
                                  _ptr(out), _ptr(colsum), _ptr(kept), _ptr(dec))
        return {"out": out, "colsum": colsum, "kept": kept.astype(bool), "dec": dec}
