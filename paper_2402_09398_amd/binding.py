"""ctypes binding of liblessdec.so: argument marshalling only.

The three calls have the names and meaning of include/lessdec.h.  Everything they
compute runs in the HIP kernels; torch is used for device memory and streams.
There is no fallback: if the library is not built, or no GPU is present when a
call is made, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path

_HERE = Path(__file__).resolve().parent
LIB_PATH = _HERE / "liblessdec.so"

DTYPE_F32, DTYPE_F16 = 0, 1
FLAG_SPARSE_DENOM = 1
FLAG_LAMBDA = 2
FLAG_PROMPT_STEPWISE = 4
OK, EINVAL, EWORKSPACE, EHIP, ESCRATCH = 0, -1, -2, -3, -4
STATIC_SCRATCH_BYTES = 4 << 20

EXPORTS = ("lessdec_workspace_bytes", "lessdec_state_reset", "lessdec_state_sync", "lessdec_prefill", "lessdec_step", "lessdec_step_features", "lessdec_step_attend", "lessdec_step_static",
           "lessdec_probe_stream_read", "lessdec_step_launches",
           "lessdec_strerror", "lessdec_budget_tokens")


class LessdecError(RuntimeError):
    pass


class Desc(C.Structure):
    """Mirror of struct lessdec_desc."""
    _fields_ = [
        ("batch", C.c_int32), ("heads", C.c_int32), ("head_dim", C.c_int32),
        ("n_heavy", C.c_int32), ("n_recent", C.c_int32),
        ("rank", C.c_int32), ("hidden", C.c_int32),
        ("dtype", C.c_int32), ("flags", C.c_uint32), ("q_per_kv", C.c_int32),
        ("k_cache", C.c_void_p), ("v_cache", C.c_void_p),
        ("acc", C.c_void_p), ("pos", C.c_void_p), ("psi", C.c_void_p),
        ("H", C.c_void_p), ("z", C.c_void_p), ("n_seen", C.c_void_p),
        ("pend_slot", C.c_void_p), ("pend_v", C.c_void_p), ("pend_psi", C.c_void_p),
        ("Wq1", C.c_void_p), ("Wq2", C.c_void_p),
        ("Wk1", C.c_void_p), ("Wk2", C.c_void_p), ("Wk3", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
    ]


_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise LessdecError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2402_09398_amd.build)")
        L = C.CDLL(str(LIB_PATH))
        L.lessdec_workspace_bytes.restype = C.c_size_t
        L.lessdec_workspace_bytes.argtypes = [C.POINTER(Desc), C.c_int32]
        L.lessdec_state_reset.restype = C.c_int
        L.lessdec_state_reset.argtypes = [C.POINTER(Desc), C.c_void_p]
        L.lessdec_state_sync.restype = C.c_int
        L.lessdec_state_sync.argtypes = [C.POINTER(Desc), C.c_void_p]
        L.lessdec_prefill.restype = C.c_int
        L.lessdec_prefill.argtypes = [C.POINTER(Desc)] + [C.c_void_p] * 3 + [C.c_int32] + [C.c_void_p] * 2
        L.lessdec_step.restype = C.c_int
        L.lessdec_step.argtypes = [C.POINTER(Desc)] + [C.c_void_p] * 6
        L.lessdec_step_static.restype = C.c_int
        L.lessdec_step_static.argtypes = [C.POINTER(Desc)] + [C.c_void_p] * 6
        L.lessdec_step_features.restype = C.c_int
        L.lessdec_step_features.argtypes = [C.POINTER(Desc)] + [C.c_void_p] * 3
        L.lessdec_step_attend.restype = C.c_int
        L.lessdec_step_attend.argtypes = [C.POINTER(Desc)] + [C.c_void_p] * 6
        L.lessdec_probe_stream_read.restype = C.c_int
        L.lessdec_probe_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.c_void_p]
        L.lessdec_step_launches.restype = C.c_int
        L.lessdec_step_launches.argtypes = [C.POINTER(Desc)]
        L.lessdec_strerror.restype = C.c_char_p
        L.lessdec_strerror.argtypes = [C.c_int]
        L.lessdec_budget_tokens.restype = C.c_int32
        L.lessdec_budget_tokens.argtypes = [C.c_double, C.c_int32]
        _lib = L
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        raise LessdecError(f"{what}: {lib().lessdec_strerror(rc).decode()} ({rc})")


def _p(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def lessdec_budget_tokens(percent: float, max_len: int) -> int:
    return int(lib().lessdec_budget_tokens(float(percent), int(max_len)))


def lessdec_workspace_bytes(desc: Desc, max_prompt: int) -> int:
    return int(lib().lessdec_workspace_bytes(C.byref(desc), int(max_prompt)))


def lessdec_state_reset(desc: Desc, stream=None):
    _check(lib().lessdec_state_reset(C.byref(desc), _stream(stream)), "lessdec_state_reset")


def lessdec_state_sync(desc: Desc, stream=None):
    _check(lib().lessdec_state_sync(C.byref(desc), _stream(stream)), "lessdec_state_sync")


def lessdec_prefill(desc: Desc, Q, K, V, P: int, out=None, stream=None):
    _check(lib().lessdec_prefill(C.byref(desc), _p(Q), _p(K), _p(V), int(P), _p(out),
                                 _stream(stream)), "lessdec_prefill")


def lessdec_step_features(desc: Desc, q, k, stream=None):
    _check(lib().lessdec_step_features(C.byref(desc), _p(q), _p(k), _stream(stream)), "lessdec_step_features")


def lessdec_step_attend(desc: Desc, q, k, v, out, evicted_pos=None, stream=None):
    _check(lib().lessdec_step_attend(C.byref(desc), _p(q), _p(k), _p(v), _p(out), _p(evicted_pos),
                                     _stream(stream)), "lessdec_step_attend")


def lessdec_step(desc: Desc, q, k, v, out, evicted_pos=None, stream=None):
    _check(lib().lessdec_step(C.byref(desc), _p(q), _p(k), _p(v), _p(out), _p(evicted_pos),
                              _stream(stream)), "lessdec_step")


def lessdec_step_static(desc: Desc, q, k, v, out, evicted_pos=None, stream=None):
    _check(lib().lessdec_step_static(C.byref(desc), _p(q), _p(k), _p(v), _p(out), _p(evicted_pos),
                                     _stream(stream)), "lessdec_step_static")


def lessdec_step_launches(desc: Desc) -> int:
    return int(lib().lessdec_step_launches(C.byref(desc)))


def lessdec_probe_stream_read(buf, nbytes: int, waves: int, sink, stream=None):
    _check(lib().lessdec_probe_stream_read(_p(buf), int(nbytes), int(waves), _p(sink), _stream(stream)),
           "lessdec_probe_stream_read")


def pack_weights(weights, device="cuda:0"):
    """Equation-layout numpy weights (Wq1 [Hh,D,R'], Wq2 [Hh,R',R], Wk1, Wk2, Wk3 [Hh,R,R])
    to the library's output-major device tensors ([Hh,R',D], [Hh,R,R'], [Hh,R,R])."""
    import numpy as np
    import torch
    return {k: torch.from_numpy(np.ascontiguousarray(np.swapaxes(v, 1, 2))).to(device)
            for k, v in weights.items()}


class LessDec:
    """Owns the device buffers of one attention layer's state and its descriptor.

    Plumbing only: allocation with torch, pointer marshalling, no arithmetic.
    weights: dict of torch tensors on the device in the library's output-major layout,
    Wq1 [Hh,R',D], Wq2 [Hh,R,R'], Wk1 [Hh,R',D], Wk2 [Hh,R,R'], Wk3 [Hh,R,R], storage dtype
    (see pack_weights).
    """

    # every buffer that makes up the state of the method (a checkpoint copies these)
    STATE = ("k_cache", "v_cache", "acc", "pos", "psi", "H", "z", "n_seen",
             "pend_slot", "pend_v", "pend_psi")

    def __init__(self, batch, heads, head_dim, n_heavy, n_recent, rank, hidden, dtype, weights,
                 flags=0, max_prompt=0, device="cuda:0", q_per_kv=1):
        import torch
        if not torch.cuda.is_available():
            raise LessdecError("no GPU visible: lessdec has no CPU path")
        lib()
        self.torch = torch
        self.device = torch.device(device)
        self.tdtype = torch.float16 if dtype in ("f16", DTYPE_F16) else torch.float32
        self.B, self.Hh, self.D = batch, heads, head_dim
        self.Nh, self.Nr, self.C = n_heavy, n_recent, n_heavy + n_recent
        self.R, self.Rp = rank, hidden
        self.G = G = int(q_per_kv)            # query heads per unit; q, out and Wq1, Wq2 carry this axis
        U, Cc, D, R = batch * heads, self.C, head_dim, rank
        dev = self.device
        self.k_cache = torch.zeros((U, Cc, D), dtype=self.tdtype, device=dev)
        self.v_cache = torch.zeros((U, Cc, D), dtype=self.tdtype, device=dev)
        self.acc = torch.zeros((U, Cc), dtype=torch.float64, device=dev)
        self.pos = torch.full((U, Cc), -1, dtype=torch.int32, device=dev)
        self.psi = torch.zeros((U, Cc, R), dtype=torch.float32, device=dev)
        self.H = torch.zeros((U, R, D), dtype=torch.float32, device=dev)
        self.z = torch.zeros((U, R), dtype=torch.float64, device=dev)
        self.n_seen = torch.zeros((U,), dtype=torch.int32, device=dev)
        self.pend_slot = torch.full((U,), -1, dtype=torch.int32, device=dev)
        self.pend_v = torch.zeros((U, D), dtype=self.tdtype, device=dev)
        self.pend_psi = torch.zeros((U, R), dtype=torch.float32, device=dev)
        self.W = {}
        for name, shape in (("Wq1", (heads * G, hidden, D)), ("Wq2", (heads * G, R, hidden)),
                            ("Wk1", (heads, hidden, D)), ("Wk2", (heads, R, hidden)),
                            ("Wk3", (heads, R, R))):
            w = weights[name]
            if tuple(w.shape) != shape or w.dtype != self.tdtype or w.device != self.k_cache.device:
                raise LessdecError(f"weight {name}: expected {shape} {self.tdtype} on {dev}")
            self.W[name] = w.contiguous()
        d = Desc()
        d.batch, d.heads, d.head_dim = batch, heads, head_dim
        d.n_heavy, d.n_recent, d.rank, d.hidden = n_heavy, n_recent, rank, hidden
        d.dtype = DTYPE_F16 if self.tdtype == torch.float16 else DTYPE_F32
        d.flags = flags
        d.q_per_kv = G
        for name in self.STATE:
            setattr(d, name, getattr(self, name).data_ptr())
        for name in self.W:
            setattr(d, name, self.W[name].data_ptr())
        need = lessdec_workspace_bytes(d, max_prompt)
        if need == 0:
            raise LessdecError("lessdec_workspace_bytes: invalid shape")
        # 0xFF bytes: the per-step exchange array of the one-launch step reads as empty (lessdec.h)
        self.workspace = torch.full((need,), 255, dtype=torch.uint8, device=dev)
        d.workspace = self.workspace.data_ptr()
        d.workspace_bytes = need
        self.desc = d
        self.max_prompt = max_prompt

    def state_reset(self, stream=None):
        lessdec_state_reset(self.desc, stream)

    def state_sync(self, stream=None):
        lessdec_state_sync(self.desc, stream)

    def prefill(self, Q, K, V, out=None, stream=None):
        """K, V: [B*Hh, P, D] (or [B,Hh,P,D]), Q, out: the same with an axis G before P if
        q_per_kv > 1; contiguous device tensors of the storage dtype."""
        P = K.shape[-2]
        for t, g in ((Q, self.G), (K, 1), (V, 1)) + (((out, self.G),) if out is not None else ()):
            if t.dtype != self.tdtype or not t.is_contiguous() or t.numel() != self.B * self.Hh * g * P * self.D:
                raise LessdecError("prefill: tensors must be contiguous [B,Hh,(G,)P,D] of the storage dtype")
        if P > self.max_prompt:
            raise LessdecError(f"prefill: P={P} exceeds max_prompt={self.max_prompt} the workspace was sized for")
        lessdec_prefill(self.desc, Q, K, V, P, out, stream)

    def step(self, q, k, v, out, evicted_pos=None, stream=None):
        """q, k, v, out: [B*Hh, D] contiguous device tensors; evicted_pos: int32 [B*Hh] or None."""
        for t, g in ((q, self.G), (k, 1), (v, 1), (out, self.G)):
            if t.dtype != self.tdtype or not t.is_contiguous() or t.numel() != self.B * self.Hh * g * self.D:
                raise LessdecError("step: tensors must be contiguous [B,Hh,(G,)D] of the storage dtype")
        if evicted_pos is not None and (evicted_pos.dtype != self.torch.int32 or
                                        evicted_pos.numel() != self.B * self.Hh):
            raise LessdecError("step: evicted_pos must be int32 [B,Hh]")
        lessdec_step(self.desc, q, k, v, out, evicted_pos, stream)

    def step_features(self, q, k, stream=None):
        """First half of step(): phi(q), psi(k) of the step into the workspace."""
        for t, g in ((q, self.G), (k, 1)):
            if t.dtype != self.tdtype or not t.is_contiguous() or t.numel() != self.B * self.Hh * g * self.D:
                raise LessdecError("step_features: tensors must be contiguous [B,Hh,(G,)D] of the storage dtype")
        lessdec_step_features(self.desc, q, k, stream)

    def step_attend(self, q, k, v, out, evicted_pos=None, stream=None):
        """Second half of step(), after step_features(q, k) on the same tensors."""
        for t, g in ((q, self.G), (k, 1), (v, 1), (out, self.G)):
            if t.dtype != self.tdtype or not t.is_contiguous() or t.numel() != self.B * self.Hh * g * self.D:
                raise LessdecError("step_attend: tensors must be contiguous [B,Hh,(G,)D] of the storage dtype")
        if evicted_pos is not None and (evicted_pos.dtype != self.torch.int32 or
                                        evicted_pos.numel() != self.B * self.Hh):
            raise LessdecError("step_attend: evicted_pos must be int32 [B,Hh]")
        lessdec_step_attend(self.desc, q, k, v, out, evicted_pos, stream)
