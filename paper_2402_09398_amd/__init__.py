"""lessdec: the LESS decode hot path (H2O-evicted KV cache + low-rank state) for MI355X.

`binding` is the ctypes front end of the HIP library, `workloads` the seeded synthetic
inputs, `build` the in-tree build of liblessdec.so.
"""
from . import binding, workloads  # noqa: F401
from .binding import (LessDec, LessdecError, lessdec_budget_tokens, lessdec_prefill, lessdec_probe_stream_read,  # noqa: F401
                      lessdec_state_reset, lessdec_state_sync, lessdec_step, lessdec_step_attend,
                      lessdec_step_features, lessdec_step_static, lessdec_workspace_bytes, pack_weights)
