"""lessdec: the LESS decode hot path (H2O-evicted KV cache + low-rank state) for MI355X."""
