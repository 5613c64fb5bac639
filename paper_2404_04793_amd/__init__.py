"""SqueezeAttention hot path for MI355X (gfx950): cosine-similarity layer
probe, per-layer KV budgets, prefill compression and decode attention over a
per-layer variable-length compact KV cache.  All compute runs in the HIP
library behind the C ABI of include/sqa.h; this package only marshals
arguments (see binding.py) and makes synthetic inputs (workloads.py)."""
