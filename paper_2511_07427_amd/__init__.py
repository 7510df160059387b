"""MI355X-native cluster-indexed sparse attention over an HBM-resident KVCache (DynaKV decode path).

`binding` is the thin ctypes layer over the C-ABI library built from `csrc/`; `workload` holds the
seeded synthetic inputs.  Nothing here falls back to a CPU implementation: without the built HIP
library every call raises.
"""
__all__ = ["binding", "workload"]
