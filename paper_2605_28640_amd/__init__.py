"""MI355X-native hot path of recurrence-augmented attention under query-aware KV sparsity.

`binding` holds the thin ctypes layer over the C-ABI library (libratsparse.so, built
from csrc/ with hipcc for gfx950); `synth` holds the seeded synthetic workloads.
Nothing here computes any step of the method on the CPU: without the built HIP
library every call raises.
"""

__all__ = ["binding", "synth"]
