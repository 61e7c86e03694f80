"""MI355X-native batched inside / inside-backward for simple PCFGs (pi(A->BC) = L[A,B] * R[A,C]).

`binding` wraps the C-ABI library built from csrc/ (HIP kernels for gfx950); `synth` draws seeded
synthetic workloads.  The binding is imported lazily so that CPU-only tools can use `synth` without
the built library; any call into the path without the library raises.
"""
__all__ = ["binding", "synth"]
