"""libgka on MI355X: the Gated KalmaNet (GKA) layer forward pass as hand-written gfx950 HIP kernels.

`paper_2511_21016_amd.binding` wraps the C-ABI library (include/gka.h); `synth` draws the seeded
synthetic workloads.  Importing the package does not load the native library; the binding loads it
on first use and fails loudly when it has not been built.
"""
__all__ = ["binding", "synth"]
