"""MI355X-native incremental TGN / TGAT inference step (StreamTGN's per-batch index refresh).

`binding.StreamTGN` wraps the C-ABI library `libstreamtgn.so` (hand-written HIP kernels for
gfx950); `synth` holds the seeded synthetic workloads.  Importing the package loads nothing;
the library is loaded on first use and its absence is an error, never a fallback.
"""
__all__ = ["binding", "synth", "build"]
