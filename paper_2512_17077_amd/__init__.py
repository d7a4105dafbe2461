"""Head-Centric Sparse Attention for diffusion-LLM serving on AMD MI355X (gfx950).

`hcsa` is the thin binding over the C-ABI library (hand-written HIP kernels);
`synth` draws the seeded synthetic workloads.  Importing this package loads
nothing native; the library is opened on first use and a missing build is an
error, never a fallback.
"""

__all__ = ["hcsa", "synth", "build"]
