"""MI355X-native hot path of GAD's per-processor GCN training step (arXiv 2110.02987).

`paper_2110_02987_amd.gad` is the thin binding over the C-ABI library `libgad.so`
(hand-written HIP kernels for gfx950); `paper_2110_02987_amd.workloads` generates
the seeded synthetic inputs.  Importing the package loads nothing native.
"""
__all__ = ["workloads"]
