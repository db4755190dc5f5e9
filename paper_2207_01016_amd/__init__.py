"""MI355X-native Nystrom factor G = K(X, L) W^T and margin sweep G w (LPD-SVM, Figure 1 steps 1d and 2a).

`paper_2207_01016_amd.lpd` is the thin binding over the C-ABI library (HIP, gfx950);
`paper_2207_01016_amd.workloads` draws the seeded synthetic inputs.  Nothing is loaded at import time.
"""
__all__ = ["lpd", "workloads"]
