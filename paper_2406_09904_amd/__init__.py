"""MI355X-native W4A8 GEMM hot path of QQQ (arXiv 2406.09904): thin Python binding over a
C-ABI library of hand-written gfx950 kernels.  ``synth`` holds the seeded input generators."""
