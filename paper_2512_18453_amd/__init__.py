"""MI355X-native Winograd F(m x m, 3 x 3) convolution with Cook-Toom transforms built
from arbitrary interpolation points.  `paper_2512_18453_amd.nova` is the thin binding
over the C-ABI library; `paper_2512_18453_amd.synth` the seeded synthetic workloads."""
