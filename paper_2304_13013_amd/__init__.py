"""SwitchBack int8 linear layer (arxiv 2304.13013, Algorithm 1) as hand-written gfx950 HIP kernels.

`paper_2304_13013_amd.switchback` is the thin binding over the C-ABI library (it needs the built library and a
GPU and raises if either is missing); `paper_2304_13013_amd.inputs` draws the seeded synthetic tensors.
"""
