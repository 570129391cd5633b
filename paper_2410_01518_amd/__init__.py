"""libinfinipot: the CCD compression step of InfiniPot as hand-written HIP for gfx950.

`paper_2410_01518_amd.infinipot` is the ctypes binding of the C-ABI library
(include/infinipot.h); `paper_2410_01518_amd.synth` draws the seeded synthetic inputs.
"""
