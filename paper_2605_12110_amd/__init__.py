"""absb: adaptive-block sparse decode attention for AMD MI355X (gfx950).

`paper_2605_12110_amd.absb` is the thin binding over the C-ABI library libabsb.so
(hand-written HIP kernels); `paper_2605_12110_amd.synth` draws the seeded synthetic
workloads.  Nothing is imported eagerly: importing the package needs neither a GPU nor
the built library, calling into `absb` needs both and fails loudly without them.
"""
__all__ = ["absb", "synth"]
