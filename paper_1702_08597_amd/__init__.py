"""swconv: sparse Winograd convolution forward pass (arxiv 1702.08597, Section 5) for MI355X.

``binding`` mirrors the C ABI of ``include/swconv.h``; ``synth`` draws the seeded synthetic
inputs; ``build`` compiles the HIP library in-tree.  Nothing here computes on the CPU.
"""
