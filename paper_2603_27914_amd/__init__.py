"""ITQ3_S fused 3-bit ternary matmul for AMD MI355X (gfx950).

``paper_2603_27914_amd.binding`` wraps the C-ABI library ``libitq3s`` (hand-written HIP kernels);
``paper_2603_27914_amd.synth`` draws the seeded synthetic tensors.  Importing the package itself
loads nothing heavy.
"""
__all__ = ["binding", "synth"]
