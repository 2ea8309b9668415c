"""Causal polynomial-sketch attention (PolySketchFormer, arXiv 2310.01655) for MI355X.

The product is the C-ABI library built from csrc/ (see include/psf.h); `binding`
marshals torch device tensors into it, `autograd` wraps the forward / backward pair
as a torch.autograd.Function and `inputs` draws the seeded synthetic workloads.  Nothing here falls back to a CPU implementation: if the HIP library
is missing or no GPU is present, calls raise.
"""
__all__ = ["autograd", "binding", "inputs"]
