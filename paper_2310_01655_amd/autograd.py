"""torch.autograd glue over the C ABI, for callers that train.

Only marshalling happens here: the forward is psf_causal_attn_fwd_save where the library keeps
the forward state for the backward pass (psf_fwd_save_bytes(desc) > 0), psf_causal_attn_fwd
elsewhere; the backward is psf_causal_attn_bwd_saved / psf_causal_attn_bwd.  The Gaussian
sketch matrices G are constants of the layer (Algorithm 1 draws them once): they receive no
gradient.  With learned sketches (Algorithm 2) G holds the networks' parameters, which are
trained with the model: when G requires a gradient the backward is
psf_causal_attn_bwd_saved_learned / psf_causal_attn_bwd_learned and G receives the parameter gradient (accumulated in fp32 by the library, returned in G's dtype).
"""
import torch

from . import binding as psf


class _CausalPolysketchAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, G, desc):
        Q, K, V = Q.contiguous(), K.contiguous(), V.contiguous()
        stream = torch.cuda.current_stream(Q.device)
        if psf.fwd_save_bytes(desc) > 0:
            O, save = psf.psf_causal_attn_fwd_save(desc, Q, K, V, G, stream=stream)
        else:
            O, save = psf.psf_causal_attn_fwd(desc, Q, K, V, G, stream=stream), None
        ctx.desc, ctx.save = desc, save
        ctx.g_grad = bool(desc.learned) and G is not None and G.requires_grad
        ctx.save_for_backward(Q, K, V, G if G is not None else Q.new_empty(0), O)
        return O

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, G, O = ctx.saved_tensors
        G = G if G.numel() else None
        dO = dO.contiguous()
        stream = torch.cuda.current_stream(Q.device)
        if ctx.g_grad:
            if ctx.save is not None:
                dQ, dK, dV, dG = psf.psf_causal_attn_bwd_saved_learned(ctx.desc, Q, K, V, G, O, dO, ctx.save,
                                                                       stream=stream)
            else:
                dQ, dK, dV, dG = psf.psf_causal_attn_bwd_learned(ctx.desc, Q, K, V, G, dO, stream=stream)
            return dQ, dK, dV, dG.to(G.dtype), None
        if ctx.save is not None:
            dQ, dK, dV = psf.psf_causal_attn_bwd_saved(ctx.desc, Q, K, V, G, O, dO, ctx.save, stream=stream)
        else:
            dQ, dK, dV = psf.psf_causal_attn_bwd(ctx.desc, Q, K, V, G, dO, stream=stream)
        return dQ, dK, dV, None, None


def causal_polysketch_attention(Q, K, V, G, p, r, b, local=psf.LOCAL_EXACT, per_head=False, learned=False):
    """Differentiable causal Polysketch attention (Sections 3, 3.1, 3.2 of the paper) of
    Q, K [batch, heads, n, d] and V [batch, heads, n, dv] on the GPU; G as for
    psf_causal_attn_fwd ([1 or heads, g_len(d, r, p)], None for p = 2; with learned = True the
    networks' parameters of Algorithm 2, [1 or heads, learned_len(d, r, p)]).  Gradients flow to
    Q, K and V, and to G when it holds learned parameters that require a gradient."""
    B, H, n, d = Q.shape
    dtype = {torch.float32: "f32", torch.bfloat16: "bf16"}[Q.dtype]
    desc = psf.make_desc(B, H, n, d, p, r, b, dtype, dv=V.shape[-1], local=local, per_head=per_head,
                         learned=learned)
    return _CausalPolysketchAttention.apply(Q, K, V, G, desc)
