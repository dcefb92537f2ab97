"""torch.autograd wrapper over the C-ABI calls of binding.py (fine-tuning use of Section 5).

    O = sla_attention(Q, K, V, W, k_h=0.05, k_l=0.10)

runs sla_build_mask + sla_forward and records sla_backward; every step is a kernel of
libsla_hip.so, this module only keeps the buffers alive between the two passes.  The mask is a
constant of the graph (no gradient flows into the block scores); a mask built once can be passed
back in through `mask=` and reused, e.g. across the steps of a diffusion sampler.
"""
from __future__ import annotations

from typing import Optional, Tuple

import torch

from . import binding as sla


class _SLAFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, W, p, Mc, luts):
        # the library reads W in the storage type of Q, K, V (a float parameter next to bf16
        # activations is cast here; its gradient goes back in the parameter's own type)
        ctx.w_dtype = W.dtype
        W = W.detach().to(Q.dtype).contiguous()
        O, saved = sla.sla_forward(p, Q, K, V, W, Mc, luts, need_saved=True)
        ctx.p = p
        ctx.save_for_backward(Q, K, V, W, Mc, luts, saved)
        return O

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, W, Mc, luts, saved = ctx.saved_tensors
        dQ, dK, dV, dW = sla.sla_backward(ctx.p, Q, K, V, W, Mc, luts, saved, dO.contiguous())
        return dQ, dK, dV, dW.to(ctx.w_dtype), None, None, None


def build_mask(Q: torch.Tensor, K: torch.Tensor, k_h: float, k_l: float,
               phi: int = sla.SLA_PHI_SOFTMAX, token_major: bool = False, bq: int = 64
               ) -> Tuple[sla.sla_params, torch.Tensor, torch.Tensor]:
    """(params, M_c int8 [B,H,ceil(N/bq),ceil(N/64)], lookup tables) for contiguous [B,H,N,d]
    tensors, or [B,N,H,d] ones with token_major.  bq: query block size of the mask (64 .. 256)."""
    if token_major:
        B, N, H, d = Q.shape
    else:
        B, H, N, d = Q.shape
    p = sla.make_params(B, H, N, d, k_h, k_l, Q.dtype, phi=phi, bq=bq,
                        layout=sla.SLA_BNHD if token_major else sla.SLA_BHND)
    Mc, luts, _ = sla.sla_build_mask(p, Q.detach(), K.detach())
    return p, Mc, luts


def sla_attention(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, W: torch.Tensor,
                  k_h: float = 0.05, k_l: float = 0.10, phi: int = sla.SLA_PHI_SOFTMAX,
                  mask: Optional[Tuple[sla.sla_params, torch.Tensor, torch.Tensor]] = None,
                  token_major: bool = False, bq: int = 64) -> torch.Tensor:
    """O = O^s + Proj(O^l) (Eq. 6) with gradients to Q, K, V and the Proj weight W [d, d].
    Q, K, V (and O, and the gradients) are [B,H,N,d], or [B,N,H,d] with token_major -- the order
    in which a transformer block's projections leave them, no transpose needed."""
    if mask is None:
        mask = build_mask(Q, K, k_h, k_l, phi, token_major, bq)
    p, Mc, luts = mask
    return _SLAFunction.apply(Q, K, V, W, p, Mc, luts)
