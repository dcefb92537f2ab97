"""Independent definitions the oracle is pinned against (CPU, torch float64).

Nothing here follows the oracle's loop structure: masks are expanded to N x N, softmax is
taken over full rows, the linear branch is written in its quadratic form (Section 4.2's
display: phi(Q) phi(K)^T restricted to marginal blocks, row-normalised), and gradients come
from torch.autograd, not from Algorithm 2.
"""
import math

import numpy as np
import torch


def expand(Mc: np.ndarray, N: int, bq: int, bkv: int, value: int) -> torch.Tensor:
    """[Tm,Tn] block labels -> [N,N] boolean indicator of label == value."""
    m = torch.from_numpy(np.asarray(Mc) == value)
    return m.repeat_interleave(bq, 0).repeat_interleave(bkv, 1)[:N, :N]


def phi_t(x: torch.Tensor, phi: int) -> torch.Tensor:
    if phi == 0:
        return torch.softmax(x, dim=-1)
    return torch.where(x > 0, x + 1, torch.exp(x))


def sla_dense(Q, K, V, W, Mc, bq, bkv, phi=0):
    """One head, torch float64 tensors [N,d].  Returns O, Os, Ol."""
    N, d = Q.shape
    E1 = expand(Mc, N, bq, bkv, 1)
    E0 = expand(Mc, N, bq, bkv, 0)
    S = (Q @ K.T) / math.sqrt(d)
    S = S.masked_fill(~E1, float("-inf"))
    has1 = E1.any(dim=1, keepdim=True)
    P = torch.softmax(torch.where(has1, S, torch.zeros_like(S)), dim=-1) * E1
    Os = P @ V
    A = (phi_t(Q, phi) @ phi_t(K, phi).T) * E0
    den = A.sum(dim=1, keepdim=True)
    has0 = E0.any(dim=1, keepdim=True)
    Ol = torch.where(has0, (A @ V) / torch.where(has0, den, torch.ones_like(den)),
                     torch.zeros_like(Os))
    return Os + Ol @ W, Os, Ol


def sla_dense_grads(Q, K, V, W, Mc, dO, bq, bkv, phi=0):
    t = [torch.tensor(np.asarray(a, np.float64), requires_grad=True) for a in (Q, K, V, W)]
    O, Os, Ol = sla_dense(*t, Mc, bq, bkv, phi)
    (O * torch.tensor(np.asarray(dO, np.float64))).sum().backward()
    return (O.detach().numpy(), Os.detach().numpy(), Ol.detach().numpy(),
            [a.grad.numpy() for a in t])


def mask_by_rank_count(s: np.ndarray, n_h: int, n_l: int) -> np.ndarray:
    """Eq. 3 by counting: an entry is critical iff fewer than n_h entries precede it in
    (score descending, index ascending) order; negligible likewise among non-critical ones."""
    s = np.asarray(s, np.float32)
    rows, Tn = s.shape
    M = np.zeros((rows, Tn), np.int8)
    for i in range(rows):
        r = s[i]
        for j in range(Tn):
            before = np.sum(r > r[j]) + np.sum((r == r[j])[:j])
            if before < n_h:
                M[i, j] = 1
        rest = [j for j in range(Tn) if M[i, j] == 0]
        for j in rest:
            before = sum(1 for k in rest if r[k] < r[j] or (r[k] == r[j] and k < j))
            if before < n_l:
                M[i, j] = -1
    return M


def rel_l2(x, ref) -> float:
    x = np.asarray(x, np.float64)
    ref = np.asarray(ref, np.float64)
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((x - ref).ravel())
    return float(num / den) if den > 0 else float(num)
