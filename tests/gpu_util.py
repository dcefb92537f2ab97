"""Helpers for the GPU parity tests: upload seeded inputs, run the C-ABI path, fetch results."""
import numpy as np
import torch

from paper_2509_24006_amd import binding as sla

TOL = {"fp32": 1e-5, "bf16": 1e-2}   # relative L2, per tensor
# relative L2 of every block of 64 consecutive tokens (or of every state row): three times the
# whole-tensor bound.  One wrong row of 64 moves its block's figure by about 1/8, whereas at
# N = 32760 it moves the whole-tensor figure by 5e-3 only and would pass that bound alone.
BLOCK_TOL = {"fp32": 3e-5, "bf16": 3e-2}


def max_block_rel_l2(got: np.ndarray, ref: np.ndarray, token_axis: int = 2, rows: int = 64,
                     floor_frac: float = 0.25):
    """Largest relative L2 error over the blocks of `rows` consecutive indices along token_axis
    (everything behind that axis belongs to the token).  A block whose reference norm is below
    floor_frac times the typical block norm is measured against that floor: its error is
    rounding noise of terms that cancel, not a fraction of what is left.
    Returns (worst error, index of the worst block as (leading index..., block))."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape
    lead = ref.shape[:token_axis + 1]
    e2 = ((got - ref) ** 2).reshape(lead + (-1,)).sum(-1)
    r2 = (ref ** 2).reshape(lead + (-1,)).sum(-1)
    n = lead[-1]
    nb = -(-n // rows)
    pad = [(0, 0)] * (len(lead) - 1) + [(0, nb * rows - n)]
    e2 = np.pad(e2, pad).reshape(lead[:-1] + (nb, rows)).sum(-1)
    r2 = np.pad(r2, pad).reshape(lead[:-1] + (nb, rows)).sum(-1)
    typical = np.sqrt(r2.mean())
    err = np.sqrt(e2) / np.maximum(np.sqrt(r2), floor_frac * typical + 1e-300)
    k = np.unravel_index(int(np.argmax(err)), err.shape)
    return float(err[k]), tuple(int(v) for v in k)


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x, np.float32))
    return t.to(torch.bfloat16 if dtype == "bf16" else torch.float32).cuda()


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def run_gpu(x, dtype: str, k_h: float, k_l: float, phi: int = 0, backward: bool = True,
            token_major: bool = False, bq: int = 64):
    """x: dict of float32 arrays Q,K,V[,dO] [B,H,N,d] and Proj [d,d].  Runs mask, forward
    and (optionally) backward through the C ABI and returns numpy results ([B,H,N,d] again).
    token_major: hand the library [B,N,H,d] tensors (the same values, transposed on the device).
    bq: query block size of the mask."""
    B, H, N, d = x["Q"].shape
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    p = sla.make_params(B, H, N, d, k_h, k_l, tdt, phi, bq=bq, layout=sla.SLA_BNHD if token_major else sla.SLA_BHND)
    tm = (lambda t: t.transpose(1, 2).contiguous()) if token_major else (lambda t: t)
    Q, K, V = (tm(to_dev(x[k], dtype)) for k in ("Q", "K", "V"))
    W = to_dev(x["Proj"], dtype)
    Mc, luts, ws = sla.sla_build_mask(p, Q, K)
    O, saved = sla.sla_forward(p, Q, K, V, W, Mc, luts)
    torch.cuda.synchronize()
    sv = sla.saved_views(p, saved)
    out = {"Mc": Mc.cpu().numpy(), "O": f64(tm(O))}
    out.update({k: f64(v) for k, v in sv.items()})
    out.update({k: v.cpu().numpy() for k, v in sla.mask_ws_views(p, ws).items()})
    out.update({k: v.cpu().numpy() for k, v in sla.lut_views(p, luts).items()})
    if backward:
        dO = tm(to_dev(x["dO"], dtype))
        dQ, dK, dV, dW = sla.sla_backward(p, Q, K, V, W, Mc, luts, saved, dO)
        torch.cuda.synchronize()
        out.update({"dQ": f64(tm(dQ)), "dK": f64(tm(dK)), "dV": f64(tm(dV)), "dW": f64(dW)})
    return out


def per_tile(a: np.ndarray, rq: int, T: int, axis: int = 2) -> np.ndarray:
    """Rows of a per-query-block array given to each of the block's rq 64-token tiles (T in all)."""
    return np.repeat(a, rq, axis=axis).take(np.arange(T), axis=axis)


def check_luts(Mc: np.ndarray, row_idx: np.ndarray, col_ptr: np.ndarray, col_rows: np.ndarray,
               ind: np.ndarray = None, ind_t: np.ndarray = None, col_order: np.ndarray = None):
    """The tables against the mask, both over 64-token query tiles: Mc is [B,H,T,T] (for larger
    query blocks: per_tile(Mc, rq, T))."""
    B, H, T, _ = Mc.shape
    assert Mc.shape[-1] == T
    if ind is not None:
        # bit b of word q of row i: block (i, 64 q + b) is marginal; bits past T are clear
        Tw = ind.shape[-1]
        assert Tw == (T + 63) // 64

        def pack(m):
            bits = np.zeros((B, H, T, Tw * 64), np.uint8)
            bits[..., :T] = m
            return np.packbits(bits.reshape(B, H, T, Tw, 64), axis=-1, bitorder="little").view(np.uint64)[..., 0]

        assert np.array_equal(ind.view(np.uint64), pack(Mc == 0))
        assert np.array_equal(ind_t.view(np.uint64), pack(np.swapaxes(Mc == 0, -1, -2)))
    if col_order is not None:
        cnt = (Mc == 1).sum(-2)
        for b in range(B):
            for h in range(H):
                want = np.lexsort((np.arange(T), -cnt[b, h]))   # count descending, index ascending
                assert np.array_equal(col_order[b, h], want)
    for b in range(B):
        for h in range(H):
            crit = Mc[b, h] == 1
            for i in range(T):
                assert np.array_equal(row_idx[b, h, i], np.nonzero(crit[i])[0])
            ptr = col_ptr[b, h]
            assert ptr[0] == 0 and np.array_equal(np.diff(ptr), crit.sum(0))
            for j in range(T):
                assert np.array_equal(col_rows[b, h, ptr[j]:ptr[j + 1]], np.nonzero(crit[:, j])[0])
