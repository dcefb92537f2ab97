"""The torch.autograd wrapper drives the same C-ABI calls: its output and the gradients autograd
hands back are compared with the CPU oracle on a small ragged bf16 case and a float case."""
import numpy as np
import pytest
import torch

from paper_2509_24006_amd import workloads as wl
from tests import pins
from tests.gpu_util import TOL

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["small_fp32", "small_bf16_d64"])
def test_autograd_matches_oracle(oracle, name):
    from paper_2509_24006_amd.autograd import build_mask, sla_attention
    w = wl.WORKLOADS[name]
    x = wl.make_inputs(w)
    tdt = torch.float32 if w.dtype == "fp32" else torch.bfloat16
    dev = torch.device("cuda:0")
    Q, K, V = (torch.from_numpy(x[k]).to(dev).to(tdt).requires_grad_(True) for k in ("Q", "K", "V"))
    W = torch.from_numpy(x["Proj"]).to(dev).to(tdt).requires_grad_(True)
    dO = torch.from_numpy(x["dO"]).to(dev).to(tdt)
    mask = build_mask(Q, K, w.k_h, w.k_l)
    O = sla_attention(Q, K, V, W, mask=mask)
    O.backward(dO)
    torch.cuda.synchronize()
    Mc = oracle.build_mask(x["Q"], x["K"], w.k_h, w.k_l)
    assert np.array_equal(mask[1].cpu().numpy(), Mc)
    f = oracle.forward(x["Q"], x["K"], x["V"], x["Proj"], Mc)
    g = oracle.backward(x["Q"], x["K"], x["V"], x["Proj"], Mc, f, x["dO"])
    tol = TOL[w.dtype]
    for n, got, ref in (("O", O, f["O"]), ("dQ", Q.grad, g["dQ"]), ("dK", K.grad, g["dK"]),
                        ("dV", V.grad, g["dV"]), ("dW", W.grad, g["dW"])):
        err = pins.rel_l2(got.detach().float().cpu().numpy(), ref)
        print(f"  {name} {n}: rel_l2 = {err:.3e}", flush=True)
        assert err <= tol, f"{n}: {err:.3e}"


def test_autograd_with_query_blocks_of_128(oracle):
    from paper_2509_24006_amd.autograd import sla_attention
    w = wl.WORKLOADS["small_bf16_d64"]
    x = wl.make_inputs(w)
    dev = torch.device("cuda:0")
    Q, K, V = (torch.from_numpy(x[k]).to(dev).to(torch.bfloat16).requires_grad_(True) for k in ("Q", "K", "V"))
    W = torch.from_numpy(x["Proj"]).to(dev).to(torch.bfloat16).requires_grad_(True)
    O = sla_attention(Q, K, V, W, k_h=w.k_h, k_l=w.k_l, bq=128)
    O.backward(torch.from_numpy(x["dO"]).to(dev).to(torch.bfloat16))
    torch.cuda.synchronize()
    Mc = oracle.build_mask(x["Q"], x["K"], w.k_h, w.k_l, bq=128)
    f = oracle.forward(x["Q"], x["K"], x["V"], x["Proj"], Mc, bq=128)
    g = oracle.backward(x["Q"], x["K"], x["V"], x["Proj"], Mc, f, x["dO"], bq=128)
    for n, got, ref in (("O", O, f["O"]), ("dQ", Q.grad, g["dQ"]), ("dK", K.grad, g["dK"]),
                        ("dV", V.grad, g["dV"]), ("dW", W.grad, g["dW"])):
        err = pins.rel_l2(got.detach().float().cpu().numpy(), ref)
        print(f"  b_q=128 {n}: rel_l2 = {err:.3e}", flush=True)
        assert err <= TOL["bf16"], f"{n}: {err:.3e}"


def test_autograd_token_major(oracle):
    # [B,N,H,d] tensors, as a transformer block's projections leave them
    from paper_2509_24006_amd.autograd import sla_attention
    w = wl.WORKLOADS["small_bf16"]
    x = wl.make_inputs(w)
    dev = torch.device("cuda:0")
    tm = lambda a: torch.from_numpy(a).to(dev).to(torch.bfloat16).transpose(1, 2).contiguous()
    Q, K, V = (tm(x[k]).requires_grad_(True) for k in ("Q", "K", "V"))
    W = torch.from_numpy(x["Proj"]).to(dev).to(torch.bfloat16).requires_grad_(True)
    O = sla_attention(Q, K, V, W, k_h=w.k_h, k_l=w.k_l, token_major=True)
    assert O.shape == Q.shape
    O.backward(tm(x["dO"]))
    torch.cuda.synchronize()
    Mc = oracle.build_mask(x["Q"], x["K"], w.k_h, w.k_l)
    f = oracle.forward(x["Q"], x["K"], x["V"], x["Proj"], Mc)
    g = oracle.backward(x["Q"], x["K"], x["V"], x["Proj"], Mc, f, x["dO"])
    back = lambda t: t.detach().float().transpose(1, 2).cpu().numpy()
    for n, got, ref in (("O", back(O), f["O"]), ("dQ", back(Q.grad), g["dQ"]), ("dK", back(K.grad), g["dK"]),
                        ("dV", back(V.grad), g["dV"]), ("dW", W.grad.detach().float().cpu().numpy(), g["dW"])):
        err = pins.rel_l2(got, ref)
        print(f"  token-major {n}: rel_l2 = {err:.3e}", flush=True)
        assert err <= TOL["bf16"], f"{n}: {err:.3e}"


def test_autograd_casts_a_float_projection_weight():
    # a float32 parameter next to bf16 activations: the wrapper hands the library a bf16 copy
    # (same values here) and returns the gradient in the parameter's own type; the raw binding
    # refuses the mismatch instead of reading the float matrix as bf16
    from paper_2509_24006_amd import binding as sla
    from paper_2509_24006_amd.autograd import build_mask, sla_attention
    w = wl.WORKLOADS["small_bf16_d64"]
    x = wl.make_inputs(w)
    dev = torch.device("cuda:0")
    Q, K, V = (torch.from_numpy(x[k]).to(dev).to(torch.bfloat16).requires_grad_(True) for k in ("Q", "K", "V"))
    dO = torch.from_numpy(x["dO"]).to(dev).to(torch.bfloat16)
    W16 = torch.from_numpy(x["Proj"]).to(dev).to(torch.bfloat16).requires_grad_(True)
    W32 = torch.from_numpy(x["Proj"]).to(dev).requires_grad_(True)      # bf16-representable values
    mask = build_mask(Q, K, w.k_h, w.k_l)
    O16 = sla_attention(Q, K, V, W16, mask=mask)
    O16.backward(dO)
    O32 = sla_attention(Q, K, V, W32, mask=mask)
    O32.backward(dO)
    torch.cuda.synchronize()
    assert torch.equal(O16, O32)
    assert W32.grad.dtype == torch.float32 and torch.equal(W32.grad.to(torch.bfloat16), W16.grad)
    with pytest.raises(sla.SLAError, match="W"):
        sla.sla_forward(mask[0], Q.detach(), K.detach(), V.detach(), W32.detach(), mask[1], mask[2])
