"""GPU parity at the benchmark's full size (Wan-1.3B-shaped layer, N = 32760, bf16) and mask
parity at the long-sequence size.  The oracle runs on a subset of heads (heads are
independent); dW, which sums over heads, is compared on a call made with exactly those heads."""
import numpy as np
import pytest
import torch

from paper_2509_24006_amd import binding as sla
from paper_2509_24006_amd import workloads as wl
from tests import pins
from tests.gpu_util import TOL, check_luts, f64, per_tile, to_dev

pytestmark = pytest.mark.gpu


def _gpu_all(x, w, k_h, k_l, H, bq=64):
    p = sla.make_params(w.B, H, w.N, w.d, k_h, k_l, torch.bfloat16, bq=bq)
    dev = {k: to_dev(v, "bf16") for k, v in x.items()}
    Mc, luts, ws = sla.sla_build_mask(p, dev["Q"], dev["K"])
    O, saved = sla.sla_forward(p, dev["Q"], dev["K"], dev["V"], dev["Proj"], Mc, luts)
    dQ, dK, dV, dW = sla.sla_backward(p, dev["Q"], dev["K"], dev["V"], dev["Proj"], Mc, luts, saved,
                                      dev["dO"])
    torch.cuda.synchronize()
    return p, Mc, luts, ws, O, saved, dQ, dK, dV, dW


@pytest.mark.timeout(600)
def test_wan_shaped_layer_against_oracle(oracle):
    w = wl.WORKLOADS["wan"]
    heads = [0, 7]
    x_all = wl.make_inputs(w)
    p, Mc, luts, ws, O, saved, dQ, dK, dV, dW = _gpu_all(x_all, w, w.k_h, w.k_l, w.H)
    # masks and pooled scores of all 12 heads, bit for bit
    Mo, so = oracle.build_mask(x_all["Q"], x_all["K"], w.k_h, w.k_l, return_scores=True)
    assert np.array_equal(sla.mask_ws_views(p, ws)["scores"].cpu().numpy(), so)
    assert np.array_equal(Mc.cpu().numpy(), Mo)
    v = {k: t.cpu().numpy() for k, t in sla.lut_views(p, luts).items()}
    check_luts(Mo[:, :2], v["row_idx"][:, :2], v["col_ptr"][:, :2], v["col_rows"][:, :2], v["ind"][:, :2], v["ind_t"][:, :2], v["col_order"][:, :2])
    print("masks of 12 heads identical", flush=True)
    # the same two heads as a call of their own: identical results, and dW to compare
    xs = {k: (np.ascontiguousarray(a[:, heads]) if a.ndim == 4 else a) for k, a in x_all.items()}
    p2, Mc2, _, _, O2, saved2, dQ2, dK2, dV2, dW2 = _gpu_all(xs, w, w.k_h, w.k_l, len(heads))
    for a, b in ((O, O2), (dQ, dQ2), (dK, dK2), (dV, dV2)):
        assert torch.equal(a[:, heads], b), "a head's result depends on which other heads are in the call"
    f = oracle.forward(xs["Q"], xs["K"], xs["V"], xs["Proj"], Mo[:, heads])
    g = oracle.backward(xs["Q"], xs["K"], xs["V"], xs["Proj"], Mo[:, heads], f, xs["dO"])
    sv = sla.saved_views(p2, saved2)
    tol = TOL["bf16"]
    for name, got, ref in (("O", O2, f["O"]), ("Os", sv["Os"], f["Os"]), ("Ol", sv["Ol"], f["Ol"]),
                           ("L", sv["L"], f["L"]), ("Hi", sv["Hi"], f["Hi"]), ("Zi", sv["Zi"], f["Zi"]),
                           ("dQ", dQ2, g["dQ"]), ("dK", dK2, g["dK"]), ("dV", dV2, g["dV"]),
                           ("dW", dW2, g["dW"])):
        err = pins.rel_l2(f64(got), ref)
        print(f"  wan {name}: rel_l2 = {err:.3e}", flush=True)
        assert err <= tol, name


@pytest.mark.timeout(600)
def test_wan_shaped_layer_with_query_blocks_of_128(oracle):
    # b_q = 128, b_kv = 64 at the full size: masks of all heads bit for bit (256 x 512 per head),
    # the tables against the mask, and one head's forward and backward against the oracle, which
    # computes with the 128 x 64 blocks directly
    w = wl.WORKLOADS["wan"]
    x_all = wl.make_inputs(w)
    p, Mc, luts, ws, O, saved, dQ, dK, dV, dW = _gpu_all(x_all, w, w.k_h, w.k_l, w.H, bq=128)
    Mo, so = oracle.build_mask(x_all["Q"], x_all["K"], w.k_h, w.k_l, bq=128, return_scores=True)
    assert Mo.shape[-2:] == (256, 512)
    assert np.array_equal(sla.mask_ws_views(p, ws)["scores"].cpu().numpy(), so)
    assert np.array_equal(Mc.cpu().numpy(), Mo)
    v = {k: t.cpu().numpy() for k, t in sla.lut_views(p, luts).items()}
    check_luts(per_tile(Mo[:, :2], 2, 512), v["row_idx"][:, :2], v["col_ptr"][:, :2], v["col_rows"][:, :2],
               v["ind"][:, :2], v["ind_t"][:, :2], v["col_order"][:, :2])
    print("masks of 12 heads identical", flush=True)
    heads = [5]
    xs = {k: (np.ascontiguousarray(a[:, heads]) if a.ndim == 4 else a) for k, a in x_all.items()}
    p2, Mc2, _, _, O2, saved2, dQ2, dK2, dV2, dW2 = _gpu_all(xs, w, w.k_h, w.k_l, 1, bq=128)
    assert torch.equal(O[:, heads], O2) and torch.equal(dK[:, heads], dK2)
    f = oracle.forward(xs["Q"], xs["K"], xs["V"], xs["Proj"], Mo[:, heads], bq=128)
    g = oracle.backward(xs["Q"], xs["K"], xs["V"], xs["Proj"], Mo[:, heads], f, xs["dO"], bq=128)
    sv = sla.saved_views(p2, saved2)
    for name, got, ref in (("O", O2, f["O"]), ("Os", sv["Os"], f["Os"]), ("Ol", sv["Ol"], f["Ol"]),
                           ("L", sv["L"], f["L"]), ("Hi", sv["Hi"], per_tile(f["Hi"], 2, 512)),
                           ("Zi", sv["Zi"], per_tile(f["Zi"], 2, 512)),
                           ("dQ", dQ2, g["dQ"]), ("dK", dK2, g["dK"]), ("dV", dV2, g["dV"]),
                           ("dW", dW2, g["dW"])):
        err = pins.rel_l2(f64(got), ref)
        print(f"  wan b_q=128 {name}: rel_l2 = {err:.3e}", flush=True)
        assert err <= TOL["bf16"], name


@pytest.mark.timeout(600)
def test_sweep_masks_and_dense_limit(oracle):
    # sparsity sweep on the Wan-shaped layer: bit-exact masks at every k_h; forward on one
    # head against the oracle at the smallest and largest sparse setting
    w0 = wl.WORKLOADS["wan"]
    heads = [3]
    x = wl.make_inputs(w0, heads=heads)
    for k_h in (0.025, 0.10, 0.20):
        w = wl.sweep(k_h)
        p, Mc, luts, ws, O, saved, dQ, dK, dV, dW = _gpu_all(x, w, w.k_h, w.k_l, 1)
        Mo = oracle.build_mask(x["Q"], x["K"], w.k_h, w.k_l)
        assert np.array_equal(Mc.cpu().numpy(), Mo), k_h
        if k_h != 0.10:
            f = oracle.forward(x["Q"], x["K"], x["V"], x["Proj"], Mo, dtype=np.float32)
            err = pins.rel_l2(f64(O), f["O"])
            print(f"  k_h={k_h}: O rel_l2 = {err:.3e}", flush=True)
            assert err <= TOL["bf16"]


@pytest.mark.timeout(600)
def test_long_sequence_masks_and_sampled_rows(oracle):
    # N = 75600 (T = 1182, tail of 16 tokens): masks of 3 heads bit-exact; forward output of
    # sampled query blocks against the oracle's definition evaluated densely for those rows
    w = wl.WORKLOADS["long"]
    heads = [0, 17, 39]
    x = wl.make_inputs(w, heads=heads)
    p, Mc, luts, ws, O, saved, dQ, dK, dV, dW = _gpu_all(x, w, w.k_h, w.k_l, len(heads))
    Mo = oracle.build_mask(x["Q"], x["K"], w.k_h, w.k_l)
    assert np.array_equal(Mc.cpu().numpy(), Mo)
    assert np.all((Mo == 1).sum(-1) == 59) and np.all((Mo == -1).sum(-1) == 118)
    # sampled rows: O^s of a query block from its critical keys only (plain softmax), and the
    # invariants that hold at any size
    Og, sv = f64(O), sla.saved_views(p, saved)
    Os = f64(sv["Os"])
    rng = np.random.default_rng(0)
    d = w.d
    for h in range(len(heads)):
        for i in list(rng.integers(0, 1182, size=3)) + [1181]:
            rows = slice(i * 64, min((i + 1) * 64, w.N))
            cols = np.concatenate([np.arange(j * 64, min((j + 1) * 64, w.N)) for j in np.nonzero(Mo[0, h, i] == 1)[0]])
            q = x["Q"][0, h, rows].astype(np.float64)
            S = q @ x["K"][0, h, cols].astype(np.float64).T / np.sqrt(d)
            P = np.exp(S - S.max(1, keepdims=True))
            ref = (P / P.sum(1, keepdims=True)) @ x["V"][0, h, cols].astype(np.float64)
            assert pins.rel_l2(Os[0, h, rows], ref) <= TOL["bf16"]
    assert np.isfinite(Og).all() and np.isfinite(f64(dQ)).all() and np.isfinite(f64(dK)).all()
    Vmax, Vmin = x["V"].max(axis=2, keepdims=True), x["V"].min(axis=2, keepdims=True)
    assert np.all(Os <= Vmax + 1e-2) and np.all(Os >= Vmin - 1e-2)   # convex combinations of V rows


def test_image_shaped_batch_against_oracle(oracle):
    # many short (batch x head) problems: all masks bit for bit, forward and backward of the whole
    # call against the oracle on two batch entries
    w = wl.WORKLOADS["image"]
    x_all = wl.make_inputs(w)
    p, Mc, luts, ws, O, saved, dQ, dK, dV, dW = _gpu_all(x_all, w, w.k_h, w.k_l, w.H)
    Mo, so = oracle.build_mask(x_all["Q"], x_all["K"], w.k_h, w.k_l, return_scores=True)
    assert np.array_equal(sla.mask_ws_views(p, ws)["scores"].cpu().numpy(), so)
    assert np.array_equal(Mc.cpu().numpy(), Mo)
    v = {k: t.cpu().numpy() for k, t in sla.lut_views(p, luts).items()}
    check_luts(Mo, v["row_idx"], v["col_ptr"], v["col_rows"], v["ind"], v["ind_t"], v["col_order"])
    bs = [0, w.B - 1]
    xs = {k: (np.ascontiguousarray(a[bs]) if a.ndim == 4 else a) for k, a in x_all.items()}
    f = oracle.forward(xs["Q"], xs["K"], xs["V"], xs["Proj"], Mo[bs])
    g = oracle.backward(xs["Q"], xs["K"], xs["V"], xs["Proj"], Mo[bs], f, xs["dO"])
    sv = sla.saved_views(p, saved)
    tol = TOL["bf16"]
    for name, got, ref in (("O", O[bs], f["O"]), ("Os", sv["Os"][bs], f["Os"]), ("Ol", sv["Ol"][bs], f["Ol"]),
                           ("dQ", dQ[bs], g["dQ"]), ("dK", dK[bs], g["dK"]), ("dV", dV[bs], g["dV"])):
        err = pins.rel_l2(f64(got), ref)
        print(f"  image {name}: rel_l2 = {err:.3e}", flush=True)
        assert err <= tol, name
    # dW sums over every (batch, head): compare against the oracle run on the whole call
    f_all = oracle.forward(x_all["Q"], x_all["K"], x_all["V"], x_all["Proj"], Mo)
    g_all = oracle.backward(x_all["Q"], x_all["K"], x_all["V"], x_all["Proj"], Mo, f_all, x_all["dO"])
    err = pins.rel_l2(f64(dW), g_all["dW"])
    print(f"  image dW: rel_l2 = {err:.3e}", flush=True)
    assert err <= tol


@pytest.mark.parametrize("T", [200, 700, 2050, 3072])
def test_masks_of_very_long_sequences(oracle, T):
    # 200 and 700 blocks: 4 and 16 keys of a row per lane in registers (the other register widths are
    # covered by the workloads); beyond 2048 blocks the classification keeps a row's keys in LDS instead of registers;
    # 3072 blocks is the longest sequence the library takes.  Masks and tables bit for bit.
    N, d, H = 64 * T - 57, 64, 1
    rng = np.random.default_rng(T)
    base = rng.standard_normal((1, H, T, d)).astype(np.float32)            # one direction per block ...
    Q = wl.round_to_bf16(np.repeat(base, 64, axis=2)[:, :, :N] + 0.5 * rng.standard_normal((1, H, N, d)).astype(np.float32))
    K = wl.round_to_bf16(np.repeat(base[:, :, ::-1], 64, axis=2)[:, :, :N] + 0.5 * rng.standard_normal((1, H, N, d)).astype(np.float32))
    p = sla.make_params(1, H, N, d, 0.03, 0.2, torch.bfloat16)
    Mc, luts, ws = sla.sla_build_mask(p, to_dev(Q, "bf16"), to_dev(K, "bf16"))
    torch.cuda.synchronize()
    Mo, so = oracle.build_mask(Q, K, 0.03, 0.2, return_scores=True)
    assert np.array_equal(sla.mask_ws_views(p, ws)["scores"].cpu().numpy(), so)
    assert np.array_equal(Mc.cpu().numpy(), Mo)
    v = {k: t.cpu().numpy() for k, t in sla.lut_views(p, luts).items()}
    check_luts(Mo, v["row_idx"], v["col_ptr"], v["col_rows"], v["ind"], v["ind_t"], v["col_order"])
