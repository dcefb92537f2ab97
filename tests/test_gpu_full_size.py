"""GPU parity at the benchmark's full sizes: the Wan-1.3B-shaped layer (N = 32760, bf16), its
sparsity sweep, and the long-sequence layer (N = 75600, 40 heads), forward and backward.  The oracle runs on a subset of heads (heads are
independent); dW, which sums over heads, is compared on a call made with exactly those heads."""
import numpy as np
import pytest
import torch

from paper_2509_24006_amd import binding as sla
from paper_2509_24006_amd import workloads as wl
from tests import pins
from tests.gpu_util import BLOCK_TOL, TOL, check_luts, f64, max_block_rel_l2, per_tile, to_dev

pytestmark = pytest.mark.gpu


def _check(tag, name, got, ref, tol=TOL["bf16"], btol=BLOCK_TOL["bf16"], rows=64):
    """whole-tensor relative L2 and, for per-token / per-tile tensors, the worst block of `rows`"""
    got = f64(got) if isinstance(got, torch.Tensor) else got
    err = pins.rel_l2(got, ref)
    msg = f"  {tag} {name}: rel_l2 = {err:.3e}"
    assert err <= tol, f"{name}: {err:.3e}"
    if rows and ref.ndim >= 3:
        berr, where = max_block_rel_l2(got, ref, 2, rows)
        msg += f", worst block {berr:.3e} at {where}"
        assert berr <= btol, f"{name}: block {where}: {berr:.3e}"
    print(msg, flush=True)


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
    for name, got, ref in (("O", O2, f["O"]), ("Os", sv["Os"], f["Os"]), ("Ol", sv["Ol"], f["Ol"]),
                           ("L", sv["L"], f["L"]), ("dQ", dQ2, g["dQ"]), ("dK", dK2, g["dK"]), ("dV", dV2, g["dV"])):
        _check("wan", name, got, ref)
    _check("wan", "Hi", sv["Hi"], f["Hi"], rows=1)
    _check("wan", "Zi", sv["Zi"], f["Zi"], rows=1)
    _check("wan", "dW", dW2, g["dW"], rows=0)


@pytest.mark.timeout(600)
def test_wan_shaped_layer_with_query_blocks_of_128(oracle, wide_tiles):
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
                           ("L", sv["L"], f["L"]), ("dQ", dQ2, g["dQ"]), ("dK", dK2, g["dK"]), ("dV", dV2, g["dV"])):
        _check("wan b_q=128", name, got, ref)
    _check("wan b_q=128", "Hi", sv["Hi"], per_tile(f["Hi"], 2, 512), rows=1)
    _check("wan b_q=128", "Zi", sv["Zi"], per_tile(f["Zi"], 2, 512), rows=1)
    _check("wan b_q=128", "dW", dW2, g["dW"], rows=0)


@pytest.mark.timeout(600)
def test_dense_reference_is_softmax_attention(say):
    # k_h = 100 %, k_l = 0: every block critical, no linear branch -- the configuration the
    # benchmark times as its dense reference.  One head of the wan layer at full length against
    # textbook softmax attention and its gradients, computed in float64 with matrix products over
    # chunks of query rows (Eq. 4 and Eq. 7 with every block in the sums).
    w = wl.WORKLOADS["wan"]
    x_all = wl.make_inputs(w)
    head = 5
    x = {k: (np.ascontiguousarray(a[:, [head]]) if a.ndim == 4 else a) for k, a in x_all.items()}
    p, Mc, luts, ws, O, saved, dQ, dK, dV, dW = _gpu_all(x, w, 1.0, 0.0, 1)
    assert bool((Mc == 1).all()), "every block is critical"
    say("dense: GPU call done")
    t64 = lambda a: torch.from_numpy(a[0, 0]).to(torch.float64)
    Q, K, V, dO = t64(x["Q"]), t64(x["K"]), t64(x["V"]), t64(x["dO"])
    N, d = Q.shape
    scale = 1.0 / np.sqrt(d)
    Oref, dQref = torch.empty_like(Q), torch.empty_like(Q)
    dKref, dVref = torch.zeros_like(K), torch.zeros_like(V)
    for r0 in range(0, N, 2048):
        r1 = min(N, r0 + 2048)
        P = torch.softmax((Q[r0:r1] @ K.T) * scale, dim=1)
        Oc = P @ V
        Oref[r0:r1] = Oc
        dP = dO[r0:r1] @ V.T
        dS = P * (dP - (dO[r0:r1] * Oc).sum(1, keepdim=True))
        dQref[r0:r1] = (dS @ K) * scale
        dKref += (dS.T @ Q[r0:r1]) * scale
        dVref += P.T @ dO[r0:r1]
    say("dense: reference done")
    for name, got, ref in (("O", O, Oref), ("dQ", dQ, dQref), ("dK", dK, dKref), ("dV", dV, dVref)):
        _check("dense", name, got, ref.numpy()[None, None])
    assert float(dW.abs().max()) == 0.0, "no marginal block: no gradient for the projection"


@pytest.mark.timeout(900)
def test_sweep_masks_forward_and_backward(oracle, say):
    # sparsity sweep on the Wan-shaped layer: bit-exact masks at every k_h; forward and backward
    # of one head (a call of its own, so that dW belongs to it) against the oracle at the
    # smallest and the largest sparse setting
    w0 = wl.WORKLOADS["wan"]
    heads = [3]
    x = wl.make_inputs(w0, heads=heads)
    for k_h in (0.025, 0.10, 0.20):
        w = wl.sweep(k_h)
        p, Mc, luts, ws, O, saved, dQ, dK, dV, dW = _gpu_all(x, w, w.k_h, w.k_l, 1)
        Mo = oracle.build_mask(x["Q"], x["K"], w.k_h, w.k_l)
        assert np.array_equal(Mc.cpu().numpy(), Mo), k_h
        say(f"sweep k_h={k_h}: mask identical")
        if k_h != 0.10:
            f = oracle.forward(x["Q"], x["K"], x["V"], x["Proj"], Mo, dtype=np.float32)
            g = oracle.backward(x["Q"], x["K"], x["V"], x["Proj"], Mo, f, x["dO"], dtype=np.float32)
            say(f"sweep k_h={k_h}: oracle forward and backward done")
            sv = sla.saved_views(p, saved)
            tag = f"k_h={k_h}"
            for name, got, ref in (("O", O, f["O"]), ("Os", sv["Os"], f["Os"]), ("Ol", sv["Ol"], f["Ol"]),
                                   ("L", sv["L"], f["L"]), ("dQ", dQ, g["dQ"]), ("dK", dK, g["dK"]),
                                   ("dV", dV, g["dV"])):
                _check(tag, name, got, ref)
            _check(tag, "dW", dW, g["dW"], rows=0)


@pytest.mark.timeout(1100)
def test_long_sequence_forward_and_backward(oracle, say):
    # N = 75600 (T = 1182, tail of 16 tokens, 59 critical blocks per row), all 40 heads in one call
    # -- the launch configuration of the benchmark's long workload, in which the dK/dV kernel gives
    # every XCD whole heads.  Masks of three heads bit for bit; forward and backward of heads 0
    # and 39 against the float oracle run on those two heads; dW, which sums over the heads of a
    # call, from a call made with exactly those two.
    w = wl.WORKLOADS["long"]
    x_all = wl.make_inputs(w)
    say("long: inputs drawn")
    p, Mc, luts, ws, O, saved, dQ, dK, dV, dW = _gpu_all(x_all, w, w.k_h, w.k_l, w.H)
    say("long: GPU call with 40 heads done")
    mh = [0, 17, 39]
    Mo3 = oracle.build_mask(x_all["Q"][:, mh], x_all["K"][:, mh], w.k_h, w.k_l)
    assert np.array_equal(Mc[:, mh].cpu().numpy(), Mo3)
    assert np.all((Mo3 == 1).sum(-1) == 59) and np.all((Mo3 == -1).sum(-1) == 118)
    say("long: masks of heads 0, 17, 39 identical")
    heads = [0, 39]
    xs = {k: (np.ascontiguousarray(a[:, heads]) if a.ndim == 4 else a) for k, a in x_all.items()}
    Mo = Mo3[:, [0, 2]]
    sv = sla.saved_views(p, saved)
    got_all = {"O": O, "Os": sv["Os"], "Ol": sv["Ol"], "L": sv["L"], "Hi": sv["Hi"], "Zi": sv["Zi"],
               "dQ": dQ, "dK": dK, "dV": dV}
    got_all = {k: f64(v[:, heads]) for k, v in got_all.items()}
    del x_all, O, saved, sv, dQ, dK, dV
    torch.cuda.empty_cache()
    f = oracle.forward(xs["Q"], xs["K"], xs["V"], xs["Proj"], Mo, dtype=np.float32)
    say("long: oracle forward of 2 heads done")
    g = oracle.backward(xs["Q"], xs["K"], xs["V"], xs["Proj"], Mo, f, xs["dO"], dtype=np.float32)
    say("long: oracle backward of 2 heads done")
    for name in ("O", "Os", "Ol", "L", "dQ", "dK", "dV"):
        _check("long", name, got_all[name], (f if name in f else g)[name])
    _check("long", "Hi", got_all["Hi"], f["Hi"], rows=1)
    _check("long", "Zi", got_all["Zi"], f["Zi"], rows=1)
    # the two heads as a call of their own: dW
    p2, Mc2, _, _, O2, saved2, dQ2, dK2, dV2, dW2 = _gpu_all(xs, w, w.k_h, w.k_l, len(heads))
    assert np.array_equal(Mc2.cpu().numpy(), Mo)
    _check("long", "dW", dW2, g["dW"], rows=0)
    _check("long (2-head call)", "dK", dK2, g["dK"])
    # convex combinations of V rows
    Vmax, Vmin = xs["V"].max(axis=2, keepdims=True), xs["V"].min(axis=2, keepdims=True)
    assert np.all(got_all["Os"] <= Vmax + 1e-2) and np.all(got_all["Os"] >= Vmin - 1e-2)


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
        _check("image", name, got, ref)
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
