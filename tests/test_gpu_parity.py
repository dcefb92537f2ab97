"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  Masks and lookup tables bit-exact; floating-point tensors by
relative L2 (1e-5 for float tensors, 1e-2 for bf16 tensors)."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from paper_2509_24006_amd import workloads as wl
from tests import pins
from tests.gpu_util import BLOCK_TOL, TOL, check_luts, max_block_rel_l2, per_tile, run_gpu

pytestmark = pytest.mark.gpu


def _oracle_all(oracle, x, k_h, k_l, phi=0, backward=True, bq=64):
    Mc, s = oracle.build_mask(x["Q"], x["K"], k_h, k_l, bq=bq, return_scores=True)
    f = oracle.forward(x["Q"], x["K"], x["V"], x["Proj"], Mc, phi=phi, bq=bq)
    g = oracle.backward(x["Q"], x["K"], x["V"], x["Proj"], Mc, f, x["dO"], phi=phi, bq=bq) if backward else {}
    return Mc, s, f, g


def _compare(name, got, ref, tol, floor_rms=0.0, block_tol=None, token_axis=2, rows=64):
    """Whole-tensor relative L2 <= tol and, with block_tol, the same measure on every block of
    `rows` consecutive indices of token_axis <= block_tol (one bad row cannot hide in a long
    tensor).  floor_rms > 0 (short sequences' gradients only, see the callers) measures the error
    against a norm of at least floor_rms per element."""
    if np.all(ref == 0):
        assert np.all(got == 0), f"{name}: expected exact zeros"
        return
    err = pins.rel_l2(got, ref)
    print(f"  {name}: rel_l2 = {err:.3e} (tol {tol:g})", flush=True)
    # a reference that is pure rounding noise (a gradient that vanishes identically, e.g. dQ
    # of a one-token sequence) is compared absolutely, at the same tolerance
    if np.abs(ref).max() < 1e-12:
        assert np.abs(got).max() <= tol, f"{name}: expected ~0, got {np.abs(got).max():.3e}"
        return
    # floor_rms: where a key block holds one or a few keys, P is 1 (or close) and dS = P (dP - D)
    # cancels exactly in most rows: the norm of the reference gradient is then set by a handful
    # of rows while float rounding noise comes from all of them; the error is measured against a
    # norm of at least floor_rms per element (inputs have unit variance)
    scale = max(np.linalg.norm(ref.ravel()), floor_rms * np.sqrt(ref.size))
    err = np.linalg.norm((got - ref).ravel()) / scale
    assert err <= tol, f"{name}: rel L2 {err:.3e} > {tol:g}"
    if block_tol is not None and floor_rms == 0.0:
        berr, where = max_block_rel_l2(got, ref, token_axis, rows)
        print(f"  {name}: worst block rel_l2 = {berr:.3e} at {where} (tol {block_tol:g})", flush=True)
        assert berr <= block_tol, f"{name}: block {where} rel L2 {berr:.3e} > {block_tol:g}"


def _full_case(oracle, x, dtype, k_h, k_l, phi=0, floor_rms=0.0, bq=64, backward=True):
    print(f"case shape={x['Q'].shape} dtype={dtype} k_h={k_h} k_l={k_l} phi={phi} bq={bq}", flush=True)
    Mc, s, f, g = _oracle_all(oracle, x, k_h, k_l, phi, backward=backward, bq=bq)
    r = run_gpu(x, dtype, k_h, k_l, phi, backward=backward, bq=bq)
    # mask step: bit-exact
    assert np.array_equal(r["scores"], s), "pooled scores differ bitwise"
    assert np.array_equal(r["Mc"], Mc), "mask differs"
    # tables and saved states are kept per 64-token query tile: a tile has its query block's row
    T, rq = Mc.shape[-1], bq // 64
    check_luts(per_tile(r["Mc"], rq, T), r["row_idx"], r["col_ptr"], r["col_rows"], r["ind"], r["ind_t"],
               r["col_order"])
    tol, btol = TOL[dtype], BLOCK_TOL[dtype]
    for k in ("O", "Os", "Ol"):
        _compare(k, r[k], f[k], tol, block_tol=btol)
    for k in ("Hi", "Zi"):   # one state per 64-token tile: every state on its own
        _compare(k, r[k], per_tile(f[k], rq, T), tol, block_tol=btol, rows=1)
    fin = np.isfinite(f["L"])
    assert np.array_equal(np.isfinite(r["L"]), fin)
    if fin.any():
        _compare("L", r["L"][fin], f["L"][fin], tol)
    for k in ("dQ", "dK", "dV", "dW") if backward else ():
        _compare(k, r[k], g[k], tol, floor_rms, block_tol=None if k == "dW" else btol)


@pytest.mark.parametrize("name", ["tiny", "small_fp32", "small_bf16", "small_bf16_d64"])
def test_workload_parity(oracle, name):
    w = wl.WORKLOADS[name]
    x = wl.make_inputs(w)
    _full_case(oracle, x, w.dtype, w.k_h, w.k_l)


@pytest.mark.parametrize("k_h,k_l", [(1.0, 0.1), (0.0, 0.0), (0.0, 0.3), (0.4, 0.6), (0.05, 0.9)])
@pytest.mark.parametrize("name", ["small_fp32", "small_bf16", "small_bf16_d64"])
def test_degenerate_masks(oracle, name, k_h, k_l):
    # all critical (dense attention), all marginal (linear attention), no critical block,
    # no marginal block
    w = wl.WORKLOADS[name]
    x = wl.make_inputs(w)
    _full_case(oracle, x, w.dtype, k_h, k_l)


@pytest.mark.parametrize("name", ["small_fp32", "small_bf16"])
def test_elu_feature_map(oracle, name):
    w = wl.WORKLOADS[name]
    x = wl.make_inputs(w)
    _full_case(oracle, x, w.dtype, w.k_h, w.k_l, phi=1)


@pytest.mark.parametrize("name,bq,k_h,k_l", [
    ("small_bf16", 128, 0.10, 0.10),       # 18 tiles in 9 blocks; last block ragged inside its second tile
    ("small_bf16_d64", 128, 0.12, 0.15),   # 15 tiles: the last block has one tile only
    ("small_bf16_d64", 192, 0.12, 0.15),   # 5 blocks of 3 tiles
    ("small_fp32", 128, 0.15, 0.20),
    ("small_fp32", 256, 0.15, 0.20),       # 9 tiles in blocks of 4, 4, 1
    ("small_bf16", 256, 0.0, 0.3),         # no critical block
    ("small_bf16", 128, 0.4, 0.6),         # no marginal block
])
def test_query_blocks_of_several_tiles(oracle, wide_tiles, name, bq, k_h, k_l):
    # b_q = 128, 192, 256 with b_kv = 64: the mask is predicted per block of b_q queries (pooling,
    # scores and classification on T_q rows); the oracle computes with the b_q x 64 blocks
    # directly, the library gives every 64-token tile of a query block that block's mask row
    w = wl.WORKLOADS[name]
    x = wl.make_inputs(w)
    _full_case(oracle, x, w.dtype, k_h, k_l, bq=bq)


@pytest.mark.parametrize("bq", [128, 256])
def test_query_blocks_of_several_tiles_mid_length(oracle, wide_tiles, bq):
    # 41 tiles (ragged tail of 5 tokens), enough key blocks for the matrix-core state aggregation
    N, d = 2565, 128
    rng = np.random.default_rng(N + bq)
    x = {k: wl.round_to_bf16(rng.standard_normal((1, 2, N, d)).astype(np.float32)) for k in ("Q", "K", "V", "dO")}
    x["Proj"] = wl.round_to_bf16((rng.standard_normal((d, d)) * 0.05).astype(np.float32))
    _full_case(oracle, x, "bf16", 0.1, 0.2, bq=bq)


@pytest.mark.parametrize("name,scale,backward", [
    ("small_bf16", 0.02, True), ("small_bf16", 2.0, True), ("small_bf16", 6.0, False),
    ("small_fp32", 0.02, True), ("small_fp32", 2.0, True), ("small_fp32", 6.0, True)])
def test_small_and_large_score_magnitudes(oracle, name, scale, backward):
    # nearly uniform attention (scores ~ 1e-3) and peaked attention (raw scores of a hundred and
    # more before the 1/sqrt(d): exponent range of the online softmax and of its lazy rescaling).
    # At the largest scale the bf16 case compares the forward pass only: with P close to one-hot,
    # dS = P (dP - D) is a small difference of terms of which D comes from the O^s saved in the
    # storage type, so in bf16 the gradients of any implementation that follows Alg. 2 lose
    # digits there (1.6 % on dQ), which says nothing about the kernels.  Float tensors save O^s
    # in float and are compared in full.
    w = wl.WORKLOADS[name]
    x = wl.make_inputs(w)
    x["Q"] = x["Q"] * np.float32(scale)
    x["K"] = x["K"] * np.float32(scale)
    if w.dtype == "bf16":
        x["Q"], x["K"] = wl.round_to_bf16(x["Q"]), wl.round_to_bf16(x["K"])
    _full_case(oracle, x, w.dtype, w.k_h, w.k_l, backward=backward)


@pytest.mark.parametrize("N", [1, 63, 64, 65, 130])
def test_short_sequences(oracle, N):
    rng = np.random.default_rng(N)
    d = 64
    x = {k: rng.standard_normal((1, 2, N, d)).astype(np.float32) for k in ("Q", "K", "V", "dO")}
    x["Proj"] = (rng.standard_normal((d, d)) * 0.05).astype(np.float32)
    _full_case(oracle, x, "fp32", 0.34, 0.34, floor_rms=0.05)


@pytest.mark.parametrize("N,d", [(2565, 128), (4096, 64), (2048, 128)])
def test_bf16_mid_length_sequences(oracle, N, d):
    # 33..64 blocks: the short-sequence state aggregation with two row tiles, a ragged tail and
    # an exact multiple of the block size
    rng = np.random.default_rng(N + d)
    x = {k: wl.round_to_bf16(rng.standard_normal((1, 2, N, d)).astype(np.float32)) for k in ("Q", "K", "V", "dO")}
    x["Proj"] = wl.round_to_bf16((rng.standard_normal((d, d)) * 0.05).astype(np.float32))
    _full_case(oracle, x, "bf16", 0.1, 0.2)


@pytest.mark.timeout(300)
@pytest.mark.parametrize("N,d", [(300 * 64 - 9, 128), (71 * 64 + 3, 64)])
def test_bf16_ragged_tiles_of_the_state_aggregation(oracle, N, d):
    # 300 blocks: two row tiles of the aggregation GEMM, the second with 44 rows, five indicator
    # words per row, the last with 44 bits; 72 blocks: one ragged row tile, two words.  Forward and
    # backward (the column-wise aggregation uses the transposed indicator)
    rng = np.random.default_rng(N + d)
    x = {k: wl.round_to_bf16(rng.standard_normal((1, 2, N, d)).astype(np.float32)) for k in ("Q", "K", "V", "dO")}
    x["Proj"] = wl.round_to_bf16((rng.standard_normal((d, d)) * 0.05).astype(np.float32))
    _full_case(oracle, x, "bf16", 0.05, 0.15)


@pytest.mark.timeout(300)
def test_many_long_heads(oracle):
    # 32 (batch x head) problems of 128 blocks: the launch order of the dK/dV kernel in which every
    # XCD takes whole heads one after the other (chosen from 32 problems and 128 blocks on), with a
    # ragged tail; all heads against the oracle
    B, H, N, d = 4, 8, 128 * 64 - 17, 64
    rng = np.random.default_rng(4128)
    x = {k: wl.round_to_bf16(rng.standard_normal((B, H, N, d)).astype(np.float32)) for k in ("Q", "K", "V", "dO")}
    x["Proj"] = wl.round_to_bf16((rng.standard_normal((d, d)) * 0.05).astype(np.float32))
    _full_case(oracle, x, "bf16", 0.05, 0.10)


@pytest.mark.timeout(300)
@pytest.mark.parametrize("T,d,tail", [(150, 128, 23), (128, 64, 0), (200, 64, 63)])
def test_key_blocks_that_nearly_every_query_block_selects(oracle, T, d, tail):
    # a few key blocks whose pooled key points along the direction shared by every query: their
    # column lists hold (nearly) all T query tiles, so the column-wise backward kernel walks them in
    # the longest walks the kernel can be given (its launch order puts them first)
    N = 64 * T - tail
    rng = np.random.default_rng(T + d)
    u = rng.standard_normal(d).astype(np.float32)
    u /= np.linalg.norm(u)
    x = {k: rng.standard_normal((1, 2, N, d)).astype(np.float32) for k in ("Q", "K", "V", "dO")}
    x["Q"] += 1.5 * u
    hot = [3, 4, T // 2, T - 1]
    for j in hot:
        x["K"][:, :, 64 * j:64 * (j + 1)] += 4.0 * u
    x["Proj"] = (rng.standard_normal((d, d)) * 0.05).astype(np.float32)
    x = {k: wl.round_to_bf16(v) for k, v in x.items()}
    Mc = oracle.build_mask(x["Q"], x["K"], 0.08, 0.2)
    cnt = (Mc == 1).sum(-2)
    assert (cnt[0, :, hot] >= T - 2).all() and (cnt >= 64).sum() >= 2 * len(hot)
    _full_case(oracle, x, "bf16", 0.08, 0.2)


@pytest.mark.parametrize("name", ["small_bf16", "small_bf16_d64", "small_fp32"])
def test_token_major_tensors(oracle, name):
    # [B,N,H,d] tensors: the same kernels walk the same values with another row pitch, so every
    # result equals the [B,H,N,d] call's bit for bit; one of the two is checked against the oracle
    w = wl.WORKLOADS[name]
    x = wl.make_inputs(replace(w, B=2))
    a = run_gpu(x, w.dtype, w.k_h, w.k_l)
    b = run_gpu(x, w.dtype, w.k_h, w.k_l, token_major=True)
    for k in a:
        assert np.array_equal(a[k], b[k]), f"{k} differs between the two memory orders"
    Mc, s, f, g = _oracle_all(oracle, x, w.k_h, w.k_l, 0)
    assert np.array_equal(b["Mc"], Mc)
    for k in ("O", "dQ", "dK", "dV", "dW"):
        _compare(k, b[k], (f if k == "O" else g)[k], TOL[w.dtype])


@pytest.mark.parametrize("name", ["small_bf16", "small_fp32"])
def test_slices_of_a_fused_projection(oracle, name):
    # Q, K, V as views into one [B,N,3,H,d] tensor, dO / O and the gradients laid out the same way
    from paper_2509_24006_amd import binding as sla
    w = wl.WORKLOADS[name]
    x = wl.make_inputs(w)
    B, H, N, d = x["Q"].shape
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    dev = torch.device("cuda:0")
    qkv = torch.empty((B, N, 3, H, d), dtype=tdt, device=dev)
    gout = torch.empty((B, N, 3, H, d), dtype=tdt, device=dev)   # dO in slot 0
    for s_, k in enumerate(("Q", "K", "V")):
        qkv[:, :, s_] = torch.from_numpy(x[k]).to(dev).to(tdt).transpose(1, 2)
    gout[:, :, 0] = torch.from_numpy(x["dO"]).to(dev).to(tdt).transpose(1, 2)
    view = lambda t, s_: t[:, :, s_].permute(0, 2, 1, 3)          # [B,H,N,d], strides (3NHd, d, 3Hd, 1)
    Q, K, V, dO = view(qkv, 0), view(qkv, 1), view(qkv, 2), view(gout, 0)
    p = sla.make_params(B, H, N, d, w.k_h, w.k_l, tdt, layout=sla.SLA_STRIDED, strides=tuple(Q.stride()[:3]))
    W = torch.from_numpy(x["Proj"]).to(dev).to(tdt)
    Mc, luts, _ = sla.sla_build_mask(p, Q, K)
    O, saved = sla.sla_forward(p, Q, K, V, W, Mc, luts)
    dqkv = torch.zeros_like(qkv)
    out = (view(dqkv, 0), view(dqkv, 1), view(dqkv, 2), torch.empty((d, d), dtype=torch.float32, device=dev))
    sla.sla_backward(p, Q, K, V, W, Mc, luts, saved, dO, out=out)
    torch.cuda.synchronize()
    ref = run_gpu(x, w.dtype, w.k_h, w.k_l)
    f64 = lambda t: t.detach().double().cpu().numpy()
    assert np.array_equal(Mc.cpu().numpy(), ref["Mc"])
    for k, got in (("O", O), ("dQ", out[0]), ("dK", out[1]), ("dV", out[2]), ("dW", out[3])):
        assert np.array_equal(f64(got), ref[k]), f"{k} differs from the packed call"


def test_classify_given_scores_with_ties(oracle):
    from paper_2509_24006_amd import binding as sla
    rng = np.random.default_rng(0)
    T = 130
    p = sla.make_params(1, 3, T * 64, 64, 0.1, 0.2, torch.float32)
    s = rng.integers(-2, 3, size=(1, 3, T, T)).astype(np.float32)     # heavy ties
    s[0, 0, 0] = 0.0
    s[0, 0, 1, ::2] = -0.0
    s[0, 1] = rng.standard_normal((T, T)).astype(np.float32)
    nh, nl = oracle.counts(T, 0.1, 0.2)
    ref = oracle.classify(s, nh, nl)
    Mc, luts = sla.sla_classify_scores(p, torch.from_numpy(s).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(Mc.cpu().numpy(), ref)
    v = {k: t.cpu().numpy() for k, t in sla.lut_views(p, luts).items()}
    check_luts(ref, v["row_idx"], v["col_ptr"], v["col_rows"], v["ind"], v["ind_t"], v["col_order"])


@pytest.mark.parametrize("bq,N", [(128, 130 * 64), (192, 130 * 64 - 40), (256, 33 * 64)])
def test_classify_given_scores_with_ties_and_larger_query_blocks(oracle, bq, N):
    # rectangular score matrices (one row per block of bq queries), heavy ties; N is chosen so that
    # the last query block has fewer tiles than the others
    from paper_2509_24006_amd import binding as sla
    rng = np.random.default_rng(bq)
    p = sla.make_params(1, 3, N, 64, 0.1, 0.2, torch.float32, bq=bq)
    z = sla.sla_sizes(p)
    s = rng.integers(-2, 3, size=(1, 3, z.Tq, z.T)).astype(np.float32)
    s[0, 0, 0] = 0.0
    s[0, 0, 1, ::2] = -0.0
    s[0, 1] = rng.standard_normal((z.Tq, z.T)).astype(np.float32)
    nh, nl = oracle.counts(z.T, 0.1, 0.2)
    ref = oracle.classify(s, nh, nl)
    Mc, luts = sla.sla_classify_scores(p, torch.from_numpy(s).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(Mc.cpu().numpy(), ref)
    v = {k: t.cpu().numpy() for k, t in sla.lut_views(p, luts).items()}
    check_luts(per_tile(ref, bq // 64, z.T), v["row_idx"], v["col_ptr"], v["col_rows"], v["ind"], v["ind_t"],
               v["col_order"])


@pytest.mark.parametrize("T,d,k_h,k_l,bq", [(18, 64, 0.1, 0.1, 64), (71, 64, 0.05, 0.45, 64), (300, 128, 0.05, 0.10, 64),
                                            (300, 128, 0.05, 0.85, 64), (41, 64, 0.1, 0.2, 128), (9, 128, 0.0, 0.0, 64),
                                            (33, 64, 0.5, 0.5, 64)])
def test_accumulation_line_by_every_method(oracle, T, d, k_h, k_l, bq):
    # Alg. 1's accumulation line alone, by the matrix-core product the library uses and by the three
    # forms the paper describes (one addition per block, pre-aggregation, Four Russians tables),
    # on random bf16 states and the mask of random scores: each against the oracle's plain sum.
    # Densities from every block marginal to none; a tile count that is no multiple of 4 or 64.
    from paper_2509_24006_amd import binding as sla
    B, H, N = 1, 2, T * 64 - 5
    rng = np.random.default_rng(T + d)
    p = sla.make_params(B, H, N, d, k_h, k_l, torch.bfloat16, bq=bq)
    z = sla.sla_sizes(p)
    assert z.T == T
    s = rng.standard_normal((B, H, z.Tq, T)).astype(np.float32)
    Mc, luts = sla.sla_classify_scores(p, torch.from_numpy(s).cuda())
    h = wl.round_to_bf16(rng.standard_normal((B, H, T, d * d + d)).astype(np.float32))
    ref = oracle.accumulate(h, per_tile(Mc.cpu().numpy(), bq // 64, T))
    hd = torch.from_numpy(h).cuda().to(torch.bfloat16)
    for method, name in ((sla.SLA_AGG_GEMM, "product"), (sla.SLA_AGG_ADD, "additions"),
                         (sla.SLA_AGG_PREAGG, "pre-aggregation"), (sla.SLA_AGG_FOUR_RUSSIANS, "four russians")):
        Hm, Zm = sla.sla_aggregate_states(p, method, luts, hd)
        torch.cuda.synchronize()
        print(f" {name}:", flush=True)
        _compare("H", Hm.double().cpu().numpy(), ref[..., :d * d], TOL["bf16"])
        # the vector part leaves in float; pre-aggregation subtracts two long float sums
        _compare("Z", Zm.double().cpu().numpy(), ref[..., d * d:], 1e-4 if method == sla.SLA_AGG_PREAGG else 1e-5)


def test_forward_without_saved_matches(oracle):
    from paper_2509_24006_amd import binding as sla
    from tests.gpu_util import to_dev, f64
    w = wl.WORKLOADS["small_bf16"]
    x = wl.make_inputs(w)
    p = sla.make_params(w.B, w.H, w.N, w.d, w.k_h, w.k_l, torch.bfloat16)
    Q, K, V, W = (to_dev(x[k], "bf16") for k in ("Q", "K", "V", "Proj"))
    Mc, luts, _ = sla.sla_build_mask(p, Q, K)
    O1, _ = sla.sla_forward(p, Q, K, V, W, Mc, luts)
    O2, sv = sla.sla_forward(p, Q, K, V, W, Mc, luts, need_saved=False)
    torch.cuda.synchronize()
    assert sv is None and torch.equal(O1, O2)


def test_calls_follow_the_given_stream(oracle):
    # every kernel of a call is enqueued on the stream handed in: the same results on a side
    # stream (default priority) as on the current one, with no host synchronisation in between
    from paper_2509_24006_amd import binding as sla
    w = wl.WORKLOADS["small_bf16"]
    x = wl.make_inputs(w)
    ref = run_gpu(x, "bf16", w.k_h, w.k_l)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        got = run_gpu(x, "bf16", w.k_h, w.k_l)
    torch.cuda.synchronize()
    for k in ref:
        assert np.array_equal(ref[k], got[k]), k


@pytest.mark.parametrize("seed", range(24))
def test_random_small_problems(oracle, seed):
    # a seeded draw over storage type, head size, batch, heads, (ragged) length, k_h, k_l, feature
    # map and memory order
    rng = np.random.default_rng(1000 + seed)
    dtype = str(rng.choice(["bf16", "fp32"], p=[0.7, 0.3]))
    d = int(rng.choice([64, 128])) if dtype == "bf16" else 64
    B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
    N = int(rng.choice([rng.integers(1, 200), rng.integers(200, 1500), 64 * rng.integers(1, 20),
                        64 * rng.integers(1, 20) + 1]))
    k_h = float(rng.choice([0.0, 0.05, 0.1, 0.3, 0.5, 1.0]))
    k_l = float(rng.choice([0.0, 0.1, 0.3, 0.9]))
    phi, tm = int(rng.integers(0, 2)), bool(rng.integers(0, 2))
    x = {k: rng.standard_normal((B, H, N, d)).astype(np.float32) for k in ("Q", "K", "V", "dO")}
    x["Proj"] = (rng.standard_normal((d, d)) * 0.05).astype(np.float32)
    if dtype == "bf16":
        x = {k: wl.round_to_bf16(v) for k, v in x.items()}
    print(f"{dtype} d={d} B={B} H={H} N={N} k_h={k_h} k_l={k_l} phi={phi} token_major={tm}", flush=True)
    Mc, s, f, g = _oracle_all(oracle, x, k_h, k_l, phi)
    r = run_gpu(x, dtype, k_h, k_l, phi, token_major=tm)
    assert np.array_equal(r["scores"], s) and np.array_equal(r["Mc"], Mc)
    check_luts(r["Mc"], r["row_idx"], r["col_ptr"], r["col_rows"], r["ind"], r["ind_t"], r["col_order"])
    # sequences of a few blocks at most: a key block of one or a few keys makes most rows' dS
    # cancel exactly, see _compare; only the gradients of such draws get the floor
    short = N < 200
    # no critical block at all (bf16): dQ and dK are the linear branch's alone, an order of magnitude
    # smaller than with a sparse part, and dQ^phi = (dO^l H_i^T - D^l Z_i^T) / den is a difference of
    # nearly equal terms when few blocks are marginal; the H_i saved in bf16 bounds its error
    # relative to the terms (1.5e-2 of the result for one marginal block per row), so the error is
    # measured against a gradient of at least floor_rms per element there too
    lin_only = dtype == "bf16" and int((Mc == 1).sum()) == 0
    for k in ("O", "Os", "Ol", "dQ", "dK", "dV", "dW"):
        floor = 0.05 if (k in ("dQ", "dK", "dV", "dW") and short) or (k in ("dQ", "dK") and lin_only) else 0.0
        _compare(k, r[k], (f if k in f else g)[k], TOL[dtype], floor_rms=floor,
                 block_tol=None if (k == "dW" or short) else BLOCK_TOL[dtype])


def test_a_captured_step_replays_to_the_eager_results():
    # mask + forward + backward captured into one HIP graph (no allocation, no memset node, no host
    # synchronisation inside the calls); every replay, with eager calls and synchronisations in
    # between, gives what the eager calls gave
    from paper_2509_24006_amd import binding as sla
    w = wl.WORKLOADS["small_bf16"]
    x = wl.make_inputs(w)
    B, H, N, d = x["Q"].shape
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(a).to(dev).to(torch.bfloat16)
    Q, K, V, W, dO = t(x["Q"]), t(x["K"]), t(x["V"]), t(x["Proj"]), t(x["dO"])
    p = sla.make_params(B, H, N, d, w.k_h, w.k_l, torch.bfloat16)
    z = sla.sla_sizes(p)
    u8 = lambda n: torch.empty(max(int(n), 256), dtype=torch.uint8, device=dev)
    Mc = torch.empty((B, H, z.T, z.T), dtype=torch.int8, device=dev)
    luts, ws_m, ws_f, ws_b, saved = (u8(n) for n in (z.luts_bytes, z.ws_mask_bytes, z.ws_forward_bytes,
                                                    z.ws_backward_bytes, z.saved_bytes))
    O = torch.empty_like(Q)
    out = (torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V),
           torch.empty((d, d), dtype=torch.float32, device=dev))

    def step():
        sla.sla_build_mask(p, Q, K, workspace=ws_m, Mc=Mc, luts=luts)
        sla.sla_forward(p, Q, K, V, W, Mc, luts, O=O, saved=saved, workspace=ws_f)
        sla.sla_backward(p, Q, K, V, W, Mc, luts, saved, dO, workspace=ws_b, out=out)

    results = lambda: [a.clone() for a in (Mc, O) + out]
    step()
    torch.cuda.synchronize()
    ref = results()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(3):
        for a in (Mc, O) + out:
            a.zero_()
        luts.zero_()
        saved.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(ref, results()):
            assert torch.equal(a, b), f"replay {rep} differs from the eager result"
        step()   # eager work between the replays
        torch.cuda.synchronize()
