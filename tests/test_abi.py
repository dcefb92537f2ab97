"""The C-ABI library loads, exports what include/sla.h declares, and rejects bad arguments
before touching a device (no GPU needed)."""
import ctypes
import os
import re

import pytest
import torch

from paper_2509_24006_amd import binding as sla

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_match_header():
    hdr = open(os.path.join(ROOT, "include", "sla.h")).read()
    declared = set(re.findall(r"^(?:int|const char\*)\s+(sla_\w+)\s*\(", hdr, re.M))
    assert declared == set(sla.EXPORTS)
    L = sla.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_constants_match_header():
    # every enumerator of the header that the binding also defines has the same value there
    import re
    text = open(os.path.join(os.path.dirname(__file__), "..", "include", "sla.h")).read()
    found = {}
    for body in re.findall(r"enum\s*\{([^}]*)\}", text):
        for name, val in re.findall(r"(SLA_\w+)\s*=\s*(-?\d+)", body):
            found[name] = int(val)
    assert {"SLA_OK", "SLA_BF16", "SLA_BNHD", "SLA_STRIDED", "SLA_PHI_ELU1", "SLA_AGG_FOUR_RUSSIANS"} <= set(found)
    checked = 0
    for name, val in found.items():
        if hasattr(sla, name):
            assert getattr(sla, name) == val, name
            checked += 1
    assert checked >= 11


def test_struct_layout_matches_header():
    assert ctypes.sizeof(sla.sla_params) == 80
    assert ctypes.sizeof(sla.sla_sizes_t) == 24 + 20 * 8


def test_sizes_and_counts():
    p = sla.make_params(1, 12, 32760, 128, 0.05, 0.10, torch.bfloat16)
    z = sla.sla_sizes(p)
    assert (z.T, z.n_h, z.n_l, z.n_0) == (512, 26, 51, 435)
    assert z.mask_bytes == 12 * 512 * 512
    p = sla.make_params(1, 40, 75600, 128, 0.05, 0.10, torch.bfloat16)
    z = sla.sla_sizes(p)
    assert (z.T, z.n_h, z.n_l, z.n_0) == (1182, 59, 118, 1005)
    p = sla.make_params(1, 2, 1024, 64, 1.0, 0.1, torch.float32)
    z = sla.sla_sizes(p)
    assert (z.n_h, z.n_l, z.n_0) == (16, 0, 0)


def test_sizes_with_larger_query_blocks():
    # b_q = 128: half as many rows of M_c and of the scores; tables and states stay per 64-token tile
    p64 = sla.make_params(1, 12, 32760, 128, 0.05, 0.10, torch.bfloat16)
    p = sla.make_params(1, 12, 32760, 128, 0.05, 0.10, torch.bfloat16, bq=128)
    z64, z = sla.sla_sizes(p64), sla.sla_sizes(p)
    assert (z64.T, z64.Tq) == (512, 512)
    assert (z.T, z.Tq, z.n_h, z.n_l, z.n_0) == (512, 256, 26, 51, 435)
    assert z.mask_bytes == 12 * 256 * 512
    assert z.luts_bytes == z64.luts_bytes and z.saved_bytes == z64.saved_bytes
    assert z.ws_mask_bytes < z64.ws_mask_bytes
    # ragged: 15 tiles in blocks of three (192 tokens) and of four (256)
    assert sla.sla_sizes(sla.make_params(1, 1, 902, 64, 0.1, 0.1, torch.float32, bq=192)).Tq == 5
    assert sla.sla_sizes(sla.make_params(1, 1, 902, 64, 0.1, 0.1, torch.float32, bq=256)).Tq == 4


def test_aggregation_workspace_sizes():
    p = sla.make_params(1, 12, 32760, 128, 0.05, 0.10, torch.bfloat16)
    row = 128 * 128 + 128
    assert sla.sla_aggregate_ws_bytes(p, sla.SLA_AGG_GEMM) == 0
    assert sla.sla_aggregate_ws_bytes(p, sla.SLA_AGG_ADD) == 0
    assert sla.sla_aggregate_ws_bytes(p, sla.SLA_AGG_PREAGG) == 12 * row * 4
    assert sla.sla_aggregate_ws_bytes(p, sla.SLA_AGG_FOUR_RUSSIANS) == 12 * 128 * 16 * row * 4   # 128 groups of 4 blocks
    n = ctypes.c_uint64()
    assert sla.lib().sla_aggregate_ws_bytes(ctypes.byref(p), 4, ctypes.byref(n)) == -2
    pf = sla.make_params(1, 2, 1024, 64, 0.1, 0.1, torch.float32)
    assert sla.lib().sla_aggregate_ws_bytes(ctypes.byref(pf), 0, ctypes.byref(n)) == -2          # bf16 only
    assert sla.lib().sla_aggregate_states(ctypes.byref(p), 1, None, None, None, None, None, 0, None) == -1


def test_counts_agree_with_oracle(oracle):
    for N in (1, 64, 65, 1000, 32760, 75600):
        for kh, kl in ((0.05, 0.1), (0.1, 0.1), (0.025, 0.1), (0.2, 0.1), (1.0, 0.0), (0.0, 0.0), (0.5, 0.5)):
            z = sla.sla_sizes(sla.make_params(1, 1, N, 64, kh, kl, torch.float32))
            assert (z.n_h, z.n_l) == oracle.counts(z.T, kh, kl)


@pytest.mark.parametrize("kw,code", [
    (dict(N=0), -1), (dict(k_h=1.5), -1), (dict(k_l=-0.1), -1), (dict(d=96), -2),
    (dict(bq=96), -2), (dict(bq=320), -2), (dict(bq=32), -2), (dict(bkv=128), -2), (dict(phi=7), -2), (dict(N=64 * 4000), -2),
])
def test_bad_params_are_rejected(kw, code):
    base = dict(B=1, H=2, N=1024, d=64, bq=64, bkv=64, k_h=0.1, k_l=0.1, phi=0, dtype=0)
    base.update(kw)
    p = sla.sla_params(*[base[k] for k in ("B", "H", "N", "d", "bq", "bkv", "k_h", "k_l", "phi", "dtype")])
    z = sla.sla_sizes_t()
    assert sla.lib().sla_sizes(ctypes.byref(p), ctypes.byref(z)) == code
    assert sla.lib().sla_build_mask(ctypes.byref(p), None, None, None, None, None, 0, None) == code


def test_null_and_small_workspace_are_rejected():
    p = sla.make_params(1, 2, 1024, 64, 0.1, 0.1, torch.float32)
    L = sla.lib()
    assert L.sla_build_mask(ctypes.byref(p), None, None, None, None, None, 0, None) == -1
    fake = ctypes.c_void_p(4096)   # never dereferenced: the size check comes first
    assert L.sla_build_mask(ctypes.byref(p), fake, fake, fake, fake, fake, 16, None) == -3
    assert L.sla_forward(ctypes.byref(p), fake, fake, fake, fake, fake, fake, fake, None, fake, 16, None) == -3
    assert L.sla_backward(ctypes.byref(p), *([fake] * 13), 16, None) == -3
    assert L.sla_forward(ctypes.byref(p), ctypes.c_void_p(4097), fake, fake, fake, fake, fake, fake, None, fake, 1 << 40, None) == -1
    assert b"workspace" in L.sla_strerror(-3)


def test_layout_field_is_checked():
    import torch
    for dt in (torch.bfloat16, torch.float32):
        ok = sla.make_params(1, 2, 128, 64, 0.5, 0.1, dt, layout=sla.SLA_BNHD)
        assert sla.sla_sizes(ok).T == 2
    bad = sla.make_params(1, 2, 128, 64, 0.5, 0.1, torch.bfloat16, layout=7)
    with pytest.raises(sla.SLAError):
        sla.sla_sizes(bad)


def test_strided_layout_is_validated():
    import torch
    mk = lambda st, dt=torch.bfloat16: sla.make_params(2, 3, 128, 64, 0.5, 0.1, dt, layout=sla.SLA_STRIDED, strides=st)
    assert sla.sla_sizes(mk((128 * 9 * 64, 64, 9 * 64))).T == 2        # slices of a fused [B,N,3,H,d] tensor
    for bad in ((128 * 9 * 64, 64, 32), (128 * 9 * 64, 60, 9 * 64), (-8, 64, 9 * 64)):
        with pytest.raises(sla.SLAError):
            sla.sla_sizes(mk(bad))
    with pytest.raises(sla.SLAError):                                   # 16-byte pieces: 4 floats
        sla.sla_sizes(mk((128 * 9 * 64, 64, 9 * 64 + 2), torch.float32))


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_binding_rejects_tensors_of_the_wrong_type_or_size():
    # the C ABI takes bare pointers: the binding is where a tensor of another storage type, shape
    # or size has to be caught (it would be read out of bounds on the device otherwise)
    p = sla.make_params(1, 2, 256, 64, 0.1, 0.1, torch.bfloat16)
    q32 = torch.zeros((1, 2, 256, 64), dtype=torch.float32)
    with pytest.raises(sla.SLAError, match="bfloat16"):
        sla.sla_build_mask(p, q32, q32)
    with pytest.raises(sla.SLAError, match="bfloat16"):
        sla.sla_forward(p, q32, q32, q32, None, None, None)
    with pytest.raises(sla.SLAError, match="bfloat16"):
        sla.sla_backward(p, q32, q32, q32, None, None, None, None, q32)
    with pytest.raises(sla.SLAError, match="W"):
        sla._packed(torch.zeros((64, 64), dtype=torch.float32), (64, 64), torch.bfloat16, "W")
    with pytest.raises(sla.SLAError, match="W"):
        sla._packed(torch.zeros((64, 64), dtype=torch.bfloat16).t()[:, :32], (64, 32), torch.bfloat16, "W")
    with pytest.raises(sla.SLAError, match="Mc"):
        sla._packed(torch.zeros((1, 2, 4, 4), dtype=torch.int32), (1, 2, 4, 4), torch.int8, "Mc")
    with pytest.raises(sla.SLAError, match="luts"):
        sla._bytes(torch.zeros(16, dtype=torch.uint8), 32, "luts")
    with pytest.raises(sla.SLAError, match="saved"):
        sla._bytes(torch.zeros(64, dtype=torch.float32), 32, "saved")
