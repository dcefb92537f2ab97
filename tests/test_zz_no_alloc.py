"""The entry point that allocates nothing: sla_build_mask_static against sla_build_mask, through
the C ABI, on two calls in a row (the second smaller, so that the shared device array still holds
the first call's data beyond what the second overwrites)."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2509_24006_amd import binding as sla
from paper_2509_24006_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _masks(shape, seed):
    B, H, N, d = shape
    rng = np.random.default_rng(seed)
    Q, K = (torch.from_numpy(wl.round_to_bf16(rng.standard_normal(shape).astype(np.float32))).to(torch.bfloat16).cuda()
            for _ in range(2))
    p = sla.make_params(B, H, N, d, 0.08, 0.15, torch.bfloat16)
    z = sla.sla_sizes(p)
    assert z.ws_mask_bytes <= sla.SLA_STATIC_WS_BYTES
    Mc_ref, luts_ref, _ = sla.sla_build_mask(p, Q, K)
    # outputs of the call under test: allocated here, by the caller, before the call
    Mc = torch.full((B, H, z.Tq, z.T), 7, dtype=torch.int8, device="cuda")
    luts = torch.zeros(max(int(z.luts_bytes), 256), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    sla.sla_build_mask_static(p, Q, K, Mc, luts)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return p, z, Mc_ref, luts_ref, Mc, luts


def test_static_workspace_mask_equals_the_workspace_call_twice_in_a_row():
    for shape, seed in (((2, 3, 64 * 150 - 23, 128), 1), ((1, 2, 64 * 37 + 5, 64), 2)):
        p, z, Mc_ref, luts_ref, Mc, luts = _masks(shape, seed)
        assert torch.equal(Mc, Mc_ref), shape
        a, b = sla.lut_views(p, luts), sla.lut_views(p, luts_ref)
        for k in a:   # every table (the scratch words at the end of the buffer are not compared)
            assert torch.equal(a[k], b[k]), (shape, k)
        assert int((Mc == 1).sum()) == shape[0] * shape[1] * z.T * z.n_h


def test_static_workspace_refuses_what_does_not_fit():
    # the long-sequence shape needs 271 MB of workspace: refused before anything is enqueued
    p = sla.make_params(1, 40, 75600, 128, 0.05, 0.10, torch.bfloat16)
    assert sla.sla_sizes(p).ws_mask_bytes > sla.SLA_STATIC_WS_BYTES
    rc = sla.lib().sla_build_mask_static(ctypes.byref(p), ctypes.c_void_p(256), ctypes.c_void_p(256),
                                         ctypes.c_void_p(256), ctypes.c_void_p(256), None)
    assert rc == -3   # SLA_ENOSPACE
