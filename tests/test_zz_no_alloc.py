"""The allocation-free entry point against qlinear_w8a8: two calls in a row on the library's fixed scratch, the second on
a smaller input, each compared bit for bit with the workspace-taking call (which the other tests hold to the oracle)."""
import ctypes
import sys

import numpy as np
import pytest

import workload

pytestmark = pytest.mark.gpu


def _case(ql, torch, M, K, N, R, key):
    x = torch.from_numpy(workload.activations(M, K, "noalloc", key)).cuda()
    lw = workload.layer_weights("noalloc", K, N, 8, key)
    w, s, b = (torch.from_numpy(lw[k]).cuda() for k in ("w", "s_w", "bias"))
    return x, w, s, b


def test_noalloc_entry_point_matches_qlinear_w8a8_twice_in_a_row():
    import torch
    import paper_2511_11446_amd as ql
    L = ql.lib()
    assert torch.cuda.is_available()
    ql.set_gemm_variant(-1)
    limit = int(L.qlinear_noalloc_max_bytes())
    assert limit == 24 << 20
    # first a layer that fills most of the scratch (per-sample scales, so the partial maxima are in use too), then a
    # smaller one with per-token scales, then the large one again: stale contents of the shared array must not matter
    cases = [(4096, 4608, 384, 1024, "big"), (300, 1152, 200, 1, "small"), (4096, 4608, 384, 1024, "big")]
    for M, K, N, R, key in cases:
        print("[case] noalloc", M, K, N, R, flush=True)
        sys.stdout.flush()
        assert ql.qlinear_workspace_bytes(M, K, R) <= limit
        x, w, s, b = _case(ql, torch, M, K, N, R, key)
        y_ref = ql.qlinear_w8a8(x, R, w, s, b)
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        ql.qlinear_w8a8_noalloc(x, R, w, s, b, y)
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16))
    # beyond the fixed maximum: a clear error before anything is launched
    vp = ctypes.c_void_p
    rc = L.qlinear_w8a8_noalloc(vp(0x1000), 16384, 4608, 1, vp(0x1000), vp(0x1000), None, 64, vp(0x1000), None)
    assert rc == 5    # QL_ERR_WORKSPACE
