"""GPU parity at the benchmark's full size (M = 16384), every output element compared.

The launch configuration is the one bench.py times: the shape-chosen tiles, i.e. the persistent
multi-tile walk for the 8-bit layers and the 4-bit kernel at its full grid.  The oracle needs a
few seconds per layer at this size, so codes, scales, int32 accumulators / group partial sums
and fp16 outputs are compared in full, not on sampled rows."""
import sys

import numpy as np
import pytest

import workload

pytestmark = pytest.mark.gpu

M_FULL = 16384


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2511_11446_amd as ql
    ql.lib()
    assert torch.cuda.is_available()
    ql.set_gemm_variant(-1)
    return ql


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


def y_mismatches(y_gpu, y_ref):
    """Asserts |y_gpu - y_ref| <= 1e-3 |y_ref| (one subnormal step near zero); returns the number of differing bit patterns."""
    a, b = y_gpu.astype(np.float32), y_ref.astype(np.float32)
    assert np.isfinite(b).all()
    tol = np.maximum(np.float32(1e-3) * np.abs(b), np.float32(2.0 ** -24))
    bad = np.abs(a - b) > tol
    assert not bad.any(), "first mismatches at %s" % np.argwhere(bad)[:4].tolist()
    return int((y_gpu.view(np.uint16) != y_ref.view(np.uint16)).sum())


def free():
    import torch
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name,K,N", workload.BLOCK_LAYERS)
def test_w8a8_m16384_every_element(gpu, orc, name, K, N):
    """The four 8-bit layers of a block: the persistent tile walk (several tiles per workgroup) on every output."""
    M, R = M_FULL, 1
    say("full W8", name, M, K, N)
    x = workload.activations(M, K, "full8", name, sigma=1.7)
    lw = workload.layer_weights(name, K, N, 8, "full8")
    ref = orc.qlinear_w8a8(x, R, lw["w"], lw["s_w"], lw["bias"], nthreads=16)
    xd, wd, sd, bd = dev(x), dev(lw["w"]), dev(lw["s_w"]), dev(lw["bias"])
    y = gpu.qlinear_w8a8(xd, R, wd, sd, bd)               # what the benchmark launches: packed epilogue, no exports
    assert y_mismatches(host(y), ref["y"]) == 0
    out = gpu.qlinear_w8a8(xd, R, wd, sd, bd, debug=True)  # the same tiles with the integer exports
    assert np.array_equal(host(out["q"]), ref["q"])
    assert np.array_equal(host(out["s_a"]).view(np.uint32), ref["s_a"].view(np.uint32))
    assert np.array_equal(host(out["acc"]), ref["acc"])
    assert np.array_equal(host(out["y"]).view(np.uint16), host(y).view(np.uint16))
    del out, y
    free()


@pytest.mark.parametrize("name,K,N,group", [("fc1", 1152, 4608, 128), ("fc2", 4608, 1152, 128),
                                            ("fc1", 1152, 4608, 288), ("fc2", 4608, 1152, 288),
                                            ("proj", 1152, 1152, 32), ("fc2", 4608, 1152, 64)])
def test_w4a8_m16384_every_element(gpu, orc, name, K, N, group):
    """4-bit layers with weight groups of 128, 288, 32 and (72 groups along K: the large scale table, one workgroup per CU)
    64: every group partial sum and every output."""
    M, R = M_FULL, 1
    say("full W4", name, M, K, N, "group", group)
    x = workload.activations(M, K, "full4", name, sigma=0.6)
    lw = workload.layer_weights(name, K, N, 4, "full4")
    s_w = lw["s_w"] if group == 128 else workload.w4_scales_group(N, K, group, "full4", name)
    q_ref, s_ref = orc.daq(x, R, nthreads=16)
    P_ref = orc.gemm_w4g(q_ref, orc.pack_w4(lw["w"]), group, nthreads=16)
    y_ref = orc.epilogue_w4(P_ref, s_ref, R, s_w, lw["bias"])
    xd, wd, sd, bd = dev(x), dev(gpu.ql_pack_w4_host(lw["w"])), dev(s_w), dev(lw["bias"])
    y = gpu.qlinear_w4a8(xd, R, wd, sd, bd, group=group)
    assert y_mismatches(host(y), y_ref) == 0
    out = gpu.qlinear_w4a8(xd, R, wd, sd, bd, debug=True, group=group)
    assert np.array_equal(host(out["q"]), q_ref)
    assert np.array_equal(host(out["s_a"]).view(np.uint32), s_ref.view(np.uint32))
    Pg = host(out["P"])
    assert np.array_equal(Pg, P_ref)
    assert np.array_equal(host(out["y"]).view(np.uint16), host(y).view(np.uint16))
    del out, y, Pg, P_ref
    free()


@pytest.mark.parametrize("storage,rng_", [(4, (-8, 7)), (8, (-32, 31))])
def test_channel_group_scales_m16384_every_element(gpu, orc, storage, rng_):
    """Eq. (4) as printed (one activation scale per image and channel group of 128) through the pipelined grouped kernel at
    full size: proj shape, 64 images of 256 tokens."""
    M, K, N, R, group = M_FULL, 1152, 1152, 256, 128
    say("full channel-group scales", M, K, N, "storage", storage)
    x = workload.activations(M, K, "fullcg", storage, sigma=1.1)
    codes = workload.rng("fullcg-w", storage).integers(rng_[0], rng_[1] + 1, (N, K), dtype=np.int8)
    s_w = workload.w4_scales_group(N, K, group, "fullcg")
    bias = workload.bias(N, "fullcg")
    q_ref, a_ref = orc.daq_cg(x, R, group, nthreads=16)
    P_ref = orc.gemm_i8g(q_ref, codes, group, nthreads=16)
    y_ref = orc.epilogue_cg(P_ref, a_ref, R, s_w, bias)
    wd = dev(gpu.ql_pack_w4_host(codes)) if storage == 4 else dev(codes)
    y = gpu.qlinear_grouped(dev(x), R, wd, dev(s_w), group, dev(bias), act_group=group, storage=storage)
    assert y_mismatches(host(y), y_ref) == 0
    out = gpu.qlinear_grouped(dev(x), R, wd, dev(s_w), group, dev(bias), act_group=group, storage=storage, debug=True)
    assert np.array_equal(host(out["q"]), q_ref)
    assert np.array_equal(host(out["s_a"]).view(np.uint32), a_ref.view(np.uint32))
    assert np.array_equal(host(out["P"]), P_ref)
    del out
    free()


@pytest.mark.parametrize("K", [1152, 4608])
def test_daq_per_tensor_m16384(gpu, orc, K):
    """One scale for the whole tensor: R*K is 19 M / 75 M values, so the block maximum comes from more than 256 partial
    maxima and the one-workgroup-per-block reduction runs between the two passes."""
    M = M_FULL
    say("full DAQ per tensor", M, K)
    x = workload.activations(M, K, "fulldaq", K, sigma=2.3)
    x[M // 2 + 5, K - 3] = np.float16(-311.0)          # the maximum sits in a late part
    q_ref, s_ref = orc.daq(x, M, nthreads=16)
    q, s = gpu.daq_quantize(dev(x), M)
    assert np.array_equal(host(s).view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(host(q), q_ref)


@pytest.mark.parametrize("name,K,N", [("proj", 1152, 1152), ("fc2", 4608, 1152)])
def test_c4_per_sample_m16384_every_element(gpu, orc, name, K, N):
    """The paper's own granularity (one scale per image of 1024 tokens and timestep) at 16 images, in full.
    At K = 4608 an image has 288 partial maxima, so the separate reduction runs with 16 scale blocks."""
    M, R = M_FULL, 1024
    say("full C4 per sample", name, M, K, N)
    sig = workload.sigma_schedule(50)
    x = workload.activations(M, K, "c4full", name, sigma=float(sig[17]))
    # images of very different magnitude, so a scale taken from the wrong image would show
    x = (x.astype(np.float32) * np.repeat(2.0 ** (np.arange(M // R) % 5 - 2), R)[:, None].astype(np.float32)).astype(np.float16)
    lw = workload.layer_weights(name, K, N, 8, "c4full")
    ref = orc.qlinear_w8a8(x, R, lw["w"], lw["s_w"], lw["bias"], nthreads=16)
    out = gpu.qlinear_w8a8(dev(x), R, dev(lw["w"]), dev(lw["s_w"]), dev(lw["bias"]), debug=True)
    assert np.array_equal(host(out["s_a"]).view(np.uint32), ref["s_a"].view(np.uint32))
    assert np.array_equal(host(out["q"]), ref["q"])
    assert np.array_equal(host(out["acc"]), ref["acc"])
    assert y_mismatches(host(out["y"]), ref["y"]) == 0
    y = gpu.qlinear_w8a8(dev(x), R, dev(lw["w"]), dev(lw["s_w"]), dev(lw["bias"]))
    assert np.array_equal(host(y).view(np.uint16), host(out["y"]).view(np.uint16))
    del out, y
    free()


def test_row_absmax_side_output_m16384(gpu, orc):
    """fc1 (4-bit, GELU) at full size with the row-maximum side output, then fc2's DAQ from it with one scale per token
    and one per image of 1024 tokens: every row maximum, scale and code against the oracle applied to the y written."""
    import torch
    M, K, N = M_FULL, 1152, 4608
    say("full rowmax", M, K, N)
    x = workload.activations(M, K, "fullrm", sigma=0.8)
    lw = workload.layer_weights("fc1", K, N, 4, "fullrm")
    rowmax = torch.empty((M,), dtype=torch.int32, device="cuda")
    y = gpu.qlinear_fused(dev(x), 1, dev(gpu.ql_pack_w4_host(lw["w"])), dev(lw["s_w"]), dev(lw["bias"]), bits=4, group=128,
                          act=gpu.ACT_GELU_TANH, row_absmax=rowmax)
    yh = host(y)
    assert np.array_equal(host(rowmax).astype(np.uint32), orc.row_absmax_bits(yh))
    for R in (1, 1024):
        q_ref, s_ref = orc.daq(yh, R, nthreads=16)
        q, s = gpu.daq_quantize_rowmax(y, R, rowmax)
        assert np.array_equal(host(s).view(np.uint32), s_ref.view(np.uint32)), R
        assert np.array_equal(host(q), q_ref), R
        del q, s
    free()


def test_c5_plan_every_layer_on_tile_row_bands(gpu, orc):
    """The 112-layer stack under the seeded bit plan at full size, through qlinear_plan_run: EVERY layer is checked on
    two whole bands of 256 consecutive rows (all columns; the first and a late tile row of the walk) plus 40 scattered rows."""
    import torch
    M, R = M_FULL, 1
    plan_desc = workload.bit_plan()
    sig = float(workload.sigma_schedule(25)[9])
    x_by_type = {name: workload.activations(M, K, "c5full", name, sigma=sig) for name, K, N in workload.BLOCK_LAYERS}
    xd = {k: dev(v) for k, v in x_by_type.items()}
    layers, host_w = [], []
    for p in plan_desc:
        lw = workload.layer_weights(p["name"], p["K"], p["N"], p["bits"], "c5full", p["block"])
        w = dev(lw["w"]) if p["bits"] == 8 else dev(gpu.ql_pack_w4_host(lw["w"]))
        layers.append(dict(K=p["K"], N=p["N"], bits=p["bits"], w=w, w_scale=dev(lw["s_w"]), bias=dev(lw["bias"])))
        host_w.append(lw)
    plan = gpu.Plan(layers, M_max=M)
    ws = gpu.workspace(plan.workspace_bytes(M, R))
    scattered = workload.rng("c5full-rows").choice(M, size=40, replace=False)
    rows = np.unique(np.concatenate([np.arange(0, 256), np.arange(M - 768, M - 512), scattered, [M - 1]]))
    idx = torch.from_numpy(rows).cuda()
    x_in = [xd[p["name"]] for p in plan_desc]
    y_out = [torch.empty((M, p["N"]), dtype=torch.float16, device="cuda") for p in plan_desc]   # 9.5 GB: one buffer per layer
    say("C5 full plan run", len(layers), "layers,", sum(p["bits"] == 4 for p in plan_desc), "at W4,", len(rows), "rows checked per layer")
    plan.run(x_in, y_out, M, R, ws)
    torch.cuda.synchronize()
    kinds = set()
    for i, (p, lw) in enumerate(zip(plan_desc, host_w)):
        xs = x_by_type[p["name"]][rows]
        if p["bits"] == 8:
            ref = orc.qlinear_w8a8(xs, 1, lw["w"], lw["s_w"], lw["bias"], nthreads=16, want_debug=False)["y"]
        else:
            ref = orc.qlinear_w4a8(xs, 1, orc.pack_w4(lw["w"]), lw["s_w"], lw["bias"], nthreads=16, want_debug=False)["y"]
        assert y_mismatches(host(y_out[i][idx]), ref) == 0, (i, p["name"], p["bits"])
        kinds.add((p["name"], p["bits"]))
        if i % 16 == 15:
            say("C5 layers checked:", i + 1)
    assert len(kinds) == 8          # every layer type at both widths occurs in the plan
    plan.close()
