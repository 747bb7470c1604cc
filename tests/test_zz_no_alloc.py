"""flux_gemm_rs_static, the GEMM-ReduceScatter entry point that allocates nothing (its K-cut scratch
lives in an array inside the library), against flux_gemm_rs on the same inputs: bit for bit, on two
calls in a row of which the second is the smaller problem, so that what the first call left in the
shared array cannot leak into the second."""
import numpy as np
import pytest
import torch

from paper_2406_06858_amd import binding as fb
from paper_2406_06858_amd import inputs as fi

import gpu_harness as gh

pytestmark = pytest.mark.gpu


def _both(w, rank, **kw):
    A, B, peers = fi.make_rs_inputs(w, rank)
    p = fb.problem(w.M, w.N, w.K, w.R, rank, w.partial_dtype, w.out_dtype, **kw)
    dA, dB = A.to(gh.DEV), B.to(gh.DEV)
    dpeers = [None if t is None else t.to(gh.DEV) for t in peers]
    dt = torch.bfloat16 if w.out_dtype == "bf16" else torch.float32
    want = [torch.full((w.S, w.N), float("nan"), dtype=dt, device=gh.DEV) for _ in range(w.R)]
    got = [torch.full((w.S, w.N), float("nan"), dtype=dt, device=gh.DEV) for _ in range(w.R)]
    ws = gh.workspace_for(fb.FLUX_OP_RS, p)
    if ws is not None:
        fb.flux_init_buffers(fb.FLUX_OP_RS, p, ws)
    fb.flux_gemm_rs(p, dA, dB, dpeers, want, ws)
    torch.cuda.synchronize()
    return p, dA, dB, dpeers, want, got


def test_static_scratch_matches_workspace_form_twice_in_a_row():
    big = fi.WORKLOADS["c5_rs_m64"]                       # 64 x 8192 x 3584: K cut in two, 4 MB of partials
    small = fi.Workload("rs_small", "rs", 8, 1024, 2048, 8, seed=95)
    assert fb.flux_split_plan(fb.FLUX_OP_RS, fb.problem(big.M, big.N, big.K, 8, 3))[2] > 1
    assert fb.flux_split_plan(fb.FLUX_OP_RS, fb.problem(small.M, small.N, small.K, 8, 3))[2] > 1
    pb, Ab, Bb, peb, wantb, gotb = _both(big, 3)
    ps, As, Bs, pes, wants, gots = _both(small, 3)
    print("static call 1:", big.M, big.N, big.K, flush=True)
    fb.flux_gemm_rs_static(pb, Ab, Bb, peb, gotb)
    print("static call 2:", small.M, small.N, small.K, flush=True)
    fb.flux_gemm_rs_static(ps, As, Bs, pes, gots)
    torch.cuda.synchronize()
    for r in range(8):
        assert torch.equal(gotb[r].view(torch.int16), wantb[r].view(torch.int16)), f"first call, slice {r}"
        assert torch.equal(gots[r].view(torch.int16), wants[r].view(torch.int16)), f"second call, slice {r}"
    # and once more the other way round, on a stream that is kept fed
    for g in gotb + gots:
        g.fill_(float("nan"))
    for _ in range(3):
        fb.flux_gemm_rs_static(ps, As, Bs, pes, gots)
        fb.flux_gemm_rs_static(pb, Ab, Bb, peb, gotb)
    torch.cuda.synchronize()
    for r in range(8):
        assert torch.equal(gotb[r].view(torch.int16), wantb[r].view(torch.int16))
        assert torch.equal(gots[r].view(torch.int16), wants[r].view(torch.int16))


def test_static_scratch_fp32_variant_and_problems_without_a_k_cut():
    w = fi.WORKLOADS["c1_rs"]                              # fp32 partial and output, no K cut: the array is not touched
    p, A, B, peers, want, got = _both(w, 1, tile_config=fb.tile_config_for(*w.tile))
    fb.flux_gemm_rs_static(p, A, B, peers, got)
    torch.cuda.synchronize()
    for r in range(w.R):
        assert torch.equal(got[r], want[r])
    w2 = fi.Workload("rs_f32_cut", "rs", 64, 512, 4096, 8, partial_dtype="f32", out_dtype="f32", seed=96)
    p, A, B, peers, want, got = _both(w2, 5, split_k=4)
    fb.flux_gemm_rs_static(p, A, B, peers, got)
    torch.cuda.synchronize()
    for r in range(w2.R):
        assert torch.equal(got[r], want[r])


def test_static_entry_point_with_a_resident_grid():
    """Many short tiles run as a grid of resident workgroups (no scratch needed): twice in a row, then a
    K-cut problem that does use the array."""
    w = fi.Workload("rs_resident_static", "rs", 8192, 8192, 256, 8, seed=94)
    p, A, B, peers, want, got = _both(w, 3)
    assert fb.flux_rs_resident_grid(p)[0] == 256
    small = fi.Workload("rs_small", "rs", 8, 1024, 2048, 8, seed=95)
    ps, As, Bs, pes, wants, gots = _both(small, 3)
    for i in range(2):
        print("static resident call", i, flush=True)
        for g in got:
            g.fill_(float("nan"))
        fb.flux_gemm_rs_static(p, A, B, peers, got)
        torch.cuda.synchronize()
        for r in range(w.R):
            assert torch.equal(got[r].view(torch.int16), want[r].view(torch.int16)), f"call {i}, slice {r}"
    fb.flux_gemm_rs_static(ps, As, Bs, pes, gots)
    torch.cuda.synchronize()
    for r in range(8):
        assert torch.equal(gots[r].view(torch.int16), wants[r].view(torch.int16))


def test_static_scratch_rejects_what_does_not_fit():
    # 8192 x 4608 x 12288: the 64 tiles of the last round are cut four ways, 64 MB of partials
    p = fb.problem(8192, 4608, 12288, 8, 0)
    assert fb.flux_workspace_bytes(fb.FLUX_OP_RS, p) > fb.FLUX_STATIC_SCRATCH_BYTES
    dummy = torch.zeros(64, dtype=torch.bfloat16, device=gh.DEV)
    with pytest.raises(fb.FluxError) as e:
        fb.flux_gemm_rs_static(p, dummy, dummy, [dummy] * 8, [dummy] * 8)
    assert e.value.status == fb.FLUX_ERR_WORKSPACE
