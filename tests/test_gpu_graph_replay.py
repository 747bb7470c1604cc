"""Fused calls recorded in a HIP graph and replayed, with the program's own eager work and
synchronisations between the replays; every replay is checked against the eager result.  The fused
AllGather-GEMM without a copy kernel and the GEMM-ReduceScatter (K cut included) are single kernel
launches that keep all their per-call state in the workspace, so they can be recorded."""
import numpy as np
import pytest
import torch

import gpu_harness as gh
from paper_2406_06858_amd import binding as fb
from paper_2406_06858_amd import inputs as fi

pytestmark = pytest.mark.gpu
DEV = gh.DEV


def _say(*a):
    print(*a, flush=True)


@pytest.mark.parametrize("shape,gbps", [(dict(M=64, N=1024, K=2048), 0), (dict(M=1024, N=1024, K=512), 0), (dict(M=2048, N=2560, K=256), 0),
                                        (dict(M=8192, N=4608, K=2048), 0),        # two rounds: four chunks travel inside the main loops
                                        (dict(M=8192, N=4608, K=2048), 800)])     # ... all seven, on a link's schedule
def test_ag_gemm_replays_from_a_graph(shape, gbps):
    w = fi.scaled(fi.WORKLOADS["c2_ag"], **shape)
    rank = 5
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    C64, _ = gh.oracle_ag(w, chunks, B)
    p = fb.problem(w.M, w.N, w.K, w.R, rank, "bf16", w.out_dtype, spin_timeout_ticks=gh.TEST_TIMEOUT_TICKS, link_gbps=gbps)
    if shape["M"] == 8192:
        assert fb.flux_ag_deferred_tiles(p) == (7 if gbps else 4)
    dB = B.to(DEV)
    dchunks = [c.to(DEV) for c in chunks]
    A_agg = torch.full((w.M, w.K), float("nan"), dtype=torch.bfloat16, device=DEV)
    Cout = torch.full((w.M, w.N), float("nan"), dtype=torch.bfloat16, device=DEV)
    signals = torch.zeros(w.R, dtype=torch.int32, device=DEV)
    ws = gh.workspace_for(fb.FLUX_OP_AG, p)
    fb.flux_init_buffers(fb.FLUX_OP_AG, p, ws, signals)
    side = torch.cuda.Stream()
    copy = torch.cuda.Stream()

    def poison():
        A_agg.fill_(float("nan"))
        Cout.fill_(float("nan"))

    # eager result first (also takes first-call set-up out of the recording)
    _say("graph replay, AllGather-GEMM", shape, "eager call")
    fb.flux_ag_gemm(p, dchunks, A_agg, dB, Cout, signals, arrival, ws, torch.cuda.current_stream(), copy)
    torch.cuda.synchronize()
    assert fb.flux_query_status(ws) == (fb.FLUX_OK, 0)
    gh.assert_close(Cout, C64, w.out_dtype)
    eager = Cout.clone()

    g = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=side):
        fb.flux_ag_gemm(p, dchunks, A_agg, dB, Cout, signals, arrival, ws, torch.cuda.current_stream(), copy)
    torch.cuda.synchronize()
    for i in range(4):
        _say("replay", i)
        poison()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert fb.flux_query_status(ws) == (fb.FLUX_OK, 0)
        assert torch.equal(Cout.view(torch.int16), eager.view(torch.int16)), f"replay {i} differs from the eager result"
        gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")
        assert signals.cpu().tolist() == [1 if c == rank else 0 for c in range(w.R)]
        # eager work of the program between replays: the same call, not from the graph
        if i == 1:
            poison()
            fb.flux_ag_gemm(p, dchunks, A_agg, dB, Cout, signals, arrival, ws, torch.cuda.current_stream(), copy)
            torch.cuda.synchronize()
            assert torch.equal(Cout.view(torch.int16), eager.view(torch.int16))


@pytest.mark.parametrize("shape,split", [(dict(M=64, N=2048, K=1024), 4), (dict(M=1024, N=1024, K=512), 0),
                                         (dict(M=8192, N=8192, K=256), 0)])       # four rounds of short tiles: the resident grid
def test_gemm_rs_replays_from_a_graph(shape, split):
    w = fi.scaled(fi.WORKLOADS["c3_rs"], **shape)
    rank = 1
    A, B, peers = fi.make_rs_inputs(w, rank)
    want64, _ = gh.oracle_rs(w, rank, A, B, peers)
    p = fb.problem(w.M, w.N, w.K, w.R, rank, w.partial_dtype, w.out_dtype, split_k=split)
    if shape["M"] == 8192:
        assert fb.flux_rs_resident_grid(p)[0] == 256
    dA, dB = A.to(DEV), B.to(DEV)
    dpeers = [None if t is None else t.to(DEV) for t in peers]
    outs = [torch.full((w.S, w.N), float("nan"), dtype=torch.bfloat16, device=DEV) for _ in range(w.R)]
    ws = gh.workspace_for(fb.FLUX_OP_RS, p)
    if ws is not None:
        fb.flux_init_buffers(fb.FLUX_OP_RS, p, ws)
    side = torch.cuda.Stream()
    _say("graph replay, GEMM-ReduceScatter", shape, "split", split)
    fb.flux_gemm_rs(p, dA, dB, dpeers, outs, ws)
    torch.cuda.synchronize()
    for r in range(w.R):
        gh.assert_close(outs[r], want64[r], w.out_dtype, f"slice {r}")
    eager = [o.clone() for o in outs]
    g = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=side):
        fb.flux_gemm_rs(p, dA, dB, dpeers, outs, ws)
    torch.cuda.synchronize()
    for i in range(4):
        for o in outs:
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for r in range(w.R):
            assert torch.equal(outs[r].view(torch.int16), eager[r].view(torch.int16)), f"replay {i}, slice {r}"
