"""Reduce with producer -> consumer tile-ready counters (Sec. 4.2, "Reduce", second form): R virtual
producers (one fused GEMM with the Write branch each, on streams of their own) scatter their partial
products by owner and count every tile in; the owner's reducer waits tile by tile and sums what has
been staged for its slice.  Integer inputs: bit for bit against the oracle's gemm_scatter and
reduce_slice."""
import numpy as np
import pytest
import torch

from oracle import flux_oracle as fo
from paper_2406_06858_amd import binding as fb
from paper_2406_06858_amd import inputs as fi

import gpu_harness as gh

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _setup(w, cfg, dt, split_k=0):
    tdt = torch.bfloat16 if dt == "bf16" else torch.float32
    prod = []
    for j in range(w.R):
        A, B, _ = fi.make_rs_inputs(w, j)
        p = fb.problem(w.M, w.N, w.K, w.R, j, dt, dt, tile_config=cfg, split_k=split_k, spin_timeout_ticks=gh.TEST_TIMEOUT_TICKS)
        outs = [torch.full((w.S, w.N), float("nan"), dtype=tdt, device=gh.DEV) for _ in range(w.R)]
        q = fb.problem(w.M, w.N, w.K, w.R, j, dt, dt, tile_config=cfg, split_k=split_k, flags=fb.FLUX_FLAG_RS_WRITE_ONLY)
        ws = gh.workspace_for(fb.FLUX_OP_RS, q)
        if ws is not None:
            fb.flux_init_buffers(fb.FLUX_OP_RS, q, ws)
        prod.append(dict(p=p, A=A, B=B, dA=A.to(gh.DEV), dB=B.to(gh.DEV), outs=outs, ws=ws, stream=torch.cuda.Stream()))
    ready = torch.zeros(fb.flux_rs_ready_count(prod[0]["p"]), dtype=torch.int32, device=gh.DEV)
    cws = torch.zeros(16384, dtype=torch.int32, device=gh.DEV)
    fb.flux_init_buffers(fb.FLUX_OP_RS, prod[0]["p"], cws)
    torch.cuda.synchronize()
    return prod, ready, cws, tdt


@pytest.mark.parametrize("cfg", [0, 1, 4, 2])
@pytest.mark.parametrize("dt", ["bf16", "f32"])
@pytest.mark.parametrize("delay", [False, True])
def test_producers_on_their_own_streams_and_a_waiting_reducer(cfg, dt, delay):
    R, owner = 4, 1
    w = fi.Workload("rs_ready", "rs", 1024, 1280, 512, R, partial_dtype=dt, out_dtype=dt, seed=97,
                    a_dist=("int", 2), b_dist=("int", 2))
    prod, ready, cws, tdt = _setup(w, cfg, dt)
    sh = fb.flux_tile_shape(fb.FLUX_OP_RS, prod[0]["p"])
    _say("ready flags cfg", cfg, dt, "delay", delay, "tile", sh.tile_m, sh.tile_n, "counters", ready.numel())
    out = torch.full((w.S, w.N), float("nan"), dtype=tdt, device=gh.DEV)
    cstream = torch.cuda.Stream()
    if delay:           # the reducer is running and waiting before any producer starts
        for d in prod:
            with torch.cuda.stream(d["stream"]):
                torch.cuda._sleep(40_000_000)
    for d in prod:      # producers first: the reducer can then never sit ahead of one in a hardware queue
        fb.flux_gemm_rs_notify(d["p"], d["dA"], d["dB"], d["outs"], ready, d["ws"], d["stream"])
    po = prod[owner]["p"]
    fb.flux_rs_reduce_slice_ready(po, [d["outs"][owner] for d in prod], out, ready, R, cws, cstream)
    torch.cuda.synchronize()
    assert fb.flux_query_status(cws) == (fb.FLUX_OK, 0)
    assert (ready == R).all()                                 # every producer counted every tile exactly once
    staged_ref = []
    for j, d in enumerate(prod):
        _, sbits = fo.gemm_scatter(fi.to_numpy(d["A"]), fi.to_numpy(d["B"]), R, dt)
        for r in range(R):
            gh.assert_bits_equal(d["outs"][r], sbits[r], f"producer {j} slice {r}")
        staged_ref.append(sbits[owner])
    gh.assert_bits_equal(out, fo.reduce_slice(staged_ref, dt, dt)[1], "reduced slice")


def test_k_cut_tiles_and_slices_smaller_than_a_tile():
    """Decode-like shape: one m-tile spans all slices, K is cut; every tile is still counted once per
    producer, by the workgroup that writes it, and each owner's reducer finds its rows."""
    R = 8
    w = fi.Workload("rs_ready_decode", "rs", 64, 2048, 2048, R, seed=98, a_dist=("int", 2), b_dist=("int", 2))
    prod, ready, cws, tdt = _setup(w, 0, "bf16")
    assert fb.flux_split_plan(fb.FLUX_OP_RS, prod[0]["p"])[2] > 1
    for d in prod:
        fb.flux_gemm_rs_notify(d["p"], d["dA"], d["dB"], d["outs"], ready, d["ws"], d["stream"])
    outs = []
    cstream = torch.cuda.Stream()
    for owner in (0, 5, 7):
        out = torch.full((w.S, w.N), float("nan"), dtype=tdt, device=gh.DEV)
        fb.flux_rs_reduce_slice_ready(prod[owner]["p"], [d["outs"][owner] for d in prod], out, ready, R, cws, cstream)
        outs.append((owner, out))
    torch.cuda.synchronize()
    assert fb.flux_query_status(cws) == (fb.FLUX_OK, 0)
    assert (ready == R).all()
    scat = [fo.gemm_scatter(fi.to_numpy(d["A"]), fi.to_numpy(d["B"]), R, "bf16")[1] for d in prod]
    for owner, out in outs:
        gh.assert_bits_equal(out, fo.reduce_slice([s[owner] for s in scat], "bf16", "bf16")[1], f"owner {owner}")


def test_reducer_gives_up_on_a_producer_that_never_comes():
    """Failure handling forced from the host: the reducer expects one producer more than there are.
    Every kernel still exits; the status block names a counter; nothing is written for the tiles given up."""
    R, owner = 2, 0
    w = fi.Workload("rs_ready_timeout", "rs", 512, 512, 256, R, seed=99, a_dist=("int", 2), b_dist=("int", 2))
    prod, ready, cws, tdt = _setup(w, 1, "bf16")
    for d in prod:
        fb.flux_gemm_rs_notify(d["p"], d["dA"], d["dB"], d["outs"], ready, d["ws"], d["stream"])
    out = torch.full((w.S, w.N), float("nan"), dtype=tdt, device=gh.DEV)
    p = fb.problem(w.M, w.N, w.K, R, owner, tile_config=1, spin_timeout_ticks=2_000_000)     # 20 ms per tile
    fb.flux_rs_reduce_slice_ready(p, [d["outs"][owner] for d in prod], out, ready, R + 1, cws, torch.cuda.Stream())
    torch.cuda.synchronize()
    code, detail = fb.flux_query_status(cws)
    assert code == fb.FLUX_ERR_TIMEOUT and 0 <= detail < ready.numel()
    assert torch.isnan(out).all()
    # after clearing the status block the same buffers work with the right count
    fb.flux_init_buffers(fb.FLUX_OP_RS, p, cws)
    fb.flux_rs_reduce_slice_ready(p, [d["outs"][owner] for d in prod], out, ready, R, cws, torch.cuda.Stream())
    torch.cuda.synchronize()
    assert fb.flux_query_status(cws) == (fb.FLUX_OK, 0)
    scat = [fo.gemm_scatter(fi.to_numpy(d["A"]), fi.to_numpy(d["B"]), R, "bf16")[1] for d in prod]
    gh.assert_bits_equal(out, fo.reduce_slice([s[owner] for s in scat], "bf16", "bf16")[1], "after retry")
