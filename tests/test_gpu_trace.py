"""On-device evidence for TileCoord (Sec. 4.1): with a tile trace every workgroup of a fused kernel
records which tile it computed, where it ran and when.  The recorded (m_tile, n_tile) of EVERY
workgroup is compared with the oracle's tile_coord, and the start clocks are checked against the
claim of Sec. 4.1 that workgroups are dispatched in the order of the swizzled tile sequence (slice
by slice after the local rank for ReduceScatter, chunk by chunk in arrival order for AllGather)."""
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


def _records(t: torch.Tensor, grid: int) -> dict:
    w = t[:grid].cpu().numpy().view(np.uint32).reshape(grid, 16)
    q = t[:grid].cpu().numpy().view(np.uint64).reshape(grid, 8)
    return dict(block=w[:, 0].astype(np.int64), m_tile=w[:, 1].astype(np.int64), n_tile=w[:, 2].astype(np.int64),
                k_part=(w[:, 3] & 0xffff).astype(np.int64), is_split=((w[:, 3] >> 16) & 1).astype(np.int64),
                die=w[:, 4].astype(np.int64), hw_id=w[:, 5], tile=w[:, 6].astype(np.int64),
                t_start=q[:, 4].astype(np.int64), t_ready=q[:, 5].astype(np.int64), t_main_end=q[:, 6].astype(np.int64),
                t_end=q[:, 7].astype(np.int64))


def _expected_tiles(op, p, w, rank, arrival, n_xcd, ctpc=1):
    """(tile index, K part) of every workgroup from the split plan, and the oracle's coordinates of every tile."""
    opc = fb.FLUX_OP_RS if op == "rs" else fb.FLUX_OP_AG
    full, split_tiles, split_k = fb.flux_split_plan(opc, p)
    sh = fb.flux_tile_shape(opc, p)
    grid = full + split_tiles * split_k
    blocks = np.arange(grid)
    tile = np.where(blocks < full, blocks, full + (blocks - full) % max(1, split_tiles))
    part = np.where(blocks < full, 0, (blocks - full) // max(1, split_tiles))
    coords = np.array([fo.tile_coord(op, int(t), w.M, w.N, w.R, rank, sh.tile_m, sh.tile_n, arrival, n_xcd, ctpc)
                       for t in range(full + split_tiles)])
    return grid, tile, part, coords, sh, split_k


JITTER_TICKS = 100      # 1 us at 100 MHz


def _check_dispatch_order(rec, tile, sh, w, what):
    """Sec. 4.1: ascending workgroup ids walk the bands (the tiles of one slice / chunk) in visit order
    and the hardware dispatches ascending ids, so a later band never starts before an earlier one: the
    first start clock and the median start clock are non-decreasing from band to band.  The bands of
    the first round are all dispatched within a fraction of a microsecond and a workgroup's first
    instruction follows its dispatch by a varying few hundred nanoseconds, so clocks are compared with
    a slack of one microsecond (a band's main loop alone takes tens of microseconds)."""
    band_sz = fo.band_height(w.M, w.R, sh.tile_m) * (-(-w.N // sh.tile_n))
    band = tile // band_sz
    first = [int(rec["t_start"][band == b].min()) for b in range(band.max() + 1)]
    med = [float(np.median(rec["t_start"][band == b])) for b in range(band.max() + 1)]
    t0 = first[0]
    assert all(x <= y + JITTER_TICKS for x, y in zip(first, first[1:])), (what, "first start per band", [x - t0 for x in first])
    assert all(x <= y + JITTER_TICKS for x, y in zip(med, med[1:])), (what, "median start per band", [x - t0 for x in med])
    # and the order is not vacuous: the last band starts after the first one has finished its main loops
    if band.max() >= 4 and len(tile) > 2 * 256:
        assert med[-1] > np.median(rec["t_main_end"][band == 0]), (what, "last band vs first band's main loop")


@pytest.mark.parametrize("cfg", [0, 1, 3])
@pytest.mark.parametrize("flags", [0, fb.FLUX_FLAG_NO_SWIZZLE, fb.FLUX_FLAG_NO_XCD_REMAP])
def test_rs_trace_matches_oracle_tile_coord(cfg, flags):
    # 3 rounds of 256x256 tiles on 256 compute units (a partly filled last round gets its K cut)
    w = fi.Workload("rs_trace", "rs", 4096, 10240, 512, 8, seed=91)
    rank = 5
    A, B, peers = fi.make_rs_inputs(w, rank)
    p = fb.problem(w.M, w.N, w.K, w.R, rank, tile_config=cfg, flags=flags)
    n_xcd = 1 if flags else 8
    grid, tile, part, coords, sh, split_k = _expected_tiles("rs", p, w, rank, None, n_xcd)
    _say("rs trace cfg", cfg, "flags", flags, "tile", sh.tile_m, sh.tile_n, "grid", grid, "split_k", split_k)
    dA, dB = A.to(gh.DEV), B.to(gh.DEV)
    dpeers = [None if t is None else t.to(gh.DEV) for t in peers]
    outs = [torch.full((w.S, w.N), float("nan"), dtype=torch.bfloat16, device=gh.DEV) for _ in range(w.R)]
    ws = gh.workspace_for(fb.FLUX_OP_RS, p)
    if ws is not None:
        fb.flux_init_buffers(fb.FLUX_OP_RS, p, ws)
    trace = torch.zeros((grid + 3, 8), dtype=torch.int64, device=gh.DEV)
    fb.flux_trace_next_call(trace)
    fb.flux_gemm_rs(p, dA, dB, dpeers, outs, ws)
    torch.cuda.synchronize()
    rec = _records(trace, grid)
    assert np.array_equal(rec["block"], np.arange(grid))
    assert np.array_equal(rec["tile"], tile)
    assert np.array_equal(rec["k_part"], part)
    if flags & fb.FLUX_FLAG_NO_SWIZZLE:
        tiles_n = -(-w.N // sh.tile_n)
        want = np.stack([tile // tiles_n, tile % tiles_n], axis=1)
    else:
        want = coords[tile]
    assert np.array_equal(np.stack([rec["m_tile"], rec["n_tile"]], axis=1), want)
    assert (trace[grid:] == 0).all()                          # nothing written past the grid
    assert (rec["t_start"] <= rec["t_main_end"]).all() and (rec["t_main_end"] <= rec["t_end"]).all()
    assert (rec["die"] < 8).all() and len(set(rec["die"].tolist())) == 8
    if not flags & fb.FLUX_FLAG_NO_SWIZZLE:
        _check_dispatch_order(rec, tile, sh, w, "rs")
    # the trace changes nothing in the result
    s64, _ = gh.oracle_rs(w, rank, A, B, peers)
    for r in range(w.R):
        gh.assert_close(outs[r], s64[r], w.out_dtype, f"slice {r}")
    # the request was consumed: the next call leaves the buffer alone
    trace.zero_()
    fb.flux_gemm_rs(p, dA, dB, dpeers, outs, ws)
    torch.cuda.synchronize()
    assert (trace == 0).all()


@pytest.mark.parametrize("order", ["ring", "random", "no_swizzle", "random_ctpc2"])
@pytest.mark.parametrize("cfg", [0, 1])
def test_ag_trace_matches_oracle_tile_coord(order, cfg):
    w = fi.Workload("ag_trace", "ag", 4096, 5120, 512, 8, seed=92)
    rank = 2
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    flags = fb.FLUX_FLAG_NO_SWIZZLE if order == "no_swizzle" else 0
    ctpc = 2 if order == "random_ctpc2" else 1          # two signals per chunk: a band is one communication tile
    if order == "ring":
        arrival = fo.default_order(rank, w.R)
    p = fb.problem(w.M, w.N, w.K, w.R, rank, tile_config=cfg, flags=flags, comm_tiles_per_chunk=ctpc,
                   spin_timeout_ticks=gh.TEST_TIMEOUT_TICKS)
    grid, tile, part, coords, sh, split_k = _expected_tiles("ag", p, w, rank, arrival, 1 if flags else 8, ctpc)
    _say("ag trace", order, "cfg", cfg, "tile", sh.tile_m, sh.tile_n, "grid", grid, "split_k", split_k)
    dchunks = [c.to(gh.DEV) for c in chunks]
    A_agg = torch.full((w.M, w.K), float("nan"), dtype=torch.bfloat16, device=gh.DEV)
    Cout = torch.full((w.M, w.N), float("nan"), dtype=torch.bfloat16, device=gh.DEV)
    signals = torch.zeros(w.R * ctpc, dtype=torch.int32, device=gh.DEV)
    ws = gh.workspace_for(fb.FLUX_OP_AG, p)
    fb.flux_init_buffers(fb.FLUX_OP_AG, p, ws, signals)
    trace = torch.zeros((grid, 8), dtype=torch.int64, device=gh.DEV)
    fb.flux_trace_next_call(trace)
    fb.flux_ag_gemm(p, dchunks, A_agg, B.to(gh.DEV), Cout, signals, arrival, ws, torch.cuda.current_stream(), torch.cuda.Stream())
    torch.cuda.synchronize()
    assert fb.flux_query_status(ws) == (fb.FLUX_OK, 0)
    rec = _records(trace, grid)
    assert np.array_equal(rec["block"], np.arange(grid))
    assert np.array_equal(rec["tile"], tile)
    if flags:
        tiles_n = -(-w.N // sh.tile_n)
        want = np.stack([tile // tiles_n, tile % tiles_n], axis=1)
    else:
        want = coords[tile]
    assert np.array_equal(np.stack([rec["m_tile"], rec["n_tile"]], axis=1), want)
    assert (rec["t_start"] <= rec["t_ready"]).all() and (rec["t_ready"] <= rec["t_main_end"]).all()
    assert (rec["t_main_end"] <= rec["t_end"]).all()
    if not flags:
        _check_dispatch_order(rec, tile, sh, w, "ag")
        # the tiles of the local chunk (the first band) need no transfer of their own rows: none of
        # them can be past its wait later than the last tile of the last chunk to arrive
        band_sz = fo.band_height(w.M, w.R, sh.tile_m) * (-(-w.N // sh.tile_n))
        assert rec["t_ready"][tile < band_sz].max() <= rec["t_ready"][tile >= (w.R - 1) * band_sz].max()
    C64, _ = gh.oracle_ag(w, chunks, B)
    gh.assert_close(Cout, C64, w.out_dtype)


def test_rs_resident_grid_walks_the_same_blocks_in_order():
    """A reduce-scatter grid of many short tiles runs as one resident workgroup per compute unit (256 of
    them) that walks the block sequence of Sec. 4.1 with the grid's stride, half of them starting late.
    Every block still leaves one record with the oracle's tile; blocks b and b + 256 ran on the same
    compute unit one after the other; the late half starts late by what the library says; the result is
    the one-workgroup-per-tile form's bit for bit, and the oracle's within tolerance."""
    w = fi.Workload("rs_resident", "rs", 8192, 8192, 256, 8, seed=94)
    rank = 3
    A, B, peers = fi.make_rs_inputs(w, rank)
    p = fb.problem(w.M, w.N, w.K, w.R, rank)
    wgs, delay = fb.flux_rs_resident_grid(p)
    assert wgs == 256 and delay > 0
    q = fb.problem(w.M, w.N, w.K, w.R, rank, flags=fb.FLUX_FLAG_NO_RESIDENT_GRID)
    assert fb.flux_rs_resident_grid(q) == (0, 0)
    grid, tile, part, coords, sh, split_k = _expected_tiles("rs", p, w, rank, None, 8)
    assert (sh.tile_m, sh.tile_n) == (256, 256) and split_k == 1 and grid == 1024
    _say("rs resident grid", grid, "blocks on", wgs, "workgroups, delay", delay, "ticks")
    dA, dB = A.to(gh.DEV), B.to(gh.DEV)
    dpeers = [None if t is None else t.to(gh.DEV) for t in peers]
    outs = [torch.full((w.S, w.N), float("nan"), dtype=torch.bfloat16, device=gh.DEV) for _ in range(w.R)]
    outs1 = [torch.full((w.S, w.N), float("nan"), dtype=torch.bfloat16, device=gh.DEV) for _ in range(w.R)]
    trace = torch.zeros((grid, 8), dtype=torch.int64, device=gh.DEV)
    fb.flux_trace_next_call(trace)
    fb.flux_gemm_rs(p, dA, dB, dpeers, outs)
    fb.flux_gemm_rs(q, dA, dB, dpeers, outs1)
    torch.cuda.synchronize()
    rec = _records(trace, grid)
    assert np.array_equal(rec["block"], np.arange(grid))
    assert np.array_equal(rec["tile"], tile)
    assert np.array_equal(np.stack([rec["m_tile"], rec["n_tile"]], axis=1), coords[tile])
    assert (rec["t_start"] <= rec["t_main_end"]).all() and (rec["t_main_end"] <= rec["t_end"]).all()
    where = rec["die"] * 256 + ((rec["hw_id"].astype(np.int64) >> 8) & 0xff)     # die, shader engine, array, compute unit
    for b in range(grid - wgs):
        assert where[b] == where[b + wgs], ("blocks of one workgroup on different units", b)
        assert rec["t_end"][b] <= rec["t_start"][b + wgs] + JITTER_TICKS, ("a workgroup's blocks overlap", b)
    assert len(set(where[:wgs].tolist())) == wgs                 # one workgroup per compute unit
    late = ((np.arange(wgs) >> 3) & 1) == 1
    t0 = rec["t_start"][:wgs]
    shift = float(np.median(t0[late]) - np.median(t0[~late]))
    assert 0.7 * delay <= shift <= 1.3 * delay + 2 * JITTER_TICKS, (shift, delay)
    # the order of Sec. 4.1, in time: a later round of blocks starts after an earlier one
    med = [float(np.median(rec["t_start"][i:i + wgs])) for i in range(0, grid, wgs)]
    assert all(x < y for x, y in zip(med, med[1:])), med
    s64, _ = gh.oracle_rs(w, rank, A, B, peers)
    for r in range(w.R):
        gh.assert_close(outs[r], s64[r], w.out_dtype, f"slice {r}")
        assert torch.equal(outs[r].view(torch.int16), outs1[r].view(torch.int16)), f"slice {r}: the two grid forms differ"


def test_trace_buffer_too_small_is_rejected():
    w = fi.Workload("rs_trace_small", "rs", 1024, 1024, 256, 8, seed=93)
    rank = 0
    A, B, peers = fi.make_rs_inputs(w, rank)
    p = fb.problem(w.M, w.N, w.K, w.R, rank, tile_config=4)
    outs = [torch.zeros((w.S, w.N), dtype=torch.bfloat16, device=gh.DEV) for _ in range(w.R)]
    trace = torch.zeros((8, 8), dtype=torch.int64, device=gh.DEV)        # 256 workgroups do not fit
    fb.flux_trace_next_call(trace)
    with pytest.raises(fb.FluxError) as e:
        fb.flux_gemm_rs(p, A.to(gh.DEV), B.to(gh.DEV), [None if t is None else t.to(gh.DEV) for t in peers], outs)
    assert e.value.status == fb.FLUX_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert (trace == 0).all()
