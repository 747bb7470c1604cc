"""GPU parity with row pitches (lda / ldb / ldc of the problem) and with B given as [N,K]
(b_is_nk): the operands and results sit in wider allocations, B may be handed over transposed, the
oracle gets the packed [K,N] views.  Integer inputs, so every comparison is bit for bit.  What lies between the end of a row and the next row is NaN on the input side (a kernel
that read it would poison its result) and a sentinel on the output side that must survive."""
import numpy as np
import pytest
import torch

from paper_2406_06858_amd import binding as fb
from paper_2406_06858_amd import inputs as fi

import gpu_harness as gh

pytestmark = pytest.mark.gpu

SENTINEL = 7.0
_T = {"bf16": torch.bfloat16, "f32": torch.float32}


def _say(*a):
    print(*a, flush=True)


def wide(t: torch.Tensor, ld: int, fill=float("nan")):
    """A copy of the matrix t inside an allocation of `ld` columns; returns (store, view)."""
    store = torch.full((t.shape[0], ld), fill, dtype=t.dtype, device=gh.DEV)
    view = store[:, :t.shape[1]]
    view.copy_(t)
    return store, view


def wide_out(rows: int, cols: int, ld: int, dtype: str):
    store = torch.full((rows, ld), SENTINEL, dtype=_T[dtype], device=gh.DEV)
    view = store[:, :cols]
    view.fill_(float("nan"))
    return store, view


def assert_gap_untouched(store: torch.Tensor, cols: int, what: str):
    gap = store[:, cols:]
    assert gap.numel() == 0 or bool((gap == SENTINEL).all()), f"{what}: the gap between rows was written"


def b_operand(B: torch.Tensor, pad: int, nk: bool):
    """B on the device as the library is to see it: [K,N], or its transpose [N,K], in rows `pad` elements longer."""
    Bm = B.t().contiguous() if nk else B
    ldb = Bm.shape[1] + pad
    return wide(Bm.to(gh.DEV), ldb)[1], (ldb if pad else 0)


def _rs_call(w, rank, A, B, peers, pads, tile_config=0, split_k=0, flags=0, static=False, nk=False):
    pa, pb, pc = pads
    lda, ldc = w.K + pa, w.N + pc
    dB, ldb = b_operand(B, pb, nk)
    p = fb.problem(w.M, w.N, w.K, w.R, rank, w.partial_dtype, w.out_dtype, tile_config, split_k, flags,
                   lda=lda if pa else 0, ldb=ldb, ldc=ldc if pc else 0, b_is_nk=int(nk))
    _, dA = wide(A.to(gh.DEV), lda)
    dpeers = [None if t is None else t.to(gh.DEV) for t in peers]
    outs = [wide_out(w.S, w.N, ldc, w.out_dtype) for _ in range(w.R)]
    if flags & fb.FLUX_FLAG_RS_ATOMIC:
        for _, v in outs:
            v.zero_()
    if static:
        fb.flux_gemm_rs_static(p, dA, dB, dpeers, [v for _, v in outs])
    else:
        ws = gh.workspace_for(fb.FLUX_OP_RS, p)
        if ws is not None:
            fb.flux_init_buffers(fb.FLUX_OP_RS, p, ws)
        fb.flux_gemm_rs(p, dA, dB, dpeers, [v for _, v in outs], ws)
    torch.cuda.synchronize()
    for r, (store, _) in enumerate(outs):
        assert_gap_untouched(store, w.N, f"slice {r}")
    return p, outs


RS_SHAPES = {
    # two rounds of 256x256 tiles would be too slow for the oracle; these span several tiles of every configuration
    "tiles": fi.Workload("pitch_rs", "rs", 1024, 768, 320, 4, a_dist=("int", 2), b_dist=("int", 2), peer_dist=("int", 8), seed=91),
    "ragged": fi.Workload("pitch_rs_ragged", "rs", 1000, 520, 200, 8, a_dist=("int", 2), b_dist=("int", 2), peer_dist=("int", 8), seed=92),
    "few_rows": fi.Workload("pitch_rs_decode", "rs", 64, 1024, 1792, 8, a_dist=("int", 2), b_dist=("int", 2), peer_dist=("int", 8), seed=93),
}


@pytest.mark.parametrize("pads", [(8, 16, 24), (64, 0, 0), (0, 128, 0), (0, 0, 8)])
@pytest.mark.parametrize("shape", list(RS_SHAPES))
@pytest.mark.parametrize("pd,od", [("bf16", "bf16"), ("f32", "f32")])
def test_rs_with_row_pitches(shape, pads, pd, od):
    w = fi.scaled(RS_SHAPES[shape], partial_dtype=pd, out_dtype=od)
    rank = w.R - 2
    A, B, peers = fi.make_rs_inputs(w, rank)
    _, want = gh.oracle_rs(w, rank, A, B, peers)
    for cfg in (0, 1, 4):
        _say("rs pitches", shape, pads, pd, od, "cfg", cfg)
        _, outs = _rs_call(w, rank, A, B, peers, pads, tile_config=cfg)
        for r in range(w.R):
            gh.assert_bits_equal(outs[r][1], want[r], f"cfg {cfg} slice {r}")


@pytest.mark.parametrize("cfg", [2, 3, 5, 6, 7, 8, 9, 10])
def test_rs_with_row_pitches_every_configuration(cfg):
    for shape in ("tiles", "ragged"):
        w = RS_SHAPES[shape]
        rank = 1
        _say("rs pitches cfg", cfg, shape)
        A, B, peers = fi.make_rs_inputs(w, rank)
        _, want = gh.oracle_rs(w, rank, A, B, peers)
        _, outs = _rs_call(w, rank, A, B, peers, (16, 8, 40), tile_config=cfg)
        for r in range(w.R):
            gh.assert_bits_equal(outs[r][1], want[r], f"slice {r}")


def test_rs_with_row_pitches_k_cut_resident_grid_and_static_scratch():
    """The forms that go beyond one workgroup per tile: K cut over several workgroups (partials parked in
    the workspace or in the library's own array), and the resident grid."""
    w = RS_SHAPES["tiles"]
    rank = 2
    A, B, peers = fi.make_rs_inputs(w, rank)
    _, want = gh.oracle_rs(w, rank, A, B, peers)
    for static in (False, True):
        _say("rs pitches split_k 2 static", static)
        _, outs = _rs_call(w, rank, A, B, peers, (8, 8, 8), tile_config=1, split_k=2, static=static)
        for r in range(w.R):
            gh.assert_bits_equal(outs[r][1], want[r], f"split slice {r}")
    wr = fi.Workload("pitch_rs_resident", "rs", 8192, 8192, 256, 8, a_dist=("int", 2), b_dist=("int", 2), peer_dist=("int", 8), seed=94)
    A, B, peers = fi.make_rs_inputs(wr, 3)
    _, want = gh.oracle_rs(wr, 3, A, B, peers)
    _say("rs pitches resident grid")
    p, outs = _rs_call(wr, 3, A, B, peers, (8, 64, 128))
    assert fb.flux_rs_resident_grid(p)[0] > 0
    for r in range(wr.R):
        gh.assert_bits_equal(outs[r][1], want[r], f"resident slice {r}")


@pytest.mark.parametrize("od", ["bf16", "f32"])
def test_rs_write_only_and_slice_reduce_with_row_pitches(od):
    """Write branch of Alg. 1 into pitched staging slices, then the owner's reduction of the R staged
    slices into a pitched output: equal to the fused reduce of the same inputs' oracle forms."""
    from oracle import flux_oracle as fo
    w = fi.scaled(RS_SHAPES["ragged"], partial_dtype=od, out_dtype=od)
    pads = (8, 16, 24)
    ldc = w.N + pads[2]
    own = 3
    staged = []
    for rank in range(w.R):
        A, B, _ = fi.make_rs_inputs(fi.scaled(w, seed=w.seed + rank), rank)
        _say("write-only pitched, producer", rank)
        _, outs = _rs_call(w, rank, A, B, [None] * w.R, pads, flags=fb.FLUX_FLAG_RS_WRITE_ONLY)
        _, want = fo.gemm_scatter(fi.to_numpy(A), fi.to_numpy(B), w.R, od)
        for r in range(w.R):
            gh.assert_bits_equal(outs[r][1], want[r], f"producer {rank} slice {r}")
        staged.append(outs[own])
    p = fb.problem(w.M, w.N, w.K, w.R, own, od, od, ldc=ldc)
    store, out = wide_out(w.S, w.N, ldc, od)
    fb.flux_rs_reduce_slice(p, [v for _, v in staged], out)
    torch.cuda.synchronize()
    assert_gap_untouched(store, w.N, "reduced slice")
    _, want = fo.reduce_slice([fi.to_numpy(v) for _, v in staged], od, od)
    gh.assert_bits_equal(out, want, "reduced slice")


def test_rs_atomic_with_row_pitches():
    from oracle import flux_oracle as fo
    w = fi.scaled(RS_SHAPES["ragged"], partial_dtype="f32", out_dtype="f32")
    rank = 4
    A, B, _ = fi.make_rs_inputs(w, rank)
    _, outs = _rs_call(w, rank, A, B, [None] * w.R, (8, 8, 8), flags=fb.FLUX_FLAG_RS_ATOMIC)
    zeros = [np.zeros((w.S, w.N), dtype=np.float32) for _ in range(w.R)]
    _, want = fo.gemm_reduce_into(fi.to_numpy(A), fi.to_numpy(B), zeros, w.R)
    for r in range(w.R):
        gh.assert_bits_equal(outs[r][1], want[r], f"slice {r}")


@pytest.mark.parametrize("nk", [False, True])
def test_tile_ready_producers_and_reducer_with_row_pitches(nk):
    """Reduce with tile-ready counters (Sec. 4.2, second form): producers write pitched staging slices and
    count their tiles in, the owner's reducer reads them at that pitch and writes a pitched slice."""
    from oracle import flux_oracle as fo
    R, owner, dt = 4, 2, "bf16"
    w = fi.Workload("pitch_rs_ready", "rs", 1024, 1280, 512, R, partial_dtype=dt, out_dtype=dt, seed=99,
                    a_dist=("int", 2), b_dist=("int", 2))
    pads = (8, 16, 40)
    lda, ldc = w.K + pads[0], w.N + pads[2]
    prods = []
    for j in range(R):
        A, B, _ = fi.make_rs_inputs(w, j)
        dB, ldb = b_operand(B, pads[1], nk)
        p = fb.problem(w.M, w.N, w.K, R, j, dt, dt, lda=lda, ldb=ldb, ldc=ldc, b_is_nk=int(nk), spin_timeout_ticks=gh.TEST_TIMEOUT_TICKS)
        outs = [wide_out(w.S, w.N, ldc, dt) for _ in range(R)]
        prods.append(dict(p=p, A=A, B=B, dA=wide(A.to(gh.DEV), lda)[1], dB=dB, outs=outs, stream=torch.cuda.Stream()))
    ready = torch.zeros(fb.flux_rs_ready_count(prods[0]["p"]), dtype=torch.int32, device=gh.DEV)
    cws = torch.zeros(16384, dtype=torch.int32, device=gh.DEV)
    fb.flux_init_buffers(fb.FLUX_OP_RS, prods[0]["p"], cws)
    store, out = wide_out(w.S, w.N, ldc, dt)
    torch.cuda.synchronize()
    _say("tile-ready with pitches, B as [N,K]:", nk)
    for d in prods:
        fb.flux_gemm_rs_notify(d["p"], d["dA"], d["dB"], [v for _, v in d["outs"]], ready, None, d["stream"])
    fb.flux_rs_reduce_slice_ready(prods[owner]["p"], [d["outs"][owner][1] for d in prods], out, ready, R, cws, torch.cuda.Stream())
    torch.cuda.synchronize()
    assert fb.flux_query_status(cws) == (fb.FLUX_OK, 0)
    assert (ready == R).all()
    staged = []
    for j, d in enumerate(prods):
        _, sbits = fo.gemm_scatter(fi.to_numpy(d["A"]), fi.to_numpy(d["B"]), R, dt)
        for r in range(R):
            assert_gap_untouched(d["outs"][r][0], w.N, f"producer {j} slice {r}")
            gh.assert_bits_equal(d["outs"][r][1], sbits[r], f"producer {j} slice {r}")
        staged.append(sbits[owner])
    assert_gap_untouched(store, w.N, "reduced slice")
    gh.assert_bits_equal(out, fo.reduce_slice(staged, dt, dt)[1], "reduced slice")


# ---------------------------------------------------------------------------------------------
# B as [N,K] (a linear layer's weight as it is stored): same bits as with its transpose
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("cfg", list(range(0, 11)))
@pytest.mark.parametrize("pads", [(0, 0, 0), (8, 24, 16)])
def test_rs_with_b_as_n_by_k(cfg, pads):
    for shape in RS_SHAPES:
        w = RS_SHAPES[shape]
        rank = 1
        _say("rs, B as [N,K], cfg", cfg, shape, pads)
        A, B, peers = fi.make_rs_inputs(w, rank)
        _, want = gh.oracle_rs(w, rank, A, B, peers)
        _, outs = _rs_call(w, rank, A, B, peers, pads, tile_config=cfg, nk=True)
        for r in range(w.R):
            gh.assert_bits_equal(outs[r][1], want[r], f"{shape} slice {r}")


def test_rs_with_b_as_n_by_k_k_cut_and_resident_grid():
    w = RS_SHAPES["tiles"]
    A, B, peers = fi.make_rs_inputs(w, 2)
    _, want = gh.oracle_rs(w, 2, A, B, peers)
    for static in (False, True):
        _say("rs, B as [N,K], split_k 2, static", static)
        _, outs = _rs_call(w, 2, A, B, peers, (0, 8, 0), tile_config=1, split_k=2, static=static, nk=True)
        for r in range(w.R):
            gh.assert_bits_equal(outs[r][1], want[r], f"split slice {r}")
    wr = fi.Workload("nk_rs_resident", "rs", 8192, 8192, 256, 8, a_dist=("int", 2), b_dist=("int", 2), peer_dist=("int", 8), seed=94)
    A, B, peers = fi.make_rs_inputs(wr, 3)
    _, want = gh.oracle_rs(wr, 3, A, B, peers)
    _say("rs, B as [N,K], resident grid")
    p, outs = _rs_call(wr, 3, A, B, peers, (0, 0, 0), nk=True)
    assert fb.flux_rs_resident_grid(p)[0] > 0
    for r in range(wr.R):
        gh.assert_bits_equal(outs[r][1], want[r], f"resident slice {r}")


@pytest.mark.parametrize("cfg", list(range(0, 11)))
@pytest.mark.parametrize("pads", [(0, 0, 0), (8, 24, 16)])
def test_ag_with_b_as_n_by_k(cfg, pads):
    for shape in ("tiles", "ragged", "few_rows"):
        w = AG_SHAPES[shape]
        rank = 2
        _say("ag, B as [N,K], cfg", cfg, shape, pads)
        chunks, B, arrival = fi.make_ag_inputs(w, rank)
        _, want = gh.oracle_ag(w, chunks, B)
        _, Cg, A_agg = _ag_call(w, rank, chunks, B, arrival, pads, tile_config=cfg, nk=True)
        gh.assert_bits_equal(Cg, want, f"{shape} C")
        gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")


def test_ag_with_b_as_n_by_k_chunks_carried_inside_the_main_loops():
    w = AG_SHAPES["two_rounds"]
    rank = 5
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    _, want = gh.oracle_ag(w, chunks, B)
    for kw in (dict(), dict(link_gbps=800)):
        _say("ag, B as [N,K], carried transfer", kw)
        p, Cg, A_agg = _ag_call(w, rank, chunks, B, arrival, (0, 0, 0), nk=True, **kw)
        assert fb.flux_ag_deferred_tiles(p) > 0
        gh.assert_bits_equal(Cg, want, "C")
        gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")


# ---------------------------------------------------------------------------------------------
# AllGather-GEMM: the gathered matrix, B and C pitched; the chunk sources stay packed
# ---------------------------------------------------------------------------------------------

def _ag_call(w, rank, chunks, B, arrival, pads, repeat=2, local_in_place=False, nk=False, **kw):
    pa, pb, pc = pads
    lda, ldc = w.K + pa, w.N + pc
    dB, ldb = b_operand(B, pb, nk)
    p = fb.problem(w.M, w.N, w.K, w.R, rank, "bf16", w.out_dtype, spin_timeout_ticks=gh.TEST_TIMEOUT_TICKS,
                   lda=lda if pa else 0, ldb=ldb, ldc=ldc if pc else 0, b_is_nk=int(nk), **kw)
    agg_store = torch.full((w.M, lda), SENTINEL, dtype=torch.bfloat16, device=gh.DEV)
    A_agg = agg_store[:, :w.K]
    dchunks = [c.to(gh.DEV) for c in chunks]
    if local_in_place:
        A_agg[rank * w.S:(rank + 1) * w.S].copy_(dchunks[rank])
        dchunks[rank] = A_agg[rank * w.S:(rank + 1) * w.S]
    c_store, Cout = wide_out(w.M, w.N, ldc, w.out_dtype)
    ctpc = max(1, kw.get("comm_tiles_per_chunk", 0))
    signals = torch.full((w.R * ctpc,), 999, dtype=torch.int32, device=gh.DEV)
    ws = gh.workspace_for(fb.FLUX_OP_AG, p)
    ws.fill_(-1)
    fb.flux_init_buffers(fb.FLUX_OP_AG, p, ws, signals)
    compute, copy = torch.cuda.current_stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for i in range(repeat):
        A_agg[:rank * w.S].fill_(float("nan"))
        A_agg[(rank + 1) * w.S:].fill_(float("nan"))
        Cout.fill_(float("nan"))
        fb.flux_ag_gemm(p, dchunks, A_agg, dB, Cout, signals, arrival, ws, compute, copy)
        torch.cuda.synchronize()
        assert fb.flux_query_status(ws) == (fb.FLUX_OK, 0), f"call {i}"
    assert_gap_untouched(agg_store, w.K, "gathered matrix")
    assert_gap_untouched(c_store, w.N, "C")
    assert signals.tolist() == [1 if i // ctpc == rank else 0 for i in range(w.R * ctpc)]
    return p, Cout, A_agg


AG_SHAPES = {
    "tiles": fi.Workload("pitch_ag", "ag", 1024, 512, 448, 4, a_dist=("int", 2), b_dist=("int", 2), seed=95),
    "ragged": fi.Workload("pitch_ag_ragged", "ag", 1000, 520, 200, 8, a_dist=("int", 2), b_dist=("int", 2), seed=96),
    "few_rows": fi.Workload("pitch_ag_decode", "ag", 64, 1792, 1024, 8, a_dist=("int", 2), b_dist=("int", 2), seed=97),
    "two_rounds": fi.Workload("pitch_ag_two_rounds", "ag", 8192, 4608, 1024, 8, a_dist=("int", 2), b_dist=("int", 2), seed=98),
}

AG_FORMS = {
    "grid_moves_the_chunks": dict(),
    "copy_kernel": dict(copy_workgroups=16),
    "copy_kernel_paced": dict(copy_workgroups=8, link_gbps=200),
    "paced_without_a_driver_request": dict(link_gbps=400),
    "library_copies": dict(flags=fb.FLUX_FLAG_COPY_MEMCPY),
    "two_signals_per_chunk": dict(comm_tiles_per_chunk=2),
}


@pytest.mark.parametrize("form", list(AG_FORMS))
@pytest.mark.parametrize("shape", list(AG_SHAPES))
@pytest.mark.parametrize("pads", [(8, 16, 24), (64, 0, 0)])
def test_ag_with_row_pitches(shape, form, pads):
    w = AG_SHAPES[shape]
    kw = dict(AG_FORMS[form])
    if form == "two_signals_per_chunk" and w.S % 2:
        pytest.skip("the chunk height is odd")
    rank = w.R - 1
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    _, want = gh.oracle_ag(w, chunks, B)
    _say("ag pitches", shape, form, pads)
    p, Cg, A_agg = _ag_call(w, rank, chunks, B, arrival, pads, **kw)
    if pads[0]:
        assert fb.flux_ag_deferred_tiles(p) == 0     # a pitched tile is not one run of memory: nothing is carried inside the main loops
    gh.assert_bits_equal(Cg, want, "C")
    gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")


def test_ag_with_row_pitches_local_chunk_in_place_and_every_configuration():
    w = AG_SHAPES["tiles"]
    rank = 1
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    _, want = gh.oracle_ag(w, chunks, B)
    for cfg in range(1, 11):
        _say("ag pitches cfg", cfg)
        _, Cg, A_agg = _ag_call(w, rank, chunks, B, arrival, (24, 8, 8), tile_config=cfg, local_in_place=(cfg % 2 == 0))
        gh.assert_bits_equal(Cg, want, f"cfg {cfg}")
        gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")


# ---------------------------------------------------------------------------------------------
# the unfused and chunked references take the same pitches
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("nk", [False, True])
def test_references_with_row_pitches(nk):
    pads = (8, 16, 24)
    w = RS_SHAPES["ragged"]
    rank = 2
    lda, ldc = w.K + pads[0], w.N + pads[2]
    A, B, peers = fi.make_rs_inputs(w, rank)
    _, want = gh.oracle_rs(w, rank, A, B, peers)
    dB, ldb = b_operand(B, pads[1], nk)
    p = fb.problem(w.M, w.N, w.K, w.R, rank, w.partial_dtype, w.out_dtype, lda=lda, ldb=ldb, ldc=ldc, b_is_nk=int(nk))
    _, dA = wide(A.to(gh.DEV), lda)
    dpeers = [None if t is None else t.to(gh.DEV) for t in peers]
    for which in ("unfused", "chunked"):
        _say("rs reference with pitches:", which)
        outs = [wide_out(w.S, w.N, ldc, w.out_dtype) for _ in range(w.R)]
        c_store, Cfull = wide_out(w.M, w.N, ldc, w.out_dtype)
        if which == "unfused":
            ws = gh.workspace_for(fb.FLUX_OP_RS, p)
            if ws is not None:
                fb.flux_init_buffers(fb.FLUX_OP_RS, p, ws)
            fb.flux_gemm_ref_unfused(fb.FLUX_OP_RS, fb.FLUX_PHASE_GEMM | fb.FLUX_PHASE_COMM, p, A=dA, B=dB, peer_partials=dpeers,
                                     out_slices=[v for _, v in outs], Cout=Cfull, workspace=ws)
        else:
            n = fb.flux_chunked_workspace_bytes(fb.FLUX_OP_RS, p)
            ws = torch.zeros(max(1, (n + 3) // 4), dtype=torch.int32, device=gh.DEV) if n else None
            fb.flux_gemm_ref_chunked(fb.FLUX_OP_RS, p, A=dA, B=dB, peer_partials=dpeers, out_slices=[v for _, v in outs], Cout=Cfull,
                                     workspace=ws, compute_stream=torch.cuda.current_stream(), comm_stream=torch.cuda.Stream())
        torch.cuda.synchronize()
        assert_gap_untouched(c_store, w.N, "C")
        for r in range(w.R):
            assert_gap_untouched(outs[r][0], w.N, f"slice {r}")
            gh.assert_bits_equal(outs[r][1], want[r], f"{which} slice {r}")

    wa = AG_SHAPES["ragged"]
    lda, ldc = wa.K + pads[0], wa.N + pads[2]
    chunks, B, arrival = fi.make_ag_inputs(wa, rank)
    _, want = gh.oracle_ag(wa, chunks, B)
    dB, ldb = b_operand(B, pads[1], nk)
    p = fb.problem(wa.M, wa.N, wa.K, wa.R, rank, "bf16", wa.out_dtype, lda=lda, ldb=ldb, ldc=ldc, b_is_nk=int(nk))
    dchunks = [c.to(gh.DEV) for c in chunks]
    for which in ("unfused", "chunked"):
        _say("ag reference with pitches:", which)
        agg_store = torch.full((wa.M, lda), SENTINEL, dtype=torch.bfloat16, device=gh.DEV)
        A_agg = agg_store[:, :wa.K]
        A_agg.fill_(float("nan"))
        c_store, Cout = wide_out(wa.M, wa.N, ldc, wa.out_dtype)
        if which == "unfused":
            ws = gh.workspace_for(fb.FLUX_OP_AG, p)
            fb.flux_init_buffers(fb.FLUX_OP_AG, p, ws)
            fb.flux_gemm_ref_unfused(fb.FLUX_OP_AG, fb.FLUX_PHASE_GEMM | fb.FLUX_PHASE_COMM, p, A_chunks=dchunks, A_agg=A_agg, B=dB,
                                     Cout=Cout, workspace=ws)
        else:
            n = fb.flux_chunked_workspace_bytes(fb.FLUX_OP_AG, p)
            ws = torch.zeros(max(1, (n + 3) // 4), dtype=torch.int32, device=gh.DEV) if n else None
            fb.flux_gemm_ref_chunked(fb.FLUX_OP_AG, p, A_chunks=dchunks, A_agg=A_agg, B=dB, Cout=Cout, arrival_order=arrival,
                                     workspace=ws, compute_stream=torch.cuda.current_stream(), comm_stream=torch.cuda.Stream())
        torch.cuda.synchronize()
        assert_gap_untouched(agg_store, wa.K, "gathered matrix")
        assert_gap_untouched(c_store, wa.N, "C")
        gh.assert_bits_equal(Cout, want, which)
        gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")
