"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Placement and exact-integer cases are bit-exact; floating-point cases use
|gpu - ref64| <= tol * max(1, |ref64|) with tol = 1e-2 (bf16 out) or 1e-5 (fp32 variant)."""
import numpy as np
import pytest
import torch

from oracle import flux_oracle as fo
from paper_2406_06858_amd import binding as fb
from paper_2406_06858_amd import inputs as fi

import gpu_harness as gh

pytestmark = pytest.mark.gpu

W = fi.WORKLOADS
ALL_CFGS = [1, 2, 3, 4, 5, 6, 7, 8, 9, 10]


def _say(*a):
    print(*a, flush=True)


# ---------------------------------------------------------------------------------------------
# c1: the small fp32 case, every rank, forced 64x64 tiles and every other configuration
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("rank", [0, 1])
@pytest.mark.parametrize("cfg", [4, 0, 1, 3])
def test_c1_rs_fp32_variant(rank, cfg):
    w = W["c1_rs"]
    _say("c1_rs rank", rank, "cfg", cfg)
    A, B, peers = fi.make_rs_inputs(w, rank)
    outs = gh.run_rs(w, rank, A, B, peers, tile_config=cfg)
    s64, _ = gh.oracle_rs(w, rank, A, B, peers)
    for r in range(w.R):
        gh.assert_close(outs[r], s64[r], "f32", f"slice {r}")


# ---------------------------------------------------------------------------------------------
# exact-integer inputs: every partial sum is an integer < 2^24, so fp32 and fp64 agree exactly
# and the single bf16 rounding is unique -> whole outputs compared bitwise
# ---------------------------------------------------------------------------------------------

INT_RS = fi.Workload("int_rs", "rs", 640, 384, 320, 4, a_dist=("int", 2), b_dist=("int", 2),
                     peer_dist=("int", 8), seed=77)


@pytest.mark.parametrize("cfg", ALL_CFGS)
@pytest.mark.parametrize("pd,od", [("bf16", "bf16"), ("f32", "f32"), ("bf16", "f32")])
def test_rs_exact_integers_bitwise(cfg, pd, od):
    w = fi.scaled(INT_RS, partial_dtype=pd, out_dtype=od)
    for rank in (0, 3):
        _say("int_rs cfg", cfg, pd, od, "rank", rank)
        A, B, peers = fi.make_rs_inputs(w, rank)
        outs = gh.run_rs(w, rank, A, B, peers, tile_config=cfg)
        _, want = gh.oracle_rs(w, rank, A, B, peers)
        for r in range(w.R):
            gh.assert_bits_equal(outs[r], want[r], f"cfg {cfg} slice {r}")


@pytest.mark.parametrize("R,rank", [(16, 0), (16, 9), (12, 11), (1, 0), (3, 1)])
@pytest.mark.parametrize("pd,od", [("bf16", "bf16"), ("f32", "f32")])
def test_rank_counts_bitwise(R, rank, pd, od):
    """Other numbers of virtual ranks than 8: up to 8 ranks the epilogue issues 7 peer loads per piece,
    above that 15; one rank has no peers at all.  Same for the AllGather signals and chunks."""
    wr = fi.Workload("int_rs_r", "rs", 192 * R // (R if R < 4 else 4), 256, 192, R, a_dist=("int", 2), b_dist=("int", 2),
                     peer_dist=("int", 4), partial_dtype=pd, out_dtype=od, seed=83)
    _say("ranks", R, rank, pd, od, "M", wr.M)
    A, B, peers = fi.make_rs_inputs(wr, rank)
    _, want = gh.oracle_rs(wr, rank, A, B, peers)
    for cfg in (0, 1, 4):
        outs = gh.run_rs(wr, rank, A, B, peers, tile_config=cfg)
        for r in range(R):
            gh.assert_bits_equal(outs[r], want[r], f"cfg {cfg} slice {r}")
    if pd == "bf16":
        wa = fi.Workload("int_ag_r", "ag", wr.M, 256, 192, R, a_dist=("int", 2), b_dist=("int", 2), seed=84)
        chunks, Ba, arrival = fi.make_ag_inputs(wa, rank)
        _, want = gh.oracle_ag(wa, chunks, Ba)
        for cw in (0, 8):
            Cg, _, signals, status = gh.run_ag(wa, rank, chunks, Ba, arrival, copy_workgroups=cw, repeat=2)
            assert status == (fb.FLUX_OK, 0)
            gh.assert_bits_equal(Cg, want, f"ag cw {cw}")
            assert signals.cpu().tolist() == [1 if c == rank else 0 for c in range(R)]


@pytest.mark.parametrize("cfg", ALL_CFGS)
def test_rs_ragged_shapes_bitwise(cfg):
    # M, N, K are multiples of neither tile size; slice height 125 straddles tiles
    w = fi.Workload("int_rs_ragged", "rs", 1000, 520, 200, 8, a_dist=("int", 2), b_dist=("int", 2),
                    peer_dist=("int", 8), seed=78)
    rank = 5
    _say("ragged rs cfg", cfg)
    A, B, peers = fi.make_rs_inputs(w, rank)
    outs = gh.run_rs(w, rank, A, B, peers, tile_config=cfg)
    _, want = gh.oracle_rs(w, rank, A, B, peers)
    for r in range(w.R):
        gh.assert_bits_equal(outs[r], want[r], f"slice {r}")


@pytest.mark.parametrize("cfg", ALL_CFGS)
def test_ag_exact_integers_bitwise(cfg):
    w = fi.Workload("int_ag", "ag", 768, 320, 448, 4, a_dist=("int", 2), b_dist=("int", 2), seed=79)
    for rank in (0, 2):
        _say("int_ag cfg", cfg, "rank", rank)
        chunks, B, arrival = fi.make_ag_inputs(w, rank)
        # three calls in a row on the same buffers: each must leave signals and counters ready
        Cg, A_agg, signals, status = gh.run_ag(w, rank, chunks, B, arrival, tile_config=cfg, repeat=3,
                                               copy_workgroups=16 if rank else 0)    # copy kernel / none
        assert status == (fb.FLUX_OK, 0)
        _, want = gh.oracle_ag(w, chunks, B)
        gh.assert_bits_equal(Cg, want, f"cfg {cfg}")
        # A_agg is the row-wise concatenation of the chunks, bit for bit
        gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")
        # signals are left in the preset state: local 1, the others 0
        assert signals.cpu().tolist() == [1 if c == rank else 0 for c in range(w.R)]


def test_rs_placement_probe():
    """A.B carries the global row index, peers are zero: every output element says which global
    row it came from; all R slices, every row, bit-exact."""
    M, N, K, R, rank = 512, 256, 256, 8, 6
    w = fi.Workload("probe", "rs", M, N, K, R, partial_dtype="f32", out_dtype="f32")
    A = torch.zeros(M, K)
    A[torch.arange(M), torch.arange(M) % K] = torch.arange(M, dtype=torch.float32) % 251   # exact in bf16
    B = torch.ones(K, N)
    peers = [None if j == rank else torch.zeros(M, N) for j in range(R)]
    outs = gh.run_rs(w, rank, A.bfloat16(), B.bfloat16(), peers)
    for r in range(R):
        want = ((torch.arange(w.S) + r * w.S) % 251).to(torch.float32)[:, None].expand(w.S, N)
        assert torch.equal(outs[r].cpu(), want), f"slice {r}"


# ---------------------------------------------------------------------------------------------
# floating-point parity at reduced and full sizes
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("name,shrink", [("c3_rs", dict(M=1024, N=1024, K=768)), ("c4_rs", dict(M=2048, N=1536, K=512))])
def test_rs_reduced_size_all_elements(name, shrink):
    w = fi.scaled(W[name], **shrink)
    for rank, cfg in ((0, 0), (5, 1), (7, 2), (2, 3)):
        _say(name, "reduced rank", rank, "cfg", cfg)
        A, B, peers = fi.make_rs_inputs(w, rank)
        outs = gh.run_rs(w, rank, A, B, peers, tile_config=cfg)
        s64, _ = gh.oracle_rs(w, rank, A, B, peers)
        for r in range(w.R):
            gh.assert_close(outs[r], s64[r], w.out_dtype, f"slice {r}")


@pytest.mark.parametrize("name,shrink", [("c2_ag", dict(M=1024, N=896, K=1024)), ("c4_ag", dict(M=2048, N=768, K=1536))])
def test_ag_reduced_size_all_elements(name, shrink):
    w = fi.scaled(W[name], **shrink)
    for rank, cfg in ((0, 0), (3, 1), (7, 2), (4, 3)):
        _say(name, "reduced rank", rank, "cfg", cfg)
        chunks, B, arrival = fi.make_ag_inputs(w, rank)
        Cg, _, _, status = gh.run_ag(w, rank, chunks, B, arrival, tile_config=cfg)
        assert status == (fb.FLUX_OK, 0)
        C64, _ = gh.oracle_ag(w, chunks, B)
        gh.assert_close(Cg, C64, w.out_dtype)


@pytest.mark.parametrize("name", ["c3_rs", "c4_rs", "op_rs_m64", "op_rs_m2048", "op_rs_m8192"])
def test_rs_full_size_all_elements(name):
    """Full benchmark shape in the launch configuration the benchmark uses (the library's own pick of
    tile, K cut and order); every element of every slice against the oracle."""
    w = W[name]
    rank = 3
    _say(name, "full size: generating inputs")
    A, B, peers = fi.make_rs_inputs(w, rank)
    _say(name, "running")
    outs = gh.run_rs(w, rank, A, B, peers)
    _say(name, "oracle, all", w.M, "rows")
    s64, _ = gh.oracle_rs(w, rank, A, B, peers)
    for r in range(w.R):
        gh.assert_close(outs[r], s64[r], w.out_dtype, f"slice {r}")


@pytest.mark.parametrize("name", ["c2_ag", "c4_ag", "op_ag_m64", "op_ag_m2048", "op_ag_m8192"])
def test_ag_full_size_all_elements(name):
    w = W[name]
    rank = 2
    _say(name, "full size: generating inputs")
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    _say(name, "running, arrival order", arrival)
    Cg, A_agg, signals, status = gh.run_ag(w, rank, chunks, B, arrival)
    assert status == (fb.FLUX_OK, 0)
    _say(name, "oracle, all", w.M, "rows")
    C64, _ = gh.oracle_ag(w, chunks, B)
    gh.assert_close(Cg, C64, w.out_dtype)
    assert torch.equal(A_agg.view(torch.int16).cpu(), torch.cat(chunks).view(torch.int16))


@pytest.mark.parametrize("M", [8, 64, 256])
@pytest.mark.parametrize("op", ["ag", "rs"])
def test_decode_shapes_all_elements(op, M):
    w = W[f"c5_{op}_m{M}"]
    rank = 1
    _say(w.name)
    if op == "rs":
        A, B, peers = fi.make_rs_inputs(w, rank)
        outs = gh.run_rs(w, rank, A, B, peers)
        s64, _ = gh.oracle_rs(w, rank, A, B, peers)
        for r in range(w.R):
            gh.assert_close(outs[r], s64[r], w.out_dtype, f"slice {r}")
    else:
        chunks, B, arrival = fi.make_ag_inputs(w, rank)
        Cg, _, _, status = gh.run_ag(w, rank, chunks, B, arrival)
        assert status == (fb.FLUX_OK, 0)
        C64, _ = gh.oracle_ag(w, chunks, B)
        gh.assert_close(Cg, C64, w.out_dtype)


@pytest.mark.parametrize("split", [2, 3, 7])
def test_split_k_bitwise_on_integers(split):
    w = fi.Workload("int_rs_split", "rs", 64, 512, 1024, 8, a_dist=("int", 2), b_dist=("int", 2),
                    peer_dist=("int", 8), seed=80)
    rank = 4
    A, B, peers = fi.make_rs_inputs(w, rank)
    _, want = gh.oracle_rs(w, rank, A, B, peers)
    dA, dB = A.to(gh.DEV), B.to(gh.DEV)
    dpeers = [None if t is None else t.to(gh.DEV) for t in peers]
    for cfg in (5, 6, 4):
        _say("split-k", split, "cfg", cfg)
        p = fb.problem(w.M, w.N, w.K, w.R, rank, w.partial_dtype, w.out_dtype, cfg, split)
        ws = gh.workspace_for(fb.FLUX_OP_RS, p)
        ws.fill_(-1)
        fb.flux_init_buffers(fb.FLUX_OP_RS, p, ws)
        for rep in range(3):        # later launches reuse the counters the earlier ones put back
            outs = [torch.full((w.S, w.N), float("nan"), dtype=torch.bfloat16, device=gh.DEV) for _ in range(w.R)]
            fb.flux_gemm_rs(p, dA, dB, dpeers, outs, ws)
            torch.cuda.synchronize()
            for r in range(w.R):
                gh.assert_bits_equal(outs[r], want[r], f"rep {rep} slice {r}")


@pytest.mark.parametrize("cfg", ALL_CFGS)
@pytest.mark.parametrize("M", [256, 40])
def test_split_k_hand_over_every_config(cfg, M):
    """The workgroup that arrives last at a K-cut tile reads the parked parts back in batches (several
    parts at once for a small tile, a part in several batches for a large one) and, with a ragged M,
    leaves out the vectors past the last row: every configuration, part counts that are and are
    not multiples of a batch, whole and ragged tiles, bitwise on integer-valued inputs."""
    w = fi.Workload("int_rs_parts", "rs", M, 512, 1152, 8, a_dist=("int", 2), b_dist=("int", 2),
                    peer_dist=("int", 8), seed=81)
    rank = 3
    A, B, peers = fi.make_rs_inputs(w, rank)
    _, want = gh.oracle_rs(w, rank, A, B, peers)
    for split in (2, 5, 9):
        _say("hand-over cfg", cfg, "M", M, "parts", split)
        outs = gh.run_rs(w, rank, A, B, peers, tile_config=cfg, split_k=split)
        for r in range(w.R):
            gh.assert_bits_equal(outs[r], want[r], f"cfg {cfg} parts {split} slice {r}")


@pytest.mark.parametrize("cfg,M,N,K", [(4, 1536, 1536, 1024), (1, 8192, 4608, 512), (3, 4608, 2048, 576)])
def test_tail_split_bitwise_on_integers(cfg, M, N, K):
    """Only the tiles of the partly filled last round are cut along K; the rest are computed whole."""
    R = 8
    wr = fi.Workload("int_rs_tail", "rs", M, N, K, R, a_dist=("int", 2), b_dist=("int", 2), peer_dist=("int", 8), seed=81)
    wa = fi.Workload("int_ag_tail", "ag", M, N, K, R, a_dist=("int", 2), b_dist=("int", 2), seed=82)
    p = fb.problem(M, N, K, R, 0, tile_config=cfg)
    full, cut, k = fb.flux_split_plan(fb.FLUX_OP_RS, p)
    assert full > 0 and cut > 0 and k > 1, (full, cut, k)
    rank = 6
    _say("tail split rs cfg", cfg, (full, cut, k))
    A, B, peers = fi.make_rs_inputs(wr, rank)
    _, want = gh.oracle_rs(wr, rank, A, B, peers)
    p = fb.problem(M, N, K, R, rank, wr.partial_dtype, wr.out_dtype, cfg)
    dA, dB = A.to(gh.DEV), B.to(gh.DEV)
    dpeers = [None if t is None else t.to(gh.DEV) for t in peers]
    ws = gh.workspace_for(fb.FLUX_OP_RS, p)
    ws.fill_(-1)
    fb.flux_init_buffers(fb.FLUX_OP_RS, p, ws)
    for rep in range(2):
        outs = [torch.full((wr.S, N), float("nan"), dtype=torch.bfloat16, device=gh.DEV) for _ in range(R)]
        fb.flux_gemm_rs(p, dA, dB, dpeers, outs, ws)
        torch.cuda.synchronize()
        for r in range(R):
            gh.assert_bits_equal(outs[r], want[r], f"rep {rep} slice {r}")
    _say("tail split ag cfg", cfg)
    chunks, B, arrival = fi.make_ag_inputs(wa, rank)
    Cg, _, signals, status = gh.run_ag(wa, rank, chunks, B, arrival, tile_config=cfg, repeat=2)
    assert status == (fb.FLUX_OK, 0)
    _, want = gh.oracle_ag(wa, chunks, B)
    gh.assert_bits_equal(Cg, want, f"cfg {cfg}")
    # the flag switches the cut off; same bits
    Cn, _, _, status = gh.run_ag(wa, rank, chunks, B, arrival, tile_config=cfg, flags=fb.FLUX_FLAG_NO_TAIL_SPLIT)
    assert status == (fb.FLUX_OK, 0)
    gh.assert_bits_equal(Cn, want, f"cfg {cfg} no tail split")


def test_resident_grid_with_a_k_cut_tail_bitwise_on_integers():
    """Four whole rounds of 256x256 tiles plus 32 tiles cut along K, all walked by 256 resident workgroups:
    a K part that is not its tile's last ends its block early and the workgroup goes on to the next one."""
    M, N, K, R, rank = 8192, 8448, 1024, 8, 5
    w = fi.Workload("int_rs_resident_tail", "rs", M, N, K, R, a_dist=("int", 2), b_dist=("int", 2), peer_dist=("int", 8), seed=83)
    p = fb.problem(M, N, K, R, rank)
    full, cut, k = fb.flux_split_plan(fb.FLUX_OP_RS, p)
    assert (full, cut) == (1024, 32) and k > 1, (full, cut, k)
    assert fb.flux_rs_resident_grid(p)[0] == 256
    _say("resident grid with tail", (full, cut, k))
    A, B, peers = fi.make_rs_inputs(w, rank)
    _, want = gh.oracle_rs(w, rank, A, B, peers)
    dA, dB = A.to(gh.DEV), B.to(gh.DEV)
    dpeers = [None if t is None else t.to(gh.DEV) for t in peers]
    ws = gh.workspace_for(fb.FLUX_OP_RS, p)
    ws.fill_(-1)
    fb.flux_init_buffers(fb.FLUX_OP_RS, p, ws)
    for rep in range(2):
        outs = [torch.full((w.S, N), float("nan"), dtype=torch.bfloat16, device=gh.DEV) for _ in range(R)]
        fb.flux_gemm_rs(p, dA, dB, dpeers, outs, ws)
        torch.cuda.synchronize()
        for r in range(R):
            gh.assert_bits_equal(outs[r], want[r], f"rep {rep} slice {r}")


# ---------------------------------------------------------------------------------------------
# AllGather protocol: orders, signals, copy engines, timing
# ---------------------------------------------------------------------------------------------

AG_SMALL = fi.scaled(W["c2_ag"], M=2048, N=512, K=512)


@pytest.mark.parametrize("order", ["ring", "reversed", "random"])
@pytest.mark.parametrize("flags", [0, fb.FLUX_FLAG_COPY_MEMCPY, fb.FLUX_FLAG_NO_SWIZZLE])
def test_ag_arrival_orders_and_copy_engines(order, flags):
    w = AG_SMALL
    rank = 5
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    if order == "ring":
        arrival = None
    elif order == "reversed":
        arrival = list(reversed(fo.default_order(rank, w.R)))
    _say("ag order", order, "flags", flags)
    C64, _ = gh.oracle_ag(w, chunks, B)
    # copy_workgroups = 0 lets the library choose: for a transfer this small, no copy kernel at all
    # (the waiting workgroups pull the tiles); a number asks for the copy kernel on the copy stream
    for ctpc, cw in ((0, 0), (2, 0), (4, 0), (0, 48), (2, 48), (4, 7)):
        Cg, _, signals, status = gh.run_ag(w, rank, chunks, B, arrival, flags=flags, comm_tiles_per_chunk=ctpc,
                                           tile_config=3, copy_workgroups=cw)
        assert status == (fb.FLUX_OK, 0)
        gh.assert_close(Cg, C64, w.out_dtype, f"ctpc {ctpc} cw {cw}")
        n = max(1, ctpc)
        assert signals.cpu().tolist() == [1 if i // n == rank else 0 for i in range(w.R * n)]


@pytest.mark.parametrize("ctpc", [1, 2])
def test_ag_library_copies_starved_of_compute_units(ctpc):
    """FLUX_FLAG_COPY_MEMCPY on a grid that fills the chip: the first 256 workgroups take every compute
    unit and most of them wait for signals, so the library copies (kernels of their own on this chip)
    cannot start.  A workgroup that has waited 100 us fetches its own rows; the call completes without
    a timeout, with the right result, the gathered matrix complete and the signals preset again."""
    w = fi.Workload("ag_starved", "ag", 4096, 4608, 512, 8, seed=89, a_dist=("int", 2), b_dist=("int", 2))
    rank = 6
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    _say("ag memcpy driver, 288 tiles on 256 compute units, ctpc", ctpc)
    Cg, A_agg, signals, status = gh.run_ag(w, rank, chunks, B, arrival, flags=fb.FLUX_FLAG_COPY_MEMCPY, tile_config=1,
                                           comm_tiles_per_chunk=ctpc, repeat=3)
    assert status == (fb.FLUX_OK, 0)
    C64, Cbits = gh.oracle_ag(w, chunks, B)
    gh.assert_bits_equal(Cg, Cbits, "C")
    gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")
    assert signals.cpu().tolist() == [1 if i // ctpc == rank else 0 for i in range(w.R * ctpc)]


def test_ag_delayed_copy_stream_still_correct():
    """The copy driver starts ~10 ms late (host-forced); every remote tile has to spin."""
    w = AG_SMALL
    rank = 0
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    C64, _ = gh.oracle_ag(w, chunks, B)
    Cg, _, _, status = gh.run_ag(w, rank, chunks, B, arrival, delay_copy_cycles=20_000_000, copy_workgroups=64)
    assert status == (fb.FLUX_OK, 0)
    gh.assert_close(Cg, C64, w.out_dtype)


def test_ag_waiting_workgroups_move_the_data_themselves():
    """The copy driver is held back ~10 ms (host-forced) while a GEMM grid larger than the chip, in
    natural tile order from a non-zero rank, starts with tiles that all have to wait.  The waiting
    workgroups claim and move the pieces themselves: the GEMM kernel is over long before the copy
    driver may even start, and the driver then finds nothing left to do."""
    w = fi.scaled(W["c2_ag"], M=4096, N=2048, K=512)
    rank = 5
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    C64, _ = gh.oracle_ag(w, chunks, B)
    for flags in (fb.FLUX_FLAG_NO_SWIZZLE, 0):
        _say("cooperative copy, flags", flags)
        e0, e1 = fb.HipEvent(), fb.HipEvent()
        fb.flux_profile_next_gemm(e0, e1)
        Cg, A_agg, signals, status = gh.run_ag(w, rank, chunks, B, arrival, tile_config=4, flags=flags,
                                               delay_copy_cycles=20_000_000, copy_workgroups=256)
        assert status == (fb.FLUX_OK, 0)
        gh.assert_close(Cg, C64, w.out_dtype)
        gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")
        assert signals.cpu().tolist() == [1 if c == rank else 0 for c in range(w.R)]
        assert e0.elapsed_ms(e1) < 5.0, "the GEMM kernel waited for the delayed copy driver"


@pytest.mark.parametrize("shape", [dict(M=4096, N=2048, K=512), dict(M=2048, N=1024, K=1024), dict(M=64, N=1024, K=2048)])
@pytest.mark.parametrize("ctpc", [1, 4])
def test_ag_without_copy_kernel(shape, ctpc):
    """The default: no copy kernel, the first workgroups of the GEMM grid share the pieces out by index
    (a grid of several rounds, one that leaves compute units free, a decode shape).  With
    FLUX_FLAG_AG_ABSENT_OWNERS every second piece belongs to a workgroup that never runs, so the
    workgroups that wait for it have to take it over through the claim table.  Two calls in a row:
    the second relies on the counters, claims and signals the first left behind."""
    w = fi.scaled(W["c2_ag"], **shape)
    rank = 6
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    C64, _ = gh.oracle_ag(w, chunks, B)
    for flags in (0, fb.FLUX_FLAG_AG_ABSENT_OWNERS, fb.FLUX_FLAG_AG_ABSENT_OWNERS | fb.FLUX_FLAG_NO_SWIZZLE):
        _say("no copy kernel", shape, "ctpc", ctpc, "flags", flags)
        Cg, A_agg, signals, status = gh.run_ag(w, rank, chunks, B, arrival, flags=flags, comm_tiles_per_chunk=ctpc,
                                               repeat=2)
        assert status == (fb.FLUX_OK, 0)
        gh.assert_close(Cg, C64, w.out_dtype)
        gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")
        assert signals.cpu().tolist() == [1 if i // ctpc == rank else 0 for i in range(w.R * ctpc)]


def test_ag_tile_waiting_for_many_signals():
    """One 256-row tile that waits for 32 signals of 1 MiB communication tiles in 256 pieces each: more
    pieces than one search of a waiting workgroup covers, so its search window has to move on as
    tiles complete.  The copy driver is held back, the waiting workgroups move everything."""
    w = fi.Workload("int_ag_many", "ag", 256, 256, 65536, 2, a_dist=("int", 2), b_dist=("int", 2), seed=85)
    rank = 1
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    _, want = gh.oracle_ag(w, chunks, B)
    for delay, cw in ((20_000_000, 256), (0, 256), (0, 0)):     # copy_workgroups 0: no copy kernel, 64 pieces per owner
        _say("many signals, delay", delay, "copy_workgroups", cw)
        Cg, A_agg, signals, status = gh.run_ag(w, rank, chunks, B, arrival, tile_config=1, comm_tiles_per_chunk=16,
                                               copy_workgroups=cw, delay_copy_cycles=delay, repeat=2)
        assert status == (fb.FLUX_OK, 0)
        gh.assert_bits_equal(Cg, want, "C")
        gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")
        assert signals.cpu().tolist() == [1 if i // 16 == rank else 0 for i in range(32)]


def test_ag_link_paced_copy_driver():
    """Emulated slow link (20 GB/s: each 256 KB chunk is released ~13 us after the previous one):
    tiles really wait for their chunk; results and the signal reset are unaffected."""
    w = AG_SMALL
    rank = 4
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    C64, _ = gh.oracle_ag(w, chunks, B)
    for ctpc, flags in ((1, 0), (4, 0), (2, fb.FLUX_FLAG_NO_SWIZZLE)):
        Cg, _, signals, status = gh.run_ag(w, rank, chunks, B, arrival, comm_tiles_per_chunk=ctpc, flags=flags,
                                           link_gbps=20, repeat=2)
        assert status == (fb.FLUX_OK, 0)
        gh.assert_close(Cg, C64, w.out_dtype, f"ctpc {ctpc} flags {flags}")
        assert signals.cpu().tolist() == [1 if i // ctpc == rank else 0 for i in range(w.R * ctpc)]


def test_ag_local_chunk_in_place():
    w = AG_SMALL
    rank = 6
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    C64, _ = gh.oracle_ag(w, chunks, B)
    Cg, _, _, status = gh.run_ag(w, rank, chunks, B, arrival, local_in_place=True)
    assert status == (fb.FLUX_OK, 0)
    gh.assert_close(Cg, C64, w.out_dtype)


def test_ag_r1_needs_no_copy():
    w = fi.Workload("ag_r1", "ag", 256, 256, 256, 1, seed=81)
    chunks, B, arrival = fi.make_ag_inputs(w, 0)
    assert arrival == []
    Cg, _, signals, status = gh.run_ag(w, 0, chunks, B, None)
    C64, _ = gh.oracle_ag(w, chunks, B)
    gh.assert_close(Cg, C64, w.out_dtype)
    assert signals.cpu().tolist() == [1]


@pytest.mark.parametrize("cw", [0, 16])
def test_ag_gathered_matrix_not_line_aligned(cw):
    """A gathered matrix whose rows do not start on cache line boundaries (base 16 bytes into a
    line): rows of two communication tiles can then share a line, and the wait ends with the
    acquire that also drops stale lines from the die's L2 (the cheaper one is only taken when
    every row starts and ends on a line boundary).  Two calls on the same buffers, the remote
    rows poisoned in between."""
    w = fi.scaled(W["c2_ag"], M=1024, N=512, K=448)
    rank = 5
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    C64, _ = gh.oracle_ag(w, chunks, B)
    for ctpc in (1, 2):
        _say("unaligned gathered matrix, copy workgroups", cw, "ctpc", ctpc)
        Cg, A_agg, _, status = gh.run_ag(w, rank, chunks, B, arrival, copy_workgroups=cw, comm_tiles_per_chunk=ctpc,
                                         repeat=2, agg_offset_elems=8)
        assert status == (fb.FLUX_OK, 0)
        assert A_agg.data_ptr() % 128 == 16
        gh.assert_close(Cg, C64, w.out_dtype)
        want = torch.cat(chunks).view(torch.int16)
        assert torch.equal(A_agg.cpu().view(torch.int16), want)


AG_TWO_ROUNDS = fi.Workload("int_ag_two_rounds", "ag", 8192, 4608, 2048, 8, a_dist=("int", 2), b_dist=("int", 2), seed=84)


@pytest.mark.parametrize("order", ["ring", "random"])
def test_ag_later_chunks_travel_inside_the_main_loops(order):
    """A grid of more than one round moves only the chunks its first round needs before the signal
    wait; the others are carried inside the first round's main loops (Sec. 3.2: compute on what has
    arrived while the rest is on its way).  Same bits as with everything moved up front, and as the
    oracle's; the gathered matrix is complete; the second call finds the state the first one left."""
    w, rank = AG_TWO_ROUNDS, 5
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    if order == "ring":
        arrival = fo.default_order(rank, w.R)
    p = fb.problem(w.M, w.N, w.K, w.R, rank)
    q = fb.problem(w.M, w.N, w.K, w.R, rank, flags=fb.FLUX_FLAG_AG_COPY_UPFRONT)
    assert fb.flux_ag_deferred_tiles(p) == 4 and fb.flux_ag_deferred_tiles(q) == 0
    _say("ag deferred transfer", order, "plan", fb.flux_split_plan(fb.FLUX_OP_AG, p))
    _, want = gh.oracle_ag(w, chunks, B)
    Cd, A_agg, signals, status = gh.run_ag(w, rank, chunks, B, arrival, repeat=2)
    assert status == (fb.FLUX_OK, 0)
    gh.assert_bits_equal(Cd, want, "C, later chunks inside the main loops")
    gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")
    assert signals.tolist() == [1 if r == rank else 0 for r in range(w.R)]
    Cu, A_agg, signals, status = gh.run_ag(w, rank, chunks, B, arrival, flags=fb.FLUX_FLAG_AG_COPY_UPFRONT)
    assert status == (fb.FLUX_OK, 0)
    gh.assert_bits_equal(Cu, want, "C, everything up front")


@pytest.mark.parametrize("R,gbps", [(2, 0), (16, 0), (16, 800), (4, 0)])
def test_ag_carried_transfer_with_other_rank_counts(R, gbps):
    """Two ranks: the first round is all local tiles and the one remote chunk travels inside its main
    loops, nothing is moved up front.  Sixteen ranks: half as many pieces per chunk as the first round
    has workgroups, so half of them carry nothing."""
    w = fi.Workload(f"int_ag_two_rounds_r{R}", "ag", 8192, 4608, 2048, R, a_dist=("int", 2), b_dist=("int", 2), seed=86 + R)
    rank = R - 1
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    p = fb.problem(w.M, w.N, w.K, w.R, rank, link_gbps=gbps)
    deferred = fb.flux_ag_deferred_tiles(p)
    _say("ag carried transfer, ranks", R, "link", gbps, "tiles carried", deferred)
    assert deferred == (R - 1 if gbps else {2: 1, 4: 2, 16: 8}[R])
    _, want = gh.oracle_ag(w, chunks, B)
    Cg, A_agg, signals, status = gh.run_ag(w, rank, chunks, B, arrival, link_gbps=gbps, repeat=2)
    assert status == (fb.FLUX_OK, 0)
    gh.assert_bits_equal(Cg, want, "C")
    gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")
    assert signals.tolist() == [1 if r == rank else 0 for r in range(w.R)]


@pytest.mark.parametrize("shape,ctpc,gbps", [("two_rounds", 1, 400), ("two_rounds", 2, 800), ("one_round", 1, 400)])
def test_ag_link_paced_transfer_carried_by_the_grid(shape, ctpc, gbps):
    """A transfer that stands for a link, without a copy kernel: the first round's workgroups carry every
    remote tile (in batches while they wait, inside their main loops afterwards) and count a tile in
    no earlier than the link would have delivered it.  Bits as the oracle's; the trace shows that no
    tile got past its wait before its communication tile was due."""
    w = AG_TWO_ROUNDS if shape == "two_rounds" else fi.Workload("int_ag_one_round", "ag", 4096, 3584, 1024, 8, a_dist=("int", 2), b_dist=("int", 2), seed=85)
    rank = 6
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    p = fb.problem(w.M, w.N, w.K, w.R, rank, comm_tiles_per_chunk=ctpc, link_gbps=gbps, spin_timeout_ticks=gh.TEST_TIMEOUT_TICKS)
    assert fb.flux_ag_deferred_tiles(p) == (w.R - 1) * ctpc
    _, want = gh.oracle_ag(w, chunks, B)
    Cg, A_agg, signals, status = gh.run_ag(w, rank, chunks, B, arrival, comm_tiles_per_chunk=ctpc, link_gbps=gbps, repeat=2)
    assert status == (fb.FLUX_OK, 0)
    gh.assert_bits_equal(Cg, want, "C")
    gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")
    assert signals.tolist() == [1 if i // ctpc == rank else 0 for i in range(w.R * ctpc)]
    # pacing, from the tile trace of one more call
    full, cut, k = fb.flux_split_plan(fb.FLUX_OP_AG, p)
    grid = full + cut * k
    sh = fb.flux_tile_shape(fb.FLUX_OP_AG, p)
    dchunks = [c.to(gh.DEV) for c in chunks]
    A2 = torch.full((w.M, w.K), float("nan"), dtype=torch.bfloat16, device=gh.DEV)
    C2 = torch.full((w.M, w.N), float("nan"), dtype=torch.bfloat16, device=gh.DEV)
    sig = torch.zeros(w.R * ctpc, dtype=torch.int32, device=gh.DEV)
    ws = gh.workspace_for(fb.FLUX_OP_AG, p)
    fb.flux_init_buffers(fb.FLUX_OP_AG, p, ws, sig)
    trace = torch.zeros((grid, 8), dtype=torch.int64, device=gh.DEV)
    fb.flux_trace_next_call(trace)
    fb.flux_ag_gemm(p, dchunks, A2, B.to(gh.DEV), C2, sig, arrival, ws, torch.cuda.current_stream(), torch.cuda.Stream())
    torch.cuda.synchronize()
    assert fb.flux_query_status(ws) == (fb.FLUX_OK, 0)
    t = trace.cpu().numpy()
    w32 = t.view(np.uint32).reshape(grid, 16)
    m_tile = w32[:, 1].astype(np.int64)
    t_start, t_ready = t[:, 4].astype(np.int64), t[:, 5].astype(np.int64)
    t0 = int(t_start.min())
    tile_bytes = w.S * w.K * 2 // ctpc
    pace = tile_bytes / gbps / 10.0                      # 100 MHz ticks per communication tile
    rows_per_tile = w.S // ctpc
    position = {c: i for i, c in enumerate(arrival)}     # chunk -> place in the transfer order
    checked = 0
    for b in range(grid):
        lo, hi = m_tile[b] * sh.tile_m, (m_tile[b] + 1) * sh.tile_m - 1
        last_due = 0.0
        for f in range(lo // rows_per_tile, hi // rows_per_tile + 1):        # communication tiles the block's rows lie in
            chunk, sub = f // ctpc, f % ctpc
            if chunk != rank:
                last_due = max(last_due, (position[chunk] * ctpc + sub + 1) * pace)
        if last_due > 0:
            assert t_ready[b] - t0 >= last_due - 300, ("block past its wait before its data was due", b, t_ready[b] - t0, last_due)
            checked += 1
    assert checked > 0
    gh.assert_bits_equal(C2, want, "C of the traced call")


@pytest.mark.parametrize("gbps", [0, 50])
def test_ag_carried_pieces_are_moved_whatever_happens_to_the_tiles(gbps):
    """Failure handling forced from the host: with a spin limit of one tick a workgroup that finds a
    signal missing when it gets to its wait gives up at once.  Whether any does depends on timing (a
    workgroup with pieces to carry keeps moving them until its own signals are there, and the later
    rounds start when the first has finished); either way the kernel exits, the status block is
    consistent with the result, and the gathered matrix is complete: the workgroups that carry the
    pieces move all of them and count them in on schedule, whether or not anybody still waits."""
    w, rank = AG_TWO_ROUNDS, 1
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    assert fb.flux_ag_deferred_tiles(fb.problem(w.M, w.N, w.K, w.R, rank, link_gbps=gbps)) == (7 if gbps else 4)
    Cg, A_agg, signals, status = gh.run_ag(w, rank, chunks, B, arrival, timeout_ticks=1, link_gbps=gbps)
    code, detail = status
    _, want = gh.oracle_ag(w, chunks, B)
    gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")
    lo, hi = rank * w.S, (rank + 1) * w.S
    gh.assert_bits_equal(Cg[lo:hi], want[lo:hi], "rows of the local chunk")
    assert code in (fb.FLUX_OK, fb.FLUX_ERR_TIMEOUT)
    if code == fb.FLUX_OK:
        gh.assert_bits_equal(Cg, want, "C")
    else:
        assert 0 <= detail < w.R and detail != rank
    # after flux_init_buffers (run_ag does it) the same problem runs clean
    Cg, _, _, status = gh.run_ag(w, rank, chunks, B, arrival, link_gbps=gbps)
    assert status == (fb.FLUX_OK, 0)
    gh.assert_bits_equal(Cg, want, "C after re-initialisation")


def test_ag_signal_wait_times_out_cleanly():
    """Failure handling, forced from the host: the copy stream is held back and the spin limit
    is one tick, so waiting tiles give up, the kernel still exits, and the status block says
    which signal was missing.  Tiles of the local chunk (preset signal) are still computed.

    Streams share a few hardware queues, and a queue hands out its packets in order: when the copy
    stream shares one with the compute stream, the kernel that holds the copies back holds the GEMM
    back as well, every signal is set by the time it starts and the call succeeds (checked too).
    Consecutive streams go to different queues, so one of the first few must show the timeout."""
    w = AG_SMALL
    rank = 2
    chunks, B, arrival = fi.make_ag_inputs(w, rank)
    C64, _ = gh.oracle_ag(w, chunks, B)
    lo, hi = rank * w.S, (rank + 1) * w.S
    timed_out = False
    for attempt in range(8):
        _say("timeout test, copy stream", attempt)
        Cg, _, signals, status = gh.run_ag(w, rank, chunks, B, arrival, delay_copy_cycles=20_000_000, timeout_ticks=1,
                                           flags=fb.FLUX_FLAG_COPY_MEMCPY,      # plain waiting: nobody else moves the data
                                           copy_stream=torch.cuda.Stream())
        code, detail = status
        if code == fb.FLUX_OK:               # the GEMM was held back with the copies
            assert detail == 0
            gh.assert_close(Cg, C64, w.out_dtype)
            continue
        assert code == fb.FLUX_ERR_TIMEOUT
        assert 0 <= detail < w.R and detail != rank
        gh.assert_close(Cg[lo:hi], C64[lo:hi], w.out_dtype, "local chunk rows")
        timed_out = True
        break
    assert timed_out
    # and the library is usable afterwards
    Cg, _, _, status = gh.run_ag(w, rank, chunks, B, arrival)
    assert status == (fb.FLUX_OK, 0)
    gh.assert_close(Cg, C64, w.out_dtype)


def test_results_are_deterministic():
    w = fi.scaled(W["c3_rs"], M=1024, N=1024, K=512)
    A, B, peers = fi.make_rs_inputs(w, 1)
    for split in (0, 1, 4):          # the K-split sum runs in split order whoever arrives last
        a = gh.run_rs(w, 1, A, B, peers, split_k=split)
        for _ in range(3):
            b = gh.run_rs(w, 1, A, B, peers, split_k=split)
            for x, y in zip(a, b):
                assert torch.equal(x.view(torch.int16), y.view(torch.int16))


# ---------------------------------------------------------------------------------------------
# non-overlapped baseline
# ---------------------------------------------------------------------------------------------

def test_unfused_baseline_matches_oracle():
    w = fi.scaled(W["c3_rs"], M=1024, N=1024, K=768)
    rank = 3
    A, B, peers = fi.make_rs_inputs(w, rank)
    p = fb.problem(w.M, w.N, w.K, w.R, rank, w.partial_dtype, w.out_dtype)
    dA, dB = A.to(gh.DEV), B.to(gh.DEV)
    dpeers = [None if t is None else t.to(gh.DEV) for t in peers]
    outs = [torch.full((w.S, w.N), float("nan"), dtype=torch.bfloat16, device=gh.DEV) for _ in range(w.R)]
    tmp = torch.empty((w.M, w.N), dtype=torch.bfloat16, device=gh.DEV)
    ws = gh.workspace_for(fb.FLUX_OP_RS, p)
    if ws is not None:
        fb.flux_init_buffers(fb.FLUX_OP_RS, p, ws)
    fb.flux_gemm_ref_unfused(fb.FLUX_OP_RS, fb.FLUX_PHASE_GEMM | fb.FLUX_PHASE_COMM, p, A=dA, B=dB,
                             peer_partials=dpeers, out_slices=outs, Cout=tmp, workspace=ws)
    torch.cuda.synchronize()
    s64, _ = gh.oracle_rs(w, rank, A, B, peers)
    for r in range(w.R):
        # the baseline rounds the GEMM result to bf16 before adding: one extra half-ulp
        gh.assert_close(outs[r], s64[r], w.out_dtype, f"slice {r}")

    wa = fi.scaled(W["c2_ag"], M=1024, N=896, K=1024)
    chunks, B, _ = fi.make_ag_inputs(wa, 1)
    pa = fb.problem(wa.M, wa.N, wa.K, wa.R, 1, "bf16", wa.out_dtype)
    A_agg = torch.full((wa.M, wa.K), float("nan"), dtype=torch.bfloat16, device=gh.DEV)
    Cout = torch.full((wa.M, wa.N), float("nan"), dtype=torch.bfloat16, device=gh.DEV)
    wsa = gh.workspace_for(fb.FLUX_OP_AG, pa)
    fb.flux_init_buffers(fb.FLUX_OP_AG, pa, wsa)
    fb.flux_gemm_ref_unfused(fb.FLUX_OP_AG, fb.FLUX_PHASE_GEMM | fb.FLUX_PHASE_COMM, pa,
                             A_chunks=[c.to(gh.DEV) for c in chunks], A_agg=A_agg, B=B.to(gh.DEV), Cout=Cout,
                             workspace=wsa)
    torch.cuda.synchronize()
    C64, _ = gh.oracle_ag(wa, chunks, B)
    gh.assert_close(Cout, C64, wa.out_dtype)


def _chunk_ws(op, p):
    n = fb.flux_chunked_workspace_bytes(op, p)
    if n == 0:
        return None
    ws = torch.full(((n + 3) // 4,), -1, dtype=torch.int32, device=gh.DEV)
    fb.flux_init_buffers(fb.FLUX_OP_RS, p, ws)
    return ws


@pytest.mark.parametrize("R,rank", [(8, 3), (4, 0), (1, 0)])
def test_chunked_baseline_matches_oracle(R, rank):
    """The medium-grained decomposition (one GEMM per slice / chunk, communication of one part beside
    the GEMM of the next on a second stream) gives the same results as the other two paths: on
    integer-valued inputs bit for bit, on random inputs within the tolerance."""
    comm = torch.cuda.Stream()
    compute = torch.cuda.current_stream()
    for ints in (True, False):
        kw = dict(a_dist=("int", 2), b_dist=("int", 2), peer_dist=("int", 8)) if ints else {}
        w = fi.Workload("rs_chunked", "rs", 128 * R, 384, 320, R, seed=86, **kw)
        _say("chunked rs", R, rank, "ints" if ints else "random")
        A, B, peers = fi.make_rs_inputs(w, rank)
        p = fb.problem(w.M, w.N, w.K, w.R, rank, w.partial_dtype, w.out_dtype)
        dA, dB = A.to(gh.DEV), B.to(gh.DEV)
        dpeers = [None if t is None else t.to(gh.DEV) for t in peers]
        ws = _chunk_ws(fb.FLUX_OP_RS, p)
        for rep in range(2):
            outs = [torch.full((w.S, w.N), float("nan"), dtype=torch.bfloat16, device=gh.DEV) for _ in range(w.R)]
            tmp = torch.full((w.M, w.N), float("nan"), dtype=torch.bfloat16, device=gh.DEV)
            fb.flux_gemm_ref_chunked(fb.FLUX_OP_RS, p, A=dA, B=dB, peer_partials=dpeers, out_slices=outs, Cout=tmp,
                                     workspace=ws, compute_stream=compute, comm_stream=comm)
            torch.cuda.synchronize()
            s64, sbits = gh.oracle_rs(w, rank, A, B, peers)
            if ints:
                # this path rounds A.B to bf16 before the peers are added; that extra rounding is exact
                # (and the result bitwise the oracle's) as long as every element of A.B is an integer
                # of magnitude at most 256
                assert np.abs(A.double().numpy() @ B.double().numpy()).max() <= 256
            for r in range(w.R):
                if ints:
                    gh.assert_bits_equal(outs[r], sbits[r], f"slice {r}")
                else:
                    gh.assert_close(outs[r], s64[r], w.out_dtype, f"slice {r}")
        wa = fi.Workload("ag_chunked", "ag", 128 * R, 384, 320, R, seed=87, **kw)
        _say("chunked ag", R, rank)
        chunks, Ba, arrival = fi.make_ag_inputs(wa, rank)
        pa = fb.problem(wa.M, wa.N, wa.K, wa.R, rank, "bf16", wa.out_dtype)
        dchunks = [c.to(gh.DEV) for c in chunks]
        C64, Cbits = gh.oracle_ag(wa, chunks, Ba)
        ws = _chunk_ws(fb.FLUX_OP_AG, pa)
        for rep in range(2):
            A_agg = torch.full((wa.M, wa.K), float("nan"), dtype=torch.bfloat16, device=gh.DEV)
            Cout = torch.full((wa.M, wa.N), float("nan"), dtype=torch.bfloat16, device=gh.DEV)
            fb.flux_gemm_ref_chunked(fb.FLUX_OP_AG, pa, A_chunks=dchunks, A_agg=A_agg, B=Ba.to(gh.DEV), Cout=Cout,
                                     arrival_order=arrival, workspace=ws, compute_stream=compute, comm_stream=comm)
            torch.cuda.synchronize()
            if ints:
                gh.assert_bits_equal(Cout, Cbits, "C")
            else:
                gh.assert_close(Cout, C64, wa.out_dtype)
            gh.assert_bits_equal(A_agg, np.concatenate([fi.to_numpy(c) for c in chunks]), "A_agg")


@pytest.mark.parametrize("cfg", [0, 1, 3, 4, 7])
@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_rs_write_only_then_slice_reduce(cfg, dt):
    """The AlltoAll flavour (Write branch of Alg. 1 + local reduction): every virtual rank scatters its
    own partial product by owner; one owner then sums the R partials staged for its slice.  Integer
    inputs: bit for bit against the oracle at both steps; random inputs: within the tolerance, and
    the reduction bit for bit when both sides start from the same staged values."""
    R, owner = 4, 2
    for ints in (True, False):
        kw = dict(a_dist=("int", 2), b_dist=("int", 2)) if ints else {}
        w = fi.Workload("rs_wo", "rs", 512, 384, 256, R, partial_dtype=dt, out_dtype=dt, seed=88, **kw)
        tdt = torch.bfloat16 if dt == "bf16" else torch.float32
        staged_gpu, staged_ref = [], []
        for j in range(R):
            _say("write-only cfg", cfg, dt, "ints" if ints else "random", "rank", j)
            A, B, _ = fi.make_rs_inputs(w, j)
            p = fb.problem(w.M, w.N, w.K, R, j, dt, dt, tile_config=cfg, flags=fb.FLUX_FLAG_RS_WRITE_ONLY)
            outs = [torch.full((w.S, w.N), float("nan"), dtype=tdt, device=gh.DEV) for _ in range(R)]
            ws = gh.workspace_for(fb.FLUX_OP_RS, p)
            if ws is not None:
                fb.flux_init_buffers(fb.FLUX_OP_RS, p, ws)
            fb.flux_gemm_rs(p, A.to(gh.DEV), B.to(gh.DEV), None, outs, ws)
            torch.cuda.synchronize()
            s64, sbits = fo.gemm_scatter(fi.to_numpy(A), fi.to_numpy(B), R, dt)
            for r in range(R):
                if ints:
                    gh.assert_bits_equal(outs[r], sbits[r], f"rank {j} slice {r}")
                else:
                    gh.assert_close(outs[r], s64[r], dt, f"rank {j} slice {r}")
            staged_gpu.append(outs[owner])
            staged_ref.append(sbits[owner])
        p = fb.problem(w.M, w.N, w.K, R, owner, dt, dt)
        out = torch.full((w.S, w.N), float("nan"), dtype=tdt, device=gh.DEV)
        fb.flux_rs_reduce_slice(p, staged_gpu, out)
        torch.cuda.synchronize()
        total, rounded = fo.reduce_slice([fi.to_numpy(t) for t in staged_gpu], dt, dt)
        gh.assert_close(out, total, dt, "slice reduce")
        if ints:
            gh.assert_bits_equal(out, fo.reduce_slice(staged_ref, dt, dt)[1], "slice reduce, integers")


@pytest.mark.parametrize("shape", [dict(M=1024, N=1024, K=512), dict(M=64, N=1024, K=2048)])
def test_autotune_returns_a_problem_that_still_matches_the_oracle(shape):
    """The tuner times every tile configuration (and, for the AllGather, the communication tile sizes)
    on the caller's buffers; whatever it returns must give the oracle's result, be no slower than the
    library's own pick by its own measurement, and leave workspace and signals ready for use."""
    # GEMM-ReduceScatter
    w = fi.scaled(W["c3_rs"], **shape)
    rank = 4
    A, B, peers = fi.make_rs_inputs(w, rank)
    s64, _ = gh.oracle_rs(w, rank, A, B, peers)
    p = fb.problem(w.M, w.N, w.K, w.R, rank, w.partial_dtype, w.out_dtype)
    dA, dB = A.to(gh.DEV), B.to(gh.DEV)
    dpeers = [None if t is None else t.to(gh.DEV) for t in peers]
    outs = [torch.full((w.S, w.N), float("nan"), dtype=torch.bfloat16, device=gh.DEV) for _ in range(w.R)]
    n = fb.flux_autotune_workspace_bytes(fb.FLUX_OP_RS, p)
    ws = torch.zeros(n // 4 + 1, dtype=torch.int32, device=gh.DEV) if n else None
    _say("autotune rs", shape)
    tuned, best, default = fb.flux_autotune_rs(p, dA, dB, dpeers, outs, ws, reps=3)
    assert 0 < best <= default
    assert 0 <= tuned.tile_config <= fb.lib().flux_tile_config_count()
    for o in outs:
        o.fill_(float("nan"))
    fb.flux_gemm_rs(tuned, dA, dB, dpeers, outs, ws)
    torch.cuda.synchronize()
    for r in range(w.R):
        gh.assert_close(outs[r], s64[r], w.out_dtype, f"slice {r}")
    # AllGather-GEMM
    wa = fi.scaled(W["c2_ag"], **shape)
    chunks, Ba, arrival = fi.make_ag_inputs(wa, rank)
    C64, _ = gh.oracle_ag(wa, chunks, Ba)
    pa = fb.problem(wa.M, wa.N, wa.K, wa.R, rank, "bf16", wa.out_dtype, spin_timeout_ticks=gh.TEST_TIMEOUT_TICKS)
    dchunks = [c.to(gh.DEV) for c in chunks]
    dBa = Ba.to(gh.DEV)
    A_agg = torch.full((wa.M, wa.K), float("nan"), dtype=torch.bfloat16, device=gh.DEV)
    Cout = torch.full((wa.M, wa.N), float("nan"), dtype=torch.bfloat16, device=gh.DEV)
    signals = torch.zeros(fb.flux_autotune_signal_count(pa), dtype=torch.int32, device=gh.DEV)
    wsa = torch.zeros(fb.flux_autotune_workspace_bytes(fb.FLUX_OP_AG, pa) // 4 + 1, dtype=torch.int32, device=gh.DEV)
    copy = torch.cuda.Stream()
    _say("autotune ag", shape)
    tuned_a, best_a, default_a = fb.flux_autotune_ag(pa, dchunks, A_agg, dBa, Cout, signals, arrival, wsa,
                                                     torch.cuda.current_stream(), copy, reps=3)
    assert 0 < best_a <= default_a
    ctpc = max(1, tuned_a.comm_tiles_per_chunk)
    assert signals.cpu().tolist()[:wa.R * ctpc] == [1 if i // ctpc == rank else 0 for i in range(wa.R * ctpc)]
    A_agg.fill_(float("nan"))
    Cout.fill_(float("nan"))
    fb.flux_ag_gemm(tuned_a, dchunks, A_agg, dBa, Cout, signals, arrival, wsa, torch.cuda.current_stream(), copy)
    torch.cuda.synchronize()
    assert fb.flux_query_status(wsa) == (fb.FLUX_OK, 0)
    gh.assert_close(Cout, C64, wa.out_dtype)
    with pytest.raises(fb.FluxError):       # too few signal words for the finest communication tile
        fb.flux_autotune_ag(pa, dchunks, A_agg, dBa, Cout, signals[:wa.R - 1], arrival, wsa,
                            torch.cuda.current_stream(), copy, reps=1)


@pytest.mark.parametrize("cfg", [0, 1, 2, 4, 7])
def test_rs_reduce_by_atomic_additions(cfg):
    """FLUX_FLAG_RS_ATOMIC: the tile is added to the owner's fp32 slice with atomic additions (Sec. 4.2,
    "Reduce", first form).  Integer inputs: bit-exact against the oracle, starting from slices that
    hold other ranks' contributions; a second call adds the product once more; bf16 output is refused."""
    w = fi.Workload("int_rs_atomic", "rs", 1024 if cfg else 64, 512, 320, 8, a_dist=("int", 2), b_dist=("int", 2),
                    peer_dist=("int", 4), partial_dtype="f32", out_dtype="f32", seed=91)
    rank = 6
    _say("atomic reduce cfg", cfg, "M", w.M)
    A, B, peers = fi.make_rs_inputs(w, rank)
    # what the slices hold before the call: the sum of the peers' partials (small integers: exact)
    held = [sum(fi.to_numpy(peers[j])[r * w.S:(r + 1) * w.S] for j in range(w.R) if j != rank).astype(np.float32)
            for r in range(w.R)]
    _, want1 = fo.gemm_reduce_into(fi.to_numpy(A), fi.to_numpy(B), held, w.R)
    _, want2 = fo.gemm_reduce_into(fi.to_numpy(A), fi.to_numpy(B), want1, w.R)
    # the pull form of the Reduce branch gives the same slices
    _, pull = gh.oracle_rs(w, rank, A, B, peers)
    for r in range(w.R):
        assert np.array_equal(want1[r], pull[r])
    p = fb.problem(w.M, w.N, w.K, w.R, rank, "f32", "f32", tile_config=cfg, flags=fb.FLUX_FLAG_RS_ATOMIC)
    dA, dB = A.to(gh.DEV), B.to(gh.DEV)
    outs = [torch.from_numpy(h.copy()).to(gh.DEV) for h in held]
    ws = gh.workspace_for(fb.FLUX_OP_RS, p)
    if ws is not None:
        fb.flux_init_buffers(fb.FLUX_OP_RS, p, ws)
    fb.flux_gemm_rs(p, dA, dB, None, outs, ws)
    torch.cuda.synchronize()
    for r in range(w.R):
        gh.assert_bits_equal(outs[r], want1[r], f"first call, slice {r}")
    fb.flux_gemm_rs(p, dA, dB, None, outs, ws)
    torch.cuda.synchronize()
    for r in range(w.R):
        gh.assert_bits_equal(outs[r], want2[r], f"second call, slice {r}")
    with pytest.raises(fb.FluxError):
        fb.flux_gemm_rs(fb.problem(w.M, w.N, w.K, w.R, rank, "bf16", "bf16", flags=fb.FLUX_FLAG_RS_ATOMIC), dA, dB, None,
                        [o.bfloat16() for o in outs], None)


def test_rs_reduce_by_atomic_additions_random_data():
    w = fi.scaled(W["c3_rs"], M=1024, N=1024, K=768)
    w = fi.Workload(w.name, "rs", w.M, w.N, w.K, w.R, a_dist=w.a_dist, b_dist=w.b_dist, peer_dist=w.peer_dist,
                    partial_dtype="f32", out_dtype="f32", seed=w.seed)
    rank = 3
    A, B, _ = fi.make_rs_inputs(w, rank)
    rng = np.random.default_rng(5)
    held = [rng.standard_normal((w.S, w.N)).astype(np.float32) for _ in range(w.R)]
    s64, _ = fo.gemm_reduce_into(fi.to_numpy(A), fi.to_numpy(B), held, w.R)
    p = fb.problem(w.M, w.N, w.K, w.R, rank, "f32", "f32", flags=fb.FLUX_FLAG_RS_ATOMIC)
    outs = [torch.from_numpy(h.copy()).to(gh.DEV) for h in held]
    fb.flux_gemm_rs(p, A.to(gh.DEV), B.to(gh.DEV), None, outs, gh.workspace_for(fb.FLUX_OP_RS, p))
    torch.cuda.synchronize()
    for r in range(w.R):
        gh.assert_close(outs[r], s64[r], "f32", f"slice {r}")
