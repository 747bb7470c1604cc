"""Pins for the oracle's integer definitions: orders, TileCoord, signals, metric (CPU only)."""
import itertools
import os

import numpy as np
import pytest

from oracle import flux_oracle as fo

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_default_order_matches_printed_example():
    for row in _rows("comm_order_sec4_3.txt"):
        rank, R, want = int(row[0]), int(row[1]), [int(x) for x in row[2:]]
        assert fo.default_order(rank, R) == want
        assert fo.visit_order_ag(rank, R) == [rank] + want
        assert fo.visit_order_rs(rank, R) == want + [rank]


def test_default_order_is_permutation_of_remote_ranks():
    for R in range(1, 10):
        for rank in range(R):
            assert sorted(fo.default_order(rank, R) + [rank]) == list(range(R))


def test_overlap_efficiency_limits():
    for tg, tn, to, want in _rows("overlap_efficiency_sec2_3.txt"):
        assert fo.overlap_efficiency(float(to), float(tn), float(tg)) == pytest.approx(float(want))


def test_flag_and_owner_of_row():
    M, R = 64, 8
    assert [fo.owner_of_row(i, M, R) for i in (0, 7, 8, 63)] == [0, 0, 1, 7]
    assert [fo.flag_of_row(i, M, R) for i in (0, 7, 8, 63)] == [0, 0, 1, 7]
    assert [fo.flag_of_row(i, M, R, 2) for i in (0, 3, 4, 8, 63)] == [0, 0, 1, 2, 15]
    with pytest.raises(ValueError):
        fo.slice_rows(10, 4)


CASES = [
    # (M, N, R, BM, BN)
    (128, 256, 2, 64, 64),       # S multiple of BM
    (4096, 3584, 8, 256, 128),
    (4096, 8192, 8, 256, 256),
    (64, 3584, 8, 64, 256),      # S < BM, one m-tile
    (256, 512, 8, 64, 128),      # S < BM, several m-tiles
    (1000, 520, 8, 64, 64),      # S = 125: neither divides, ragged tail
    (24, 40, 3, 16, 16),
]


@pytest.mark.parametrize("M,N,R,BM,BN", CASES)
@pytest.mark.parametrize("op", ["rs", "ag"])
@pytest.mark.parametrize("n_xcd", [1, 8])
def test_tile_coord_is_a_bijection(M, N, R, BM, BN, op, n_xcd):
    tiles_m, tiles_n = -(-M // BM), -(-N // BN)
    for rank in {0, R // 2, R - 1}:
        arr = None
        if op == "ag":
            rng = np.random.default_rng(rank)
            remote = [c for c in range(R) if c != rank]
            arr = [remote[p] for p in rng.permutation(len(remote))]
        seen = {fo.tile_coord(op, b, M, N, R, rank, BM, BN, arr, n_xcd) for b in range(tiles_m * tiles_n)}
        assert seen == set(itertools.product(range(tiles_m), range(tiles_n)))


@pytest.mark.parametrize("M,N,R,BM,BN", [c for c in CASES if (c[0] // c[2]) % c[3] == 0])
@pytest.mark.parametrize("n_xcd", [1, 8])
def test_order_property_when_tiles_divide_slices(M, N, R, BM, BN, n_xcd):
    """Ascending workgroup ids walk slices (rs) / chunks (ag) in visit order, each for
    g * tiles_n consecutive ids."""
    S = M // R
    g, tiles_n = S // BM, -(-N // BN)
    nblocks = R * g * tiles_n
    for rank in range(R):
        owners = [fo.tile_coord("rs", b, M, N, R, rank, BM, BN, None, n_xcd)[0] * BM // S for b in range(nblocks)]
        want = [r for r in fo.visit_order_rs(rank, R) for _ in range(g * tiles_n)]
        assert owners == want
        arr = list(reversed(fo.default_order(rank, R)))
        chunks = [fo.tile_coord("ag", b, M, N, R, rank, BM, BN, arr, n_xcd)[0] * BM // S for b in range(nblocks)]
        assert chunks == [c for c in [rank] + arr for _ in range(g * tiles_n)]


@pytest.mark.parametrize("M,N,R,BM,BN", [c for c in CASES if (c[0] // c[2]) % c[3] == 0])
def test_rs_ranks_hit_distinct_destinations_at_each_step(M, N, R, BM, BN):
    """The contention-avoidance claim of Sec. 4.1: at the same step index all ranks write to
    pairwise different destination ranks."""
    S = M // R
    nblocks = (M // BM) * -(-N // BN)
    for b in range(nblocks):
        dests = [fo.tile_coord("rs", b, M, N, R, rank, BM, BN)[0] * BM // S for rank in range(R)]
        assert len(set(dests)) == R


def test_rs_last_slice_is_own_and_first_is_next_rank():
    M, N, R, BM, BN = 4096, 8192, 8, 256, 256
    for rank in range(R):
        order = fo.m_tile_order("rs", M, R, rank, BM)
        assert order[0] * BM // (M // R) == (rank + 1) % R
        assert order[-1] * BM // (M // R) == rank


def test_rs_order_is_a_rotation_for_any_tile_height():
    for M, R, BM in [(1000, 8, 64), (256, 8, 64), (64, 8, 64), (24, 3, 16), (96, 4, 32)]:
        tiles_m = -(-M // BM)
        for rank in range(R):
            order = fo.m_tile_order("rs", M, R, rank, BM)
            t0 = order[0]
            assert order == [(t0 + i) % tiles_m for i in range(tiles_m)]


def test_ag_ragged_order_never_precedes_arrival():
    """A tile spanning several chunks is scheduled no earlier than any tile that needs only a
    subset of earlier-arriving chunks: keys are non-decreasing along the order."""
    M, R, BM = 1000, 8, 64
    S = M // R
    for rank in range(R):
        arr = list(reversed(fo.default_order(rank, R)))
        pos = {c: p for p, c in enumerate([rank] + arr)}
        order = fo.m_tile_order("ag", M, R, rank, BM, arr)
        keys = [max(pos[c] for c in range(t * BM // S, (min(M, t * BM + BM) - 1) // S + 1)) for t in order]
        assert keys == sorted(keys)
        assert sorted(order) == list(range(-(-M // BM)))


def test_xcd_remap_gives_each_die_a_contiguous_run():
    M, N, R, BM, BN, X = 4096, 3584, 8, 256, 128, 8
    gb, tiles_n = (M // R) // BM, N // BN
    band = gb * tiles_n
    assert band % X == 0
    rank = 3
    plain = [fo.tile_coord("ag", b, M, N, R, rank, BM, BN, None, 1) for b in range(band)]
    for die in range(X):
        mine = [fo.tile_coord("ag", b, M, N, R, rank, BM, BN, None, X) for b in range(die, band, X)]
        assert mine == plain[die * (band // X):(die + 1) * (band // X)]


def test_protocol_replay_waits_only_when_copy_lags():
    rng = np.random.default_rng(3)
    S, K, N, R, rank = 4, 6, 8, 4, 2
    to_bits = lambda a: fo.f64_to_bf16_bits(a)
    chunks = [to_bits(rng.integers(-3, 4, (S, K)).astype(np.float64)) for _ in range(R)]
    B = to_bits(rng.integers(-3, 4, (K, N)).astype(np.float64))
    want, _ = fo.ag_gemm(chunks, B, "f32")
    arr = [0, 3, 1]
    tiles_per_chunk = (S // 2) * (N // 4)
    # copy keeps pace with the tile order: nobody waits, nothing poisoned is read
    C, waits = fo.simulate_ag_protocol(chunks, B, rank, 2, 4, arr, tiles_per_step=tiles_per_chunk)
    assert waits == 0 and np.array_equal(C, want)
    # copy never advances by itself: the first tile of every remote chunk has to wait
    C, waits = fo.simulate_ag_protocol(chunks, B, rank, 2, 4, arr, tiles_per_step=None)
    assert waits == R - 1 and np.array_equal(C, want)
    # tile order NOT aligned with arrival (kernel told the default order, driver uses arr):
    # still correct, because WaitSignal blocks
    with pytest.raises(ValueError):
        fo.visit_order_ag(rank, R, [0, 1])


@pytest.mark.parametrize("R", [2, 3, 5, 8])
def test_protocol_replay_wait_counts_have_a_closed_form(R):
    """Alg. 2 + Alg. 3 replayed with a driver that delivers a chunk of its own accord every `mult`
    bands of tiles (a band = the tiles of one chunk, visited in arrival order, Sec. 4.1): the first
    tile of band j finds its signal unset exactly when j is not a multiple of `mult` (the chunks
    before it were forced in by the bands before, the driver's own step comes only at multiples), so
    the number of waiting tiles is #{1 <= j < R : j mod mult != 0}.  Whatever the pace and the
    arrival order, the result is the plain gathered GEMM and no poisoned row is ever read."""
    rng = np.random.default_rng(50 + R)
    S, K, N, BM, BN = 4, 6, 8, 2, 4
    band = (S // BM) * (N // BN)
    to_bits = lambda a: fo.f64_to_bf16_bits(a)
    chunks = [to_bits(rng.integers(-3, 4, (S, K)).astype(np.float64)) for _ in range(R)]
    B = to_bits(rng.integers(-3, 4, (K, N)).astype(np.float64))
    want, _ = fo.ag_gemm(chunks, B, "f32")
    for rank in range(R):
        orders = [None, list(reversed(fo.default_order(rank, R)))]
        for order in orders:
            for mult in (1, 2, 3):
                C, waits = fo.simulate_ag_protocol(chunks, B, rank, BM, BN, order, tiles_per_step=mult * band)
                assert np.array_equal(C, want)
                assert waits == sum(1 for j in range(1, R) if j % mult != 0)


@pytest.mark.parametrize("ctpc", [1, 2, 4, 8])
@pytest.mark.parametrize("n_xcd", [1, 8])
def test_ag_bands_follow_the_communication_tile(ctpc, n_xcd):
    """Sec. 4.3 + 4.1: with several signals per chunk the tiles are still a bijection, ascending
    workgroup ids never ask for a communication tile that is transferred later than one asked for
    before, and where whole tiles make up a communication tile a band holds the m-tiles of exactly
    one of them (they wait for the same signal and are dispatched together)."""
    M, N, R, rank, BM, BN = 8192, 4608, 8, 2, 256, 256
    arr = [0, 6, 3, 1, 5, 7, 4]
    tiles_m, tiles_n = M // BM, N // BN
    coords = [fo.tile_coord("ag", b, M, N, R, rank, BM, BN, arr, n_xcd, ctpc) for b in range(tiles_m * tiles_n)]
    assert set(coords) == set(itertools.product(range(tiles_m), range(tiles_n)))
    S = M // R
    rows_per_signal = S // ctpc
    visit = fo.visit_order_ag(rank, R, arr)
    # transfer position of the communication tile that holds the tile's last row
    def position(mt):
        last = (mt + 1) * BM - 1
        return visit.index(last // S) * ctpc + (last % S) // rows_per_signal
    pos = [position(mt) for mt, _ in coords]
    gb = fo.band_height(M, R, BM, ctpc)
    band_sz = gb * tiles_n
    per_band = [pos[i:i + band_sz] for i in range(0, len(pos), band_sz)]
    assert all(max(a) <= min(b) for a, b in zip(per_band, per_band[1:]))
    if rows_per_signal % BM == 0:
        assert gb == rows_per_signal // BM
        assert all(len(set(band)) == 1 for band in per_band)
    else:
        assert gb == S // BM           # a tile spans several communication tiles: bands stay per chunk
