"""CPU-only checks of the C-ABI library: it loads, exports what include/flux.h declares, rejects
bad arguments before enqueuing anything, and its TileCoord agrees with the oracle's."""
import os
import re

import numpy as np
import pytest

from oracle import flux_oracle as fo
from paper_2406_06858_amd import binding as fb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_loads_and_exports_every_declared_symbol():
    L = fb.lib()
    header = open(os.path.join(ROOT, "include", "flux.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(flux_[a-z0-9_]+)\s*\(", header))
    assert declared == set(fb.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name
    assert fb.flux_version() >= 1


def test_problem_struct_layout_matches_header():
    # 14 int32/uint32 fields, one uint64, three int64 row pitches, two int32, naturally aligned
    import ctypes
    assert ctypes.sizeof(fb.flux_problem_t) == 96
    assert fb.flux_problem_t.b_is_nk.offset == 88
    assert fb.flux_problem_t.spin_timeout_ticks.offset == 56
    assert (fb.flux_problem_t.lda.offset, fb.flux_problem_t.ldb.offset, fb.flux_problem_t.ldc.offset) == (64, 72, 80)


def test_status_strings():
    L = fb.lib()
    assert L.flux_status_string(0) == b"ok"
    assert b"timed out" in L.flux_status_string(fb.FLUX_ERR_TIMEOUT)


def test_default_order_matches_oracle():
    for R in range(1, 9):
        for rank in range(R):
            assert fb.flux_default_order(rank, R) == fo.default_order(rank, R)


@pytest.mark.parametrize("bad,status", [
    (dict(M=100, R=8), fb.FLUX_ERR_SHAPE),          # M % R != 0
    (dict(N=100), fb.FLUX_ERR_SHAPE),               # N % 8 != 0
    (dict(K=100), fb.FLUX_ERR_SHAPE),
    (dict(M=0), fb.FLUX_ERR_SHAPE),
    (dict(R=17), fb.FLUX_ERR_SHAPE),
    (dict(rank=8), fb.FLUX_ERR_INVALID_ARG),
    (dict(out_dtype=7), fb.FLUX_ERR_INVALID_ARG),
    (dict(tile_config=99), fb.FLUX_ERR_INVALID_ARG),
])
def test_invalid_problems_are_rejected(bad, status):
    kw = dict(M=128, N=256, K=256, R=8, rank=0)
    kw.update(bad)
    out_dtype = kw.pop("out_dtype", None)
    p = fb.problem(**kw)
    if out_dtype is not None:
        p.out_dtype = out_dtype
    with pytest.raises(fb.FluxError) as e:
        fb.flux_tile_shape(fb.FLUX_OP_RS, p)
    assert e.value.status == status
    assert fb.flux_workspace_bytes(fb.FLUX_OP_RS, p) == 0


def test_null_pointers_are_rejected_before_any_enqueue():
    import ctypes as C
    p = fb.problem(128, 256, 256, 2, 0)
    L = fb.lib()
    null_list = (C.c_void_p * 2)()
    assert L.flux_gemm_rs(C.byref(p), None, None, null_list, null_list, None, 0, None) == fb.FLUX_ERR_INVALID_ARG
    assert L.flux_ag_gemm(C.byref(p), null_list, None, None, None, None, None, None, 0, None, None) == fb.FLUX_ERR_INVALID_ARG
    # misaligned base pointer
    assert L.flux_gemm_rs(C.byref(p), 8, 16, null_list, null_list, None, 0, None) == fb.FLUX_ERR_INVALID_ARG


def test_bad_arrival_order_is_rejected():
    p = fb.problem(128, 256, 256, 4, 1)
    for arr in ([0, 2, 2], [0, 1, 3], [0, 2, 5]):
        with pytest.raises(fb.FluxError) as e:
            fb.flux_tile_coord(fb.FLUX_OP_AG, p, arr, 0)
        assert e.value.status == fb.FLUX_ERR_INVALID_ARG


def test_comm_tiles_must_divide_chunk():
    p = fb.problem(128, 256, 256, 4, 1, comm_tiles_per_chunk=5)
    with pytest.raises(fb.FluxError) as e:
        fb.flux_tile_shape(fb.FLUX_OP_AG, p)
    assert e.value.status == fb.FLUX_ERR_SHAPE


def _all_configs():
    return [(i,) + fb.flux_tile_config_info(i) for i in range(1, fb.flux_tile_config_count() + 1)]


SHAPES = [
    # (M, N, R)
    (128, 256, 2), (4096, 3584, 8), (4096, 8192, 8), (64, 3584, 8), (8, 8192, 8), (256, 3584, 8),
    (1000, 520, 8), (96, 40, 3), (8192, 4608, 8),
]


@pytest.mark.parametrize("M,N,R", SHAPES)
@pytest.mark.parametrize("op", ["rs", "ag"])
def test_tile_coord_matches_oracle(M, N, R, op):
    """The library's TileCoord and the oracle's are written independently; they must agree on
    every workgroup id, for every tile configuration, rank and swizzle flag."""
    opc = fb.FLUX_OP_RS if op == "rs" else fb.FLUX_OP_AG
    for cfg, bm, bn, _ in _all_configs():
        tiles = -(-M // bm) * -(-N // bn)
        step = max(1, tiles // 97)
        for rank in sorted({0, R // 2, R - 1}):
            arr = None
            if op == "ag":
                rng = np.random.default_rng(1000 * rank + M)
                remote = [c for c in range(R) if c != rank]
                arr = [remote[i] for i in rng.permutation(len(remote))]
            for flags, n_xcd in ((0, 8), (fb.FLUX_FLAG_NO_XCD_REMAP, 1)):
                p = fb.problem(M, N, 256, R, rank, tile_config=cfg, flags=flags)
                shape = fb.flux_tile_shape(opc, p)
                assert (shape.tile_m, shape.tile_n, shape.n_xcd) == (bm, bn, n_xcd)
                for b in list(range(0, tiles, step)) + [tiles - 1]:
                    got = fb.flux_tile_coord(opc, p, arr, b)
                    want = fo.tile_coord(op, b, M, N, R, rank, bm, bn, arr, n_xcd)
                    assert got == want, (cfg, rank, flags, b)


def test_tile_coord_bands_follow_the_communication_tile():
    """With several signals per chunk (Sec. 4.3) a band is the set of m-tiles that wait for the same
    signal: library and oracle agree for every workgroup, and the m-tiles of a band all lie in
    one communication tile."""
    M, N, R, rank = 8192, 4608, 8, 2
    arr = [0, 6, 3, 1, 5, 7, 4]
    for cfg, ctpc in ((1, 1), (1, 2), (1, 4), (2, 4), (3, 8), (1, 8)):
        p = fb.problem(M, N, 256, R, rank, tile_config=cfg, comm_tiles_per_chunk=ctpc)
        sh = fb.flux_tile_shape(fb.FLUX_OP_AG, p)
        tiles_n = N // sh.tile_n
        tiles = (M // sh.tile_m) * tiles_n
        gb = fo.band_height(M, R, sh.tile_m, ctpc)
        rows_per_signal = M // R // ctpc
        assert gb == (rows_per_signal // sh.tile_m if rows_per_signal % sh.tile_m == 0 else M // R // sh.tile_m)
        for b in range(0, tiles, 7):
            got = fb.flux_tile_coord(fb.FLUX_OP_AG, p, arr, b)
            assert got == fo.tile_coord("ag", b, M, N, R, rank, sh.tile_m, sh.tile_n, arr, sh.n_xcd, ctpc), (cfg, ctpc, b)
        if rows_per_signal % sh.tile_m == 0:
            for band in range(0, tiles // (gb * tiles_n), 3):
                sig = {fb.flux_tile_coord(fb.FLUX_OP_AG, p, arr, band * gb * tiles_n + q)[0] * sh.tile_m // rows_per_signal
                       for q in range(gb * tiles_n)}
                assert len(sig) == 1


def test_no_swizzle_flag_gives_natural_order():
    M, N, R, rank = 4096, 3584, 8, 3
    p = fb.problem(M, N, 256, R, rank, tile_config=1, flags=fb.FLUX_FLAG_NO_SWIZZLE)
    tiles_n = N // 256
    for b in (0, 1, tiles_n, 5 * tiles_n + 3):
        assert fb.flux_tile_coord(fb.FLUX_OP_RS, p, None, b) == (b // tiles_n, b % tiles_n)


def test_workspace_bytes():
    p = fb.problem(4096, 8192, 3584, 8, 0)
    assert fb.flux_workspace_bytes(fb.FLUX_OP_RS, p) == 0          # no K split: nothing needed
    assert fb.flux_workspace_bytes(fb.FLUX_OP_AG, p) > 0           # status + counters
    d = fb.problem(64, 8192, 3584, 8, 0, split_k=4)
    shape = fb.flux_tile_shape(fb.FLUX_OP_RS, d)
    assert shape.split_k == 4
    tiles = -(-64 // shape.tile_m) * (8192 // shape.tile_n)
    assert fb.flux_workspace_bytes(fb.FLUX_OP_RS, d) >= 4 * tiles * shape.tile_m * shape.tile_n * 4


def test_split_plan_cuts_only_a_partly_filled_last_round():
    # 32 x 18 tiles of 256x256 on 256 CUs: two full rounds, then 64 tiles -> those are cut 4 ways
    p = fb.problem(8192, 4608, 12288, 8, 0)
    for op in (fb.FLUX_OP_RS, fb.FLUX_OP_AG):
        full, cut, k = fb.flux_split_plan(op, p)
        assert (full, cut, k) == (512, 64, 4)
        shape = fb.flux_tile_shape(op, p)
        assert (shape.tile_m, shape.tile_n, shape.split_k) == (256, 256, 4)
        assert fb.flux_workspace_bytes(op, p) >= 4 * 64 * 256 * 256 * 4
    # switched off by flag, and an explicit split_k is a uniform one
    q = fb.problem(8192, 4608, 12288, 8, 0, tile_config=1, flags=fb.FLUX_FLAG_NO_TAIL_SPLIT)
    assert fb.flux_split_plan(fb.FLUX_OP_AG, q) == (0, 576, 1)
    assert fb.flux_workspace_bytes(fb.FLUX_OP_RS, q) == 0
    u = fb.problem(8192, 4608, 12288, 8, 0, tile_config=1, split_k=2)
    assert fb.flux_split_plan(fb.FLUX_OP_AG, u) == (0, 576, 2)
    # a last round that is more than half full, or a grid of exactly whole rounds, is left alone
    assert fb.flux_split_plan(fb.FLUX_OP_RS, fb.problem(8192, 6144, 12288, 8, 0, tile_config=1)) == (0, 768, 1)
    assert fb.flux_split_plan(fb.FLUX_OP_RS, fb.problem(8192, 5632, 12288, 8, 0, tile_config=1))[2] == 1   # 704 = 2.75 rounds
    # short K: every part keeps at least four K slabs
    assert fb.flux_split_plan(fb.FLUX_OP_RS, fb.problem(8192, 4608, 512, 8, 0, tile_config=1)) == (512, 64, 2)
    assert fb.flux_split_plan(fb.FLUX_OP_RS, fb.problem(8192, 4608, 256, 8, 0, tile_config=1)) == (0, 576, 1)


def test_tile_choice_follows_how_well_the_grid_fills_the_chip():
    """The library picks among the 256x256, 256x128 and 128x128 tiles by estimated time: the largest
    tile where its grid fills the chip round by round, a smaller one where that leaves units idle."""
    def tile(M, N, K):
        s = fb.flux_tile_shape(fb.FLUX_OP_AG, fb.problem(M, N, K, 8, 0))
        return (s.tile_m, s.tile_n)
    assert tile(4096, 3584, 8192) == (256, 256)      # 224 tiles, one round
    assert tile(4096, 8192, 3584) == (256, 256)      # 512 tiles, two rounds
    assert tile(8192, 6144, 12288) == (256, 256)     # 768 tiles, three rounds
    assert tile(8192, 4608, 12288) == (256, 256)     # 2.25 rounds, the last one cut along K
    assert tile(2048, 6144, 12288) == (256, 128)     # 192 tiles of 256x256 would leave a quarter of the chip idle
    assert tile(1024, 8192, 3584) == (256, 128)      # 128 tiles of 256x256: half the chip
    assert tile(2048, 8192, 3584) == (256, 256)      # exactly one round
    assert tile(512, 6144, 12288)[0] in (128, 256) and tile(512, 6144, 12288) != (256, 256)
    # one m-tile of 256 rows over a long K whose 256x128 tiles would need more than five K parts to
    # fill the chip: 64x128 tiles, two workgroups per CU, K cut so that every slot has a part
    assert tile(256, 3584, 8192) == (64, 128)
    assert fb.flux_split_plan(fb.FLUX_OP_AG, fb.problem(256, 3584, 8192, 8, 0)) == (0, 112, 4)
    # ... five parts or fewer: 256x128, the weights read once
    assert tile(256, 12288, 6144) == (256, 128)
    assert fb.flux_split_plan(fb.FLUX_OP_AG, fb.problem(256, 6144, 12288, 8, 0)) == (0, 48, 5)
    assert tile(256, 8192, 3584) == (64, 128)          # short K: no
    assert tile(512, 3584, 8192) == (256, 128)         # more rows: the estimate decides
    # 64 rows: 64x64 tiles on six stages, or 64x128 on four where at most five K parts fill the chip
    assert tile(64, 3584, 8192) == (64, 64)
    assert fb.flux_split_plan(fb.FLUX_OP_AG, fb.problem(64, 6144, 12288, 8, 0)) == (0, 48, 5)
    assert tile(64, 12288, 6144) == (64, 128)
    # two m-tiles, long K, few columns: the two-per-CU tile with a finer K cut
    assert fb.flux_split_plan(fb.FLUX_OP_AG, fb.problem(128, 6144, 12288, 8, 0)) == (0, 96, 5)
    assert fb.flux_split_plan(fb.FLUX_OP_AG, fb.problem(128, 3584, 8192, 8, 0)) == (0, 56, 4)     # 64x128 on four stages, one per CU


def test_autotune_sizes_cover_every_candidate():
    """Host side of the tuner: the workspace it asks for holds every candidate's, the signal count
    covers the finest communication tile (chunk height halved down to the tile height, at most 8)."""
    p = fb.problem(8192, 4608, 12288, 8, 2)
    need = fb.flux_autotune_workspace_bytes(fb.FLUX_OP_AG, p)
    for cfg in range(1, fb.lib().flux_tile_config_count() + 1):
        for ctpc in (1, 2, 4):
            q = fb.problem(8192, 4608, 12288, 8, 2, tile_config=cfg, comm_tiles_per_chunk=ctpc)
            if q.M // q.R // ctpc < fb.flux_tile_shape(fb.FLUX_OP_AG, q).tile_m:
                continue
            assert fb.flux_workspace_bytes(fb.FLUX_OP_AG, q) <= need
    # chunk = 1024 rows; 32-row tiles allow 8 communication tiles per chunk, the cap
    assert fb.flux_autotune_signal_count(p) == 8 * 8
    # decode: the chunk (8 rows) is below every tile height, one signal per chunk
    assert fb.flux_autotune_signal_count(fb.problem(64, 3584, 8192, 8, 2)) == 8
    assert fb.flux_autotune_workspace_bytes(fb.FLUX_OP_RS, fb.problem(64, 8192, 3584, 8, 2)) >= \
        fb.flux_workspace_bytes(fb.FLUX_OP_RS, fb.problem(64, 8192, 3584, 8, 2))


def test_offsets_stay_in_32_bits_at_the_edges_of_validation():
    """The kernels address A and B through unsigned 32-bit byte offsets and a tile of partials through a
    signed 31-bit one: validation admits only shapes for which that holds."""
    ok = fb.problem(16384, 65536, 65536, 8, 0)                 # M*K = M*N = 2^30, K*N = 2^32: too many
    with pytest.raises(fb.FluxError) as e:
        fb.flux_tile_shape(fb.FLUX_OP_RS, ok)
    assert e.value.status == fb.FLUX_ERR_SHAPE
    # largest admitted element counts: 2^31 - 2^15 elements per matrix -> byte offsets below 2^32
    p = fb.problem(32768, 65528, 65528, 8, 0)
    assert 32768 * 65528 < 2 ** 31 and 65528 * 65528 >= 2 ** 31
    with pytest.raises(fb.FluxError):
        fb.flux_tile_shape(fb.FLUX_OP_RS, p)
    q = fb.problem(32768, 65528, 32768, 8, 0)
    assert (q.M * q.K) * 2 < 2 ** 32 and (q.K * q.N) * 2 < 2 ** 32
    assert fb.flux_tile_shape(fb.FLUX_OP_RS, q).tile_m == 256
    # a tile of 256 rows of fp32 partials: 256 * N * 4 bytes must stay below 2^31
    wide = fb.problem(8, 1 << 21, 8, 8, 0)
    with pytest.raises(fb.FluxError) as e:
        fb.flux_tile_shape(fb.FLUX_OP_RS, wide)
    assert e.value.status == fb.FLUX_ERR_SHAPE
    assert fb.flux_tile_shape(fb.FLUX_OP_RS, fb.problem(8, (1 << 21) - 8, 8, 8, 0)).tile_n > 0
    assert 256 * ((1 << 21) - 8) * 4 < 2 ** 31


@pytest.mark.parametrize("bad,status", [
    (dict(lda=248), fb.FLUX_ERR_SHAPE),              # shorter than a row
    (dict(ldb=260), fb.FLUX_ERR_SHAPE),              # rows would lose their 16-byte alignment
    (dict(ldc=250), fb.FLUX_ERR_SHAPE),
    (dict(lda=-8), fb.FLUX_ERR_INVALID_ARG),
    (dict(ldc=1 << 21), fb.FLUX_ERR_SHAPE),          # a tile of the slice would pass 2^31 bytes
    (dict(lda=1 << 25), fb.FLUX_ERR_SHAPE),          # the last element's index would pass 2^31
    (dict(b_is_nk=2), fb.FLUX_ERR_INVALID_ARG),
    (dict(b_is_nk=1, ldb=256), fb.FLUX_ERR_SHAPE),   # rows of B as [N,K] hold K = 512 values
])
def test_row_pitches_are_validated(bad, status):
    p = fb.problem(128, 256, 512 if "b_is_nk" in bad else 256, 8, 0, **bad)
    with pytest.raises(fb.FluxError) as e:
        fb.flux_tile_shape(fb.FLUX_OP_RS, p)
    assert e.value.status == status
    assert fb.flux_tile_shape(fb.FLUX_OP_RS, fb.problem(128, 256, 512, 8, 0, b_is_nk=1, ldb=512)).tile_m > 0


def test_row_pitches_in_planning():
    """A pitch equal to the row length is the packed layout; a gathered matrix with a longer pitch is
    moved before the signal wait (its communication tiles are not single runs of memory)."""
    packed = fb.problem(8192, 4608, 2048, 8, 1)
    same = fb.problem(8192, 4608, 2048, 8, 1, lda=2048, ldb=4608, ldc=4608)
    assert fb.flux_ag_deferred_tiles(packed) == fb.flux_ag_deferred_tiles(same) > 0
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 2048, 8, 1, lda=2048 + 64)) == 0
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 2048, 8, 1, lda=2048 + 64, link_gbps=400)) == 0
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 2048, 8, 1, ldb=4608 + 64, ldc=4608 + 8)) > 0
    # the largest pitch that keeps the last element's index below 2^31
    assert fb.flux_tile_shape(fb.FLUX_OP_RS, fb.problem(128, 256, 256, 8, 0, lda=(2 ** 31 - 256) // 127 // 8 * 8)).tile_m > 0


def test_trace_request_arguments():
    import ctypes as C
    L = fb.lib()
    assert L.flux_trace_next_call(None, 0) == fb.FLUX_OK                      # cancels
    assert L.flux_trace_next_call(8, 4096) == fb.FLUX_ERR_INVALID_ARG         # misaligned
    assert L.flux_trace_next_call(4096, 32) == fb.FLUX_ERR_INVALID_ARG        # not even one record
    assert fb.TRACE_RECORD_BYTES == 64
    # a pending request does not survive a call that is rejected for its own reasons ...
    assert L.flux_trace_next_call(4096, 1 << 20) == fb.FLUX_OK
    assert L.flux_trace_next_call(None, 0) == fb.FLUX_OK


def test_resident_grid_is_planned_for_many_short_reduce_scatter_tiles():
    """flux_rs_resident_grid: four rounds or more of 256x256 tiles with K <= 3072 and the Reduce epilogue."""
    c4 = fb.problem(8192, 12288, 1536, 8, 2)
    n, d = fb.flux_rs_resident_grid(c4)
    assert n == 256 and 3000 <= d <= 3800                       # half of (36 us main loop + 32 us epilogue)
    assert fb.flux_rs_resident_grid(fb.problem(8192, 12288, 1536, 8, 2, flags=fb.FLUX_FLAG_NO_RESIDENT_GRID)) == (0, 0)
    assert fb.flux_rs_resident_grid(fb.problem(8192, 12288, 1536, 8, 2, flags=fb.FLUX_FLAG_RS_WRITE_ONLY)) == (0, 0)
    assert fb.flux_rs_resident_grid(fb.problem(4096, 8192, 3584, 8, 2)) == (0, 0)       # two rounds, long K
    assert fb.flux_rs_resident_grid(fb.problem(8192, 12288, 6144, 8, 2)) == (0, 0)      # long K
    assert fb.flux_rs_resident_grid(fb.problem(8192, 12288, 1536, 8, 2, tile_config=2)) == (0, 0)
    assert fb.flux_rs_resident_grid(fb.problem(8192 + 8, 12288, 1536, 8, 2)) == (0, 0)  # ragged: other kernel
    # the blocks and their order do not depend on the form
    assert fb.flux_split_plan(fb.FLUX_OP_RS, c4) == fb.flux_split_plan(
        fb.FLUX_OP_RS, fb.problem(8192, 12288, 1536, 8, 2, flags=fb.FLUX_FLAG_NO_RESIDENT_GRID))


def test_deferred_transfer_is_planned_for_grids_of_several_rounds():
    """flux_ag_deferred_tiles: the chunks the first round of workgroups does not touch, when every condition holds."""
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 12288, 8, 2)) == 4        # 2.25 rounds; the first covers 4 bands of 72 tiles
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 6144, 12288, 8, 2)) == 5        # three rounds, bands of 96 tiles
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 12288, 8, 2, flags=fb.FLUX_FLAG_AG_COPY_UPFRONT)) == 0
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 12288, 8, 2, flags=fb.FLUX_FLAG_NO_SWIZZLE)) == 0
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 12288, 8, 2, comm_tiles_per_chunk=2)) == 0
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 12288, 8, 2, copy_workgroups=16)) == 0   # a copy kernel moves the data
    # a transfer that stands for a link and has no driver of its own is carried whole, on the link's schedule
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 12288, 8, 2, link_gbps=400)) == 7
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 12288, 8, 2, link_gbps=400, comm_tiles_per_chunk=4)) == 28
    assert fb.flux_ag_deferred_tiles(fb.problem(4096, 3584, 8192, 8, 2, link_gbps=400)) == 7
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 12288, 8, 2, link_gbps=400, copy_workgroups=20)) == 0
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 12288, 8, 2, link_gbps=400, flags=fb.FLUX_FLAG_COPY_MEMCPY)) == 0
    assert fb.flux_ag_deferred_tiles(fb.problem(4096, 3584, 8192, 8, 2)) == 0         # one round: every chunk is needed at once
    assert fb.flux_ag_deferred_tiles(fb.problem(2048, 6144, 12288, 8, 2)) == 0        # the first round touches every chunk
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 512, 8, 2)) == 0          # K too short to carry the vectors
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 12288, 8, 2, tile_config=2)) == 0   # other kernel
    assert fb.flux_ag_deferred_tiles(fb.problem(8192, 4608, 12288, 1, 0)) == 0
