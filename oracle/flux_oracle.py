"""CPU oracle for the tile-fused tensor-parallel GEMMs (GEMM-ReduceScatter, AllGather-GEMM).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module: it exists so
that tests, the smoke check and the benchmark's CPU-baseline leg have a slow, plain,
independent statement of what the GPU library must compute.  It shares no code, table or
constant with the HIP library and imports nothing from it.

What the method computes (paper, Sec. 3): the fused kernels are a *schedule*, not an
approximation, so numerically the result is the textbook one:

  * GEMM-ReduceScatter (Alg. 1, Sec. 3.1): every rank r holds a K-shard (A_r, B_r); the
    reduce-scattered output is  sum_r A_r . B_r, and row i of it belongs to rank
    i // (M / N_TP) ("selection based on the row index").  Seen from one rank, the other
    ranks' products arrive as ready-made partial matrices ("peer partials").
  * AllGather-GEMM (Alg. 2/3, Sec. 3.2): C = A_agg . B where A_agg is the row-wise
    concatenation of the N_TP chunks; the arrival order of chunks must not change C.

All floating-point work is fp64 (numpy matmul as the library primitive for the contraction);
results are returned in fp64 and, separately, rounded once (round-to-nearest-even) to the
output type.  bfloat16 tensors cross this interface as uint16 bit patterns, float32 tensors
as numpy float32 arrays.

The integer part (which tile a workgroup computes, which rank owns a row, which signal
covers a row, in which order chunks are visited) is written out step by step because the
paper only describes it in prose (Sec. 4.1, Sec. 4.3); the readings taken are listed with
each function.

Pins (tests/test_oracle_*.py): literal triple-loop brute force on tiny shapes, exact-integer
closed forms, the reduce-scatter and all-gather invariants, one-hot placement probes, the
communication-order example printed in Sec. 4.3, exhaustive bf16 round trips and hand-built
rounding midpoints, and the limits of Eq. 2.  The protocol simulation `simulate_ag_protocol`
has no value in the paper to compare with; it is pinned by the all-gather invariant (for every
arrival order and driver pace its result is the plain gathered GEMM, with every row poisoned until
its transfer) and by closed-form counts of the tiles that have to wait.
"""
from __future__ import annotations

import numpy as np

BF16 = "bf16"
F32 = "f32"

# --------------------------------------------------------------------------------------
# bfloat16 / float32 helpers (bit-level, independent of torch)
# --------------------------------------------------------------------------------------


def bf16_bits_to_f64(bits) -> np.ndarray:
    """bf16 bit pattern -> fp64, exact (a bf16 is the top half of an IEEE float32)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    with np.errstate(invalid="ignore"):     # signalling-NaN patterns are quietened by the cast
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f32_bits_to_bf16_bits(u32) -> np.ndarray:
    """float32 bit pattern -> bf16 bit pattern, round-to-nearest, ties to even."""
    u = np.ascontiguousarray(u32, dtype=np.uint32)
    exp_all_ones = (u & np.uint32(0x7F800000)) == np.uint32(0x7F800000)
    is_nan = exp_all_ones & ((u & np.uint32(0x007FFFFF)) != 0)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u.astype(np.uint64) + np.uint64(0x7FFF) + lsb.astype(np.uint64)) >> np.uint64(16)
    out = rounded.astype(np.uint16)
    # Inf stays Inf (adding the bias to 0x7F800000 does not change the top half); NaN -> quiet NaN
    out = np.where(is_nan, ((u >> np.uint32(16)) | np.uint32(0x0040)).astype(np.uint16), out)
    return out.astype(np.uint16)


def f64_to_bf16_bits(x) -> np.ndarray:
    """fp64 -> bf16 bits with a single round-to-nearest-even.

    Going fp64 -> fp32 -> bf16 with two nearest roundings can land on the wrong side of a bf16
    midpoint, so the first step rounds to *odd* instead (truncate toward zero and set the last
    bit if anything was lost); fp32 keeps 16 more bits than bf16, which makes the second,
    nearest-even step exact with respect to the original fp64 value.
    """
    x = np.ascontiguousarray(x, dtype=np.float64)
    with np.errstate(over="ignore", invalid="ignore"):
        f = x.astype(np.float32)
    u = f.view(np.uint32).copy()
    back = f.astype(np.float64)
    finite = np.isfinite(x) & np.isfinite(back)
    inexact = finite & (back != x)
    too_big = inexact & (np.abs(back) > np.abs(x))
    u = np.where(too_big, u - np.uint32(1), u)  # one ulp toward zero (same sign, magnitude bits)
    u = np.where(inexact, u | np.uint32(1), u)
    # |x| beyond the fp32 range but finite: astype gives inf, which is also what bf16 gives
    return f32_bits_to_bf16_bits(u)


def f64_to_f32(x) -> np.ndarray:
    """fp64 -> fp32, round-to-nearest-even (the IEEE conversion numpy performs)."""
    with np.errstate(over="ignore"):
        return np.ascontiguousarray(x, dtype=np.float64).astype(np.float32)


def to_f64(x, dtype: str) -> np.ndarray:
    if dtype == BF16:
        return bf16_bits_to_f64(x)
    if dtype == F32:
        a = np.ascontiguousarray(x)
        if a.dtype != np.float32:
            raise TypeError("f32 tensors must be numpy float32")
        return a.astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


def round_to(x64, dtype: str) -> np.ndarray:
    """Round an fp64 array once to `dtype`; bf16 is returned as uint16 bit patterns."""
    if dtype == BF16:
        return f64_to_bf16_bits(x64)
    if dtype == F32:
        return f64_to_f32(x64)
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------------------
# Integer definitions: ownership, signals, orders, TileCoord
# --------------------------------------------------------------------------------------


def slice_rows(M: int, R: int) -> int:
    if R < 1 or M % R != 0:
        raise ValueError("M must be a positive multiple of the tensor-parallel degree")
    return M // R


def owner_of_row(i: int, M: int, R: int) -> int:
    """GetOutput, Sec. 3.1: the output pointer is selected by the row index."""
    return i // slice_rows(M, R)


def local_row(i: int, M: int, R: int) -> int:
    return i % slice_rows(M, R)


def flag_of_row(i: int, M: int, R: int, comm_tiles_per_chunk: int = 1) -> int:
    """GetSignal, Sec. 3.2: the signal is selected by the row index.

    One signal per communication tile; a chunk (M / N_TP rows) is cut into
    `comm_tiles_per_chunk` equal communication tiles (Sec. 4.3, "communication tile size":
    the chunk size divided by a power of two)."""
    S = slice_rows(M, R)
    if comm_tiles_per_chunk < 1 or S % comm_tiles_per_chunk != 0:
        raise ValueError("communication tiles must divide the chunk")
    return i // (S // comm_tiles_per_chunk)


def default_order(rank: int, R: int) -> list[int]:
    """Sec. 4.3, communication order on an all-to-all interconnect: a ring order that starts
    right after the local rank."""
    return [(rank + d) % R for d in range(1, R)]


def visit_order_ag(rank: int, R: int, arrival_order=None) -> list[int]:
    """Chunk order in which AllGather-GEMM tiles are scheduled: the local chunk first (its
    signal is preset, Sec. 3.3), then the chunks in the order the host driver transfers them
    (Sec. 4.1: TileCoord aligned with the signal arrival order)."""
    arr = default_order(rank, R) if arrival_order is None else [int(c) for c in arrival_order]
    if sorted(arr) != sorted(c for c in range(R) if c != rank):
        raise ValueError("arrival_order must be a permutation of the remote ranks")
    return [rank] + arr


def visit_order_rs(rank: int, R: int) -> list[int]:
    """Destination order of GEMM-ReduceScatter tiles.  The paper only says the tile coordinate
    is shifted by the rank index so that ranks write to different devices at the same time
    step (Sec. 4.1).  Reading taken: rank r starts at slice r+1 and ends on its own slice, the
    same ring as the communication order of Sec. 4.3."""
    return default_order(rank, R) + [rank]


def m_tile_order(op: str, M: int, R: int, rank: int, BM: int, arrival_order=None) -> list[int]:
    """Order in which the m-tiles (BM rows each, the last one possibly ragged) are scheduled.

    Every m-tile gets a key and tiles are sorted by (key, tile index):
      * "rs": key = position in visit_order_rs of the rank owning the tile's first row;
      * "ag": key = the latest position in visit_order_ag among the chunks the tile's rows
        touch (a tile can start only when all of its rows have arrived).
    When the slice height is a multiple of BM this is "all tiles of the first visited slice,
    then all tiles of the second ...".
    """
    S = slice_rows(M, R)
    tiles_m = -(-M // BM)
    if op == "rs":
        order = visit_order_rs(rank, R)
    elif op == "ag":
        order = visit_order_ag(rank, R, arrival_order)
    else:
        raise ValueError(op)
    pos = {c: p for p, c in enumerate(order)}
    keyed = []
    for t in range(tiles_m):
        r0 = t * BM
        r1 = min(M, r0 + BM) - 1
        if op == "rs":
            key = pos[r0 // S]
        else:
            key = max(pos[c] for c in range(r0 // S, r1 // S + 1))
        keyed.append((key, t))
    keyed.sort()
    return [t for _, t in keyed]


def band_height(M: int, R: int, BM: int, comm_tiles_per_chunk: int = 1) -> int:
    """Number of consecutive scheduled m-tiles enumerated together with all n-tiles: the m-tiles
    of one communication tile (Sec. 4.3: a chunk, or the given fraction of one; tiles that wait for
    the same signal are then dispatched together and those of the next communication tile after
    them) when its height is a multiple of BM; else those of one slice/chunk when that is a
    multiple of BM; else one."""
    S = slice_rows(M, R)
    t = max(1, comm_tiles_per_chunk)
    if S % t == 0 and (S // t) % BM == 0:
        return S // t // BM
    return S // BM if S % BM == 0 else 1


def tile_coord(op: str, block: int, M: int, N: int, R: int, rank: int, BM: int, BN: int,
               arrival_order=None, n_xcd: int = 1, comm_tiles_per_chunk: int = 1) -> tuple[int, int]:
    """TileCoord of Alg. 1 / Alg. 2: linear workgroup id -> (m_tile, n_tile).

    Workgroups are dispatched in id order, so ascending ids must walk the m-tiles in
    `m_tile_order`.  The grid is cut into bands of `band_height` scheduled m-tiles times all
    n-tiles.  Inside a band the enumeration is m-fastest.  With n_xcd > 1 (and a band size that
    is a multiple of it) the in-band index q is first replaced by
    (q % n_xcd) * (band / n_xcd) + q // n_xcd, so that the workgroups that land on one
    accelerator die (ids congruent mod n_xcd) own a contiguous run of the band and share
    operand panels in that die's L2; which band a workgroup belongs to is unchanged.
    """
    tiles_m = -(-M // BM)
    tiles_n = -(-N // BN)
    if not (0 <= block < tiles_m * tiles_n):
        raise ValueError("block out of range")
    gb = band_height(M, R, BM, comm_tiles_per_chunk if op == "ag" else 1)
    band_sz = gb * tiles_n
    band = block // band_sz
    q = block % band_sz
    # bands are never short: tiles_m is a multiple of gb by construction
    if n_xcd > 1 and band_sz % n_xcd == 0:
        q = (q % n_xcd) * (band_sz // n_xcd) + q // n_xcd
    i = band * gb + q % gb
    j = q // gb
    order = m_tile_order(op, M, R, rank, BM, arrival_order)
    return order[i], j


# --------------------------------------------------------------------------------------
# Numerical definitions
# --------------------------------------------------------------------------------------


def gemm_f64(A, B, ab_dtype: str = BF16) -> np.ndarray:
    """A[M,K] . B[K,N] in fp64."""
    a = to_f64(A, ab_dtype)
    b = to_f64(B, ab_dtype)
    if a.ndim != 2 or b.ndim != 2 or a.shape[1] != b.shape[0]:
        raise ValueError("shape mismatch")
    return a @ b


def gemm_rs(A, B, peers, R: int, rank: int, partial_dtype: str, out_dtype: str,
            ab_dtype: str = BF16):
    """GEMM-ReduceScatter seen from `rank` (Alg. 1 with the Reduce branch, Sec. 3.1).

    A[M,K], B[K,N]: this rank's K-shard.  peers: sequence of length R; entry j != rank is rank
    j's partial product [M,N] in `partial_dtype`; entry `rank` is ignored.
    Returns (slices64, slices_rounded): R arrays [M/R, N]; slice r is what rank r ends up
    owning = rows [r*M/R, (r+1)*M/R) of  A.B + sum_{j != rank} peers[j]  (peers added in
    ascending j; in fp64 the order is immaterial at the tolerances used).
    """
    full = gemm_f64(A, B, ab_dtype)
    M = full.shape[0]
    S = slice_rows(M, R)
    if len(peers) != R:
        raise ValueError("need one peer entry per rank")
    for j in range(R):
        if j == rank:
            continue
        p = to_f64(peers[j], partial_dtype)
        if p.shape != full.shape:
            raise ValueError("peer partial has the wrong shape")
        full = full + p
    slices64 = [full[r * S:(r + 1) * S, :] for r in range(R)]
    return slices64, [round_to(s, out_dtype) for s in slices64]


def gemm_scatter(A, B, R: int, out_dtype: str, ab_dtype: str = BF16):
    """GEMM with the Write branch of Alg. 1 (Sec. 3.1, 4.2: the AlltoAll flavour of ReduceScatter):
    the tile is not reduced, each row of this rank's partial product A.B goes to the slice of the
    rank that owns the row.  Returns (slices64, slices_rounded): R arrays [M/R, N]."""
    full = gemm_f64(A, B, ab_dtype)
    S = slice_rows(full.shape[0], R)
    slices64 = [full[r * S:(r + 1) * S, :] for r in range(R)]
    return slices64, [round_to(s, out_dtype) for s in slices64]


def gemm_reduce_into(A, B, held, R: int, ab_dtype: str = BF16):
    """GEMM with the Reduce branch of Alg. 1 carried out by additions on the destination (Sec. 4.2,
    "Reduce", first form): `held[r]` is what slice r, an fp32 array [M/R, N], holds before the call
    (the other ranks' contributions so far, or zeros); afterwards it holds that plus the rows of
    this rank's A.B that the slice owns.  Returns (slices64, slices_f32)."""
    full = gemm_f64(A, B, ab_dtype)
    S = slice_rows(full.shape[0], R)
    if len(held) != R:
        raise ValueError("need one held slice per rank")
    slices64 = []
    for r in range(R):
        h = to_f64(held[r], F32)
        if h.shape != (S, full.shape[1]):
            raise ValueError("held slice has the wrong shape")
        slices64.append(h + full[r * S:(r + 1) * S, :])
    return slices64, [round_to(s, F32) for s in slices64]


def reduce_slice(staged, staged_dtype: str, out_dtype: str):
    """The local reduction that follows the AlltoAll (Sec. 3.1): `staged` holds, for one slice, the
    R partial results [M/R, N] the R ranks wrote for it (in `staged_dtype`); the slice is their sum,
    rounded once.  Returns (sum64, rounded)."""
    if len(staged) == 0:
        raise ValueError("need at least one partial")
    total = to_f64(staged[0], staged_dtype).copy()
    for s in staged[1:]:
        t = to_f64(s, staged_dtype)
        if t.shape != total.shape:
            raise ValueError("partials differ in shape")
        total = total + t
    return total, round_to(total, out_dtype)


def gemm_rs_rows(A, B, peers, R: int, rank: int, partial_dtype: str, rows, ab_dtype: str = BF16):
    """The same definition as `gemm_rs`, evaluated for a subset of global rows only (used where
    the full problem is too large to finish in seconds).  Returns a list of
    (owner_rank, local_row, values64[N]) in the order of `rows`."""
    rows = [int(i) for i in rows]
    a = to_f64(A, ab_dtype)
    M = a.shape[0]
    S = slice_rows(M, R)
    vals = a[rows, :] @ to_f64(B, ab_dtype)
    for j in range(R):
        if j == rank:
            continue
        pj = peers[j]
        if pj.shape[0] != M:
            raise ValueError("peer partial has the wrong shape")
        vals = vals + to_f64(pj[rows, :], partial_dtype)
    return [(owner_of_row(i, M, R), local_row(i, M, R), vals[t]) for t, i in enumerate(rows)]


def ag_gemm_rows(A_chunks, B, rows, ab_dtype: str = BF16) -> np.ndarray:
    """`ag_gemm` for a subset of global rows: row i lives in chunk i // S at local row i % S."""
    S = A_chunks[0].shape[0]
    picked = np.stack([to_f64(A_chunks[int(i) // S][int(i) % S], ab_dtype) for i in rows])
    return picked @ to_f64(B, ab_dtype)


def rs_from_factors(A_list, B_list, ab_dtype: str = BF16) -> np.ndarray:
    """The reduce-scatter result written from its definition: sum over ranks of A_r . B_r,
    before scattering (Sec. 2.1: the second GEMM of the MLP is sharded along K)."""
    total = None
    for A, B in zip(A_list, B_list):
        prod = gemm_f64(A, B, ab_dtype)
        total = prod if total is None else total + prod
    return total


def partial_of(A, B, partial_dtype: str, ab_dtype: str = BF16):
    """What a peer rank would hand over: its own product rounded to the partial dtype."""
    return round_to(gemm_f64(A, B, ab_dtype), partial_dtype)


def ag_gemm(A_chunks, B, out_dtype: str, ab_dtype: str = BF16):
    """AllGather-GEMM (Alg. 2, Sec. 3.2): C = concat_r(A_chunks[r]) . B, chunk r occupying
    rows [r*S, (r+1)*S).  Returns (C64, C_rounded).  Arrival order does not enter."""
    rows = [to_f64(c, ab_dtype) for c in A_chunks]
    S = rows[0].shape[0]
    if any(r.shape != rows[0].shape for r in rows):
        raise ValueError("all chunks must have the same shape")
    A_agg = np.concatenate(rows, axis=0) if S > 0 else np.zeros((0, rows[0].shape[1]))
    C = A_agg @ to_f64(B, ab_dtype)
    return C, round_to(C, out_dtype)


def simulate_ag_protocol(A_chunks, B, rank: int, BM: int, BN: int, arrival_order=None,
                         tiles_per_step: int | None = None, n_xcd: int = 1,
                         ab_dtype: str = BF16):
    """Step-by-step replay of Alg. 2 + Alg. 3 (pull form) on one device, sequentially.

    A_agg starts poisoned with NaN except the local chunk, whose signal is preset (Sec. 3.3).
    The host driver (Alg. 3) then, chunk by chunk in `arrival_order`, copies the chunk into
    A_agg and sets its signal.  Workgroups are taken in id order; a workgroup whose signals
    are not all set makes the driver advance until they are (this models WaitSignal: the tile
    blocks, the copy continues).  `tiles_per_step` lets the driver advance on its own after
    that many tiles, modelling a copy that runs ahead.  Returns (C64, waits) where `waits` is
    the number of tiles that found a signal unset when first reached.
    """
    R = len(A_chunks)
    rows = [to_f64(c, ab_dtype) for c in A_chunks]
    S, K = rows[0].shape
    M = S * R
    b = to_f64(B, ab_dtype)
    N = b.shape[1]
    A_agg = np.full((M, K), np.nan)
    flags = [0] * R
    A_agg[rank * S:(rank + 1) * S] = rows[rank]
    flags[rank] = 1
    pending = list(visit_order_ag(rank, R, arrival_order)[1:])

    def driver_step():
        c = pending.pop(0)
        A_agg[c * S:(c + 1) * S] = rows[c]      # DataTransfer
        flags[c] = 1                            # SetSignal, after the transfer

    tiles_m = -(-M // BM)
    tiles_n = -(-N // BN)
    C = np.full((M, N), np.nan)
    waits = 0
    for block in range(tiles_m * tiles_n):
        if tiles_per_step and block and block % tiles_per_step == 0 and pending:
            driver_step()
        mt, nt = tile_coord("ag", block, M, N, R, rank, BM, BN, arrival_order, n_xcd)
        r0, r1 = mt * BM, min(M, mt * BM + BM)
        c0, c1 = nt * BN, min(N, nt * BN + BN)
        need = range(flag_of_row(r0, M, R), flag_of_row(r1 - 1, M, R) + 1)
        if not all(flags[f] for f in need):
            waits += 1
            while not all(flags[f] for f in need):  # WaitSignal
                driver_step()
        C[r0:r1, c0:c1] = A_agg[r0:r1] @ b[:, c0:c1]
    while pending:
        driver_step()
    return C, waits


# --------------------------------------------------------------------------------------
# Metric (Sec. 2.3)
# --------------------------------------------------------------------------------------


def effective_comm_time(overall: float, gemm_non_split: float) -> float:
    """Eq. 1: ECT = OverallTime - GEMM_non-split."""
    return overall - gemm_non_split


def overlap_efficiency(t_overlap: float, t_non_overlap: float, t_gemm: float) -> float:
    """Eq. 2: E = 1 - ECT_overlap / ECT_non-overlap, both ECTs against the same GEMM time."""
    return 1.0 - effective_comm_time(t_overlap, t_gemm) / effective_comm_time(t_non_overlap, t_gemm)
