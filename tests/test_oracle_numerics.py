"""Pins for the oracle's numerical definitions (CPU only): brute force, closed forms,
invariants and placement probes.  Each test is meant to fail for one plausible mistake
(dropped peer, transposed operand, wrong slice owner, wrong chunk position ...)."""
import numpy as np
import pytest

from oracle import flux_oracle as fo


def bf16(x):
    """float array of bf16-representable values -> bit patterns (asserts exactness)."""
    bits = fo.f64_to_bf16_bits(np.asarray(x, dtype=np.float64))
    assert np.array_equal(fo.bf16_bits_to_f64(bits), np.asarray(x, dtype=np.float64))
    return bits


def rand_int(rng, shape, lim):
    return rng.integers(-lim, lim + 1, size=shape).astype(np.float64)


# ---- brute force on tiny shapes: literal loops, no library contraction -------------------

@pytest.mark.parametrize("M,N,K,R,rank", [(4, 3, 5, 1, 0), (4, 6, 2, 2, 1), (8, 5, 7, 4, 2), (8, 8, 8, 2, 0)])
def test_gemm_rs_brute_force(M, N, K, R, rank):
    rng = np.random.default_rng(M * 100 + N * 10 + K + R)
    A = rand_int(rng, (M, K), 3)
    B = rand_int(rng, (K, N), 3)
    peers = [None if j == rank else rand_int(rng, (M, N), 9) for j in range(R)]
    S = M // R
    want = [[[0.0] * N for _ in range(S)] for _ in range(R)]
    for i in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                acc += A[i][k] * B[k][n]
            for j in range(R):
                if j != rank:
                    acc += peers[j][i][n]
            want[i // S][i % S][n] = acc
    s64, srnd = fo.gemm_rs(bf16(A), bf16(B), [None if p is None else bf16(p) for p in peers],
                           R, rank, "bf16", "f32")
    assert len(s64) == R
    for r in range(R):
        assert s64[r].shape == (S, N)
        assert np.array_equal(s64[r], np.array(want[r]))
        assert np.array_equal(srnd[r].astype(np.float64), np.array(want[r]))


@pytest.mark.parametrize("S,N,K,R", [(1, 3, 5, 1), (2, 4, 3, 2), (2, 5, 7, 4), (1, 8, 8, 8)])
def test_ag_gemm_brute_force(S, N, K, R):
    rng = np.random.default_rng(S * 1000 + N * 100 + K * 10 + R)
    chunks = [rand_int(rng, (S, K), 3) for _ in range(R)]
    B = rand_int(rng, (K, N), 3)
    want = np.zeros((S * R, N))
    for r in range(R):
        for i in range(S):
            for n in range(N):
                acc = 0.0
                for k in range(K):
                    acc += chunks[r][i][k] * B[k][n]
                want[r * S + i][n] = acc
    C64, Crnd = fo.ag_gemm([bf16(c) for c in chunks], bf16(B), "bf16")
    assert np.array_equal(C64, want)
    assert np.array_equal(fo.bf16_bits_to_f64(Crnd), want)  # |values| small: exact in bf16


# ---- closed forms --------------------------------------------------------------------------

def test_closed_form_ones_and_ramps():
    M, N, K, R, rank = 12, 10, 16, 4, 1
    # A = all ones, B[k][n] = n  ->  (A.B)[i][n] = K * n ; peers j constant (j+1)
    A = np.ones((M, K))
    B = np.tile(np.arange(N, dtype=np.float64), (K, 1))
    peers = [None if j == rank else np.full((M, N), float(j + 1)) for j in range(R)]
    s64, _ = fo.gemm_rs(bf16(A), bf16(B), [None if p is None else bf16(p) for p in peers],
                        R, rank, "bf16", "f32")
    peer_sum = R * (R + 1) / 2 - (rank + 1)
    for r in range(R):
        assert np.array_equal(s64[r], np.tile(K * np.arange(N) + peer_sum, (M // R, 1)))


def test_closed_form_detects_transposed_operands():
    # A[i][k] = i (rows differ), B[k][n] = [k == 0] * (n + 1)  ->  C[i][n] = i * (n + 1)
    M, N, K = 6, 4, 6
    A = np.tile(np.arange(M, dtype=np.float64)[:, None], (1, K))
    B = np.zeros((K, N))
    B[0, :] = np.arange(1, N + 1)
    C = fo.gemm_f64(bf16(A), bf16(B))
    assert np.array_equal(C, np.outer(np.arange(M), np.arange(1, N + 1)))


def test_exact_integer_inputs_round_once_to_bf16():
    # |result| up to a few thousand: not all exact in bf16, so the single rounding is exercised
    rng = np.random.default_rng(5)
    M, N, K, R, rank = 16, 24, 512, 2, 0
    A = rand_int(rng, (M, K), 2)
    B = rand_int(rng, (K, N), 2)
    P = rand_int(rng, (M, N), 8)
    s64, srnd = fo.gemm_rs(bf16(A), bf16(B), [None, bf16(P)], R, rank, "bf16", "bf16")
    exact = A.astype(np.int64) @ B.astype(np.int64) + P.astype(np.int64)
    assert np.array_equal(np.concatenate(s64), exact.astype(np.float64))
    got = fo.bf16_bits_to_f64(np.concatenate(srnd))
    # nearest bf16: error at most half an ulp (ulp = 2^(e-7))
    e = np.floor(np.log2(np.maximum(np.abs(exact), 1)))
    assert np.all(np.abs(got - exact) <= 2.0 ** (e - 8))


# ---- invariants ------------------------------------------------------------------------------

def test_reduce_scatter_invariant_equals_unsharded_gemm():
    """Sum over ranks of A_r.B_r == one GEMM over the concatenated K; every rank's view of the
    fused op (own product + the others' partials) gives the same slices."""
    rng = np.random.default_rng(11)
    M, N, Kr, R = 8, 6, 5, 4
    As = [rand_int(rng, (M, Kr), 2) for _ in range(R)]
    Bs = [rand_int(rng, (Kr, N), 2) for _ in range(R)]
    full = fo.rs_from_factors([bf16(a) for a in As], [bf16(b) for b in Bs])
    unsharded = np.concatenate(As, axis=1).astype(np.int64) @ np.concatenate(Bs, axis=0).astype(np.int64)
    assert np.array_equal(full, unsharded.astype(np.float64))
    partials = [fo.partial_of(bf16(a), bf16(b), "f32") for a, b in zip(As, Bs)]
    for rank in range(R):
        peers = [None if j == rank else partials[j] for j in range(R)]
        s64, _ = fo.gemm_rs(bf16(As[rank]), bf16(Bs[rank]), peers, R, rank, "f32", "f32")
        assert np.array_equal(np.concatenate(s64), full)
        for r in range(R):
            assert np.array_equal(s64[r], full[r * (M // R):(r + 1) * (M // R)])


def test_all_gather_invariant_and_order_independence():
    rng = np.random.default_rng(12)
    S, N, K, R = 3, 5, 7, 4
    chunks = [rand_int(rng, (S, K), 3) for _ in range(R)]
    B = rand_int(rng, (K, N), 3)
    C64, _ = fo.ag_gemm([bf16(c) for c in chunks], bf16(B), "f32")
    want = np.vstack(chunks).astype(np.int64) @ B.astype(np.int64)
    assert np.array_equal(C64, want.astype(np.float64))
    for rank in range(R):
        for order in (None, list(reversed(fo.default_order(rank, R)))):
            Csim, _ = fo.simulate_ag_protocol([bf16(c) for c in chunks], bf16(B), rank, 2, 2, order)
            assert np.array_equal(Csim, C64)


def test_r1_reduces_to_plain_gemm():
    rng = np.random.default_rng(13)
    A = rand_int(rng, (5, 4), 3)
    B = rand_int(rng, (4, 6), 3)
    s64, _ = fo.gemm_rs(bf16(A), bf16(B), [None], 1, 0, "bf16", "f32")
    C64, _ = fo.ag_gemm([bf16(A)], bf16(B), "f32")
    want = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64)
    assert len(s64) == 1 and np.array_equal(s64[0], want) and np.array_equal(C64, want)


# ---- placement probes ------------------------------------------------------------------------

def test_rs_placement_one_hot_rows():
    """A.B is made to carry the global row index in every element, peers carry 1024*(j+1) in
    every element: each output element then says which row and which peers it came from."""
    M, N, K, R = 12, 4, 12, 3
    A = np.zeros((M, K))
    for i in range(M):
        A[i, i % K] = float(i)            # A[i][k] = i * [k == i]
    B = np.ones((K, N))
    for rank in range(R):
        peers = [None if j == rank else bf16(np.full((M, N), 1024.0 * (j + 1))) for j in range(R)]
        s64, _ = fo.gemm_rs(bf16(A), bf16(B), peers, R, rank, "bf16", "f32")
        others = sum(1024.0 * (j + 1) for j in range(R) if j != rank)
        for r in range(R):
            for lr in range(M // R):
                gi = r * (M // R) + lr
                assert fo.owner_of_row(gi, M, R) == r and fo.local_row(gi, M, R) == lr
                assert np.all(s64[r][lr] == gi + others)


def test_ag_chunk_placement():
    S, K, N, R = 2, 4, 3, 4
    B = np.ones((K, N))
    chunks = [np.full((S, K), float(r + 1)) for r in range(R)]   # chunk r -> rows all K*(r+1)
    C64, _ = fo.ag_gemm([bf16(c) for c in chunks], bf16(B), "f32")
    for i in range(S * R):
        assert np.all(C64[i] == K * (i // S + 1))


def test_peer_partial_shape_and_count_are_checked():
    A = bf16(np.ones((4, 2)))
    B = bf16(np.ones((2, 2)))
    with pytest.raises(ValueError):
        fo.gemm_rs(A, B, [None], 2, 0, "bf16", "f32")
    with pytest.raises(ValueError):
        fo.gemm_rs(A, B, [None, bf16(np.ones((2, 2)))], 2, 0, "bf16", "f32")
    with pytest.raises(ValueError):
        fo.gemm_rs(bf16(np.ones((3, 2))), B, [None, bf16(np.ones((3, 2)))], 2, 0, "bf16", "f32")


def test_row_subset_variants_agree_with_full_definitions():
    rng = np.random.default_rng(21)
    M, N, K, R, rank = 12, 5, 6, 3, 1
    A = rand_int(rng, (M, K), 3)
    B = rand_int(rng, (K, N), 3)
    peers = [None if j == rank else bf16(rand_int(rng, (M, N), 9)) for j in range(R)]
    s64, _ = fo.gemm_rs(bf16(A), bf16(B), peers, R, rank, "bf16", "f32")
    rows = [11, 0, 5, 4]
    for (owner, lr, vals), i in zip(fo.gemm_rs_rows(bf16(A), bf16(B), peers, R, rank, "bf16", rows), rows):
        assert owner * (M // R) + lr == i
        assert np.array_equal(vals, s64[owner][lr])
    chunks = [bf16(A[r * 4:(r + 1) * 4]) for r in range(R)]
    C64, _ = fo.ag_gemm(chunks, bf16(B), "f32")
    assert np.array_equal(fo.ag_gemm_rows(chunks, bf16(B), rows), C64[rows])


def test_alltoall_flavour_equals_reduce_scatter():
    """Write branch + local reduction (Sec. 3.1: ReduceScatter = AlltoAll + reduction): every rank
    scatters its partial product by owner, every owner sums the R partials staged for its slice.
    On integer inputs that is exactly the unsharded GEMM over the concatenated K, slice by slice,
    and exactly what the Reduce branch gives; a dropped rank or a wrong row range changes it."""
    rng = np.random.default_rng(21)
    M, N, Kr, R = 8, 6, 5, 4
    S = M // R
    As = [rand_int(rng, (M, Kr), 2) for _ in range(R)]
    Bs = [rand_int(rng, (Kr, N), 2) for _ in range(R)]
    unsharded = np.concatenate(As, axis=1).astype(np.int64) @ np.concatenate(Bs, axis=0).astype(np.int64)
    scattered = [fo.gemm_scatter(bf16(a), bf16(b), R, "f32")[1] for a, b in zip(As, Bs)]   # [rank][slice]
    for j in range(R):      # brute force: slice r of rank j's scatter is rows r*S.. of its own product
        own = As[j].astype(np.int64) @ Bs[j].astype(np.int64)
        for r in range(R):
            assert np.array_equal(fo.to_f64(scattered[j][r], "f32"), own[r * S:(r + 1) * S].astype(np.float64))
    for r in range(R):
        total, rounded = fo.reduce_slice([scattered[j][r] for j in range(R)], "f32", "f32")
        assert np.array_equal(total, unsharded[r * S:(r + 1) * S].astype(np.float64))
        assert np.array_equal(fo.to_f64(rounded, "f32"), total)
    # same as the Reduce branch seen from any rank
    partials = [fo.partial_of(bf16(a), bf16(b), "f32") for a, b in zip(As, Bs)]
    s64, _ = fo.gemm_rs(bf16(As[1]), bf16(Bs[1]), [None if j == 1 else partials[j] for j in range(R)], R, 1, "f32", "f32")
    for r in range(R):
        assert np.array_equal(s64[r], fo.reduce_slice([scattered[j][r] for j in range(R)], "f32", "f32")[0])
    with pytest.raises(ValueError):
        fo.reduce_slice([scattered[0][0], scattered[0][0][:1]], "f32", "f32")


def test_reduce_slice_rounds_once():
    # three bf16 values whose exact sum needs more than 8 significand bits: rounded once, to even
    vals = [bf16(np.array([[256.0]])), bf16(np.array([[1.0]])), bf16(np.array([[2.0]]))]   # 259 -> 260 (tie 258/260? no: 259 is between 258 and 260)
    total, rounded = fo.reduce_slice(vals, "bf16", "bf16")
    assert total[0, 0] == 259.0
    assert fo.to_f64(rounded, "bf16")[0, 0] == 260.0      # 259 = 258 + 1 is a tie of (258, 260): even significand wins


def test_reduce_by_additions_on_the_destination():
    """Reduce branch carried out on the destination (Sec. 4.2, "Reduce", first form): every rank adds
    its partial product into the slices, starting from zeros.  On integer inputs, after all R ranks
    (in any order) the slices are exactly the unsharded GEMM over the concatenated K; after one rank
    they are its Write-branch scatter; and adding onto the sum of the peers' partials gives what the
    pull form of the Reduce branch gives.  A dropped term, a wrong slice or a wrong row range fails."""
    rng = np.random.default_rng(33)
    M, N, Kr, R = 12, 5, 7, 3
    S = M // R
    As = [rand_int(rng, (M, Kr), 2) for _ in range(R)]
    Bs = [rand_int(rng, (Kr, N), 2) for _ in range(R)]
    unsharded = np.concatenate(As, axis=1).astype(np.int64) @ np.concatenate(Bs, axis=0).astype(np.int64)
    zeros = [np.zeros((S, N), dtype=np.float32) for _ in range(R)]
    # one rank onto zeros = its scatter; brute force for one element
    _, after0 = fo.gemm_reduce_into(bf16(As[0]), bf16(Bs[0]), zeros, R)
    _, scat0 = fo.gemm_scatter(bf16(As[0]), bf16(Bs[0]), R, "f32")
    for r in range(R):
        assert np.array_equal(after0[r], scat0[r])
    assert float(after0[2][1, 3]) == float(sum(int(As[0][2 * S + 1, k]) * int(Bs[0][k, 3]) for k in range(Kr)))
    # all ranks, two different orders
    for order in ((0, 1, 2), (2, 0, 1)):
        held = zeros
        for j in order:
            _, held = fo.gemm_reduce_into(bf16(As[j]), bf16(Bs[j]), held, R)
        for r in range(R):
            assert np.array_equal(held[r].astype(np.int64), unsharded[r * S:(r + 1) * S])
    # onto the peers' sum = the pull form seen from rank 1
    partials = [fo.partial_of(bf16(a), bf16(b), "f32") for a, b in zip(As, Bs)]
    peers_sum = [sum(fo.to_f64(partials[j], "f32")[r * S:(r + 1) * S] for j in range(R) if j != 1).astype(np.float32)
                 for r in range(R)]
    s64_add, _ = fo.gemm_reduce_into(bf16(As[1]), bf16(Bs[1]), peers_sum, R)
    s64_pull, _ = fo.gemm_rs(bf16(As[1]), bf16(Bs[1]), [None if j == 1 else partials[j] for j in range(R)], R, 1, "f32", "f32")
    for r in range(R):
        assert np.array_equal(s64_add[r], s64_pull[r])
    with pytest.raises(ValueError):
        fo.gemm_reduce_into(bf16(As[0]), bf16(Bs[0]), zeros[:2], R)
    with pytest.raises(ValueError):
        fo.gemm_reduce_into(bf16(As[0]), bf16(Bs[0]), [z[:1] for z in zeros], R)
