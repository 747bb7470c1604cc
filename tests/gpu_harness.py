"""Helpers for the GPU parity tests: run the library through its C ABI on seeded inputs and
compare with the CPU oracle.  Not a test module."""
from __future__ import annotations

import numpy as np
import torch

from oracle import flux_oracle as fo
from paper_2406_06858_amd import binding as fb
from paper_2406_06858_amd import inputs as fi

DEV = "cuda:0"
TEST_TIMEOUT_TICKS = 300_000_000      # 3 s at 100 MHz: a lost signal ends the kernel, not the box

_TORCH = {"bf16": torch.bfloat16, "f32": torch.float32}


def tol_for(out_dtype: str) -> float:
    """Elementwise bound |gpu - ref| <= tol * max(1, |ref|): 1e-2 for bf16 outputs (bf16 has 8
    significand bits: half an ulp is 2^-9 ~ 2e-3 relative, the rest is fp32 accumulation
    order), 1e-5 for the fp32 variant."""
    return 1e-2 if out_dtype == "bf16" else 1e-5


def assert_close(got: torch.Tensor, ref64: np.ndarray, out_dtype: str, what: str = ""):
    g = got.detach().cpu().to(torch.float64).numpy()
    assert g.shape == ref64.shape, (what, g.shape, ref64.shape)
    err = np.abs(g - ref64)
    bound = tol_for(out_dtype) * np.maximum(1.0, np.abs(ref64))
    bad = ~(err <= bound)            # also catches NaN
    if bad.any():
        idx = np.argwhere(bad)[0]
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements out of tolerance; first at {tuple(idx)}: "
                             f"gpu={g[tuple(idx)]} ref={ref64[tuple(idx)]}")


def assert_bits_equal(got: torch.Tensor, want_np: np.ndarray, what: str = ""):
    g = fi.to_numpy(got)
    if not np.array_equal(g, want_np):
        bad = np.argwhere(g != want_np)
        i = tuple(bad[0])
        raise AssertionError(f"{what}: {len(bad)} elements differ bitwise; first at {i}: gpu={g[i]} want={want_np[i]}")


def workspace_for(op: int, p) -> torch.Tensor | None:
    n = fb.flux_workspace_bytes(op, p)
    if n == 0:
        return None
    return torch.zeros((n + 3) // 4, dtype=torch.int32, device=DEV)


def run_rs(w: fi.Workload, rank: int, A, B, peers, tile_config=0, split_k=0, flags=0, poison=True):
    """Fused GEMM-ReduceScatter through the C ABI.  Returns the list of R output slices."""
    p = fb.problem(w.M, w.N, w.K, w.R, rank, w.partial_dtype, w.out_dtype, tile_config, split_k, flags)
    dA, dB = A.to(DEV), B.to(DEV)
    dpeers = [None if t is None else t.to(DEV) for t in peers]
    fill = float("nan") if poison else 0.0
    outs = [torch.full((w.S, w.N), fill, dtype=_TORCH[w.out_dtype], device=DEV) for _ in range(w.R)]
    ws = workspace_for(fb.FLUX_OP_RS, p)
    if ws is not None:
        ws.fill_(-1)                                  # garbage until initialised
        fb.flux_init_buffers(fb.FLUX_OP_RS, p, ws)
    fb.flux_gemm_rs(p, dA, dB, dpeers, outs, ws)
    torch.cuda.synchronize()
    return outs


def run_ag(w: fi.Workload, rank: int, chunks, B, arrival, tile_config=0, split_k=0, flags=0,
           comm_tiles_per_chunk=0, copy_workgroups=0, local_in_place=False, delay_copy_cycles=0,
           timeout_ticks=TEST_TIMEOUT_TICKS, repeat=1, link_gbps=0, copy_stream=None, agg_offset_elems=0):
    """Fused AllGather-GEMM through the C ABI.  A_agg starts NaN-poisoned so a tile that reads
    rows before their signal shows up in C.  Returns (C, A_agg, signals, status)."""
    p = fb.problem(w.M, w.N, w.K, w.R, rank, "bf16", w.out_dtype, tile_config, split_k, flags,
                   comm_tiles_per_chunk, copy_workgroups, timeout_ticks, link_gbps)
    dB = B.to(DEV)
    # (agg_offset_elems: start the gathered matrix that many elements into its allocation, e.g. 8
    # for a base that is 16-byte but not cache-line aligned)
    agg_store = torch.full((w.M * w.K + agg_offset_elems,), float("nan"), dtype=torch.bfloat16, device=DEV)
    A_agg = agg_store[agg_offset_elems:].view(w.M, w.K)
    dchunks = [c.to(DEV) for c in chunks]
    if local_in_place:
        A_agg[rank * w.S:(rank + 1) * w.S].copy_(dchunks[rank])
        dchunks[rank] = A_agg[rank * w.S:(rank + 1) * w.S]
    Cout = torch.full((w.M, w.N), float("nan"), dtype=_TORCH[w.out_dtype], device=DEV)
    nsig = w.R * max(1, comm_tiles_per_chunk)
    signals = torch.full((nsig,), 12345, dtype=torch.int32, device=DEV)     # garbage until initialised
    ws = workspace_for(fb.FLUX_OP_AG, p)
    ws.fill_(-1)
    fb.flux_init_buffers(fb.FLUX_OP_AG, p, ws, signals)
    compute = torch.cuda.current_stream()
    copy = copy_stream if copy_stream is not None else torch.cuda.Stream()
    torch.cuda.synchronize()
    if delay_copy_cycles:
        with torch.cuda.stream(copy):
            torch.cuda._sleep(int(delay_copy_cycles))
    results = []
    for _ in range(repeat):      # later calls rely on the state the previous call left behind
        if results:
            A_agg[:rank * w.S].fill_(float("nan"))
            A_agg[(rank + 1) * w.S:].fill_(float("nan"))
            Cout.fill_(float("nan"))
        fb.flux_ag_gemm(p, dchunks, A_agg, dB, Cout, signals, arrival, ws, compute, copy)
        torch.cuda.synchronize()
        results.append(fb.flux_query_status(ws))
    status = results[-1] if all(r == results[0] for r in results) else results
    return Cout, A_agg, signals, status


def oracle_rs(w, rank, A, B, peers):
    return fo.gemm_rs(fi.to_numpy(A), fi.to_numpy(B), [None if t is None else fi.to_numpy(t) for t in peers],
                      w.R, rank, w.partial_dtype, w.out_dtype)


def oracle_ag(w, chunks, B):
    return fo.ag_gemm([fi.to_numpy(c) for c in chunks], fi.to_numpy(B), w.out_dtype)
