#!/usr/bin/env python3
"""Benchmark of the fused tensor-parallel GEMMs on one MI355X.

A step is one pass of the whole hot path on one batch of the largest configuration that fits one
GPU, the GPT-3-175B-like layer at TP=8 with 8192 tokens: the fused AllGather-GEMM of the QKV
projection (8 chunks of [1024,12288] gathered in a seeded random arrival order, times [12288,4608])
followed by the fused GEMM-ReduceScatter of the attention output projection ([8192,1536] times
[1536,12288], 7 peer partials added in the epilogue, 8 row slices written).  Inputs are seeded
synthetic tensors, already resident in HBM when the timed region starts.

Prints ONE JSON line (the README names the fields).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
# bytes per launch behind the L2 of the two kernels of the timed step (rocprofv3 FETCH_SIZE + WRITE_SIZE)
TRAFFIC_BYTES = {"rs": 2170.7e6 + 205.8e6, "ag": 2619.6e6 + 319.2e6}     # profiles/bench_c4_pmc_traffic.txt
HBM_PEAK_GBS = 8000.0
TIMEOUT_TICKS = 500_000_000        # 5 s: a lost signal ends the run with an error, not a hang


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--ramp-seconds", type=float, default=2.0, help="untimed load before the warm-up steps")
    ap.add_argument("--ag-flags", type=int, default=0,
                    help="FLUX_FLAG_* bits for the AllGather-GEMM of the timed step")
    ap.add_argument("--serial-kernels", type=int, default=0, metavar="N",
                    help="counter-collection mode: run N rounds of [chunk copy, AllGather-GEMM kernel on the gathered "
                         "matrix, fused GEMM-ReduceScatter, fused AllGather-GEMM call] and exit (rocprofv3 --pmc runs "
                         "kernels one at a time)")
    ap.add_argument("--serial-decode", type=int, default=0, metavar="N",
                    help="counter-collection mode for the few-row shapes (M = 8, 64, 256): N plain GEMMs, N fused "
                         "AllGather-GEMM calls and N fused GEMM-ReduceScatter calls each, over rotating copies of the "
                         "weight matrix, then exit")
    ap.add_argument("--event-every", type=int, default=8, metavar="E",
                    help="record the per-kernel HIP events on every E-th timed step (1 = every step)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the per-config / overlap-efficiency section")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (R virtual ranks inside one MI355X); --gpus must be 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    t_begin = time.perf_counter()

    def say(msg):
        """Progress on stderr (the JSON line is the only thing on stdout)."""
        print(f"[bench {time.perf_counter() - t_begin:6.1f}s] {msg}", file=sys.stderr, flush=True)

    from paper_2406_06858_amd import binding as fb
    from paper_2406_06858_amd import inputs as fi

    dev = "cuda:0"
    torch.cuda.set_device(0)
    W = fi.WORKLOADS
    compute = torch.cuda.current_stream()
    copy = torch.cuda.Stream()

    def chunk_workspace(op, p):
        n = fb.flux_chunked_workspace_bytes(op, p)
        if n == 0:
            return None
        ws = torch.zeros(n // 4 + 1, dtype=torch.int32, device=dev)
        fb.flux_init_buffers(fb.FLUX_OP_RS, p, ws)
        return ws

    class RotatingB:
        """Few-row shapes: the weight matrix (58.7 MB) would stay in the 256 MB Infinity Cache from one
        call to the next, which no decode step of a real model enjoys (every layer has its own
        weights).  Such operators cycle through enough copies of B to exceed that cache."""
        def rotate_weights(self, copies):
            self._Bs = [self.B] + [self.B.clone() for _ in range(copies - 1)]
            self._bi = 0

        def next_B(self):
            if not hasattr(self, "_Bs"):
                return self.B
            self._bi = (self._bi + 1) % len(self._Bs)
            return self._Bs[self._bi]

    class AG(RotatingB):
        def __init__(self, w, rank, **kw):
            self.w, self.rank = w, rank
            self.chunks_cpu, self.B_cpu, self.arrival = fi.make_ag_inputs(w, rank)
            self.p = fb.problem(w.M, w.N, w.K, w.R, rank, "bf16", w.out_dtype, spin_timeout_ticks=TIMEOUT_TICKS, **kw)
            self.chunks = [c.to(dev) for c in self.chunks_cpu]
            self.B = self.B_cpu.to(dev)
            self.A_agg = torch.zeros((w.M, w.K), dtype=torch.bfloat16, device=dev)
            # the local chunk lives in place inside A_agg (its signal is preset), as a rank's own
            # activations would; only the R-1 remote chunks are transferred
            self.A_agg[rank * w.S:(rank + 1) * w.S].copy_(self.chunks[rank])
            self.chunks[rank] = self.A_agg[rank * w.S:(rank + 1) * w.S]
            self.C = torch.zeros((w.M, w.N), dtype=torch.bfloat16, device=dev)
            self.signals = torch.zeros(w.R * max(1, kw.get("comm_tiles_per_chunk", 0)), dtype=torch.int32, device=dev)
            self.ws = torch.zeros(fb.flux_workspace_bytes(fb.FLUX_OP_AG, self.p) // 4 + 1, dtype=torch.int32, device=dev)
            fb.flux_init_buffers(fb.FLUX_OP_AG, self.p, self.ws, self.signals)
            # steady state: A_agg holds the previous step's gathered activations, not zeros (a GEMM
            # over zeros draws less power and runs at a higher clock: a flattering baseline)
            self.unfused(fb.FLUX_PHASE_COMM)

        def fused(self, stream=None):
            fb.flux_ag_gemm(self.p, self.chunks, self.A_agg, self.next_B(), self.C, self.signals, self.arrival,
                            self.ws, stream or compute, copy)

        def unfused(self, phases):
            fb.flux_gemm_ref_unfused(fb.FLUX_OP_AG, phases, self.p, A_chunks=self.chunks, A_agg=self.A_agg,
                                     B=self.next_B(), Cout=self.C, workspace=self.ws, stream=compute)

        def chunked(self):
            if not hasattr(self, "ws_chunk"):
                self.ws_chunk = chunk_workspace(fb.FLUX_OP_AG, self.p)
            fb.flux_gemm_ref_chunked(fb.FLUX_OP_AG, self.p, A_chunks=self.chunks, A_agg=self.A_agg, B=self.next_B(),
                                     Cout=self.C, arrival_order=self.arrival, workspace=self.ws_chunk,
                                     compute_stream=compute, comm_stream=copy)

        def copy_upfront(self):
            # the same fused call with every remote chunk moved before the signal wait (only differs where
            # the library would carry the later chunks inside the first round's main loops)
            if not hasattr(self, "p_up"):
                w = self.w
                self.p_up = fb.problem(w.M, w.N, w.K, w.R, self.rank, "bf16", w.out_dtype, spin_timeout_ticks=TIMEOUT_TICKS,
                                       flags=fb.FLUX_FLAG_AG_COPY_UPFRONT)
            fb.flux_ag_gemm(self.p_up, self.chunks, self.A_agg, self.next_B(), self.C, self.signals, self.arrival,
                            self.ws, compute, copy)

        def b_as_n_by_k(self):
            # the same fused call with the weight handed over as [N,K] (a linear layer's own layout)
            if not hasattr(self, "p_nk"):
                w = self.w
                self.p_nk = fb.problem(w.M, w.N, w.K, w.R, self.rank, "bf16", w.out_dtype, spin_timeout_ticks=TIMEOUT_TICKS, b_is_nk=1)
                self.B_nk = self.B.t().contiguous()
            fb.flux_ag_gemm(self.p_nk, self.chunks, self.A_agg, self.B_nk, self.C, self.signals, self.arrival,
                            self.ws, compute, copy)

        def alg_bytes(self):     # fused kernel: A_agg + B read once, C written once; the default call has no
            w = self.w           # copy kernel, so the R-1 remote chunks are read and written by this kernel too
            return 2.0 * (w.M * w.K + w.K * w.N + w.M * w.N) + 2 * 2.0 * (w.R - 1) * w.S * w.K

    class RS(RotatingB):
        def __init__(self, w, rank, **kw):
            self.w, self.rank = w, rank
            self.A_cpu, self.B_cpu, self.peers_cpu = fi.make_rs_inputs(w, rank)
            self.p = fb.problem(w.M, w.N, w.K, w.R, rank, w.partial_dtype, w.out_dtype, **kw)
            self.A, self.B = self.A_cpu.to(dev), self.B_cpu.to(dev)
            self.peers = [None if t is None else t.to(dev) for t in self.peers_cpu]
            dt = torch.bfloat16 if w.out_dtype == "bf16" else torch.float32
            self.outs = [torch.zeros((w.S, w.N), dtype=dt, device=dev) for _ in range(w.R)]
            self.tmp = torch.zeros((w.M, w.N), dtype=dt, device=dev)
            n = fb.flux_workspace_bytes(fb.FLUX_OP_RS, self.p)
            self.ws = torch.zeros(n // 4 + 1, dtype=torch.int32, device=dev) if n else None
            if self.ws is not None:
                fb.flux_init_buffers(fb.FLUX_OP_RS, self.p, self.ws)

        def fused(self, stream=None):
            fb.flux_gemm_rs(self.p, self.A, self.next_B(), self.peers, self.outs, self.ws, stream or compute)

        def unfused(self, phases):
            fb.flux_gemm_ref_unfused(fb.FLUX_OP_RS, phases, self.p, A=self.A, B=self.next_B(), peer_partials=self.peers,
                                     out_slices=self.outs, Cout=self.tmp, workspace=self.ws, stream=compute)

        def chunked(self):
            if not hasattr(self, "ws_chunk"):
                self.ws_chunk = chunk_workspace(fb.FLUX_OP_RS, self.p)
            fb.flux_gemm_ref_chunked(fb.FLUX_OP_RS, self.p, A=self.A, B=self.next_B(), peer_partials=self.peers,
                                     out_slices=self.outs, Cout=self.tmp, workspace=self.ws_chunk,
                                     compute_stream=compute, comm_stream=copy)

        def alltoall_flavour(self):
            # Write branch + local reduction: what ONE rank of a real group does (its GEMM scattered
            # by owner, then the sum of the R partials staged for its own slice)
            if not hasattr(self, "p_wo"):
                w = self.w
                self.p_wo = fb.problem(w.M, w.N, w.K, w.R, self.rank, w.partial_dtype, w.out_dtype,
                                       flags=fb.FLUX_FLAG_RS_WRITE_ONLY)
                lo, hi = self.rank * w.S, (self.rank + 1) * w.S
                self.staged = [self.outs[self.rank] if j == self.rank else self.peers[j][lo:hi] for j in range(w.R)]
                self.own = torch.zeros_like(self.outs[self.rank])
            fb.flux_gemm_rs(self.p_wo, self.A, self.next_B(), None, self.outs, self.ws, compute)
            fb.flux_rs_reduce_slice(self.p_wo, self.staged, self.own, compute)

        def atomic_flavour(self):
            # Reduce by fp32 atomic additions into the owners' slices (Sec. 4.2, first form of Reduce)
            if not hasattr(self, "p_at"):
                w = self.w
                self.p_at = fb.problem(w.M, w.N, w.K, w.R, self.rank, "f32", "f32", flags=fb.FLUX_FLAG_RS_ATOMIC)
                self.outs_f32 = [torch.zeros((w.S, w.N), dtype=torch.float32, device=dev) for _ in range(w.R)]
                n = fb.flux_workspace_bytes(fb.FLUX_OP_RS, self.p_at)
                self.ws_at = torch.zeros(n // 4 + 1, dtype=torch.int32, device=dev) if n else None
                if self.ws_at is not None:
                    fb.flux_init_buffers(fb.FLUX_OP_RS, self.p_at, self.ws_at)
            fb.flux_gemm_rs(self.p_at, self.A, self.next_B(), None, self.outs_f32, self.ws_at, compute)

        def one_workgroup_per_tile(self):
            # the same fused call without the resident grid (only differs where the library plans one)
            if not hasattr(self, "p_1pt"):
                w = self.w
                self.p_1pt = fb.problem(w.M, w.N, w.K, w.R, self.rank, w.partial_dtype, w.out_dtype,
                                        flags=fb.FLUX_FLAG_NO_RESIDENT_GRID)
            fb.flux_gemm_rs(self.p_1pt, self.A, self.next_B(), self.peers, self.outs, self.ws, compute)

        def b_as_n_by_k(self):
            if not hasattr(self, "p_nk"):
                w = self.w
                self.p_nk = fb.problem(w.M, w.N, w.K, w.R, self.rank, w.partial_dtype, w.out_dtype, b_is_nk=1)
                self.B_nk = self.B.t().contiguous()
            fb.flux_gemm_rs(self.p_nk, self.A, self.B_nk, self.peers, self.outs, self.ws, compute)

        def alg_bytes(self):
            w = self.w
            ps = 2 if w.partial_dtype == "bf16" else 4
            os_ = 2 if w.out_dtype == "bf16" else 4
            return 2.0 * (w.M * w.K + w.K * w.N) + (w.R - 1) * w.M * w.N * ps + w.M * w.N * os_

    def time_calls(fn, reps, warm, batch=8):
        """Median time per call (ms), measured with events on the compute stream around `batch` calls
        enqueued back to back: the steady state of a stream that is kept fed (the way an operator runs
        inside a model), not the latency of one call on an idle device."""
        t_w = time.perf_counter()
        while time.perf_counter() - t_w < 0.3:      # keep the clocks where sustained load puts them
            fn()
            torch.cuda.synchronize()
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0, e1 = fb.HipEvent(), fb.HipEvent()
            e0.record(compute)
            for _ in range(batch):
                fn()
            e1.record(compute)
            e1.synchronize()
            ts.append(e0.elapsed_ms(e1) / batch)
        return statistics.median(ts)

    def overlap_block(op, reps=20, warm=5, graph=False, nk=False):
        """Eq. 1-2 with GEMM_non-split := the plain kernel of the same tile configuration."""
        t_gemm = time_calls(lambda: op.unfused(fb.FLUX_PHASE_GEMM), reps, warm)
        t_comm = time_calls(lambda: op.unfused(fb.FLUX_PHASE_COMM), reps, warm)
        t_unf = time_calls(lambda: op.unfused(fb.FLUX_PHASE_GEMM | fb.FLUX_PHASE_COMM), reps, warm)
        t_fus = time_calls(op.fused, reps, warm)
        t_chk = time_calls(op.chunked, reps, warm)      # medium-grained: R GEMMs, communication beside the next one
        # duration of the fused GEMM kernel alone (events recorded by the library around its
        # launch): what the per-kernel roofline figures use; the per-call times above also carry
        # what is left of launch and cross-stream latencies in a stream that is kept fed
        ks = []
        for _ in range(reps):
            k0, k1 = fb.HipEvent(), fb.HipEvent()
            fb.flux_profile_next_gemm(k0, k1)
            op.fused()
            torch.cuda.synchronize()
            ks.append(k0.elapsed_ms(k1))
        t_k = statistics.median(ks)
        t_a2a = time_calls(op.alltoall_flavour, reps, warm) if hasattr(op, "alltoall_flavour") else None
        t_atomic = time_calls(op.atomic_flavour, reps, warm) if hasattr(op, "atomic_flavour") else None
        # the same fused call recorded once in a HIP graph (8 calls per graph) and replayed: what a
        # serving loop that cannot afford per-call launch work would run
        t_graph = None
        if graph:
            side = torch.cuda.Stream()
            side.wait_stream(compute)
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for _ in range(8):
                    op.fused(torch.cuda.current_stream())
            torch.cuda.synchronize()
            t_graph = time_calls(g.replay, reps, warm, batch=1) / 8
            del g
        ect_no, ect_ov = t_unf - t_gemm, t_fus - t_gemm
        E = 1.0 - ect_ov / ect_no if ect_no > 0 else None
        w = op.w
        more = {} if t_a2a is None else {"ms_write_only_plus_slice_reduce": round(t_a2a, 4)}
        if t_graph is not None:
            more["ms_fused_graph_replay"] = round(t_graph, 4)
        if t_atomic is not None:
            more["ms_atomic_reduce_f32"] = round(t_atomic, 4)
        if hasattr(op, "copy_upfront") and op.p.flags == 0 and op.p.link_gbps == 0 and fb.flux_ag_deferred_tiles(op.p) > 0:
            more["chunks_moved_inside_main_loops"] = fb.flux_ag_deferred_tiles(op.p)
            more["ms_fused_all_chunks_up_front"] = round(time_calls(op.copy_upfront, reps, warm), 4)
        if hasattr(op, "one_workgroup_per_tile") and fb.flux_rs_resident_grid(op.p)[0] > 0:
            more["resident_grid"] = dict(zip(("workgroups", "late_start_ticks_100MHz"), fb.flux_rs_resident_grid(op.p)))
            more["ms_fused_one_workgroup_per_tile"] = round(time_calls(op.one_workgroup_per_tile, reps, warm), 4)
        if nk:
            more["ms_fused_b_as_n_by_k"] = round(time_calls(op.b_as_n_by_k, reps, warm), 4)
        return {**more, "ms_gemm_only": round(t_gemm, 4), "ms_comm_only": round(t_comm, 4), "ms_unfused": round(t_unf, 4),
                "ms_fused": round(t_fus, 4), "ms_fused_kernel": round(t_k, 4), "ms_chunked": round(t_chk, 4),
                "overlap_efficiency_chunked": None if ect_no <= 0 else round(1.0 - (t_chk - t_gemm) / ect_no, 4),
                "kernel_alg_GBs": round(op.alg_bytes() / t_k / 1e6, 1),
                "kernel_frac_hbm_peak": round(op.alg_bytes() / t_k / 1e6 / HBM_PEAK_GBS, 4),
                "kernel_tflops": round(w.flops / t_k / 1e9, 1),
                "overlap_efficiency": None if E is None else round(E, 4),
                "fused_tflops": round(w.flops / t_fus / 1e9, 1),
                "fused_frac_mfma_peak": round(w.flops / t_fus / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                "fused_alg_GBs": round(op.alg_bytes() / t_fus / 1e6, 1),
                "fused_frac_hbm_peak": round(op.alg_bytes() / t_fus / 1e6 / HBM_PEAK_GBS, 4)}

    if args.serial_decode > 0:
        # per few-row shape: N plain GEMMs (no communication), then N fused AllGather-GEMM calls, then N
        # fused GEMM-ReduceScatter calls, each over rotating copies of the weight matrix; synchronised
        # between the groups so that a trace shows them apart
        for m in (8, 64, 256):
            ag_op = AG(W[f"c5_ag_m{m}"], 2)
            ag_op.rotate_weights(9)
            for _ in range(args.serial_decode):
                ag_op.unfused(fb.FLUX_PHASE_GEMM)
            torch.cuda.synchronize()
            for _ in range(args.serial_decode):
                ag_op.fused()
            torch.cuda.synchronize()
            del ag_op
            rs_op = RS(W[f"c5_rs_m{m}"], 2)
            rs_op.rotate_weights(9)
            for _ in range(args.serial_decode):
                rs_op.fused()
            torch.cuda.synchronize()
            del rs_op
        print(json.dumps({"mode": "serial-decode", "launches_per_shape_and_kind": args.serial_decode,
                          "order": "per M in (8, 64, 256): plain GEMM (AllGather shape), fused AllGather-GEMM, fused GEMM-ReduceScatter"}))
        return 0

    # ---- the timed workload: QKV projection (AG-GEMM) + attention output projection (GEMM-RS) ----
    say("generating the inputs of c4_ag and c4_rs")
    ag = AG(W["c4_ag"], rank=2, flags=args.ag_flags)
    rs = RS(W["c4_rs"], rank=2)
    flops_step = ag.w.flops + rs.w.flops

    if args.serial_kernels > 0:
        for _ in range(args.serial_kernels):
            ag.unfused(fb.FLUX_PHASE_COMM)      # plain copy of 7 chunks: 176.2 MB read + 176.2 MB written
            ag.unfused(fb.FLUX_PHASE_GEMM)      # same tile configuration as the fused kernel, no signal wait
            rs.fused()
            # the fused AllGather call also completes when its two kernels cannot overlap: whichever
            # runs first, the GEMM's waiting workgroups move what the copy driver has not
            ag.fused()
            torch.cuda.synchronize()
        print(json.dumps({"mode": "serial-kernels", "rounds": args.serial_kernels,
                          "copy_bytes_read": 7 * ag.w.S * ag.w.K * 2, "copy_bytes_written": 7 * ag.w.S * ag.w.K * 2}))
        return 0

    def step(prof=None):
        if prof is not None:
            fb.flux_profile_next_gemm(prof[0], prof[1])
        ag.fused()
        if prof is not None:
            fb.flux_profile_next_gemm(prof[2], prof[3])
        rs.fused()

    say("clock ramp, warm-up and timed steps")
    # clock ramp: the engine clock takes about a second of sustained load to leave its idle
    # state and settle at the power-limited level; the W warm-up steps come after that
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < args.ramp_seconds:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # The kernels' own durations come from HIP events the library records around their launches, on
    # every `event_every`-th step of the timed region: four event records per step cost about 12 us
    # of a 500 us step (measured), which is the step's time, not the kernels'.
    every = max(1, args.event_every)
    profs = [[fb.HipEvent() for _ in range(4)] if i % every == 0 else None for i in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(profs[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = flops_step / (ms_per_step * 1e-3) / 1e12
    ag_ms = statistics.mean(p[0].elapsed_ms(p[1]) for p in profs if p is not None)
    rs_ms = statistics.mean(p[2].elapsed_ms(p[3]) for p in profs if p is not None)
    status = fb.flux_query_status(ag.ws)
    if status[0] != fb.FLUX_OK:
        print(f"bench.py: AllGather-GEMM reported status {status}", file=sys.stderr)
        return 1

    say(f"timed region done: {ms_per_step:.4f} ms per step; spot check against the oracle")
    # spot check against the oracle on a few rows (outside the timed region)
    from oracle import flux_oracle as fo
    rows = [0, 1023, 1024, 4095, 8191]
    ref = fo.ag_gemm_rows([fi.to_numpy(c) for c in ag.chunks_cpu], fi.to_numpy(ag.B_cpu), rows)
    got = ag.C[rows].float().cpu().double().numpy()
    ok_ag = bool(np.all(np.abs(got - ref) <= 1e-2 * np.maximum(1.0, np.abs(ref))))
    refr = fo.gemm_rs_rows(fi.to_numpy(rs.A_cpu), fi.to_numpy(rs.B_cpu),
                           [None if t is None else fi.to_numpy(t) for t in rs.peers_cpu], rs.w.R, rs.rank,
                           rs.w.partial_dtype, rows)
    ok_rs = all(bool(np.all(np.abs(rs.outs[o][lr].float().cpu().double().numpy() - v) <= 1e-2 * np.maximum(1.0, np.abs(v))))
                for o, lr, v in refr)
    if not (ok_ag and ok_rs):
        print("bench.py: result check against the CPU oracle FAILED", file=sys.stderr)
        return 1

    # Traffic behind the L2 per launch, from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) of
    # `bench.py --serial-kernels 5`, each scaled by what the same counter reads for the 176.2 MB chunk
    # copy of the same run (1.9986 and 1.0000 KiB per count); profiles/bench_c4_pmc_traffic.txt.
    traffic = TRAFFIC_BYTES
    alg = {"rs": rs.alg_bytes(), "ag": ag.alg_bytes()}

    def kernel_line(name, which, w, ms, bound):
        tf = w.flops / (ms * 1e-3) / 1e12
        gbs = alg[which] / ms / 1e6
        line = {"kernel": name, "bound": bound}
        if bound == "mfma":
            line.update({"achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4)})
        else:
            line.update({"achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4)})
        line.update({"traffic": traffic[which],
                     "traffic_note": "bytes per launch requested by the L2s from Infinity Cache/HBM; algorithmic %.1fe6"
                                     % (alg[which] / 1e6),
                     "avg_kernel_ms": round(ms, 4), "tflops": round(tf, 1), "frac_mfma": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                     "alg_GBs": round(gbs, 1), "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)})
        return line

    # The roofline line is for the kernel of the step that takes longer, each against the roof that
    # binds it: the AllGather-GEMM (927.7 GFLOP over 390 MB + 352 MB gathered: MFMA), the
    # GEMM-ReduceScatter of this shape (309 GFLOP over 1673.5 MB: 123 us of MFMA work against
    # 209 us of memory traffic at peak: HBM).  The other one follows as "second_kernel".
    lines = [kernel_line("GEMM kernel <ReduceScatter epilogue> on c4_rs", "rs", rs.w, rs_ms, "hbm"),
             kernel_line("GEMM kernel <AllGather prologue> on c4_ag", "ag", ag.w, ag_ms, "mfma")]
    lines.sort(key=lambda d: -d["avg_kernel_ms"])
    roofline = dict(lines[0])
    roofline["second_kernel"] = lines[1]

    extra = {}
    if not args.no_extra:
        say("extra: c4_ag")
        extra["c4_ag"] = overlap_block(ag, nk=True)
        say("extra: c4_rs")
        extra["c4_rs"] = overlap_block(rs, nk=True)
        say("extra: vendor library GEMM on the same operands")
        # Context, not a target and not part of the path: the vendor library's plain GEMM (hipBLASLt
        # behind torch.matmul) on the same operands, and on zeros.  With normally distributed operands
        # the chip runs into its power limit and every GEMM, this one included, slows down by a
        # fifth or so; the MFMA peak is not reachable on such data by any kernel.
        lib = {}
        for key, A_, B_ in (("c4_ag", ag.A_agg, ag.B), ("c4_rs", rs.A, rs.B)):
            out_ = torch.empty((A_.shape[0], B_.shape[1]), dtype=torch.bfloat16, device=dev)
            fl = 2.0 * A_.shape[0] * A_.shape[1] * B_.shape[1]
            t_data = time_calls(lambda: torch.matmul(A_, B_, out=out_), 20, 5)
            Az, Bz = torch.zeros_like(A_), torch.zeros_like(B_)
            t_zero = time_calls(lambda: torch.matmul(Az, Bz, out=out_), 20, 5)
            lib[key] = {"ms_workload_operands": round(t_data, 4), "tflops_workload_operands": round(fl / t_data / 1e9, 1),
                        "ms_zero_operands": round(t_zero, 4), "tflops_zero_operands": round(fl / t_zero / 1e9, 1)}
            del Az, Bz, out_
        extra["library_gemm_context"] = lib
        # Eq. 1-2 once more with GEMM_non-split := the faster of this library's plain kernel and the
        # vendor library's GEMM on the same operands (the paper takes the fastest GEMM known)
        for key in ("c4_ag", "c4_rs"):
            tg = min(extra[key]["ms_gemm_only"], lib[key]["ms_workload_operands"])
            ect_no = extra[key]["ms_unfused"] - tg
            extra[key]["overlap_efficiency_vs_fastest_gemm"] = (
                None if ect_no <= 0 else round(1.0 - (extra[key]["ms_fused"] - tg) / ect_no, 4))
        del ag, rs
        torch.cuda.empty_cache()
        for name in ("c2_ag", "c3_rs", "c5_ag_m64", "c5_rs_m64", "c5_ag_m8", "c5_rs_m8", "c5_ag_m256", "c5_rs_m256"):
            say(f"extra: {name}")
            op = AG(W[name], 2) if W[name].op == "ag" else RS(W[name], 2)
            if name.startswith("c5"):
                op.rotate_weights(9)        # 9 x 58.7 MB = 528 MB, twice the Infinity Cache
            extra[name] = overlap_block(op, reps=20 if not name.startswith("c5") else 50, graph=name.startswith("c5"))
            del op
            torch.cuda.empty_cache()
        # The tuner (Sec. 4.4) on three shapes: what it picks and what that gains over the library's own choice
        tuned = {}
        for name in ("c4_ag", "c4_rs", "op_ag_m2048", "op_rs_m2048", "c5_ag_m64", "c5_rs_m64", "c5_ag_m256"):
            w = W[name]
            say(f"extra: tuner on {name}")
            if w.op == "ag":
                op = AG(w, 2)
                op.signals = torch.zeros(fb.flux_autotune_signal_count(op.p), dtype=torch.int32, device=dev)
                op.ws = torch.zeros(fb.flux_autotune_workspace_bytes(fb.FLUX_OP_AG, op.p) // 4 + 1, dtype=torch.int32, device=dev)
                t, ms_best, ms_def = fb.flux_autotune_ag(op.p, op.chunks, op.A_agg, op.B, op.C, op.signals, op.arrival,
                                                         op.ws, compute, copy, reps=5)
            else:
                op = RS(w, 2)
                n = fb.flux_autotune_workspace_bytes(fb.FLUX_OP_RS, op.p)
                op.ws = torch.zeros(n // 4 + 1, dtype=torch.int32, device=dev) if n else None
                t, ms_best, ms_def = fb.flux_autotune_rs(op.p, op.A, op.B, op.peers, op.outs, op.ws, compute, reps=5)
            tuned[name] = {"tile_config": t.tile_config, "split_k": t.split_k, "comm_tiles_per_chunk": t.comm_tiles_per_chunk,
                           "flags": int(t.flags), "ms_tuned": round(ms_best, 4), "ms_library_pick": round(ms_def, 4)}
            del op
            torch.cuda.empty_cache()
        extra["autotune"] = tuned
        # Second workload: the paper's op-level sweep (Sec. 5.1), GPT-3-175B MLP shapes at TP=8
        sweep = {}
        for name in ("op_ag_m8", "op_rs_m8", "op_ag_m64", "op_rs_m64",
                     "op_ag_m512", "op_rs_m512", "op_ag_m2048", "op_rs_m2048", "op_ag_m8192", "op_rs_m8192"):
            say(f"extra: op-level sweep {name}")
            op = AG(W[name], 2) if W[name].op == "ag" else RS(W[name], 2)
            if W[name].M <= 64:
                op.rotate_weights(3)        # 3 x 151 MB: a decode step never finds its weights in the Infinity Cache
            sweep[name] = overlap_block(op, reps=10 if W[name].M > 64 else 30, warm=3)
            del op
            torch.cuda.empty_cache()
        extra["op_level_sweep"] = sweep
        # Secondary, labelled: the transfer paced to an inbound link of 7 x 153 GB/s (what one rank
        # of an 8-GPU xGMI mesh receives), so that communication is a paper-like fraction of the GEMM
        # time; communication tile = chunk / ctpc (Sec. 4.3), swizzle on and off.  Without a driver
        # (the grid carries the tiles itself and counts them in on the link's schedule), and for
        # comparison with the paced copy kernel as driver (54 workgroups move 1071 GB/s).
        link = {}
        for name, variants in (("c4_ag", ((1, 0, 0), (2, 0, 0), (4, 0, 0), (2, fb.FLUX_FLAG_NO_SWIZZLE, 0), (1, 0, 54))),
                               ("c2_ag", ((1, 0, 0), (2, 0, 0)))):
            for ctpc, flags, driver in variants:
                op = AG(W[name], 2, link_gbps=1071, comm_tiles_per_chunk=ctpc, flags=flags, copy_workgroups=driver)
                key = f"{name}_ctpc{ctpc}" + ("_noswizzle" if flags else "") + (f"_driver{driver}" if driver else "")
                say(f"extra: link-paced {key}")
                link[key] = overlap_block(op)
                link[key]["tiles_carried_by_the_grid"] = fb.flux_ag_deferred_tiles(op.p)
                del op
                torch.cuda.empty_cache()
        extra["link_paced_1071GBps"] = link
        # The SDMA-style driver of Alg. 3: hipMemcpyAsync per communication tile plus a stream write of its
        # signal on the copy stream, the GEMM grid only waits (no workgroup moves data)
        mc = {}
        for name in ("c2_ag", "c4_ag"):
            say(f"extra: memcpy driver {name}")
            op = AG(W[name], 2, flags=fb.FLUX_FLAG_COPY_MEMCPY)
            mc[name] = {"ms_fused": round(time_calls(op.fused, 20, 5), 4)}
            del op
            torch.cuda.empty_cache()
        extra["copy_memcpy_driver"] = mc
    cpu_baseline = None
    if not args.no_cpu_baseline:
        say("cpu baseline: the oracle on whole steps of the same workload")
        # the oracle as it stands, on the host cores: full AllGather-GEMM of the timed shape
        try:
            from threadpoolctl import threadpool_info
            cores = max([d.get("num_threads", 1) for d in threadpool_info()] + [1])
        except Exception:
            cores = len(os.sched_getaffinity(0))
        # one step of the same workload (c4_ag AllGather-GEMM, then c4_rs GEMM-ReduceScatter with its
        # 7 peer partials), whole matrices, repeated until about 10 s of CPU time have gone by
        wa, wr = W["c4_ag"], W["c4_rs"]
        chunks, Ba, _ = fi.make_ag_inputs(wa, 2)
        cn, Ban = [fi.to_numpy(c) for c in chunks], fi.to_numpy(Ba)
        Ar, Br, peers = fi.make_rs_inputs(wr, 2)
        Arn, Brn = fi.to_numpy(Ar), fi.to_numpy(Br)
        pn = [None if t is None else fi.to_numpy(t) for t in peers]
        reps, t0 = 0, time.perf_counter()
        while True:
            fo.ag_gemm(cn, Ban, wa.out_dtype)
            fo.gemm_rs(Arn, Brn, pn, wr.R, 2, wr.partial_dtype, wr.out_dtype)
            reps += 1
            dt = time.perf_counter() - t0
            if dt >= 10.0 or reps >= 50:
                break
        cpu_baseline = {"value": round(reps * (wa.flops + wr.flops) / dt / 1e12, 4), "unit": "TFLOP/s",
                        "cores": cores, "kind": "oracle",
                        "sample": f"{reps} whole steps of the timed workload (oracle ag_gemm on c4_ag + gemm_rs on c4_rs, "
                                  f"fp64 numpy) in {dt:.1f} s"}

    out = {
        "metric": "fused GEMM-RS/AG-GEMM TFLOP/s (% MFMA peak) + % comm time hidden, 1 MI355X",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c4_ag + c4_rs: GPT-3-175B-like layer at TP=8, 8192 tokens - fused AllGather-GEMM "
                               "[8x1024,12288]x[12288,4608] then fused GEMM-ReduceScatter [8192,1536]x[1536,12288] + 7 peers",
                   "virtual_ranks": 8, "rank": 2, "frac_mfma_peak": round(value / MFMA_BF16_PEAK_TFLOPS, 4)},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "extra": extra,
    }
    say("done")
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
