#!/usr/bin/env python3
"""Benchmark of the vector-LUT ternary x INT8 mpGeMM hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: per-token INT8 quantisation of the fp32 activations, streamed LDS table build,
lookup-accumulate and scale epilogue, through vlut_mpgemm_f32 (which runs the quantisation inside the
lookup kernel or as a kernel of its own ahead of it, whichever its cost model prefers for the shape; the
two-call form vlut_quantize_act + vlut_mpgemm is timed next to it).  Weight packing is the paper's
offline stage and is not timed.  The packed weights rotate through a pool larger than the last-level
cache, so every step streams its weights from HBM.

Default run (`python bench.py [--gpus 1 --steps K --warmup W]`): every benchmark shape is timed -- the
2B FFN up projection at N = 128, the 3B up/down projections at N = 256, the 8B linears at N = 512 and the
seven linears of one 2.4B-style decoder layer at N in {1, 16, 64, 256, 1024} (plus the layer as four stacked
launches from fp32 inputs) -- and reported under `sweep` / `layer`, one entry per (shape, N) with its time, GOPS,
weight-stream GB/s, the roof that binds it and the fraction of that roof.  The headline (`value`,
`ms_per_step`, `roofline`, `cpu_baseline`) is the largest single-GPU shape, the 8B gate/up projection
M = 14336, K = 4096, N = 512.  `--workload/--linear/--tokens` pick another headline; `--no-sweep` times the
headline only (the form the rocprofv3 summaries under profiles/ use).

Timing: K = --steps launches are captured into one HIP graph; after W warm-up calls and one untimed replay
(clock ramp) the graph is replayed REPS >= 10 times, each replay bracketed by a device synchronise and by HIP
events on the launch stream; the figures are medians over the replays.

Prints ONE JSON line on stdout; a per-shape table goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X published peaks used for the roofline fractions
HBM_PEAK_GBS = 8000.0
CUS, CLOCK_GHZ = 256, 2.4
# packed INT16 adds: 64 lanes x 2 per CU per clock; table reads: 256 B per CU per clock (2 B per add)
ALU_PEAK_TADDS = CUS * 64 * 2 * CLOCK_GHZ / 1e3          # 78.64 T INT16 adds/s
LDS_PEAK_GBS = CUS * 256 * CLOCK_GHZ                      # 157286 GB/s
# what microbenchmarks reach on this device: 240 B/clk/CU of conflict-free 16-byte table reads at the ~2.1 GHz the
# shader clock holds under this load
LDS_MEASURED_PEAK_GBS = CUS * 240 * 2.1                   # 129024 GB/s
MFMA_INT8_PEAK_TOPS = 5000.0                              # dense INT8 matrix-core peak (the comparison kernel's roof)

# HBM bytes per launch of the lookup kernel measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), see profiles/
MEASURED_TRAFFIC_BYTES = {
    "llama8b_linears/gateup/512": 75.8e6,  # profiles/lookup_kernel_llama8b_gateup_n512_stats_sq_counters_hbm_traffic.md
    "bitnet3b_prefill/up/256": 22.6e6,     # profiles/lookup_kernel_bitnet3b_up_n256_stats_sq_counters_hbm_traffic.md
    "bitnet2b_ffn_up/up/128": 10.85e6,     # profiles/lookup_kernel_bitnet2b_ffn_up_n128_stats_sq_counters_hbm_traffic.md
    "layer2b4_nsweep/gate/16": 6.33e6,     # profiles/layer2b4_gate_n16_kernel_stats_hbm_traffic.md
    "layer2b4_nsweep/gate/1": 4.66e6,      # profiles/narrow_kernel_layer2b4_gate_n1_stats_and_hbm_traffic.md
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama8b_linears")
    ap.add_argument("--linear", default="", help="linear of the workload (default: gateup for the 8B linears, else its first)")
    ap.add_argument("--tokens", type=int, default=0, help="N of the workload's sweep (default: its first)")
    ap.add_argument("--reps", type=int, default=int(os.environ.get("VLUT_BENCH_REPS", "12")),
                    help="timed replays of the captured graph per figure (median reported; at least 10)")
    ap.add_argument("--no-sweep", action="store_true", help="time the headline shape only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-rotate", action="store_true", help="keep one weight buffer (cache-warm weights)")
    ap.add_argument("--all", action="store_true", help="kept for compatibility: the sweep is the default now")
    ap.add_argument("--plan", default="", help="force J,R,S for the lookup kernel (tuning)")
    ap.add_argument("--layer", action="store_true",
                    help="also time one decoder layer's seven linears at every N of the sweep: one launch per linear "
                         "against stacked launches (q/k/v and gate/up share their input and their tables)")
    ap.add_argument("--ablation", action="store_true",
                    help="also time the un-streamed variant (table materialised in HBM by vlut_build_lut, then read "
                         "by vlut_mpgemm) against the streamed default, Sec. 5.6 of the paper (table on stderr)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 64 MiB device-to-device copy (known size: the reference a rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE run of this command is scaled by)")
    return ap.parse_args()


class Case:
    """Device-resident tensors of one linear layer at one N, with the C-ABI calls pre-marshalled."""

    def __init__(self, B, torch, wl, W, w_scale, x, rotate_bytes, w_rows=None):
        self.M, self.K = W.shape
        self.N = x.shape[0]
        self.w_scale = float(w_scale)
        packed = B.pack_weights(torch.from_numpy(W).cuda())
        n_pool = 1 if rotate_bytes <= 0 else max(1, min(256, -(-rotate_bytes // packed.numel())))
        self.pool = [packed] + [packed.clone() for _ in range(n_pool - 1)]
        self.x = torch.from_numpy(x).cuda()
        self.a_q = torch.empty(((self.N + 7) // 8, self.K, 8), dtype=torch.int8, device="cuda")
        self.a_s = torch.empty(self.N, dtype=torch.float32, device="cuda")
        self.y = torch.empty((self.N, self.M), dtype=torch.float32, device="cuda")
        ws = B.workspace_bytes(self.M, self.K, self.N)
        self.ws = torch.empty(max(ws, 16), dtype=torch.uint8, device="cuda")
        self.plan = B.query_plan(self.M, self.K, self.N)
        L = B.lib()
        self._check = B._check
        self._quant = L.vlut_quantize_act
        self._gemm = L.vlut_mpgemm
        self._qargs = (self.x.data_ptr(), self.N, self.K, self.x.stride(0), self.a_q.data_ptr(), self.a_s.data_ptr())
        # stacked matrices (one launch for several projections of the same input): per-row weight scales
        self.w_rows = None if w_rows is None else torch.from_numpy(w_rows).cuda()
        if self.w_rows is not None:
            self._gemm = L.vlut_mpgemm_rows
        first = self.w_scale if self.w_rows is None else self.w_rows.data_ptr()
        self._gargs = [(pk.data_ptr(), first, self.a_q.data_ptr(), self.a_s.data_ptr(), None, self.M, self.K,
                        self.N, self.y.data_ptr(), self.y.stride(0), None, self.ws.data_ptr(), self.ws.numel())
                       for pk in self.pool]
        # the in-run comparison path (INT8 matrix cores) with its own scratch
        self._mfma = L.vlut_mpgemm_mfma
        self.mws = torch.empty(max(L.vlut_mfma_workspace_bytes(self.M, self.K, self.N), 16), dtype=torch.uint8, device="cuda")
        self._margs = [(pk.data_ptr(), self.w_scale, self.a_q.data_ptr(), self.a_s.data_ptr(), None, self.M, self.K,
                        self.N, self.y.data_ptr(), self.y.stride(0), None, self.mws.data_ptr(), self.mws.numel())
                       for pk in self.pool]

        # quantisation fused into the lookup kernel: fp32 activations in, one launch per step
        self._f32 = L.vlut_mpgemm_f32
        self.ws32 = torch.empty(max(L.vlut_workspace_bytes_f32(self.M, self.K, self.N), 16), dtype=torch.uint8, device="cuda")
        self.plan32 = B.query_plan_f32(self.M, self.K, self.N)
        rows_ptr = None if self.w_rows is None else self.w_rows.data_ptr()
        self._fargs = [(pk.data_ptr(), self.w_scale, rows_ptr, self.x.data_ptr(), self.x.stride(0), self.M, self.K, self.N,
                        self.y.data_ptr(), self.y.stride(0), None, None, self.ws32.data_ptr(), self.ws32.numel())
                       for pk in self.pool]

    def step_fused(self, i, stream):
        self._check(self._f32(*self._fargs[i % len(self._fargs)], stream), "vlut_mpgemm_f32")

    def enable_g5(self, B, torch, W, rotate_bytes):
        """Adds the 1.60-bit blob of the same weights (K % 20 == 0 only) and pre-marshals vlut_mpgemm_g5."""
        L = B.lib()
        packed = B.pack_weights_g5(torch.from_numpy(W).cuda())
        n_pool = 1 if rotate_bytes <= 0 else max(1, min(256, -(-rotate_bytes // packed.numel())))
        self.pool5 = [packed] + [packed.clone() for _ in range(n_pool - 1)]
        ws = L.vlut_workspace_bytes_g5(self.M, self.K, self.N)
        self.ws5 = torch.empty(max(ws, 16), dtype=torch.uint8, device="cuda")
        self.plan5 = B.query_plan_g5(self.M, self.K, self.N)
        self._gemm5 = L.vlut_mpgemm_g5
        self._g5args = [(pk.data_ptr(), self.w_scale, self.a_q.data_ptr(), self.a_s.data_ptr(), self.M, self.K, self.N,
                         self.y.data_ptr(), self.y.stride(0), None, self.ws5.data_ptr(), self.ws5.numel())
                        for pk in self.pool5]

    def enable_mixed(self, B, torch, W, rotate_bytes):
        """Adds the blob of the mixed 1.60-bit / 2-bit packing of the same weights and pre-marshals vlut_mpgemm_mixed."""
        L = B.lib()
        packed = B.pack_weights_mixed(torch.from_numpy(W).cuda())
        n_pool = 1 if rotate_bytes <= 0 else max(1, min(256, -(-rotate_bytes // packed.numel())))
        self.poolx = [packed] + [packed.clone() for _ in range(n_pool - 1)]
        self.wsx = torch.empty(max(L.vlut_workspace_bytes_mixed(self.M, self.K, self.N), 16), dtype=torch.uint8, device="cuda")
        self._gemmx = L.vlut_mpgemm_mixed
        self._gxargs = [(pk.data_ptr(), self.w_scale, self.a_q.data_ptr(), self.a_s.data_ptr(), self.M, self.K, self.N,
                         self.y.data_ptr(), self.y.stride(0), None, self.wsx.data_ptr(), self.wsx.numel())
                        for pk in self.poolx]

    def gemm_mixed(self, i, stream):
        self._check(self._gemmx(*self._gxargs[i % len(self._gxargs)], stream), "vlut_mpgemm_mixed")

    def gemm_g5(self, i, stream):
        self._check(self._gemm5(*self._g5args[i % len(self._g5args)], stream), "vlut_mpgemm_g5")

    def quantize(self, stream):
        self._check(self._quant(*self._qargs, stream), "vlut_quantize_act")

    def gemm(self, i, stream):
        self._check(self._gemm(*self._gargs[i % len(self._gargs)], stream), "vlut_mpgemm")

    def gemm_mfma(self, i, stream):
        self._check(self._mfma(*self._margs[i % len(self._margs)], stream), "vlut_mpgemm_mfma")

    def step(self, i, stream):
        self.quantize(stream)
        self.gemm(i, stream)


REPS = 12


def run_timed(torch, fn, count, warmup, use_graph=True):
    """Times `count` calls of fn(i, stream) that are enqueued back to back.

    The calls are captured once into a HIP graph (so the host's launch cost is not part of the GPU timeline); after
    `warmup` direct calls and one untimed replay the graph is replayed REPS times, each replay between two device
    synchronisations and two HIP events recorded on the launch stream.  If capture is not possible the calls are
    enqueued directly.  Returns (median wall ms per call, median GPU ms per call from the events, launch mode)."""
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for i in range(warmup):
            fn(i, side.cuda_stream)
    side.synchronize()
    graph = None
    try:
        if not use_graph:
            raise RuntimeError("stream launches requested")
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for i in range(count):
                fn(i, torch.cuda.current_stream().cuda_stream)
        graph = g
    except Exception as e:  # noqa: BLE001 - fall back to plain stream launches
        if use_graph:
            print(f"bench.py: graph capture unavailable ({type(e).__name__}: {e}); timing stream launches", file=sys.stderr)
    walls, gpus = [], []
    with torch.cuda.stream(side):
        if graph is not None:
            graph.replay()          # untimed replay: first-use costs of the graph itself, clocks back up
        for _ in range(max(1, REPS)):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e0.record(side)
            if graph is not None:
                graph.replay()
            else:
                for i in range(count):
                    fn(i, side.cuda_stream)
            e1.record(side)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            walls.append((t1 - t0) * 1e3 / count)
            gpus.append(e0.elapsed_time(e1) / count)
    return float(np.median(walls)), float(np.median(gpus)), ("hipGraph" if graph is not None else "stream")


def time_case(B, torch, case, steps, warmup):
    """(wall ms per whole step through vlut_mpgemm_f32, GPU ms per launch of the dominant kernel, launch mode, wall ms
    per step of the two-call form, GPU ms per vlut_mpgemm launch).  The dominant kernel is the lookup kernel: when
    the step is one fused launch its time is the step's own GPU time (HIP events on the launch stream), otherwise it
    comes from a timed region that holds only the vlut_mpgemm launches, after quantising once."""
    # The device clocks fall while the host prepares a case; whichever region is timed first would pay for the ramp.
    # One untimed pass of the same steps brings them back before any figure is taken.
    run_timed(torch, case.step_fused, steps, warmup)
    ms_step, ms_step_gpu, mode = run_timed(torch, case.step_fused, steps, warmup)
    ms_two, _, _ = run_timed(torch, case.step, steps, warmup)
    _, ms_gemm, _ = run_timed(torch, case.gemm, steps, warmup)
    one_launch = case.plan32[4] and case.plan32[2] == 1
    return ms_step, (ms_step_gpu if one_launch else ms_gemm), mode, ms_two, ms_gemm


def time_mfma(torch, case, steps, warmup):
    """GPU ms per vlut_mpgemm_mfma call (activation re-layout + INT8 matrix-core GEMM), same inputs."""
    _, ms, _ = run_timed(torch, case.gemm_mfma, steps, warmup)
    return ms


def time_ablation(B, torch, case, steps, warmup):
    """Streamed (tables built in LDS on the fly) against materialised (whole table written to HBM, then read back
    tile by tile), and the materialised table token-contiguous (the method's layout) against token-outermost (one
    table per token, one value per lookup): the ablations of Sec. 5.6.  Returns GPU ms per call: streamed mpgemm,
    build_lut + mpgemm(lut), mpgemm(lut) alone, build + mpgemm on the token-outermost table, that mpgemm alone."""
    L = B.lib()
    lut = torch.empty(L.vlut_lut_bytes(case.K, case.N) // 2, dtype=torch.int16, device="cuda")
    bargs = (case.a_q.data_ptr(), case.K, case.N, lut.data_ptr(), lut.numel() * 2)
    largs = [a[:4] + (lut.data_ptr(),) + a[5:] for a in case._gargs]

    def build(i, stream):
        case._check(L.vlut_build_lut(*bargs, stream), "vlut_build_lut")

    def gemm_lut(i, stream):
        case._check(case._gemm(*largs[i % len(largs)], stream), "vlut_mpgemm")

    def both(i, stream):
        build(i, stream)
        gemm_lut(i, stream)

    case.quantize(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    _, t_stream, _ = run_timed(torch, case.gemm, steps, warmup)
    y_streamed = case.y.clone()
    _, t_both, _ = run_timed(torch, both, steps, warmup)
    if not torch.equal(y_streamed, case.y):
        print("bench.py: the un-streamed variant disagrees with the streamed one", file=sys.stderr)
        sys.exit(4)
    _, t_lut, _ = run_timed(torch, gemm_lut, steps, warmup)

    oargs = [(a[0], a[1], case.a_s.data_ptr(), lut.data_ptr(), case.M, case.K, case.N, case.y.data_ptr(), case.y.stride(0),
              None) for a in case._gargs]

    def build_outer(i, stream):
        case._check(L.vlut_build_lut_token_outer(*bargs, stream), "vlut_build_lut_token_outer")

    def gemm_outer(i, stream):
        case._check(L.vlut_mpgemm_token_outer(*oargs[i % len(oargs)], stream), "vlut_mpgemm_token_outer")

    def both_outer(i, stream):
        build_outer(i, stream)
        gemm_outer(i, stream)

    few = max(5, steps // 4)                      # the slow leg: fewer repetitions
    _, t_both_outer, _ = run_timed(torch, both_outer, few, 2)
    if not torch.equal(y_streamed, case.y):
        print("bench.py: the token-outermost table disagrees with the streamed path", file=sys.stderr)
        sys.exit(4)
    _, t_outer, _ = run_timed(torch, gemm_outer, few, 2)
    return t_stream, t_both, t_lut, t_both_outer, t_outer


def cpu_baseline(wl, W, w_scale, x):
    """The oracle as it stands on the host cores, on the same workload (one full pass, repeated to ~10 s)."""
    from oracle import oracle as O
    O.mpgemm(W[:64], w_scale, x)  # build + page in
    M, K = W.shape
    N = x.shape[0]
    t_total, reps = 0.0, 0
    while t_total < 10.0 and reps < 300:
        t0 = time.perf_counter()
        O.mpgemm(W, w_scale, x)
        t_total += time.perf_counter() - t0
        reps += 1
    sec = t_total / reps
    return {"value": 2.0 * M * K * N / sec / 1e9, "unit": "GOPS", "cores": O.num_threads(), "kind": "oracle",
            "sample": f"whole workload (quantise + triple-loop GEMM + scale), {reps} passes, {sec * 1e3:.0f} ms each"}


def roof(M, K, N, ms):
    """The roof that binds a shape and the fraction of it that `ms` (milliseconds) reaches.

    N <= 16: HBM bandwidth on the algorithmic bytes (packed weights + INT8 activations + scales + fp32 output).
    N >= 256: the table-lookup roof: one 2-byte LDS read (= one INT16 add) per (row, k-group, token) at 256 B/clk/CU.
    In between: whichever of the two floors is the longer time.  frac = floor time / measured time."""
    alg = M * K // 4 + K * N + 4 * N + 4 * M * N
    lds = 2 * M * (K // 4) * N
    t_hbm = alg / (HBM_PEAK_GBS * 1e9) * 1e3
    t_lds = lds / (LDS_PEAK_GBS * 1e9) * 1e3
    if N <= 16:
        bound, floor = "hbm", t_hbm
    elif N >= 256:
        bound, floor = "lds", t_lds
    else:
        bound, floor = ("lds", t_lds) if t_lds >= t_hbm else ("hbm", t_hbm)
    return {"bound": bound, "floor_ms": floor, "frac": floor / ms, "hbm_floor_ms": t_hbm, "lds_floor_ms": t_lds}


def measure_entry(B, torch, wl, wname, lin, n, seed, rotate, steps, warmup, with_mfma=True):
    """One (shape, N) of the sweep: the whole step through vlut_mpgemm_f32, the lookup kernel alone, the comparison
    path.  Returns (dict for the JSON line, Case, (W, w_scale, x))."""
    wk = wl.WORKLOADS[wname]
    W, w_scale, x = wl.make_case(wk, lin, n, seed)
    M, K = W.shape
    c = Case(B, torch, wl, W, w_scale, x, rotate)
    ms_step, ms_kernel, mode, ms_two, ms_gemm = time_case(B, torch, c, steps, warmup)
    r_step, r_kernel = roof(M, K, n, ms_step), roof(M, K, n, ms_kernel)
    e = {"workload": wname, "linear": lin.name, "M": M, "K": K, "N": n, "seed": seed,
         "plan": {"J": c.plan32[0], "R": c.plan32[1], "split_k": c.plan32[2], "workgroups": c.plan32[3],
                  "one_launch_from_fp32": bool(c.plan32[4])},
         "ms": ms_step, "kernel_ms": ms_kernel, "two_call_ms": ms_two, "mpgemm_ms": ms_gemm,
         "GOPS": 2.0 * M * K * n / (ms_step * 1e-3) / 1e9,
         "weight_stream_GBs": (M * K / 4) / (ms_step * 1e-3) / 1e9,
         "bound": r_step["bound"], "floor_ms": r_step["floor_ms"], "frac": r_step["frac"],
         "kernel_frac": r_kernel["frac"]}
    if with_mfma:
        ms_mfma = time_mfma(torch, c, steps, warmup)
        e["mfma_ms"] = ms_mfma
        e["lut_over_mfma_time"] = ms_gemm / ms_mfma
        e["mfma_frac_of_int8_peak"] = 2.0 * M * K * n / (ms_mfma * 1e-3) / 1e12 / MFMA_INT8_PEAK_TOPS
    return e, c, (W, w_scale, x)


def measure_layer(B, torch, wl, n, seed, rotate, steps, warmup):
    """One decoder layer's seven linears at N = n as four launches from fp32 inputs: q|k|v and gate|up stacked along M
    (they share their input, hence every table a workgroup builds), o, down; quantisation included."""
    wk = wl.WORKLOADS["layer2b4_nsweep"]
    lins = {l_.name: l_ for l_ in wk.linears}
    made = {name: wl.make_case(wk, lins[name], n, seed) for name in lins}

    def stacked(names):
        Wm = np.concatenate([made[nm][0] for nm in names], axis=0)
        wr = np.concatenate([np.full(made[nm][0].shape[0], made[nm][1], np.float32) for nm in names])
        return Case(B, torch, wl, Wm, 1.0, made[names[0]][2], rotate // 4, w_rows=wr)

    cases = [stacked(("q", "k", "v")), Case(B, torch, wl, *made["o"], rotate // 4), stacked(("gate", "up")),
             Case(B, torch, wl, *made["down"], rotate // 4)]

    def fn(i, stream):
        for c in cases:
            c.step_fused(i, stream)

    run_timed(torch, fn, steps, warmup)
    ms, ms_gpu, _ = run_timed(torch, fn, steps, warmup)
    shapes = [(lins[nm].M, lins[nm].K) for nm in ("q", "k", "v", "o", "gate", "up", "down")]
    alg = sum(m * k // 4 + 4 * m * n for m, k in shapes) + 3 * (2560 * n + 4 * n) + (6912 * n + 4 * n)
    lds = sum(2 * m * (k // 4) * n for m, k in shapes)
    t_hbm, t_lds = alg / (HBM_PEAK_GBS * 1e9) * 1e3, lds / (LDS_PEAK_GBS * 1e9) * 1e3
    bound, floor = ("hbm", t_hbm) if n <= 16 else (("lds", t_lds) if (n >= 256 or t_lds >= t_hbm) else ("hbm", t_hbm))
    ops = sum(2.0 * m * k * n for m, k in shapes)
    return {"N": n, "seed": seed, "launches": 4, "what": "q|k|v, o, gate|up, down through vlut_mpgemm_f32 (quantisation included)",
            "plans": [list(c.plan32) for c in cases],
            "ms": ms, "gpu_ms": ms_gpu, "GOPS": ops / (ms * 1e-3) / 1e9,
            "weight_stream_GBs": sum(m * k // 4 for m, k in shapes) / (ms * 1e-3) / 1e9,
            "bound": bound, "floor_ms": floor, "frac": floor / ms}


def main():
    global REPS
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path shards over tokens with no exchange: every GPU "
              "would run this same kernel on its share of the tokens). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    REPS = max(10, args.reps)
    import torch
    from paper_2512_06443_amd import binding as B
    from paper_2512_06443_amd import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    B.lib()  # fails loudly if libvlut.so is missing
    if args.plan:
        j, r, s = (int(v) for v in args.plan.split(","))
        B.set_plan(j, r, 0, s)

    w = wl.WORKLOADS[args.workload]
    default_lin = "gateup" if args.workload == "llama8b_linears" else w.linears[0].name
    lin = ([l_ for l_ in w.linears if l_.name == (args.linear or default_lin)] or [w.linears[0]])[0]
    N = args.tokens if args.tokens in w.N else w.N[0]
    seed = w.seeds[w.N.index(N)] if len(w.seeds) == len(w.N) else w.seeds[0]
    rotate = 0 if args.no_rotate else 600 << 20

    # ---- headline shape
    head, case, (W, w_scale, x) = measure_entry(B, torch, wl, w.name, lin, N, seed, rotate, args.steps, args.warmup)
    M, K = W.shape
    y_ref = torch.empty_like(case.y)
    case.step(0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    y_ref.copy_(case.y)
    case.y.zero_()
    case.step_fused(0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    if not torch.equal(y_ref, case.y):
        print("bench.py: vlut_mpgemm_f32 disagrees with vlut_quantize_act + vlut_mpgemm", file=sys.stderr)
        sys.exit(4)
    ms_step, ms_kernel, ms_two_call, ms_gemm = head["ms"], head["kernel_ms"], head["two_call_ms"], head["mpgemm_ms"]
    mode = "hipGraph"
    # the same step enqueued call by call from this process (host launch cost included), beside the graph figure
    ms_step_stream, _, _ = run_timed(torch, case.step_fused, args.steps, args.warmup, use_graph=False)
    g5 = None
    if K % 20 == 0:
        case.enable_g5(B, torch, W, rotate)
        _, ms_g5, _ = run_timed(torch, case.gemm_g5, args.steps, args.warmup)
        if not torch.equal(y_ref, case.y):
            print("bench.py: the 1.60-bit path disagrees with the 2-bit path", file=sys.stderr)
            sys.exit(4)
        g5 = {"what": "vlut_mpgemm_g5 on the same weights packed 5 per byte (1.60 bits per weight, 243-row tables)",
              "ms": ms_g5, "plan": {"R": case.plan5[0], "split_k": case.plan5[1], "workgroups": case.plan5[2]},
              "packed_weight_bytes": case.pool5[0].numel(), "time_over_2bit": ms_g5 / ms_gemm}
    else:
        case.enable_mixed(B, torch, W, rotate)
        _, ms_mx, _ = run_timed(torch, case.gemm_mixed, args.steps, args.warmup)
        if not torch.equal(y_ref, case.y):
            print("bench.py: the mixed packing disagrees with the 2-bit path", file=sys.stderr)
            sys.exit(4)
        g5 = {"what": "vlut_mpgemm_mixed on the same weights (first 20*floor(K/20) features 5 per byte, the rest 4 per byte)",
              "ms": ms_mx, "packed_weight_bytes": case.poolx[0].numel(), "time_over_2bit": ms_mx / ms_gemm}
    if case.plan32[0] == 0:
        kernel_name = "narrow_kernel (few tokens: quantisation, table build, lookups and scale in one launch)"
    elif case.plan32[4] and case.plan32[2] == 1:
        kernel_name = ("lookup_kernel, quantising variant (absmax + INT8 codes, LDS table build, lookup-accumulate, "
                       "epilogue in one launch)")
    else:
        kernel_name = "lookup_kernel (LDS table build + lookup-accumulate + epilogue)"
    ops = 2.0 * M * K * N
    adds = M * (K // 4) * N                      # one INT16 add (= 2 table bytes) per (row, group, token)
    gops = ops / (ms_step * 1e-3) / 1e9
    achieved_tadds = adds / (ms_kernel * 1e-3) / 1e12
    lds_gbs = 2.0 * adds / (ms_kernel * 1e-3) / 1e9
    alg = wl.algorithmic_bytes(M, K, N)
    rk = roof(M, K, N, ms_kernel)
    traffic_key = f"{w.name}/{lin.name}/{N}"
    roofline = {
        "kernel": kernel_name, "kernel_ms": ms_kernel,
        "bound": rk["bound"],
        "achieved": lds_gbs if rk["bound"] == "lds" else alg / (ms_kernel * 1e-3) / 1e9,
        "peak": LDS_PEAK_GBS if rk["bound"] == "lds" else HBM_PEAK_GBS, "unit": "GB/s",
        "frac": rk["frac"],
        "what": ("lds: table bytes the lookups read, 2 per (row, k-group, token), against 256 CUs x 256 B/clk x 2.4 GHz; "
                 "hbm: algorithmic bytes against 8 TB/s"),
        "alu_equivalent": {"achieved_TADDs": achieved_tadds, "peak_TADDs": ALU_PEAK_TADDS,
                           "frac": achieved_tadds / ALU_PEAK_TADDS},
        "lds_frac": lds_gbs / LDS_PEAK_GBS,
        "lds_frac_of_measured_peak": lds_gbs / LDS_MEASURED_PEAK_GBS,
        "hbm_frac": alg / (ms_kernel * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "traffic": MEASURED_TRAFFIC_BYTES.get(traffic_key),
        "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary under profiles/ (a stored figure: this run "
                          "does not read counters)" if traffic_key in MEASURED_TRAFFIC_BYTES else None,
    }
    out = {
        "metric": "ternary mpGeMM GOPS (2*M*K*N) + weight-stream GB/s at N=1..1024 tokens",
        "value": gops, "unit": "GOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int16/int32 (INT8 activations, ternary weights)", "data": "synthetic",
        "config": {"workload": f"{w.name}/{lin.name}: M={M} K={K} N={N}, ternary P(0)={w.p_zero}, INT8 per-token absmax "
                               f"activations from N(0,1)" + (f" with {w.outlier_frac:.0%} outlier channels x20" if w.outlier_frac else "") +
                               "; step = vlut_mpgemm_f32 (quantise + table build + lookup + scale)",
                   "plan": head["plan"], "weight_pool_buffers": len(case.pool), "launch": mode,
                   "timing": f"median of {REPS} replays of a graph of {args.steps} steps"},
        "weight_stream_GBs": (M * K / 4) / (ms_step * 1e-3) / 1e9,
        "algorithmic_GBs": alg / (ms_step * 1e-3) / 1e9,
        "per_call_stream_launches": {"what": "the same steps enqueued one call at a time from Python (ctypes), no graph",
                                     "ms_per_step": ms_step_stream},
        "two_call_form": {"what": "vlut_quantize_act + vlut_mpgemm on the same inputs", "ms_per_step": ms_two_call,
                          "mpgemm_kernel_ms": ms_gemm},
        "mfma_comparison": {"what": "vlut_mpgemm_mfma on the same inputs (unpack to INT8 + v_mfma_i32_16x16x64_i8), "
                                    "GPU ms per call incl. its activation re-layout kernel",
                            "ms": head.get("mfma_ms"), "lut_over_mfma_time": head.get("lut_over_mfma_time"),
                            "mfma_frac_of_int8_peak": head.get("mfma_frac_of_int8_peak")},
        "g5_packing": g5,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, W, w_scale, x)
    del case
    torch.cuda.empty_cache()

    if args.copy_probe:
        src = torch.empty(64 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()

    # ---- the sweep: every benchmark shape, the decoder layer at every N
    if not args.no_sweep:
        sweep = [dict(head)]
        for wname in ("bitnet2b_ffn_up", "bitnet3b_prefill", "llama8b_linears", "layer2b4_nsweep"):
            wk = wl.WORKLOADS[wname]
            for n in wk.N:
                sd = wk.seeds[wk.N.index(n)] if len(wk.seeds) == len(wk.N) else wk.seeds[0]
                for linr in wk.linears:
                    if (wname, linr.name, n) == (w.name, lin.name, N):
                        continue
                    e, c, _ = measure_entry(B, torch, wl, wname, linr, n, sd, rotate, args.steps, args.warmup)
                    sweep.append(e)
                    del c
                    torch.cuda.empty_cache()
        out["sweep"] = sweep
        wk = wl.WORKLOADS["layer2b4_nsweep"]
        out["layer"] = [measure_layer(B, torch, wl, n, wk.seeds[wk.N.index(n)], rotate, args.steps, args.warmup)
                        for n in wk.N]
        print(f"{'workload':18s} {'lin':7s} {'M':>6s} {'K':>6s} {'N':>5s} {'plan(J,R,S,WG)':>20s} {'step us':>9s} "
              f"{'kernel us':>9s} {'TOPS':>7s} {'W GB/s':>8s} {'bound':>5s} {'frac':>6s} {'k.frac':>6s} {'mfma us':>8s}",
              file=sys.stderr)
        for e in sweep:
            pl = e["plan"]
            print(f"{e['workload']:18s} {e['linear']:7s} {e['M']:6d} {e['K']:6d} {e['N']:5d} "
                  f"{str((pl['J'], pl['R'], pl['split_k'], pl['workgroups'])):>20s} {e['ms'] * 1e3:9.1f} "
                  f"{e['kernel_ms'] * 1e3:9.1f} {e['GOPS'] / 1e3:7.1f} {e['weight_stream_GBs']:8.1f} {e['bound']:>5s} "
                  f"{e['frac']:6.3f} {e['kernel_frac']:6.3f} {e.get('mfma_ms', float('nan')) * 1e3:8.1f}", file=sys.stderr)
        for e in out["layer"]:
            print(f"layer (4 launches from fp32) N={e['N']:5d} {e['ms'] * 1e3:9.1f} us  {e['GOPS'] / 1e3:7.1f} TOPS  "
                  f"{e['weight_stream_GBs']:8.1f} GB/s  {e['bound']} frac {e['frac']:.3f}", file=sys.stderr)

    if args.ablation:
        abl = []
        for wname, lname, n in (("bitnet2b_ffn_up", "up", 128), ("bitnet3b_prefill", "up", 256),
                                ("layer2b4_nsweep", "gate", 16), ("layer2b4_nsweep", "gate", 1024)):
            wk = wl.WORKLOADS[wname]
            linr = [l_ for l_ in wk.linears if l_.name == lname][0]
            Wm, ws_, xm = wl.make_case(wk, linr, n, wk.seeds[0])
            c = Case(B, torch, wl, Wm, ws_, xm, rotate)
            ts, tb, tl, tbo, to = time_ablation(B, torch, c, max(20, args.steps // 4), 5)
            abl.append({"workload": wname, "linear": lname, "M": c.M, "K": c.K, "N": n,
                        "lut_MB": B.lib().vlut_lut_bytes(c.K, n) / 1e6, "streamed_ms": ts,
                        "build_lut_plus_mpgemm_ms": tb, "mpgemm_on_materialised_ms": tl,
                        "streaming_gain": tb / ts,
                        "token_outer_build_plus_mpgemm_ms": tbo, "token_outer_mpgemm_ms": to,
                        "layout_gain": tbo / tb})
            del c
            torch.cuda.empty_cache()
        out["ablation_streamed_vs_materialised"] = abl
        print(f"{'workload':18s} {'lin':5s} {'N':>5s} {'table MB':>9s} {'streamed us':>12s} {'build+gemm us':>14s} "
              f"{'gemm(lut) us':>13s} {'gain':>6s} {'outer build+gemm us':>20s} {'outer gemm us':>14s} {'layout gain':>12s}",
              file=sys.stderr)
        for a in abl:
            print(f"{a['workload']:18s} {a['linear']:5s} {a['N']:5d} {a['lut_MB']:9.1f} {a['streamed_ms'] * 1e3:12.1f} "
                  f"{a['build_lut_plus_mpgemm_ms'] * 1e3:14.1f} {a['mpgemm_on_materialised_ms'] * 1e3:13.1f} "
                  f"{a['streaming_gain']:6.2f} {a['token_outer_build_plus_mpgemm_ms'] * 1e3:20.1f} "
                  f"{a['token_outer_mpgemm_ms'] * 1e3:14.1f} {a['layout_gain']:12.2f}", file=sys.stderr)

    if args.layer:
        wk = wl.WORKLOADS["layer2b4_nsweep"]
        lins = {l_.name: l_ for l_ in wk.linears}
        layer_rows = []
        for n in wk.N:
            made = {name: wl.make_case(wk, lins[name], n, wk.seeds[0]) for name in lins}
            single = [Case(B, torch, wl, *made[name], rotate // 4) for name in ("q", "k", "v", "o", "gate", "up", "down")]

            def stacked(names):
                Wm = np.concatenate([made[nm][0] for nm in names], axis=0)
                wr = np.concatenate([np.full(made[nm][0].shape[0], made[nm][1], np.float32) for nm in names])
                return Case(B, torch, wl, Wm, 1.0, made[names[0]][2], rotate // 4, w_rows=wr)

            fused = [stacked(("q", "k", "v")), single[3], stacked(("gate", "up")), single[6]]
            for c in single + fused:
                c.quantize(torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()

            def run_all(cases):
                def fn(i, stream):
                    for c in cases:
                        c.gemm(i, stream)
                return fn

            def run_all_steps(cases, f32):
                def fn(i, stream):
                    for c in cases:
                        (c.step_fused if f32 else c.step)(i, stream)
                return fn

            cnt = max(10, args.steps // 8)
            _, t_single, _ = run_timed(torch, run_all(single), cnt, 3)
            _, t_fused, _ = run_timed(torch, run_all(fused), cnt, 3)
            # the same four launches from fp32 inputs: quantisation included, as a decoder layer needs them
            _, t_f32, _ = run_timed(torch, run_all_steps(fused, True), cnt, 3)
            _, t_two, _ = run_timed(torch, run_all_steps(fused, False), cnt, 3)
            wbytes = sum(c.M * c.K // 4 for c in single)
            layer_rows.append({"N": n, "launches_single": 7, "single_ms": t_single, "launches_stacked": 4,
                               "stacked_ms": t_fused, "stacked_from_fp32_ms": t_f32,
                               "stacked_from_fp32_two_call_ms": t_two, "packed_weight_MB": wbytes / 1e6,
                               "weight_stream_GBs_stacked": wbytes / (t_fused * 1e-3) / 1e9,
                               "hbm_frac_stacked": wbytes / (t_fused * 1e-3) / 1e9 / HBM_PEAK_GBS})
            del single, fused
            torch.cuda.empty_cache()
        out["layer_linears"] = layer_rows
        print(f"{'N':>5s} {'7 launches us':>14s} {'4 stacked us':>13s} {'4 from fp32 us':>15s} {'4 x (quant+gemm) us':>20s} "
              f"{'weights MB':>11s} {'GB/s stacked':>13s} {'hbm frac':>9s}", file=sys.stderr)
        for r in layer_rows:
            print(f"{r['N']:5d} {r['single_ms'] * 1e3:14.1f} {r['stacked_ms'] * 1e3:13.1f} {r['stacked_from_fp32_ms'] * 1e3:15.1f} "
                  f"{r['stacked_from_fp32_two_call_ms'] * 1e3:20.1f} {r['packed_weight_MB']:11.2f} "
                  f"{r['weight_stream_GBs_stacked']:13.1f} {r['hbm_frac_stacked']:9.3f}", file=sys.stderr)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
