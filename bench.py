#!/usr/bin/env python3
"""bench.py - one-GPU benchmark of the SFMP mixed-precision GEMM/GEMV hot path on MI355X.

A "step" is one pass of the whole hot path over one batch: the seven projections
(q, k, v, o, gate, up, down) of a Llama-3-8B-shaped decoder layer at M = 1, 128x128 tiles with
one third each of 2/3/4-bit tiles (average 3.0 code bits), group 128, random column and row
permutations - benchmark configs[1].  Inputs are synthetic and already resident in HBM.
Weights are rotated over R device copies (R * layer bytes >= 1 GiB) so that neither the L2s nor
the 256 MB Infinity Cache hold them between steps: the numbers are cold-cache numbers.

Prints ONE JSON line (see the keys below); `value` is microseconds per layer (lower is better).
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

NCPU = len(os.sched_getaffinity(0))
os.environ.setdefault("OMP_NUM_THREADS", str(NCPU))
os.environ.setdefault("OPENBLAS_NUM_THREADS", str(NCPU))

import numpy as np  # noqa: E402

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak
MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X published dense fp16 matrix peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=240)
    ap.add_argument("--warmup", type=int, default=24)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the per-shape / 70B / prefill side reports")
    ap.add_argument("--eager", action="store_true", help="time eager launches instead of HIP-graph replays")
    ap.add_argument("--separate", action="store_true",
                    help="one launch per projection (7) instead of q|k|v, o, gate|up, down sharing launches (4)")
    ap.add_argument("--section", choices=("all", "decode", "layers", "layer70b", "batch", "prefill", "prefill_sweep", "sweep",
                                          "lut"),
                    default="all",
                    help="which reports to run after the headline measurement (for profiling one kernel family at a "
                         "time): decode = per-projection and 70B M=1, layers = one layer of configs[2] and [3] at every "
                         "M, batch = M in {4, 16} both ways, prefill = M=2048 on the six shapes of configs[4] "
                         "(roofline_prefill), prefill_sweep = shorter prompts; with anything but all / decode / lut the "
                         "headline region runs 2 steps only")
    ap.add_argument("--no-prefill", action="store_true", help="skip the M=2048 matrix-core measurement")
    ap.add_argument("--prefill-launches", type=int, default=12, help="sfmp_gemm calls timed per prefill shape")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (known size) so that rocprofv3 --pmc FETCH_SIZE / "
                         "WRITE_SIZE readings can be scaled")
    return ap.parse_args()


class Layer:
    """Device-resident projections of one decoder layer, replicated R times for cold-cache timing."""

    def __init__(self, problems, replicas, device="cuda:0"):
        import torch
        import paper_2602_01027_amd as S
        self.S = S
        self.torch = torch
        self.device = device
        self.problems = problems
        self.replicas = replicas
        self.proj = []  # per projection: dict(layout, reps=[DevicePacked...], X, Y, cp, rp, ws, bytes)
        for p in problems:
            L, s2, s3, s4, index = S.sfmp_pack(p.codes, p.bitmap)
            S.sfmp_layout_set_quant(L, p.group, p.scale_format)
            reps = [S.upload_packed(L, s2, s3, s4, index, p.scales, p.zeros, p.bitmap, device) for _ in range(replicas)]
            cp = [torch.from_numpy(p.col_perm).to(device) for _ in range(replicas)] if p.col_perm is not None else None
            rp = [torch.from_numpy(p.row_perm).to(device) for _ in range(replicas)] if p.row_perm is not None else None
            X = torch.from_numpy(p.X).to(device)
            Y = torch.empty((p.M, p.N), dtype=torch.float16, device=device)
            ws = torch.empty(S.sfmp_gemm_workspace(L, p.M), dtype=torch.uint8, device=device)  # contents irrelevant
            self.proj.append(dict(p=p, layout=L, reps=reps, cp=cp, rp=rp, X=X, Y=Y, ws=ws))
        torch.cuda.synchronize()
        self._args = {}

    def _call_args(self, i, r, stream_ptr):
        """Pre-marshalled ctypes arguments of sfmp_gemm for projection i, replica r."""
        key = (i, r, stream_ptr)
        if key not in self._args:
            d = self.proj[i]
            dp = d["reps"][r]

            def ptr(t):
                return C.c_void_p(t.data_ptr()) if t is not None and t.numel() else None

            self._args[key] = (ptr(d["X"]), C.c_int32(d["p"].M), ptr(d["cp"][r]) if d["cp"] else None,
                               C.byref(dp.layout), ptr(dp.s2), ptr(dp.s3), ptr(dp.s4), ptr(dp.index), ptr(dp.scales),
                               ptr(dp.zeros), ptr(dp.bitmap), ptr(d["rp"][r]) if d["rp"] else None, ptr(d["Y"]),
                               ptr(d["ws"]), C.c_int64(d["ws"].numel()), C.c_void_p(stream_ptr))
        return self._args[key]

    def launch(self, i, r, stream_ptr):
        rc = self.S.load_library().sfmp_gemm(*self._call_args(i, r, stream_ptr))
        if rc != 0:
            raise RuntimeError(self.S.sfmp_strerror(rc))

    def step(self, r, stream_ptr):
        for i in range(len(self.proj)):
            self.launch(i, r, stream_ptr)

    def step_fused(self, r, stream_ptr, groups):
        """The same projections as `step`, independent ones sharing a launch (sfmp_gemv_batched at M = 1,
        sfmp_gemm_batched for small batches)."""
        lib = self.S.load_library()
        M = self.problems[0].M
        for gi, idxs in enumerate(groups):
            key = ("fused", gi, r)
            if key not in self._args:
                batch = []
                for i in idxs:
                    d = self.proj[i]
                    batch.append((d["X"], d["cp"][r] if d["cp"] else None, d["reps"][r],
                                  d["rp"][r] if d["rp"] else None, d["Y"]))
                arr, keep = self.S.make_gemv_batch(batch)
                ws = None
                if M > 1:
                    wkey = ("fused_ws", gi)
                    if wkey not in self._args:
                        self._args[wkey] = self.torch.empty(self.S.sfmp_gemm_batched_workspace(batch, M),
                                                            dtype=self.torch.uint8, device=self.device)
                    ws = self._args[wkey]
                self._args[key] = (arr, keep, ws)
            arr, _keep, ws = self._args[key]
            if M == 1:
                rc = lib.sfmp_gemv_batched(C.cast(arr, C.c_void_p), len(idxs), C.c_void_p(stream_ptr))
            else:
                rc = lib.sfmp_gemm_batched(C.cast(arr, C.c_void_p), len(idxs), C.c_int32(M), C.c_void_p(ws.data_ptr()),
                                           C.c_int64(ws.numel()), C.c_void_p(stream_ptr))
            if rc != 0:
                raise RuntimeError(self.S.sfmp_strerror(rc))

    def bytes_per_proj(self, W):
        out = []
        for d in self.proj:
            p = d["p"]
            out.append(W.algorithmic_bytes(p.N, p.K, p.M, p.bitmap, col_perm=p.col_perm is not None,
                                           row_perm=p.row_perm is not None, index_words=p.bitmap.size, group=p.group))
        return out


def build_problems_iter(W, cid):
    """The problems of a configuration one at a time (codes drawn directly), so that only one 70B matrix is in host
    memory at once."""
    spec = W.CONFIGS[cid]
    for si, (label, K, N) in enumerate(spec.shapes):
        yield W.make_problem(label, K, N, spec.Ms[0], 1000 * cid + si, w_std=spec.w_std[si], fractions=spec.fractions,
                             outliers=spec.outliers, use_col_perm=spec.col_perm, use_row_perm=spec.row_perm[si],
                             fast_codes=True)


def build_problems(W, cid, Ms=None, fast=False, only=None, allocated_bits=None, **fmt):
    """fmt: group / scale_format / block passed on to the generator (default: group 128, fp16, 128x128 blocks).
    allocated_bits: take the bitmap from the sorting-based allocation on synthetic salience at this average width
    (salient rows and columns first: wide tiles cluster in the top-left corner) instead of a shuffled one."""
    spec = W.CONFIGS[cid]
    out = []
    for si, (label, K, N) in enumerate(spec.shapes):
        if only is not None and label not in only:
            continue
        M = (Ms or spec.Ms)[0]
        if allocated_bits is not None:
            blk = fmt.get("block", (4, 1))
            fmt = dict(fmt, bitmap=W.allocation.allocated_layout(N, K, allocated_bits, np.random.default_rng(
                77000 + 1000 * cid + si), block=(blk[0], max(blk[1], fmt.get("group", 128) // 128)))["bitmap"])
            fmt.pop("block", None)
        out.append(W.make_problem(label, K, N, M, 1000 * cid + si, w_std=spec.w_std[si], fractions=spec.fractions,
                                  outliers=spec.outliers, use_col_perm=spec.col_perm, use_row_perm=spec.row_perm[si],
                                  fast_codes=fast, **fmt))
    return out


FUSED_GROUPS = [[0, 1, 2], [3], [4, 5], [6]]  # q|k|v, o, gate|up, down: what a decoder layer can run together


def do_step(layer, r, stream_ptr, groups):
    """One step on replica r: one launch per projection (groups None), or independent projections sharing launches."""
    if groups is None:
        layer.step(r, stream_ptr)
    else:
        layer.step_fused(r, stream_ptr, groups)


def capture_step_graphs(torch, layer, groups):
    """One HIP graph per weight replica, each holding the launches of one step (after an eager warm-up on the capture
    stream: module load, first touch).  The timed region replays them in rotation."""
    stream = torch.cuda.current_stream()
    graphs = []
    side = torch.cuda.Stream()
    side.wait_stream(stream)
    with torch.cuda.stream(side):
        for r in range(layer.replicas):
            do_step(layer, r, side.cuda_stream, groups)
    side.synchronize()
    for r in range(layer.replicas):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            do_step(layer, r, torch.cuda.current_stream().cuda_stream, groups)
        graphs.append(g)
    torch.cuda.synchronize()
    return graphs


def time_steps(torch, layer, steps, warmup, use_graph, groups=None):
    """Times `steps` steps after `warmup`; returns (ms_per_step from HIP events, wall ms_per_step).

    groups None: one launch per projection; else independent projections share a launch."""
    R = layer.replicas
    stream = torch.cuda.current_stream()
    graphs = capture_step_graphs(torch, layer, groups) if use_graph else None

    def run(i):
        if graphs is not None:
            graphs[i % R].replay()
        else:
            do_step(layer, i % R, stream.cuda_stream, groups)

    for i in range(warmup):
        run(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        run(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return e0.elapsed_time(e1) / steps, wall


def time_each_projection(torch, layer, launches=60):
    """Average microseconds per launch of every projection alone (back-to-back launches, rotating replicas)."""
    out = []
    stream = torch.cuda.current_stream()
    R = layer.replicas
    for i in range(len(layer.proj)):
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            layer.launch(i, 0, side.cuda_stream)
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for j in range(launches):
                layer.launch(i, j % R, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        g.replay()
        e1.record(stream)
        torch.cuda.synchronize()
        out.append(e0.elapsed_time(e1) * 1e3 / launches)
    return out


def dense_fp16_us(torch, M, N, K, launches):
    """Microseconds per call of a dense fp16 GEMM (torch.matmul: the vendor library) at this shape: N(0, 1) activations,
    N(0, 0.02) weights rotated over enough copies to stay out of the caches, graph of back-to-back calls."""
    dev = "cuda:0"
    X = torch.randn(M, K, device=dev, dtype=torch.float16)
    reps = max(2, min(8, int(2 ** 30 // (N * K * 2)) + 1))
    Ws = [torch.randn(N, K, device=dev, dtype=torch.float16) * 0.02 for _ in range(reps)]
    Y = torch.empty(M, N, device=dev, dtype=torch.float16)
    for w in Ws:
        torch.matmul(X, w.t(), out=Y)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        for j in range(launches):
            torch.matmul(X, Ws[j % reps].t(), out=Y)
    torch.cuda.synchronize()
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    g.replay()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / launches
    del Ws, X, Y, g
    torch.cuda.empty_cache()
    return round(us, 1)


def time_lut(torch, S, p, replicas, launches, table_format="fp32"):
    """Average microseconds per call of sfmp_lut_gemv on problem p (graph replay, weights rotated over replicas)."""
    dev = "cuda:0"
    planes, tile_off = S.sfmp_lut_pack(p.codes, p.bitmap)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    reps = [(d(planes), d(tile_off.view(np.int32)), d(p.scales), d(p.zeros)) for _ in range(replicas)]
    X, Y = d(p.X[0]), torch.zeros(p.N, dtype=torch.float16, device=dev)
    cp = d(p.col_perm) if p.col_perm is not None else None
    rp = d(p.row_perm) if p.row_perm is not None else None
    ws = torch.zeros(S.sfmp_lut_gemv_workspace(p.N, p.K), dtype=torch.uint8, device=dev)

    def call(j, stream):
        pl, to, sc, zr = reps[j % replicas]
        S.sfmp_lut_gemv(X, cp, p.N, p.K, pl, to, sc, zr, rp, Y, ws, stream=stream, table_format=table_format)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        call(0, side)
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        for j in range(launches):
            call(j, torch.cuda.current_stream())
    torch.cuda.synchronize()
    g.replay()
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    g.replay()
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / launches


def cpu_baseline(problems):
    """The CPU oracle, as it stands, on the same layer: one pass over all projections."""
    from oracle import sfmp_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([d.get("num_threads", 1) for d in threadpool_info()] + [1])
    except Exception:
        threads = NCPU
    t0 = time.perf_counter()
    for p in problems:
        O.gemm(p.X, p.col_perm, p.codes, p.scales, p.zeros, p.row_perm)
    dt = time.perf_counter() - t0
    return dict(value=dt * 1e6, unit="us/layer", cores=int(threads), kind="oracle",
                sample="the full 8B layer (7 projections, M=1), one pass of oracle.gemm (fp64 dequant + matmul); "
                       f"host has {NCPU} usable cores")


def profile_figures():
    """Figures taken from the rocprofv3 summaries under profiles/ (kernel-trace means, counter traffic); the file names
    its sources.  They are constants of the tracked profiles, not measured in this run."""
    path = os.path.join(ROOT, "profiles", "bench_profile_figures.json")
    try:
        return json.load(open(path))
    except Exception:
        return {}


def bare_read_floor_us(torch, launch_bytes, replicas, nrep, src=None):
    """The floor of a step: HIP-event microseconds per step of a step made of len(launch_bytes) launches, each a bare
    streaming read (the probe library's kernel: nothing computed, no dependent start) of the bytes its launch of the
    step moves, replayed as a graph over rotating memory (1 GiB) like the step itself."""
    from paper_2602_01027_amd import probe
    if src is None:
        src = torch.empty((1 << 30) + (64 << 20), dtype=torch.uint8, device="cuda:0").random_(0, 255)
    outp = torch.empty(2048, dtype=torch.uint8, device="cuda:0")
    launch_bytes = [(int(b) + 255) // 256 * 256 for b in launch_bytes]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graphs, off = [], 0
    for r in range(replicas):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for b in launch_bytes:
                if off + b > (1 << 30):
                    off = 0
                probe.stream_read(src[off:off + b], outp, stream=torch.cuda.current_stream())
                off += b
        graphs.append(g)
    torch.cuda.synchronize()
    for i in range(replicas):
        graphs[i].replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(nrep):
        graphs[i % replicas].replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / nrep


def layer_line(torch, W, cid, M, steps, eager, groups):
    """One transformer layer of configuration cid at batch M: microseconds per layer and its share of the bounds; at
    M = 1 also the floor of its launches (bare streaming reads of the same bytes, bare_read_floor_us)."""
    fused = groups is not None and M <= 16
    pb = build_problems(W, cid, Ms=(M,), fast=True)
    bb = sum(W.algorithmic_bytes(p.N, p.K, p.M, p.bitmap, index_words=p.bitmap.size) for p in pb)
    fl = sum(2.0 * p.M * p.N * p.K for p in pb)
    lb = Layer(pb, int(np.ceil(2 ** 30 / bb)))
    ms, _ = time_steps(torch, lb, steps, max(2, steps // 10), use_graph=not eager, groups=groups if fused else None)
    row = dict(M=M, us_per_layer=round(ms * 1e3, 2), launches="4 batched calls" if fused else "7 calls",
               MB=round(bb / 1e6, 1), GBps=round(bb / ms / 1e6, 1),
               frac_hbm_peak=round(bb / ms / 1e6 / HBM_PEAK_GBPS, 4),
               TFLOPs=round(fl / ms / 1e9, 2), frac_mfma_peak=round(fl / ms / 1e9 / MFMA_F16_PEAK_TFLOPS, 4))
    per = lb.bytes_per_proj(W)
    replicas = lb.replicas
    del lb, pb
    torch.cuda.empty_cache()
    if M == 1 and fused:
        try:
            floor = bare_read_floor_us(torch, [sum(per[i] for i in g) for g in groups], replicas, max(steps, 2 * replicas))
            row["bare_read_floor_us"] = round(floor, 2)
            row["floor_over_value"] = round(floor / (ms * 1e3), 4)
        except Exception as ex:  # the probe is an aid: never let it take the bench line down
            row["bare_read_floor_error"] = str(ex)
        torch.cuda.empty_cache()
    return row


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import sfmp_workloads as W
    import paper_2602_01027_amd as S
    S.load_library()  # fails loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    figs = profile_figures()

    problems = build_problems(W, 2)
    layer_bytes = sum(W.algorithmic_bytes(p.N, p.K, p.M, p.bitmap, index_words=p.bitmap.size) for p in problems)
    R = int(np.ceil(2 ** 30 / layer_bytes))
    layer = Layer(problems, R)
    per_proj_bytes = layer.bytes_per_proj(W)

    if args.pmc_calibration:
        src = torch.empty(256 * 2 ** 20, dtype=torch.uint8, device="cuda:0").fill_(3)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)  # reads 256 MiB and writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    groups = None if args.separate else FUSED_GROUPS
    if args.section in ("batch", "prefill", "prefill_sweep", "sweep", "layers", "layer70b"):
        args.steps, args.warmup = 2, 1
    ms_step, wall_ms = time_steps(torch, layer, args.steps, args.warmup, use_graph=not args.eager, groups=groups)
    us_layer = ms_step * 1e3
    gbps = layer_bytes / (ms_step * 1e-3) / 1e9
    n_launch = len(problems) if groups is None else len(groups)
    dec = figs.get("gemv_8b_decode", {})
    k_us = dec.get("kernel_avg_us")
    bytes_per_launch = layer_bytes / n_launch

    result = {
        "metric": "us_per_layer_M1 (Llama-3-8B-shaped decoder layer, 7 mixed 2/3/4-bit projections, avg 3.0 bits)",
        "value": round(us_layer, 3),
        "unit": "us/layer",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 (fp16 activations/scales, 2/3/4-bit codes, fp32 accumulate)",
        "data": "synthetic (seeded Gaussian weights, min-max group quantised; cold cache: weights rotated over "
                f"{R} device copies)",
        "config": {"workload": "configs[1]: 8B decode layer, M=1, q/k/v/o/gate/up/down, 128x128 tiles 1/3 each "
                               "2/3/4-bit, group 128, random col+row perms",
                   "launch": ("eager" if args.eager else "hip-graph replay") + (
                       ", one launch per projection (7)" if groups is None else
                       ", 4 launches: q|k|v, o, gate|up, down (independent projections share a launch)"),
                   "replicas": R, "layer_bytes": int(layer_bytes)},
        "effective_GBps": round(gbps, 1),
        "pct_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "wall_ms_per_step": round(wall_ms, 6),
        "roofline": {
            "bound": "hbm",
            "kernel": "sfmp::gemv_batched_kernel<16, S> / gemv_kernel<16, S> (same body)",
            "achieved": round(gbps, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(gbps / HBM_PEAK_GBPS, 4),
            "traffic": dec.get("traffic_bytes_per_launch"),
            "bytes_per_launch_avg": int(bytes_per_launch),
            "avg_launch_us": round(us_layer / n_launch, 3),
            "kernel_avg_us": k_us,
            "kernel_frac": round(bytes_per_launch / (k_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4) if k_us else None,
            "note": "achieved / frac = algorithmic bytes of all launches of a step / HIP-event time of the step "
                    "(launch gaps of the graph replay included), measured in this run; kernel_frac = the same bytes per "
                    "launch / kernel_avg_us, the mean duration of the GEMV kernels in the tracked rocprofv3 kernel trace "
                    f"({dec.get('kernel_trace_source')}; kernel time only, a constant of that profile, not measured in "
                    f"this run); traffic = FETCH_SIZE + WRITE_SIZE per launch from {dec.get('traffic_source')} (counter "
                    "run, also a constant of that profile)",
        },
    }

    # second denominator: what a plain streaming read reaches on this machine (1 GiB, cold), beside the data sheet;
    # and the floor of the step: the same number of launches, each a bare streaming read of the bytes its launch of the
    # step moves (nothing computed, no dependent start), replayed as a graph over rotating memory like the step itself
    try:
        from paper_2602_01027_amd import probe
        src = torch.empty((1 << 30) + (64 << 20), dtype=torch.uint8, device="cuda:0").random_(0, 255)
        outp = torch.empty(2048, dtype=torch.uint8, device="cuda:0")
        whole = src[:1 << 30]
        for _ in range(2):
            probe.stream_read(whole, outp)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            probe.stream_read(whole, outp)
        e1.record()
        torch.cuda.synchronize()
        stream_gbps = 5 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9
        result["roofline"]["measured_stream_read_GBps"] = round(stream_gbps, 1)
        result["roofline"]["frac_of_measured_stream_read"] = round(gbps / stream_gbps, 4)
        launch_bytes = [sum(per_proj_bytes[i] for i in g) for g in (groups or [[i] for i in range(len(problems))])]
        floor_us = bare_read_floor_us(torch, launch_bytes, R, max(args.steps, 2 * R), src=src)
        del src, outp, whole
        result["roofline"]["bare_read_floor_us"] = round(floor_us, 3)
        result["roofline"]["floor_over_value"] = round(floor_us / us_layer, 4)
        result["roofline"]["note_floor"] = ("bare_read_floor_us = HIP-event time of a step made of the same number of launches, "
                                            "each a plain streaming read (probe kernel, nothing computed) of the bytes its launch "
                                            "moves, graph replay over rotating memory: what launch overhead plus HBM transfer cost "
                                            "on this machine; floor_over_value = that floor / value")
    except Exception as ex:  # the probe is an aid: never let it take the bench line down
        result["roofline"]["measured_stream_read_GBps"] = result["roofline"].get("measured_stream_read_GBps")
        result["roofline"]["measured_stream_read_error"] = str(ex)

    extra = {}
    if not args.no_extra and args.section in ("all", "decode"):
        if groups is not None:
            ms7, _ = time_steps(torch, layer, args.steps, args.warmup, use_graph=not args.eager, groups=None)
            extra["seven_separate_launches_us_per_layer"] = round(ms7 * 1e3, 3)
        per = time_each_projection(torch, layer)
        extra["per_projection_8b_M1"] = [
            dict(shape=f"{d['p'].K}->{d['p'].N}", label=d["p"].label, us=round(t, 3), MB=round(b / 1e6, 3),
                 GBps=round(b / t / 1e3, 1), pct_hbm_peak=round(100 * b / t / 1e3 / HBM_PEAK_GBPS, 2))
            for d, t, b in zip(layer.proj, per, per_proj_bytes)]
    del layer
    torch.cuda.empty_cache()

    if not args.no_prefill and args.section in ("all", "prefill"):
        # The matrix-core half of the metric: configs[4], M = 2048, all six shapes, one sfmp_gemm call each (staging +
        # GEMM + row un-permute where the configuration has a row permutation), codes drawn directly (timing only).
        rows, tot_fl, tot_t, dense_t, tot_traffic = [], 0.0, 0.0, 0.0, 0
        kfig = figs.get("prefill_M2048", {})
        for pp in build_problems_iter(W, 5):
            lp = Layer([pp], 1)
            t = time_each_projection(torch, lp, launches=args.prefill_launches)[0]
            fl = 2.0 * pp.M * pp.N * pp.K
            kus = kfig.get("kernel_us", {}).get(f"{pp.K}->{pp.N}")
            ktr = kfig.get("kernel_traffic_bytes", {}).get(f"{pp.K}->{pp.N}")
            # what the GEMM kernel has to move at least: packed weights and parameters, the staged activations, the product
            alg = int(W.algorithmic_bytes(pp.N, pp.K, pp.M, pp.bitmap, col_perm=False, row_perm=False,
                                          index_words=pp.bitmap.size, group=pp.group))
            rows.append(dict(shape=f"{pp.K}->{pp.N}", us=round(t, 1), GFLOP=round(fl / 1e9, 1),
                             TFLOPs=round(fl / t / 1e6, 1), frac=round(fl / t / 1e6 / MFMA_F16_PEAK_TFLOPS, 4),
                             kernel_us=kus,
                             kernel_frac=round(fl / kus / 1e6 / MFMA_F16_PEAK_TFLOPS, 4) if kus else None,
                             kernel_traffic_bytes=ktr, kernel_algorithmic_bytes=alg,
                             dense_fp16_us=dense_fp16_us(torch, pp.M, pp.N, pp.K, args.prefill_launches)))
            tot_traffic = (tot_traffic + ktr) if (ktr is not None and tot_traffic is not None) else None
            tot_fl += fl
            tot_t += t
            dense_t += rows[-1]["dense_fp16_us"]
            del lp, pp
            torch.cuda.empty_cache()
        result["roofline_prefill"] = {
            "bound": "mfma",
            "kernel": "sfmp::prefill_kernel (fp16 MFMA, weights dequantised in registers) + activation staging and "
                      "row un-permute passes",
            "achieved": round(tot_fl / tot_t / 1e6, 1),
            "peak": MFMA_F16_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(tot_fl / tot_t / 1e6 / MFMA_F16_PEAK_TFLOPS, 4),
            "traffic": tot_traffic,
            "workload": "configs[4]: M=2048 on 4096->4096, 4096->1024, 4096->14336, 14336->4096, 8192->28672, "
                        "28672->8192; 50 % 3-bit / 50 % 4-bit tiles, outlier columns",
            "per_shape": rows,
            "dense_fp16_reference_TFLOPs": round(tot_fl / dense_t / 1e6, 1),
            "achieved_over_dense_fp16_reference": round(dense_t / tot_t, 4),
            "note_dense": "dense_fp16_us / dense_fp16_reference_TFLOPs = torch.matmul of fp16 [M, K] by fp16 [N, K]^T (the "
                          "vendor GEMM library, unquantised weights, no permutations) on the same shapes, timed in this "
                          "run the same way: what a dense fp16 GEMM sustains on this machine at random operands, as context "
                          "for frac (not a target and not part of value)",
            "note": "achieved / frac = FLOP-weighted aggregate: total 2*M*N*K of the six shapes / total HIP-event time of "
                    "one whole sfmp_gemm call each (graph of back-to-back calls), measured in this run; per-shape "
                    f"kernel_us / kernel_frac = GEMM kernel alone from the tracked kernel trace ({kfig.get('source')}), "
                    "constants of that profile; traffic = FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 of the GEMM kernel (counter runs "
                    "of the same profile, factors from a 256 MiB copy), summed over the six launches, per shape as "
                    "kernel_traffic_bytes beside kernel_algorithmic_bytes (packed weights and parameters once, staged "
                    "activations in, product out): the excess is the weights read once per XCD (8 L2s) and activation "
                    "blocks that left an L2 before every workgroup sharing them had read them",
        }

    if not args.no_extra:
        if args.section in ("all", "layers"):
            # the pass / fail lines of the other decode configurations: one transformer layer each
            extra["layer_8b_config3_2p5bit"] = [layer_line(torch, W, 3, M, 60 if M <= 16 else 30, args.eager, FUSED_GROUPS)
                                                for M in (1, 4, 16, 64)]
            extra["layer_70b_config4_3p25bit"] = [layer_line(torch, W, 4, M, 40, args.eager, FUSED_GROUPS) for M in (1, 8)]
        if args.section == "layer70b":  # the 70B decode layer alone, M = 1 (for a kernel trace of its own)
            extra["layer_70b_config4_3p25bit"] = [layer_line(torch, W, 4, 1, 40, args.eager, FUSED_GROUPS)]
        if args.section in ("all", "decode"):
            # 70B-shaped decode layer (configs[3]) at M = 1, one launch per projection, and every projection alone
            p70 = build_problems(W, 4, Ms=(1,), fast=True)
            b70 = sum(W.algorithmic_bytes(p.N, p.K, p.M, p.bitmap, index_words=p.bitmap.size) for p in p70)
            l70 = Layer(p70, int(np.ceil(2 ** 30 / b70)))
            ms70, _ = time_steps(torch, l70, 60, 6, use_graph=not args.eager)
            per70 = time_each_projection(torch, l70, launches=24)
            b70p = l70.bytes_per_proj(W)
            extra["layer_70b_M1_seven_launches"] = dict(
                us_per_layer=round(ms70 * 1e3, 2), MB=round(b70 / 1e6, 1), GBps=round(b70 / ms70 / 1e6, 1),
                pct_hbm_peak=round(100 * b70 / ms70 / 1e6 / HBM_PEAK_GBPS, 2),
                per_projection=[dict(shape=f"{d['p'].K}->{d['p'].N}", us=round(t, 2), GBps=round(b / t / 1e3, 1),
                                     pct_hbm_peak=round(100 * b / t / 1e3 / HBM_PEAK_GBPS, 2))
                                for d, t, b in zip(l70.proj, per70, b70p)])
            del l70, p70
            torch.cuda.empty_cache()
        if args.section in ("all", "decode"):
            # the paper's own parameter format on the 8B layer at M = 1: (512, 256) bit-allocation blocks, group 256,
            # bf16 scales and zeros (its best setting at low bit budgets), same 1/3-each width mix, 4 launches
            pf = build_problems(W, 2, fast=True, group=256, scale_format="bf16", block=(4, 2))
            bf = sum(W.algorithmic_bytes(p.N, p.K, p.M, p.bitmap, index_words=p.bitmap.size, group=p.group) for p in pf)
            lf = Layer(pf, int(np.ceil(2 ** 30 / bf)))
            msf, _ = time_steps(torch, lf, 120, 12, use_graph=not args.eager, groups=FUSED_GROUPS)
            extra["layer_8b_M1_blocks512x256_group256_bf16"] = dict(
                us_per_layer=round(msf * 1e3, 2), MB=round(bf / 1e6, 1), GBps=round(bf / msf / 1e6, 1),
                pct_hbm_peak=round(100 * bf / msf / 1e6 / HBM_PEAK_GBPS, 2))
            del lf, pf
            torch.cuda.empty_cache()
        if args.section in ("all", "decode"):
            # group length 64 (the smallest n_b of the block-size ablation: 0.5 bit per weight of parameters), fp16
            pg = build_problems(W, 2, fast=True, group=64)
            bg = sum(W.algorithmic_bytes(p.N, p.K, p.M, p.bitmap, index_words=p.bitmap.size, group=p.group) for p in pg)
            lg = Layer(pg, int(np.ceil(2 ** 30 / bg)))
            msg, _ = time_steps(torch, lg, 120, 12, use_graph=not args.eager, groups=FUSED_GROUPS)
            extra["layer_8b_M1_group64"] = dict(
                us_per_layer=round(msg * 1e3, 2), MB=round(bg / 1e6, 1), GBps=round(bg / msg / 1e6, 1),
                pct_hbm_peak=round(100 * bg / msg / 1e6 / HBM_PEAK_GBPS, 2))
            del lg, pg
            torch.cuda.empty_cache()
        if args.section in ("all", "decode"):
            # bitmaps as the method produces them: Algorithm 1 on synthetic salience, (512, 128) blocks, average 3.0
            # bits; rows and columns sorted by salience, so tile rows differ in bytes (4-bit rows first)
            pa = build_problems(W, 2, fast=True, allocated_bits=3.0)
            ba = sum(W.algorithmic_bytes(p.N, p.K, p.M, p.bitmap, index_words=p.bitmap.size, group=p.group) for p in pa)
            la = Layer(pa, int(np.ceil(2 ** 30 / ba)))
            msa, _ = time_steps(torch, la, 120, 12, use_graph=not args.eager, groups=FUSED_GROUPS)
            extra["layer_8b_M1_allocated_bitmaps"] = dict(
                us_per_layer=round(msa * 1e3, 2), MB=round(ba / 1e6, 1), GBps=round(ba / msa / 1e6, 1),
                pct_hbm_peak=round(100 * ba / msa / 1e6 / HBM_PEAK_GBPS, 2),
                avg_bits=[round(p.avg_bits, 3) for p in pa])
            del la, pa
            torch.cuda.empty_cache()
        if args.section in ("batch",):
            # small batches (configs[2]) both ways: 4 batched calls and 7 separate calls
            rows = []
            for M in (4, 16):
                pb = build_problems(W, 3, Ms=(M,), fast=True)
                bb = sum(W.algorithmic_bytes(p.N, p.K, p.M, p.bitmap, index_words=p.bitmap.size) for p in pb)
                lb = Layer(pb, int(np.ceil(2 ** 30 / bb)))
                msb, _ = time_steps(torch, lb, 60, 6, use_graph=not args.eager, groups=FUSED_GROUPS)
                ms7, _ = time_steps(torch, lb, 60, 6, use_graph=not args.eager)
                rows.append(dict(M=M, us_per_layer=round(msb * 1e3, 2), seven_separate_calls_us=round(ms7 * 1e3, 2),
                                 MB=round(bb / 1e6, 1), GBps=round(bb / msb / 1e6, 1),
                                 pct_hbm_peak=round(100 * bb / msb / 1e6 / HBM_PEAK_GBPS, 2)))
                del lb, pb
                torch.cuda.empty_cache()
            extra["layer_8b_small_batch"] = rows
        if args.section in ("prefill_sweep",):
            # the 4096 -> 14336 matrix at shorter prompts, and with the rows left in reordered order
            pp = build_problems(W, 5, fast=True, only=("8b.gate",))
            pg = pp[0]
            import dataclasses as _dc
            lf = Layer([_dc.replace(pg, row_perm=None)], 2)
            extra["prefill_M2048_4096x14336_rows_left_reordered_us"] = round(time_each_projection(torch, lf, launches=24)[0], 1)
            del lf
            sweep = []
            for M in (128, 256, 512, 1024):
                pm = [W.with_activations(pg, M, outliers=True)]
                lm = Layer(pm, 2)
                t = time_each_projection(torch, lm, launches=24)[0]
                fl = 2.0 * M * pg.N * pg.K
                sweep.append(dict(M=M, us=round(t, 1), TFLOPs=round(fl / t / 1e6, 1),
                                  pct_mfma_peak=round(100 * fl / t / 1e6 / MFMA_F16_PEAK_TFLOPS, 2)))
                del lm, pm
            extra["prefill_4096x14336_M_sweep"] = sweep
            del pp
        if args.section in ("all", "sweep"):
            # one call of sfmp_gemm at every batch size on two 8B matrices: which kernels a given M runs is the
            # library's choice (GEMV, ring kernel, its chunked form, MFMA kernel with or without a split K)
            ps = build_problems(W, 2, fast=True, only=("8b.q", "8b.down"))
            sweep = {}
            for q in ps:
                rows = []
                for M in (1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048):
                    lm = Layer([W.with_activations(q, M, outliers=False)], 8 if M <= 128 else 2)
                    t = time_each_projection(torch, lm, launches=32 if M <= 128 else 16)[0]
                    rows.append(dict(M=M, us=round(t, 1), us_per_row=round(t / M, 2),
                                     TFLOPs=round(2.0 * M * q.N * q.K / t / 1e6, 1)))
                    del lm
                sweep[f"{q.K}->{q.N}"] = rows
            extra["single_call_M_sweep"] = sweep
            del ps
        if args.section in ("all", "lut"):
            # the paper's own kernel scheme (one-bit lookup tables on a bit-plane format) beside the MFMA path, M = 1,
            # same matrices, cold cache: uniform widths (its latency should follow the width) and the 1/3-each mix
            rows = []
            for (K, N) in ((4096, 4096), (4096, 14336)):
                for label, fr in (("2-bit", {2: 1.0}), ("3-bit", {3: 1.0}), ("4-bit", {4: 1.0}), ("mixed 2/3/4", None)):
                    q = W.make_problem(f"lut.{K}x{N}.{label}", K, N, 1, 9100 + N + len(label), fractions=fr, fast_codes=True)
                    lm = Layer([q], 13)
                    t_mfma = time_each_projection(torch, lm, launches=52)[0]
                    del lm
                    t_lut = time_lut(torch, S, q, 13, 52)
                    t_lut16 = time_lut(torch, S, q, 13, 52, table_format="fp16")
                    wbytes = float(q.bitmap.astype(np.float64).sum()) * 2048.0
                    rows.append(dict(shape=f"{K}->{N}", widths=label, lut_us=round(t_lut, 2),
                                     lut_fp16_tables_us=round(t_lut16, 2), mfma_us=round(t_mfma, 2),
                                     lut_GBps=round(wbytes / t_lut / 1e3, 1)))
            extra["lut_gemv_vs_mfma_gemv_M1"] = rows
    if extra:
        result["extra"] = extra

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(problems)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
