#!/usr/bin/env python3
"""Benchmark of the libmpq hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input of the chosen
workload.  Default workload: configuration 2, the ResNet-50-shaped conv-as-GEMM stack (8 layers at
batch 32).  Per layer a step runs, through the C ABI:
    absmax(A) per tensor, absmax(W) per output channel            (calibration, Sec. 3.1)
    quant_error(A) and quant_error(W), b = 2..8 in one read each  (Eq. 2)
    noise_inject(W) at the layer's weight bit-width               (Eq. 3-5)
    fake_quant(A) -> int8 codes, fake_quant(W) -> int8 / packed int4 codes, the two step sizes
    qgemm -> fp32 Y                                               ("Evaluate f(x, w)")
    sse_pair(Y, Y_ref)                                            (candidate score)
All inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "qgemm int8 TOPS (% MFMA peak); quant+error sweep GB/s (% HBM peak)"
HBM_PEAK_GBS = 8000.0
INT8_PEAK_TOPS = 5000.0
LAMBDA = 0.28867513  # 1/sqrt(12): noise with the variance of uniform rounding error of one step

CALLS = ["absmax", "quant_error", "noise_inject", "fake_quant", "qgemm", "sse_pair"]

# HBM traffic per main-stream launch (activation tensor of a layer, averaged over the 8 layers),
# in KiB, from the rocprofv3 counter runs summarised in profiles/cfg2_hot_path_hbm_traffic.txt:
# FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000 of the call's kernels (main + finishing kernel).
TRAFFIC_KIB_PER_LAUNCH = {
    "absmax": (38243.1 + 5.0) * 2.0 + 50.1,
    "quant_error": (38284.6 + 27.7) * 2.0 + 68.6 + 0.1,
    "fake_quant": (38253.9 + 2.5) * 2.0 + 19110.0 + 1.2,
    "sse_pair": (29416.5 + 7.2) * 2.0 + 42.4,
}


class Layer:
    """Device buffers of one linear layer; allocated once, reused by every step."""

    def __init__(self, torch, mpq, idx, name, a, w, bits_a, bits_w):
        self.idx, self.name, self.bits_a, self.bits_w = idx, name, bits_a, bits_w
        self.M, self.K = a.shape
        self.N = w.shape[0]
        self.a = torch.from_numpy(a).cuda()
        self.w = torch.from_numpy(w).cuda()
        dev = self.a.device
        f32, i8, u8, f64 = torch.float32, torch.int8, torch.uint8, torch.float64
        self.am_a = torch.empty(1, dtype=f32, device=dev)
        self.am_w = torch.empty(self.N, dtype=f32, device=dev)
        self.sse_a = torch.empty((1, 7), dtype=f64, device=dev)
        self.sse_w = torch.empty((self.N, 7), dtype=f64, device=dev)
        self.w_noisy = torch.empty_like(self.w)
        self.a_codes = torch.empty((self.M, self.K), dtype=i8, device=dev)
        self.w_store = 4 if bits_w <= 4 else 8
        self.w_codes = (torch.empty((self.N, self.K // 2), dtype=u8, device=dev) if self.w_store == 4
                        else torch.empty((self.N, self.K), dtype=i8, device=dev))
        self.s_a = torch.empty(1, dtype=f32, device=dev)
        self.s_w = torch.empty(self.N, dtype=f32, device=dev)
        self.y = torch.empty((self.M, self.N), dtype=f32, device=dev)
        # reference output of the unquantized layer, computed once outside the timed region
        self.y_ref = self.a @ self.w.t()
        self.score = torch.empty(1, dtype=f64, device=dev)

    # algorithmic HBM bytes of each call of this layer (one read of every input, one write of
    # every output, nothing else)
    def bytes(self):
        mk, nk, mn = self.M * self.K, self.N * self.K, self.M * self.N
        wb = nk * self.w_store // 8
        return {
            "absmax": 4 * mk + 4 * nk,
            "quant_error": 4 * mk + 4 * nk,
            "noise_inject": 8 * nk,
            "fake_quant": (4 * mk + mk) + (4 * nk + wb),
            "qgemm": mk + wb + 4 * mn,
            "sse_pair": 8 * mn,
        }

    # the part of bytes() that the main-stream launch of each call moves (activation side)
    def main_bytes(self):
        mk, nk, mn = self.M * self.K, self.N * self.K, self.M * self.N
        wb = nk * self.w_store // 8
        return {"absmax": 4 * mk, "quant_error": 4 * mk, "fake_quant": 5 * mk,
                "qgemm": mk + wb + 4 * mn, "sse_pair": 8 * mn}

    def ops(self):
        return 2 * self.M * self.N * self.K


def run_layer(mpq, L, ws_a, ws_w, rec, torch, side):
    """The hot path on one layer.  rec(call_name) -> context manager that times the call.

    The weight-side calls (small tensors, latency-bound launches) go to the side stream and overlap
    the activation-side calls on the main stream; the GEMM waits for both.  Tensors of the two
    sides are independent, each side has its own workspace."""
    P = mpq
    main = torch.cuda.current_stream()
    side.wait_stream(main)  # the previous layer's GEMM has consumed what this side overwrites next
    with torch.cuda.stream(side):
        P.calibrate_absmax(L.w, P.PER_ROW, out=L.am_w)
        P.quant_error(L.w, L.am_w, 2, 8, P.PER_ROW, out=L.sse_w, ws=ws_w)
        P.noise_inject(L.w, L.am_w, L.bits_w, LAMBDA, 2302, L.idx, P.PER_ROW, out=L.w_noisy)
        if L.w_store == 4:
            P.fake_quant(L.w, L.am_w, L.bits_w, P.PER_ROW, want_y=False, packed4=L.w_codes)
        else:
            P.fake_quant(L.w, L.am_w, L.bits_w, P.PER_ROW, want_y=False, codes=L.w_codes)
        P.scale_from_absmax(L.am_w, L.bits_w, out=L.s_w)
    with rec("absmax"):
        P.calibrate_absmax(L.a, P.PER_TENSOR, out=L.am_a, ws=ws_a)
    with rec("quant_error"):
        P.quant_error(L.a, L.am_a, 2, 8, P.PER_TENSOR, out=L.sse_a, ws=ws_a)
    with rec("fake_quant"):
        P.fake_quant(L.a, L.am_a, L.bits_a, P.PER_TENSOR, want_y=False, codes=L.a_codes)
    P.scale_from_absmax(L.am_a, L.bits_a, out=L.s_a)
    main.wait_stream(side)
    with rec("qgemm"):
        P.qgemm(L.a_codes, L.w_codes, L.s_a, L.s_w, L.w_store, P.PER_ROW, y=L.y, ws=ws_a)
    with rec("sse_pair"):
        P.sse_pair(L.y, L.y_ref, out=L.score, ws=ws_a)


class NullRec:
    def __call__(self, name):
        return self

    def __enter__(self):
        return self

    def __exit__(self, *a):
        return False


class EventRec:
    """Brackets selected calls with HIP events on the stream the kernels are launched on
    (torch's current stream, which is the stream handed to every libmpq call)."""

    def __init__(self, torch, only=None):
        self.torch, self.only, self.pairs, self.cur = torch, only, [], None

    def __call__(self, name):
        self.cur = name
        return self

    def __enter__(self):
        if self.only is None or self.cur in self.only:
            e0 = self.torch.cuda.Event(enable_timing=True)
            e1 = self.torch.cuda.Event(enable_timing=True)
            e0.record()
            self.pairs.append((self.cur, e0, e1))
            self._open = e1
        else:
            self._open = None
        return self

    def __exit__(self, *a):
        if self._open is not None:
            self._open.record()
        return False

    def totals_ms(self):
        out = {}
        for name, e0, e1 in self.pairs:
            out[name] = out.get(name, 0.0) + e0.elapsed_time(e1)
        return out


def cpu_baseline(workloads, sample_rows):
    """The oracle, as it stands, over the same path on a bounded sample: the first `sample_rows`
    activation rows of every layer with the full weight tensors.  Layers run on a thread pool
    (the oracle itself is single threaded; ctypes releases the GIL)."""
    import numpy as np
    import oracle

    def one(idx):
        a, w, ba, bw = workloads.cfg2_layer(idx, rows=sample_rows)
        t0 = time.perf_counter()
        am_a, am_w = oracle.absmax(a), oracle.absmax(w, oracle.PER_ROW)
        oracle.quant_error(a, am_a)
        oracle.quant_error(w, am_w, gran=oracle.PER_ROW)
        oracle.noise_inject(w, am_w, bw, LAMBDA, 2302, idx, oracle.PER_ROW)
        _, ca, _ = oracle.fake_quant(a, am_a, ba)
        st = 4 if bw <= 4 else 8
        _, cw, pw = oracle.fake_quant(w, am_w, bw, oracle.PER_ROW, want_packed4=st == 4)
        y, _ = oracle.qgemm(ca, pw if st == 4 else cw, oracle.scale_from_absmax(am_a, ba),
                            oracle.scale_from_absmax(am_w, bw), st, oracle.PER_ROW)
        oracle.sse_pair(y, y)
        dt = time.perf_counter() - t0
        m, k = a.shape
        n = w.shape[0]
        mk, nk, mn = m * k, n * k, m * n
        wb = nk * st // 8
        nbytes = (4 * mk + 4 * nk) * 2 + 8 * nk + (5 * mk + 4 * nk + wb) + (mk + wb + 4 * mn) + 8 * mn
        return nbytes, dt

    oracle.lib()
    n_layers = len(workloads.CFG2)
    cores = max(1, min(n_layers, len(os.sched_getaffinity(0))))
    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        res = list(ex.map(one, range(n_layers)))
    wall = time.perf_counter() - t0
    total = sum(r[0] for r in res)
    return {
        "value": total / wall / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
        "sample": "first %d activation rows of each of the 8 layers, full weights; %.1f s wall, "
                  "%.1f s summed over threads" % (sample_rows, wall, sum(r[1] for r in res)),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--cpu-sample-rows", type=int, default=1024)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain device copy of known size (231 MB) three times before the "
                         "warm-up: the reference that rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU only (the path has no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2302_01382_amd import mpq, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; libmpq has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    mpq.lib()

    layers = []
    for idx, g in enumerate(workloads.CFG2):
        a, w, ba, bw = workloads.cfg2_layer(idx)
        layers.append(Layer(torch, mpq, idx, g.name, a, w, ba, bw))
        del a, w
    ws_a, ws_w = mpq.Workspace(), mpq.Workspace()
    ws_a.get(1 << 22)
    ws_w.get(1 << 22)
    side = torch.cuda.Stream()  # default priority
    torch.cuda.synchronize()

    if args.calibrate_copy:
        dst = torch.empty_like(layers[0].a)
        for _ in range(3):
            dst.copy_(layers[0].a)   # plain copy kernel: reads and writes layers[0].a.numel() * 4 bytes
        torch.cuda.synchronize()
        del dst

    def step(rec):
        for L in layers:
            run_layer(mpq, L, ws_a, ws_w, rec, torch, side)
        torch.cuda.current_stream().wait_stream(side)

    # warm-up; the last warm-up step is timed per call to find the dominant one
    null = NullRec()
    for _ in range(max(args.warmup - 1, 0)):
        step(null)
    def step_behind_a_blocker(rec):
        """Eager step for kernel-level timing: a ~1.5 ms spin kernel goes first, so that the host has
        enqueued the whole step before the GPU starts on it and the HIP events bracket back-to-back
        kernels instead of host launch gaps."""
        torch.cuda._sleep(3_500_000)
        step(rec)

    probe = EventRec(torch)
    step_behind_a_blocker(probe)
    torch.cuda.synchronize()
    per_call_ms = probe.totals_ms()
    dominant = max(per_call_ms, key=per_call_ms.get)

    # One step = ~130 kernel launches of a few microseconds each: issued one by one from Python the
    # host, not the GPU, sets the pace.  The step is therefore captured once into a HIP graph (both
    # streams; the library records kernels only, no memset nodes) and the timed region replays it.
    def snapshot():
        return [(L.score.clone(), L.sse_a.clone(), L.sse_w.clone(), L.am_w.clone()) for L in layers]

    eager_ref = snapshot()
    launch_mode = "hip_graph"
    graph = None
    try:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(null)
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(snapshot(), eager_ref):
            for g_, w_ in zip(got, want):
                if not torch.equal(g_, w_):
                    raise RuntimeError("graph replay differs from the eager result")
    except Exception as e:  # capture not possible here: time eager launches instead, and say so
        print("bench.py: HIP graph path unavailable (%s); timing eager launches" % e, file=sys.stderr)
        graph = None
        launch_mode = "eager"
        torch.cuda.synchronize()

    # timed region: exactly `steps` steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        if graph is not None:
            graph.replay()
        else:
            step(null)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    if graph is not None:
        for got, want in zip(snapshot(), eager_ref):
            for g_, w_ in zip(got, want):
                if not torch.equal(g_, w_):
                    raise RuntimeError("graph replay differs from the eager result after the timed region")

    # kernel-level timing for the roofline: the same `steps` steps launched eagerly right after,
    # HIP events around every launch of the dominant call and of qgemm on the stream they run on
    # (events cannot be recorded inside a graph replay)
    rec = EventRec(torch, only={dominant, "qgemm"})
    for _ in range(args.steps):
        step_behind_a_blocker(rec)
        torch.cuda.synchronize()

    call_bytes = {c: sum(L.bytes()[c] for L in layers) for c in CALLS}
    main_bytes = {c: sum(L.main_bytes()[c] for L in layers) for c in layers[0].main_bytes()}
    step_bytes = sum(call_bytes.values())
    timed = rec.totals_ms()
    dom_ms_per_step = timed[dominant] / args.steps
    gemm_ms_per_step = timed["qgemm"] / args.steps
    gemm_ops = sum(L.ops() for L in layers)
    n_launch = len(layers)  # one main-stream launch of the dominant call per layer
    if dominant == "qgemm":
        roof = {"bound": "mfma", "achieved": gemm_ops / (gemm_ms_per_step * 1e-3) / 1e12,
                "peak": INT8_PEAK_TOPS, "unit": "TOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": main_bytes[dominant] / (dom_ms_per_step * 1e-3) / 1e9,
                "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    t_kib = TRAFFIC_KIB_PER_LAUNCH.get(dominant)
    roof["traffic"] = None if t_kib is None else t_kib * 1024.0
    roof["kernel"] = dominant
    roof["avg_launch_us"] = dom_ms_per_step * 1e3 / n_launch
    roof["algorithmic_per_launch"] = (gemm_ops if dominant == "qgemm" else main_bytes[dominant]) / n_launch
    if dominant == "quant_error":
        # the sweep is co-bound by the vector ALUs: 29 lane-operations per element (7 bit-widths x
        # 4 + one clip); peak 256 CUs x 64 lanes x 2.4 GHz = 39.3 T lane-op/s without packed math
        elems = main_bytes[dominant] / 4
        roof["alu"] = {"lane_ops_per_element": 29, "achieved_Tlaneop_s": elems * 29 / (dom_ms_per_step * 1e-3) / 1e12,
                       "peak_Tlaneop_s": 39.3216,
                       "frac": elems * 29 / (dom_ms_per_step * 1e-3) / 1e12 / 39.3216}

    out = {
        "metric": METRIC,
        "value": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 elementwise, int8 x int8 -> int32 GEMM",
        "data": "synthetic",
        "config": {"workload": "cfg2: ResNet-50-shaped conv-as-GEMM stack, batch 32, 8 layers, "
                               "whole hot path per layer (absmax, quant_error b=2..8, noise, fake_quant, qgemm, sse_pair)",
                   "step_algorithmic_bytes": step_bytes, "step_gemm_ops": gemm_ops},
        "launch": launch_mode,
        "qgemm": {"tops": gemm_ops / (gemm_ms_per_step * 1e-3) / 1e12,
                  "frac_of_int8_mfma_peak": gemm_ops / (gemm_ms_per_step * 1e-3) / 1e12 / INT8_PEAK_TOPS,
                  "ms_per_step": gemm_ms_per_step},
        "main_stream_call_ms_probe_step": {k: round(v, 4) for k, v in per_call_ms.items()},
        "main_stream_call_gbs_probe_step": {k: round(main_bytes[k] / (v * 1e-3) / 1e9, 1) for k, v in per_call_ms.items()},
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(workloads, args.cpu_sample_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
