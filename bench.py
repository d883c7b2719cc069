#!/usr/bin/env python3
"""Benchmark of the libmpq hot path on one MI355X.

Default (`--workload headline`): both halves of the metric on their own workloads, in one JSON line.
  sweep  configuration 4, the sensitivity sweep over the 96 BERT-large weight tensors (302 M
         elements, 1.208 GB): a step = max calibration per output channel and per tensor, then the
         error sums of b = 2..8 per tensor and per output channel, all through the batched calls
         (5 launches).  `value` = 12 bytes per element (three reads of 4 bytes) / time; 100 timed
         steps after 60 warm-up steps by default (a step is 0.6 ms and the chip needs some 15 ms of
         work to leave its idle clocks).  Reported beside it: the same results from two reads
         (calibration and the per-row sums from one read), both granularities from one read, and
         the seven noise levels per tensor.
  gemm   mpq_qgemm on every configured GEMM shape (configurations 2, 3, 5; int8 and packed int4
         weights), cold operands: TOP/s, fraction of the int8 matrix peak and of the shape's own
         roofline.
  cfg2   the whole per-layer path of configuration 2 (below), as a block of the same line.
`--workload cfg2`: configuration 2, the ResNet-50-shaped conv-as-GEMM stack (8 layers at batch 32).
Per layer a step runs, through the C ABI:
    absmax(A) per tensor, absmax(W) per output channel            (calibration, Sec. 3.1)
    quant_error(A) and quant_error(W), b = 2..8 in one read each  (Eq. 2)
    noise_inject(W) at the layer's weight bit-width               (Eq. 3-5)
    fake_quant(A) -> int8 codes + step size, fake_quant(W) -> int8 / packed int4 codes, its step sizes
    qgemm -> fp32 Y                                               (the evaluation step)
    sse_pair(Y, Y_ref)                                            (candidate score)
Other workloads (the parity-test configurations, measured with the same machinery):
    cfg3  BERT-base encoder linears at M = 12288, same per-layer path, per-tensor scales
    cfg4  the sensitivity sweep with one call per tensor instead of the batched calls: absmax +
          quant_error per tensor and per output channel, noise at every b = 2..8 from one call per
          tensor; the tensors are independent and are dealt to 4 streams (cfg4-1stream: one after
          the other; cfg4-unfused: one call per granularity and per noise level, one stream)
    cfg5  64 candidate bit configurations of a BERT-large FFN block at M = 16384, back to back;
          GELU and the calibration of its output in the first GEMM's epilogue, the output score in
          the second's
          (cfg5-twopass: the first GEMM runs twice, absmax of GELU(H) only, then its int8 codes
           straight from the epilogue, no fp32 H in HBM;
           cfg5-unfused: mpq_qgemm, torch GELU, mpq_calibrate_absmax, mpq_sse_pair)
    search  Alg. 1 / Alg. 2 over a 24-layer stack, evaluations per second
    latency qgemm latency table at batch 1 and the mixed-precision latency estimate built from it
    gemm    mpq_qgemm on every configured GEMM shape: TOP/s, fraction of the matrix peak and of the
            shape's own roofline
    hutchinson  Hessian-trace probe (random sign vectors, quadratic forms on the fp32 matrix cores)
    kernels every streaming call of the path (a1, a2, a3, a4, a6) on one 268 MB tensor, cold: GB/s each
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
ALU_PEAK_TLANEOPS = 256 * 4 * 32 * 2.4e9 / 1e12   # 256 CUs x 4 SIMDs x 32 lanes per clock x 2.4 GHz = 78.6 (157.3 TFLOP/s fp32)
CLOCK_RAMP_S = 0.03   # untimed device work in front of the sweep's warm-up steps
LAMBDA = 0.28867513  # 1/sqrt(12): noise with the variance of uniform rounding error of one step

# HBM traffic per main-stream launch of configuration 2 (activation tensor of a layer, averaged
# over the 8 layers), in KiB, from the rocprofv3 counter runs summarised in
# profiles/cfg2_hot_path_hbm_traffic.txt: FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000 of the call's
# kernels (main + finishing kernel).
TRAFFIC_KIB_PER_LAUNCH_CFG2 = {
    "absmax": (38243.3 + 5.0) * 2.0 + 50.1,
    "quant_error": (38288.2 + 27.7) * 2.0 + 68.6 + 0.1,
    "fake_quant": 38255.3 * 2.0 + 19110.0,
    "sse_pair": (29410.9 + 7.2) * 2.0 + 42.3,
}


# ------------------------------------------------------------------------------------------------
# timing helpers
class NullRec:
    def __call__(self, name, nbytes=0, ops=0):
        return self

    def __enter__(self):
        return self

    def __exit__(self, *a):
        return False


class EventRec:
    """Brackets selected calls with HIP events on the stream the kernels are launched on (torch's
    current stream, which is the stream handed to every libmpq call).  Also adds up the algorithmic
    bytes / integer ops the bracketed launches were declared with."""

    def __init__(self, torch, only=None):
        self.torch, self.only, self.pairs, self.cur = torch, only, [], None
        self.bytes, self.ops, self.count = {}, {}, {}
        self._open = None

    def __call__(self, name, nbytes=0, ops=0):
        self.cur = name
        if self.only is None or name in self.only:
            self.bytes[name] = self.bytes.get(name, 0) + nbytes
            self.ops[name] = self.ops.get(name, 0) + ops
            self.count[name] = self.count.get(name, 0) + 1
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


def measure(torch, step, snapshot, steps, warmup):
    """Warm-up, HIP-graph capture of one step, `steps` timed replays, then the same steps launched
    eagerly with HIP events around the dominant call.  Returns a dict of measurements."""
    null = NullRec()
    for _ in range(max(warmup - 1, 0)):
        step(null)

    def step_behind_a_blocker(rec):
        # a ~1.5 ms spin kernel goes first, so that the host has enqueued (most of) the step before
        # the GPU starts on it and the events bracket back-to-back kernels, not host launch gaps
        torch.cuda._sleep(3_500_000)
        step(rec)

    probe = EventRec(torch)
    step_behind_a_blocker(probe)
    torch.cuda.synchronize()
    per_call_ms = probe.totals_ms()
    dominant = max(per_call_ms, key=per_call_ms.get)

    # A step is hundreds of kernel launches of a few microseconds each: issued one by one from
    # Python the host, not the GPU, sets the pace.  The step is therefore captured once into a HIP
    # graph (the library records kernels only, no memset nodes) and the timed region replays it.
    eager_ref = snapshot()
    launch_mode, graph = "hip_graph", None

    def same_as_eager():
        for got, want in zip(snapshot(), eager_ref):
            if not torch.equal(got, want):
                raise RuntimeError("graph replay differs from the eager result")

    try:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(null)
        graph.replay()
        torch.cuda.synchronize()
        same_as_eager()
    except Exception as e:  # capture not possible here: time eager launches instead, and say so
        print("bench.py: HIP graph path unavailable (%s); timing eager launches" % e, file=sys.stderr)
        graph, launch_mode = None, "eager"
        torch.cuda.synchronize()

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        if graph is not None:
            graph.replay()
        else:
            step(null)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    if graph is not None:
        same_as_eager()

    # kernel-level timing for the roofline: the same steps launched eagerly right after, events
    # around every launch of the dominant call and of qgemm (events cannot sit inside a replay)
    rec = EventRec(torch, only={dominant, "qgemm"})
    for _ in range(steps):
        step_behind_a_blocker(rec)
        torch.cuda.synchronize()
    return {"ms_per_step": wall * 1e3 / steps, "launch": launch_mode, "probe": probe, "rec": rec,
            "dominant": dominant, "steps": steps}


def roofline_of(m, traffic_kib=None):
    rec, dom, steps = m["rec"], m["dominant"], m["steps"]
    ms = rec.totals_ms()[dom] / steps
    n_launch = rec.count[dom] / steps
    if dom == "qgemm":
        roof = {"bound": "mfma", "achieved": rec.ops[dom] / steps / (ms * 1e-3) / 1e12, "peak": INT8_PEAK_TOPS,
                "unit": "TOP/s", "algorithmic_per_launch": rec.ops[dom] / steps / n_launch}
    else:
        roof = {"bound": "hbm", "achieved": rec.bytes[dom] / steps / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "algorithmic_per_launch": rec.bytes[dom] / steps / n_launch}
    if dom == "quant_error":
        # 28 lane-operations per element (6 bit-widths x 4, 3 for two bits, one clip) at 4 bytes per
        # element is 7 lane-op per byte, below the chip's ratio of 78.6 T lane-op/s to 8 TB/s = 9.8:
        # the sweep is bound by HBM; the vector-ALU view is kept next to it
        lane_ops = rec.bytes[dom] / steps / 4 * 28
        roof["alu_view"] = {"lane_ops_per_element": 28, "achieved": lane_ops / (ms * 1e-3) / 1e12,
                            "peak": ALU_PEAK_TLANEOPS, "unit": "T lane-op/s",
                            "frac": lane_ops / (ms * 1e-3) / 1e12 / ALU_PEAK_TLANEOPS}
    roof["frac"] = roof["achieved"] / roof["peak"]
    t = None if traffic_kib is None else traffic_kib.get(dom)
    roof["traffic"] = None if t is None else t * 1024.0
    roof["kernel"] = dom
    roof["avg_launch_us"] = ms * 1e3 / n_launch
    return roof


def gemm_summary(m):
    rec, steps = m["rec"], m["steps"]
    if "qgemm" not in rec.count:
        return None
    ms = rec.totals_ms()["qgemm"] / steps
    tops = rec.ops["qgemm"] / steps / (ms * 1e-3) / 1e12
    return {"tops": tops, "frac_of_int8_mfma_peak": tops / INT8_PEAK_TOPS, "ms_per_step": ms}


# ------------------------------------------------------------------------------------------------
# configurations 2 and 3: a stack of linear layers, whole path per layer
class Layer:
    """Device buffers of one linear layer; allocated once, reused by every step."""

    def __init__(self, torch, idx, name, a, w, bits_a, bits_w, w_gran):
        self.idx, self.name, self.bits_a, self.bits_w, self.w_gran = idx, name, bits_a, bits_w, w_gran
        self.M, self.K = a.shape
        self.N = w.shape[0]
        self.a = torch.from_numpy(a).cuda()
        self.w = torch.from_numpy(w).cuda()
        dev = self.a.device
        f32, i8, u8, f64 = torch.float32, torch.int8, torch.uint8, torch.float64
        nch = self.N if w_gran == 1 else 1
        self.am_a = torch.empty(1, dtype=f32, device=dev)
        self.am_w = torch.empty(nch, dtype=f32, device=dev)
        self.sse_a = torch.empty((1, 7), dtype=f64, device=dev)
        self.sse_w = torch.empty((nch, 7), dtype=f64, device=dev)
        self.w_noisy = torch.empty_like(self.w)
        self.a_codes = torch.empty((self.M, self.K), dtype=i8, device=dev)
        self.w_store = 4 if bits_w <= 4 else 8
        self.w_codes = (torch.empty((self.N, self.K // 2), dtype=u8, device=dev) if self.w_store == 4
                        else torch.empty((self.N, self.K), dtype=i8, device=dev))
        self.s_a = torch.empty(1, dtype=f32, device=dev)
        self.s_w = torch.empty(nch, dtype=f32, device=dev)
        self.y = torch.empty((self.M, self.N), dtype=f32, device=dev)
        # reference output of the unquantized layer, computed once outside the timed region
        self.y_ref = self.a @ self.w.t()
        self.score = torch.empty(1, dtype=f64, device=dev)

    # algorithmic HBM bytes: one read of every input, one write of every output, nothing else
    def bytes(self):
        mk, nk, mn = self.M * self.K, self.N * self.K, self.M * self.N
        wb = nk * self.w_store // 8
        return {"absmax": 4 * mk + 4 * nk, "quant_error": 4 * mk + 4 * nk, "noise_inject": 8 * nk,
                "fake_quant": (4 * mk + mk) + (4 * nk + wb), "qgemm": mk + wb + 4 * mn, "sse_pair": 8 * mn}

    def ops(self):
        return 2 * self.M * self.N * self.K


def run_layer(P, L, ws_a, ws_w, rec, torch, side):
    """The hot path on one layer.  The weight-side calls (small tensors, latency-bound launches) go
    to the side stream and overlap the activation-side calls on the main stream; the GEMM waits
    for both.  The two sides touch independent tensors and have their own workspaces."""
    mk, mn = L.M * L.K, L.M * L.N
    wb = L.N * L.K * L.w_store // 8
    main = torch.cuda.current_stream()
    side.wait_stream(main)  # the previous layer's GEMM has consumed what this side overwrites next
    with torch.cuda.stream(side):
        P.calibrate_absmax(L.w, L.w_gran, out=L.am_w, ws=ws_w)
        P.quant_error(L.w, L.am_w, 2, 8, L.w_gran, out=L.sse_w, ws=ws_w)
        P.noise_inject(L.w, L.am_w, L.bits_w, LAMBDA, 2302, L.idx, L.w_gran, out=L.w_noisy)
        wq = {"packed4": L.w_codes} if L.w_store == 4 else {"codes": L.w_codes}
        if L.w_gran == P.PER_TENSOR:   # the quantizer kernel also leaves the step size
            P.fake_quant_step(L.w, L.am_w, L.bits_w, want_y=False, step=L.s_w, **wq)
        else:
            P.fake_quant(L.w, L.am_w, L.bits_w, L.w_gran, want_y=False, **wq)
            P.scale_from_absmax(L.am_w, L.bits_w, out=L.s_w)
    with rec("absmax", 4 * mk):
        P.calibrate_absmax(L.a, P.PER_TENSOR, out=L.am_a, ws=ws_a)
    with rec("quant_error", 4 * mk):
        P.quant_error(L.a, L.am_a, 2, 8, P.PER_TENSOR, out=L.sse_a, ws=ws_a)
    with rec("fake_quant", 5 * mk):
        P.fake_quant_step(L.a, L.am_a, L.bits_a, want_y=False, codes=L.a_codes, step=L.s_a)
    main.wait_stream(side)
    with rec("qgemm", mk + wb + 4 * mn, L.ops()):
        P.qgemm(L.a_codes, L.w_codes, L.s_a, L.s_w, L.w_store, L.w_gran, y=L.y, ws=ws_a)
    with rec("sse_pair", 8 * mn):
        P.sse_pair(L.y, L.y_ref, out=L.score, ws=ws_a)


def workload_layers(torch, P, workloads, which):
    layers = []
    if which == "cfg2":
        for idx, g in enumerate(workloads.CFG2):
            a, w, ba, bw = workloads.cfg2_layer(idx)
            layers.append(Layer(torch, idx, g.name, a, w, ba, bw, P.PER_ROW))
        label = ("cfg2: ResNet-50-shaped conv-as-GEMM stack, batch 32, 8 layers, whole hot path per layer "
                 "(absmax, quant_error b=2..8, noise, fake_quant, qgemm, sse_pair)")
    else:
        for idx, g in enumerate(workloads.CFG3):
            a, w, ba, bw = workloads.cfg3_layer(idx)
            layers.append(Layer(torch, idx, g.name, a, w, ba, bw, P.PER_TENSOR))
        label = ("cfg3: BERT-base encoder linears, seq 384 x batch 32 (M = 12288), 4 layers, whole hot path "
                 "per layer, per-tensor scales")
    ws_a, ws_w = P.Workspace(), P.Workspace()
    ws_a.get(1 << 22)
    ws_w.get(1 << 22)
    side = torch.cuda.Stream()  # default priority

    def step(rec):
        for L in layers:
            run_layer(P, L, ws_a, ws_w, rec, torch, side)
        torch.cuda.current_stream().wait_stream(side)

    def snapshot():
        out = []
        for L in layers:
            out += [L.score.clone(), L.sse_a.clone(), L.sse_w.clone(), L.am_w.clone()]
        return out

    nbytes = sum(sum(L.bytes().values()) for L in layers)
    ops = sum(L.ops() for L in layers)
    return step, snapshot, nbytes, ops, label, layers


# ------------------------------------------------------------------------------------------------
# configuration 4: sensitivity sweep over the BERT-large weight set
def workload_cfg4(torch, P, workloads, fused, n_streams=1):
    tensors = [torch.from_numpy(w).cuda() for _, w in workloads.cfg4_tensors()]
    dev = tensors[0].device
    f32, f64 = torch.float32, torch.float64
    am_t = [torch.empty(1, dtype=f32, device=dev) for _ in tensors]
    am_r = [torch.empty(t.shape[0], dtype=f32, device=dev) for t in tensors]
    sse_t = [torch.empty((1, 7), dtype=f64, device=dev) for _ in tensors]
    sse_r = [torch.empty((t.shape[0], 7), dtype=f64, device=dev) for t in tensors]
    # one output buffer per shape: a plane per bit-width when the seven noise levels come from one call
    # Tensors are independent: they are dealt round-robin to n_streams streams (each with its own
    # workspace and noise buffers), so that the launch ramp of one small kernel overlaps the body
    # of another.
    noisy_s = [{tuple(t.shape): torch.empty((7 if fused else 1,) + tuple(t.shape), dtype=f32, device=dev)
                for t in tensors} for _ in range(n_streams)]
    ws_s = [P.Workspace() for _ in range(n_streams)]
    for w in ws_s:
        w.get(1 << 22)
    extra = [torch.cuda.Stream() for _ in range(n_streams - 1)]   # default priority

    def step(rec):
        # kernel-level timing (events around calls) is taken with the tensors in sequence, so that
        # a call's duration is its own and not that of whatever shares the chip with it
        lanes = 1 if isinstance(rec, EventRec) else n_streams
        main = torch.cuda.current_stream()
        for st in extra[:lanes - 1]:
            st.wait_stream(main)
        for i, t in enumerate(tensors):
            lane = i % lanes
            with torch.cuda.stream(main if lane == 0 else extra[lane - 1]):
                one_tensor(rec, i, t, ws_s[lane], noisy_s[lane])
        for st in extra[:lanes - 1]:
            main.wait_stream(st)

    def one_tensor(rec, i, t, ws, noisy):
        n = t.numel()
        if fused:   # the tensor's maximum is the maximum of its row maxima: one read of the tensor
            with rec("absmax", 4 * n):
                P.calibrate_absmax(t, P.PER_ROW, out=am_r[i])
                P.calibrate_absmax(am_r[i].view(1, -1), P.PER_TENSOR, out=am_t[i], ws=ws)
        else:
            with rec("absmax", 8 * n):
                P.calibrate_absmax(t, P.PER_TENSOR, out=am_t[i], ws=ws)
                P.calibrate_absmax(t, P.PER_ROW, out=am_r[i])
        with rec("quant_error", 8 * n):
            P.quant_error(t, am_t[i], 2, 8, P.PER_TENSOR, out=sse_t[i], ws=ws)
            P.quant_error(t, am_r[i], 2, 8, P.PER_ROW, out=sse_r[i], ws=ws)
        if fused:   # z does not depend on b: drawn once, seven outputs
            with rec("noise_inject", (4 + 7 * 4) * n):
                P.noise_inject_sweep(t, am_r[i], 2, 8, LAMBDA, 2302, i, P.PER_ROW, out=noisy[tuple(t.shape)])
        else:
            with rec("noise_inject", 7 * 8 * n):
                for b in range(2, 9):
                    P.noise_inject(t, am_r[i], b, LAMBDA, 2302, i, P.PER_ROW, out=noisy[tuple(t.shape)][0])

    def snapshot():
        return [s.clone() for s in sse_t] + [s.clone() for s in sse_r[:8]]

    n_total = sum(t.numel() for t in tensors)
    label = ("cfg4: sensitivity sweep over 96 BERT-large weight tensors (302 M elements): absmax + quant_error "
             "b=2..8 per tensor and per output channel, noise at every b"
             + (" (row maxima reused for the tensor maximum; the seven noise levels from one call)" if fused
                else " (one call per granularity and per noise level)"))
    return step, snapshot, n_total * ((4 + 8 + 32) if fused else (8 + 8 + 56)), 0, label


# ------------------------------------------------------------------------------------------------
# configuration 5: candidate scoring on a BERT-large FFN block
def workload_cfg5(torch, P, workloads, mode):
    fused = mode != "unfused"
    x, w1, w2 = workloads.cfg5_tensors()
    cands = workloads.cfg5_candidates()
    dx, dw1, dw2 = torch.from_numpy(x).cuda(), torch.from_numpy(w1).cuda(), torch.from_numpy(w2).cuda()
    dev = dx.device
    M, K1 = dx.shape
    N1, N2 = dw1.shape[0], dw2.shape[0]
    f32, i8, u8, f64 = torch.float32, torch.int8, torch.uint8, torch.float64
    gelu = torch.nn.functional.gelu
    y_ref = gelu(dx @ dw1.t()) @ dw2.t()
    am_x, am_h = torch.empty(1, dtype=f32, device=dev), torch.empty(1, dtype=f32, device=dev)
    am_w1, am_w2 = torch.empty(1, dtype=f32, device=dev), torch.empty(1, dtype=f32, device=dev)
    s_h = torch.empty(1, dtype=f32, device=dev)
    # step sizes of the tensors whose absmax does not change from candidate to candidate, per width
    s_w1 = {b: torch.empty(1, dtype=f32, device=dev) for b in (2, 4, 8)}
    s_w2 = {b: torch.empty(1, dtype=f32, device=dev) for b in (2, 4, 8)}
    s_x = {b: torch.empty(1, dtype=f32, device=dev) for b in (4, 8)}
    cx = torch.empty((M, K1), dtype=i8, device=dev)
    ch = torch.empty((M, N1), dtype=i8, device=dev)
    cw1, pw1 = torch.empty((N1, K1), dtype=i8, device=dev), torch.empty((N1, K1 // 2), dtype=u8, device=dev)
    cw2, pw2 = torch.empty((N2, N1), dtype=i8, device=dev), torch.empty((N2, N1 // 2), dtype=u8, device=dev)
    h = torch.empty((M, N1), dtype=f32, device=dev)
    y = torch.empty((M, N2), dtype=f32, device=dev)
    scores = torch.empty(len(cands), dtype=f64, device=dev)
    ws = P.Workspace()
    ws.get(1 << 22)

    def quant_w(rec, dw, am, b, codes, packed):
        with rec("fake_quant", int(dw.numel() * (4.5 if b <= 4 else 5))):
            if b <= 4:
                P.fake_quant(dw, am, b, want_y=False, packed4=packed)
            else:
                P.fake_quant(dw, am, b, want_y=False, codes=codes)
        return (packed, 4) if b <= 4 else (codes, 8)

    def step(rec):
        with rec("absmax", 4 * (dx.numel() + dw1.numel() + dw2.numel())):
            P.calibrate_absmax(dx, out=am_x, ws=ws)
            P.calibrate_absmax(dw1, out=am_w1, ws=ws)
            P.calibrate_absmax(dw2, out=am_w2, ws=ws)
        for b in (2, 4, 8):
            P.scale_from_absmax(am_w1, b, out=s_w1[b])
            P.scale_from_absmax(am_w2, b, out=s_w2[b])
        for b in (4, 8):
            P.scale_from_absmax(am_x, b, out=s_x[b])
        for c, (bw1, ba1, bw2, ba2) in enumerate(cands):
            q1, st1 = quant_w(rec, dw1, am_w1, bw1, cw1, pw1)
            q2, st2 = quant_w(rec, dw2, am_w2, bw2, cw2, pw2)
            with rec("fake_quant", 5 * dx.numel()):
                P.fake_quant(dx, am_x, ba1, want_y=False, codes=cx)
            if mode == "twopass":
                # The first GEMM runs twice and stores no fp32 output: pass one keeps only the absmax
                # of GELU(H), pass two quantizes GELU(H) with it in the epilogue and stores int8 codes.
                with rec("qgemm", M * K1 + N1 * K1 * st1 // 8, 2 * M * N1 * K1):
                    P.qgemm_act(cx, q1, s_x[ba1], s_w1[bw1], P.ACT_GELU, st1, want_y=False, absmax=am_h)
                with rec("qgemm", M * K1 + N1 * K1 * st1 // 8 + M * N1, 2 * M * N1 * K1):
                    P.qgemm_act_codes(cx, q1, s_x[ba1], s_w1[bw1], P.ACT_GELU, am_h, ba2, st1, codes=ch)
            elif fused:  # GELU and the calibration of its output happen in the first GEMM's epilogue
                with rec("qgemm", M * K1 + N1 * K1 * st1 // 8 + 4 * M * N1, 2 * M * N1 * K1):
                    P.qgemm_act(cx, q1, s_x[ba1], s_w1[bw1], P.ACT_GELU, st1, y=h, absmax=am_h)
            else:
                with rec("qgemm", M * K1 + N1 * K1 * st1 // 8 + 4 * M * N1, 2 * M * N1 * K1):
                    P.qgemm(cx, q1, s_x[ba1], s_w1[bw1], st1, y=h, ws=ws)
                torch.ops.aten.gelu_(h)  # torch, in place, same stream
                with rec("absmax", 4 * h.numel()):
                    P.calibrate_absmax(h, out=am_h, ws=ws)
            if mode != "twopass":
                with rec("fake_quant", 5 * h.numel()):
                    P.fake_quant_step(h, am_h, ba2, want_y=False, codes=ch, step=s_h)
            else:
                P.scale_from_absmax(am_h, ba2, out=s_h)
            if fused:  # the score is taken in the epilogue: Y_ref is read, Y is never written
                with rec("qgemm", M * N1 + N2 * N1 * st2 // 8 + 4 * M * N2, 2 * M * N2 * N1):
                    P.qgemm_score(ch, q2, s_h, s_w2[bw2], y_ref, st2, out=scores[c:c + 1], ws=ws)
            else:
                with rec("qgemm", M * N1 + N2 * N1 * st2 // 8 + 4 * M * N2, 2 * M * N2 * N1):
                    P.qgemm(ch, q2, s_h, s_w2[bw2], st2, y=y, ws=ws)
                with rec("sse_pair", 8 * y.numel()):
                    P.sse_pair(y, y_ref, out=scores[c:c + 1], ws=ws)

    def snapshot():
        return [scores.clone()]

    if mode == "twopass":
        first = 2 * (M * K1 + N1 * K1) + M * N1
    else:
        first = (M * K1 + N1 * K1 + 4 * M * N1) + (0 if fused else 4 * M * N1) + 5 * M * N1
    per_cand = (4.75 * (dw1.numel() + dw2.numel()) + 5 * dx.numel() + first + (M * N1 + N2 * N1 + 4 * M * N2)
                + (0 if fused else 8 * M * N2))
    nbytes = int(len(cands) * per_cand + 4 * (dx.numel() + dw1.numel() + dw2.numel()))
    ops = len(cands) * ((2 if mode == "twopass" else 1) * 2 * M * N1 * K1 + 2 * M * N2 * N1)
    label = ("cfg5: 64 candidate bit configurations of a BERT-large FFN block (1024 -> 4096 -> 1024) at "
             "M = 16384, back to back: re-quantize, qgemm, GELU, calibrate, re-quantize, qgemm, output SSE"
             + {"twopass": "; the first GEMM runs twice (absmax of GELU(H), then int8 codes of GELU(H) from the "
                           "epilogue: no fp32 H in HBM), the score in the second GEMM's epilogue",
                "onepass": "; GELU + calibration in the first GEMM's epilogue, the score in the second's",
                "unfused": "; GELU by torch, calibration and score as passes of their own"}[mode])
    return step, snapshot, nbytes, ops, label, len(cands)


# ------------------------------------------------------------------------------------------------
# the default run: the metric's two halves on their own workloads
def _timed_calls(torch, calls, reps):
    """Average duration in microseconds of each call of `calls` (name -> function), `reps` launches
    each, HIP events on the launch stream around every single call, the host kept ahead of the GPU
    by a spin kernel."""
    out = {}
    for name, fn in calls.items():
        fn()
        torch.cuda.synchronize()
        pairs = []
        torch.cuda._sleep(3_000_000)
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            pairs.append((e0, e1))
        torch.cuda.synchronize()
        out[name] = sum(a.elapsed_time(b) for a, b in pairs) * 1e3 / reps
    return out


# HBM traffic per launch of mpq_qgemm on cfg5.ffn2 (16384 x 4096 x 1024), bytes, from the counter runs
# summarised in profiles/cfg5_ffn2_qgemm_hbm_traffic.txt: (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000) KiB
TRAFFIC_BYTES_PER_LAUNCH_GEMM = {
    ("cfg5.ffn2", 8): (49275.3 * 2.0 + 67481.8) * 1024.0,
    ("cfg5.ffn2", 4): (41118.6 * 2.0 + 66957.9) * 1024.0,
}

# HBM traffic per launch of the batched sweep kernels over configuration 4, bytes, from the rocprofv3
# counter runs summarised in profiles/cfg4_batched_sweep_hbm_traffic.txt (FETCH_SIZE and WRITE_SIZE
# scaled by what the same counters read for a plain device copy of known size in the same run).
TRAFFIC_BYTES_PER_LAUNCH_CFG4 = {   # (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000) KiB of the call's two kernels
    "calibrate_absmax_batch": ((590499.1 + 451.5) * 2.0 + 1319.4 + 3.0) * 1024.0,
    "quant_error_batch_per_tensor": ((590230.9 + 157.5) * 2.0 + 360.0 + 7.5) * 1024.0,
    "quant_error_batch_per_row": (591782.5 * 2.0 + 12533.1) * 1024.0,
}


def bench_sweep_cfg4(torch, mpq, workloads, steps, warmup):
    host = [w for _, w in workloads.cfg4_tensors()]
    tensors = [torch.from_numpy(w).cuda() for w in host]
    n = sum(t.numel() for t in tensors)
    plan = mpq.sweep_plan_build(tensors)

    def step():
        mpq.calibrate_absmax_batch(plan)
        mpq.quant_error_batch(plan, mpq.PER_TENSOR)
        mpq.quant_error_batch(plan, mpq.PER_ROW)

    # From idle the chip needs some 15 ms of work before its clocks are up (a step is 0.6 ms: with
    # three warm-up steps the first 20 timed ones run 15 % slower).  Whatever --warmup says, the
    # device is first kept busy with the same steps for CLOCK_RAMP_S; then the W warm-up steps.
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < CLOCK_RAMP_S:
        for _ in range(8):
            step()
        torch.cuda.synchronize()
    for _ in range(max(warmup, 1)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    # kernel-level figures: the same steps again with HIP events (on the launch stream) around every
    # call, the host kept ahead of the GPU by a spin kernel; a call is its main kernel plus a
    # finishing kernel of a few microseconds
    names = ("calibrate_absmax_batch", "quant_error_batch_per_tensor", "quant_error_batch_per_row")
    calls = (lambda: mpq.calibrate_absmax_batch(plan), lambda: mpq.quant_error_batch(plan, mpq.PER_TENSOR),
             lambda: mpq.quant_error_batch(plan, mpq.PER_ROW))
    pairs = {k: [] for k in names}
    torch.cuda._sleep(3_000_000)
    for _ in range(steps):
        for k, fn in zip(names, calls):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            pairs[k].append((e0, e1))
    torch.cuda.synchronize()
    us = {k: sum(a.elapsed_time(b) for a, b in v) * 1e3 / len(v) for k, v in pairs.items()}
    us.update(_timed_calls(torch, {
        "quant_error_batch_both_in_one_read": lambda: mpq.quant_error_batch(plan, mpq.SWEEP_TENSOR_AND_ROW),
        "calibrate_quant_error_rows_batch": lambda: mpq.calibrate_quant_error_rows_batch(plan)}, steps))
    # the same results from two reads instead of three: calibration and the per-row sums from one read,
    # then the per-tensor sums (8 algorithmic bytes per element; reported beside the three-call step)
    def step_two_reads():
        mpq.calibrate_quant_error_rows_batch(plan)
        mpq.quant_error_batch(plan, mpq.PER_TENSOR)

    for _ in range(max(warmup // 2, 1)):
        step_two_reads()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step_two_reads()
    torch.cuda.synchronize()
    ms_two = (time.perf_counter() - t0) * 1e3 / steps
    gbs = {k: 4.0 * n / v / 1e3 for k, v in us.items()}
    # the noise levels: one call per tensor, seven planes each (4 bytes read + 28 written per element)
    noisy = {}
    for t in tensors:
        if tuple(t.shape) not in noisy:
            noisy[tuple(t.shape)] = torch.empty((7,) + tuple(t.shape), dtype=torch.float32, device=t.device)

    def noise_step():
        for i, t in enumerate(tensors):
            mpq.noise_inject_sweep(t, plan.absmax_row[i], 2, 8, LAMBDA, 2302, i, mpq.PER_ROW, out=noisy[tuple(t.shape)])

    noise_step()
    torch.cuda.synchronize()
    k_noise = max(1, min(steps, 5))
    t0 = time.perf_counter()
    for _ in range(k_noise):
        noise_step()
    torch.cuda.synchronize()
    noise_ms = (time.perf_counter() - t0) * 1e3 / k_noise
    slow = max(("quant_error_batch_per_tensor", "quant_error_batch_per_row"), key=lambda k: us[k])
    return {
        "tensors": len(tensors), "elements": n, "bytes_per_step": 12 * n, "launches_per_step": 5,
        "clock_ramp_ms_before_warmup": CLOCK_RAMP_S * 1e3,
        "ms_per_step": ms, "gbs": 12.0 * n / ms / 1e6, "frac_of_hbm_peak": 12.0 * n / ms / 1e6 / HBM_PEAK_GBS,
        "call_us": {k: round(v, 2) for k, v in us.items()},
        "same_results_from_two_reads": {"ms_per_step": ms_two, "launches_per_step": 4, "bytes_per_step": 8 * n,
                                        "gbs": 8.0 * n / ms_two / 1e6, "speedup_over_three_calls": ms / ms_two},
        "call_gbs_at_4_bytes_per_element": {k: round(v, 1) for k, v in gbs.items()},
        "call_frac_of_hbm_peak": {k: round(v / HBM_PEAK_GBS, 4) for k, v in gbs.items()},
        "both_in_one_read_alu_view": {
            "lane_ops_per_element": 56,
            "t_lane_ops_per_s": round(56.0 * n / us["quant_error_batch_both_in_one_read"] / 1e6, 2),
            "frac_of_alu_peak": round(56.0 * n / us["quant_error_batch_both_in_one_read"] / 1e6 / ALU_PEAK_TLANEOPS, 4)},
        "noise_7_levels": {"ms_per_sweep": noise_ms, "bytes_per_sweep": 32 * n, "gbs": 32.0 * n / noise_ms / 1e6,
                           "frac_of_hbm_peak": 32.0 * n / noise_ms / 1e6 / HBM_PEAK_GBS, "launches": len(tensors)},
        "roofline": {"bound": "hbm", "achieved": gbs[slow], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbs[slow] / HBM_PEAK_GBS, "traffic": TRAFFIC_BYTES_PER_LAUNCH_CFG4.get(slow),
                     "kernel": slow + " (b = 2..8, all 96 tensors in one launch + a finishing launch)",
                     "algorithmic_per_launch": 4.0 * n, "avg_launch_us": us[slow], "bar": 0.70,
                     "alu_view": {"lane_ops_per_element": 28, "achieved": 28.0 * n / us[slow] / 1e6,
                                  "peak": ALU_PEAK_TLANEOPS, "unit": "T lane-op/s",
                                  "frac": 28.0 * n / us[slow] / 1e6 / ALU_PEAK_TLANEOPS}},
    }, host


def gemm_shape_rows(workloads, reps=30, warmup=4, only=None):
    """only: "MxKxN" restricts the table to that one shape (what the counter passes profile)."""
    from paper_2302_01382_amd import latency as lat
    rows = []
    for cfg, shapes in (("cfg2", workloads.CFG2), ("cfg3", workloads.CFG3), ("cfg5", workloads.CFG5)):
        for g in shapes:
            if only and only != "%dx%dx%d" % (g.M, g.K, g.N):
                continue
            for st in (8, 4):
                us = lat.time_qgemm(g.M, g.K, g.N, st, reps=reps, warmup=warmup)
                ops = 2.0 * g.M * g.N * g.K
                nbytes = g.M * g.K + g.N * g.K * st // 8 + 4.0 * g.M * g.N
                tops = ops / us / 1e6
                roof_tops = min(INT8_PEAK_TOPS, ops / nbytes * HBM_PEAK_GBS / 1e3)
                rows.append({"shape": "%s.%s" % (cfg, g.name), "M": g.M, "K": g.K, "N": g.N, "w_storage_bits": st,
                             "us": round(us, 2), "tops": round(tops, 1), "frac_of_int8_mfma_peak": round(tops / INT8_PEAK_TOPS, 4),
                             "roofline_tops": round(roof_tops, 1), "frac_of_own_roofline": round(tops / roof_tops, 4),
                             "bound": "mfma" if roof_tops >= INT8_PEAK_TOPS else "hbm"})
    return rows


def bench_gemm_block(torch, mpq, workloads, peaks):
    rows = gemm_shape_rows(workloads)
    for r in rows:
        r["frac_of_measured_mfma_rate_random_bytes"] = round(r["tops"] / peaks["int8_mfma_tops_random_bytes"], 4)
    long_k = [r for r in rows if r["K"] >= 2048]
    best = max(rows, key=lambda r: r["tops"])
    ops = sum(2.0 * r["M"] * r["N"] * r["K"] for r in rows)
    us = sum(r["us"] for r in rows)
    ops_k = sum(2.0 * r["M"] * r["N"] * r["K"] for r in long_k)
    us_k = sum(r["us"] for r in long_k)
    return {
        "operands": "uniformly random int8 / nibbles, rotated through more buffers than the 256 MB memory-side cache holds; "
                    "per-output-channel scales, fp32 output",
        "tops_all_shapes": ops / us / 1e6, "tops_k_ge_2048_shapes": ops_k / us_k / 1e6,
        "frac_of_int8_mfma_peak_k_ge_2048_shapes": ops_k / us_k / 1e6 / INT8_PEAK_TOPS,
        "w4_over_w8_time_ratio": {"worst": max(round(b["us"] / a["us"], 3) for a, b in zip(rows[0::2], rows[1::2])),
                                  "best": min(round(b["us"] / a["us"], 3) for a, b in zip(rows[0::2], rows[1::2])),
                                  "all_shapes_together": round(sum(r["us"] for r in rows[1::2]) / sum(r["us"] for r in rows[0::2]), 3)},
        "shapes": rows,
        "roofline": {"bound": "mfma", "achieved": best["tops"], "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                     "frac": best["tops"] / INT8_PEAK_TOPS,
                     "traffic": TRAFFIC_BYTES_PER_LAUNCH_GEMM.get((best["shape"], best["w_storage_bits"])), "bar": 0.60,
                     "kernel": "qgemm %s W%d (%d x %d x %d)" % (best["shape"], best["w_storage_bits"], best["M"], best["K"], best["N"]),
                     "algorithmic_per_launch": 2.0 * best["M"] * best["N"] * best["K"], "avg_launch_us": best["us"],
                     "frac_of_measured_mfma_rate_random_bytes": best["tops"] / peaks["int8_mfma_tops_random_bytes"]},
    }


def _cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline_headline(workloads, host_tensors):
    """The oracle as it stands, on the host cores of this machine.  Sweep half: the same three passes
    (row + tensor maxima, error sums per tensor, error sums per row) at full tensor size, on one
    thread over the first 2 layers (8 tensors) and on all cores over the first 12 layers (48 tensors;
    one tensor per task -- the oracle itself is single threaded, ctypes releases the interpreter
    lock).  GEMM half: the oracle's triple loop on the first 256 rows of configuration 5's second
    GEMM (rows are independent), with the extrapolation to all 16384 rows labelled as such."""
    import numpy as np
    import oracle
    oracle.lib()

    def sweep_one(w):
        t0 = time.perf_counter()
        mr = oracle.absmax(w, oracle.PER_ROW)
        mt = oracle.absmax(w)
        oracle.quant_error(w, mt)
        oracle.quant_error(w, mr, gran=oracle.PER_ROW)
        return time.perf_counter() - t0

    one = host_tensors[:8]
    t0 = time.perf_counter()
    for w in one:
        sweep_one(w)
    t_one = time.perf_counter() - t0
    gbs_one = 12.0 * sum(w.size for w in one) / t_one / 1e9
    cores = max(1, len(os.sched_getaffinity(0)))
    many = host_tensors[:48]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        busy = sum(ex.map(sweep_one, many))
    t_all = time.perf_counter() - t0
    gbs_all = 12.0 * sum(w.size for w in many) / t_all / 1e9
    g = workloads.CFG5[1]
    r = np.random.Generator(np.random.PCG64(5))
    a = r.integers(-127, 128, (256, g.K), dtype=np.int8)
    w = r.integers(-127, 128, (g.N, g.K), dtype=np.int8)
    t0 = time.perf_counter()
    oracle.qgemm(a, w, np.ones(1, np.float32), np.ones(g.N, np.float32), 8, oracle.PER_ROW)
    t_g = time.perf_counter() - t0
    return {
        "value": gbs_all, "unit": "GB/s", "cores": cores, "kind": "oracle", "cpu": _cpu_model(),
        "sample": "configuration 4 sweep (row + tensor maxima, error sums b = 2..8 per tensor and per row; 12 bytes per "
                  "element) at full tensor size: all cores on the first 48 of the 96 tensors, %.1f s wall, %.1f s "
                  "summed over threads; one thread on the first 8 tensors, %.1f s" % (t_all, busy, t_one),
        "value_one_thread": gbs_one,
        "gemm": {"sample": "oracle triple loop on the first 256 of the 16384 rows of cfg5.ffn2 (K = 4096, N = 1024), one thread",
                 "seconds_measured": t_g, "tops_measured": 2.0 * 256 * g.K * g.N / t_g / 1e12,
                 "seconds_full_M_extrapolated": t_g * g.M / 256, "cores": 1},
    }


def run_headline(torch, mpq, workloads, args):
    peaks = measured_peaks(torch, mpq)
    sweep, host_tensors = bench_sweep_cfg4(torch, mpq, workloads, args.steps, args.warmup)
    torch.cuda.empty_cache()
    gemm = bench_gemm_block(torch, mpq, workloads, peaks)
    torch.cuda.empty_cache()
    # the per-layer path of configuration 2 as a third block
    step, snapshot, nbytes, ops, label, layers = workload_layers(torch, mpq, workloads, "cfg2")
    k2 = max(1, min(args.steps, 10))
    m = measure(torch, step, snapshot, k2, min(args.warmup, 2))
    probe_ms = m["probe"].totals_ms()
    cfg2 = {"workload": label, "steps": k2, "ms_per_step": m["ms_per_step"], "gbs": nbytes / (m["ms_per_step"] * 1e-3) / 1e9,
            "step_algorithmic_bytes": nbytes, "step_gemm_ops": ops, "launch": m["launch"], "qgemm": gemm_summary(m),
            "timed_call_ms_probe_step": {k: round(v, 4) for k, v in probe_ms.items()},
            "timed_call_gbs_probe_step": {k: round(m["probe"].bytes[k] / (v * 1e-3) / 1e9, 1) for k, v in probe_ms.items()},
            "roofline_of_dominant_call": roofline_of(m, TRAFFIC_KIB_PER_LAUNCH_CFG2)}
    del layers, step, snapshot
    torch.cuda.empty_cache()
    rooflines = [sweep.pop("roofline"), gemm.pop("roofline")]
    head = min(rooflines, key=lambda r: r["frac"] / r["bar"])   # the kernel furthest below its bar
    out = {
        "metric": METRIC, "value": sweep["gbs"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sweep["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 elementwise, int8 x int8 -> int32 GEMM", "data": "synthetic",
        "config": {"workload": "cfg4 sensitivity sweep over the 96 BERT-large weight tensors (value, ms_per_step: max calibration "
                               "per row and per tensor + error sums b = 2..8 per tensor and per row, batched calls, 12 bytes per "
                               "element); qgemm on the 14 GEMM shapes of cfg2 / cfg3 / cfg5 (block `gemm`, headline shape "
                               "cfg5.ffn2 16384 x 4096 x 1024); the cfg2 per-layer path (block `cfg2`)"},
        "value_qgemm_tops_best_shape": rooflines[1]["achieved"],
        "sweep": sweep, "gemm": gemm, "cfg2": cfg2, "roofline": head, "rooflines": rooflines, "measured_peaks": peaks,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_headline(workloads, host_tensors)
    print(json.dumps(out))


# ------------------------------------------------------------------------------------------------
def cpu_baseline(workloads, sample_rows):
    """The oracle, as it stands, over the configuration-2 path on a bounded sample: the first
    `sample_rows` activation rows of every layer with the full weight tensors.  Layers run on a
    thread pool (the oracle itself is single threaded; ctypes releases the GIL)."""
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
    cpu = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                cpu = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    busy = sum(r[1] for r in res)
    return {
        "value": total / wall / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
        "sample": "cfg2 path on the first %d activation rows of each of the 8 layers, full weights; "
                  "%.1f s wall, %.1f s summed over threads" % (sample_rows, wall, busy),
        "value_per_thread": total / busy / 1e9, "cpu": cpu,
    }


def run_search(torch, mpq, workloads, args):
    """The loop the hot path exists for: Alg. 2 (greedy) and Alg. 1 (bisection) over a 24-layer
    stack of 1024 x 1024 layers at M = 4096, every evaluation a chain of libmpq launches ending in
    one read-back of the score.  Reports evaluations per second with the evaluation issued as one
    native call (mpq_stack_evaluate), call by call from Python, and as one HIP graph per (layer,
    width)."""
    from paper_2302_01382_amd.stack import QuantStack
    layers, width, rows, bits, target = 24, 1024, 4096, [8, 4, 2], 0.9
    x, weights = workloads.search_stack(seed=6, layers=layers, width=width, rows=rows)
    dx, dws = torch.from_numpy(x).cuda(), [torch.from_numpy(w).cuda() for w in weights]
    res = {}
    for mode, graphs in (("one_native_call", False), ("python_calls", False),
                         ("python_calls_hip_graph_per_layer_and_width", True)):
        st = QuantStack(dx, dws, bits, 8, use_graphs=graphs)
        ev = st.evaluate if mode == "one_native_call" else st.evaluate_by_calls   # evaluate_by_calls counts too
        order = st.order_by(st.qe_sensitivity(2))
        for b in bits:                       # warm-up: every (layer, width) pair once
            ev([b] * layers)
        torch.cuda.synchronize()
        # Both searches ask for configurations they have scored before (the first listed width equals
        # the starting width, so the whole first round of Alg. 2 re-scores an unchanged model): the
        # native-call mode answers those from a table (evaluate_once) and reports, per search, how
        # many evaluations were asked for, how many ran on the device and how many changed the model.
        memo = mode == "one_native_call"
        out_mode = {}
        for alg in ("greedy", "bisection"):
            st.scored, st.evaluations, st.repeats = {}, 0, 0
            fn = st.evaluate_once if memo else ev
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            cfg, asked = (st.greedy(order, target, fn) if alg == "greedy" else st.bisection(order, target, evaluate=fn))
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            ran = st.evaluations
            out_mode[alg] = {"evaluations": ran, "evaluations_asked_for": asked, "answered_from_table": st.repeats,
                             "seconds": dt, "evaluations_per_s": ran / dt, "mean_weight_bits": sum(cfg) / layers,
                             "accuracy": st.evaluate(cfg), "config": cfg}
        res[mode] = out_mode
    from paper_2302_01382_amd import latency as lat
    shapes = [(rows, width, width)] * layers
    table = lat.LatencyTable().measure(shapes[:1])
    for mode in res:
        for alg in ("greedy", "bisection"):
            cfg = res[mode][alg].pop("config")
            res[mode][alg]["estimated_relative_latency"] = round(table.relative(shapes, cfg), 4)
            res[mode][alg]["relative_footprint"] = lat.relative_footprint(shapes, cfg)
    best = res["one_native_call"]["greedy"]
    ops_per_eval = 2.0 * rows * width * width * layers
    out = {
        "metric": "configuration-search evaluations/s (Alg. 2 greedy; each evaluation = the whole quantized stack)",
        "value": best["evaluations_per_s"], "unit": "evaluations/s", "n_gpus": 1, "steps": best["evaluations"],
        "warmup": len(bits), "ms_per_step": 1e3 / best["evaluations_per_s"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32 elementwise, int8 x int8 -> int32 GEMM",
        "data": "synthetic",
        "config": {"workload": "search: %d layers of %d x %d at M = %d, weight widths %s, activations 8 bit, "
                               "target accuracy %.2f (1 - SSE/||Y_ref||^2), order by E_QE at b = 2"
                               % (layers, width, width, rows, bits, target)},
        "qgemm_tops_inside_an_evaluation": ops_per_eval * best["evaluations_per_s"] / 1e12,
        "search": res,
    }
    print(json.dumps(out))


def run_hutchinson(torch, mpq, workloads, args):
    """Hessian-trace sensitivity (Sec. 3.2.3) of the BERT-large FFN block's two layers at M = 16384:
    a step takes the quadratic forms of 32 random sign vectors per tensor, drawn inside the kernel
    (mpq_hutchinson_quad_signs), for the activation tensors X [16384 x 1024] and GELU(H) [16384 x 4096].
    Five copies of the pair are rotated through so that no step finds its tensors in the 256 MB
    memory-side cache.  Also timed: 64 probes (the width at which the fp32 matrix rate is level with
    the read of the tensor)."""
    x, w1, _ = workloads.cfg5_tensors()
    dx = torch.from_numpy(x).cuda()
    dh = torch.nn.functional.gelu(dx @ torch.from_numpy(w1).cuda().t())
    copies = [(dx.clone(), dh.clone()) for _ in range(5)]
    M = dx.shape[0]
    ws = mpq.Workspace()
    ws.get(1 << 22)
    out_q = {}

    def step(i, probes, matrix, timed=None):
        for j, t in enumerate(copies[i % len(copies)]):
            K = t.shape[1]
            key = (probes, K)
            if key not in out_q:
                out_q[key] = (torch.empty((probes, K), dtype=torch.float32, device=t.device),
                              torch.empty(probes, dtype=torch.float64, device=t.device))
            v, q = out_q[key]
            if matrix:
                mpq.rademacher(7, 2 * i + j, probes, K, out=v)
            if timed is not None:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
            if matrix:
                mpq.hutchinson_quad(t, v, out=q, ws=ws)
            else:
                mpq.hutchinson_quad_signs(t, 7, 2 * i + j, probes, out=q, ws=ws)
            if timed is not None:
                e1.record()
                timed.append((j, e0, e1))

    res = {}
    for probes, matrix in ((32, False), (64, False), (32, True), (64, True)):
        for i in range(args.warmup):
            step(i, probes, matrix)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i, probes, matrix)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / args.steps
        timed = []
        for i in range(args.steps):
            torch.cuda._sleep(2_000_000)
            step(i, probes, matrix, timed)
        torch.cuda.synchronize()
        per = {0: [], 1: []}
        for j, e0, e1 in timed:
            per[j].append(e0.elapsed_time(e1) * 1e-3)
        res[(probes, matrix)] = {"wall_s": wall, "call_s": {j: sum(v) / len(v) for j, v in per.items()}}
    nbytes = 4 * (dx.numel() + dh.numel())
    r32, r64 = res[(32, False)], res[(64, False)]
    big = dh.numel()
    flops64 = 2.0 * big * 64
    est, err = None, None
    from paper_2302_01382_amd import hessian
    est, err = hessian.trace_linear_mse(dx, 32, 7, 0, ws)
    exact = 2.0 / M * float((dx.double() ** 2).sum().item())
    out = {
        "metric": "Hessian-trace probe GB/s of activations read (32 random sign vectors per tensor)",
        "value": nbytes / r32["wall_s"] / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r32["wall_s"] * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 (fp32 matrix cores, fp32 accumulate)", "data": "synthetic",
        "config": {"workload": "hutchinson: X [16384 x 1024] and GELU(H) [16384 x 4096] of configuration 5's FFN block, "
                               "32 probes each, 5 copies rotated (cold memory-side cache)", "step_algorithmic_bytes": nbytes},
        "roofline": {"bound": "hbm", "achieved": 4.0 * big / r32["call_s"][1] / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": 4.0 * big / r32["call_s"][1] / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "hutchinson_quad, 16384 x 4096, 32 probes", "algorithmic_per_launch": 4.0 * big,
                     "avg_launch_us": r32["call_s"][1] * 1e6},
        "probes_64": {"bound": "mfma", "achieved": flops64 / r64["call_s"][1] / 1e12, "peak": 157.3, "unit": "TFLOP/s",
                      "frac": flops64 / r64["call_s"][1] / 1e12 / 157.3, "avg_launch_us": r64["call_s"][1] * 1e6,
                      "hbm_gbs": 4.0 * big / r64["call_s"][1] / 1e9, "ms_per_step": r64["wall_s"] * 1e3},
        "probe_matrix_in_memory": {"probes_32_us": res[(32, True)]["call_s"][1] * 1e6,
                                   "probes_64_us": res[(64, True)]["call_s"][1] * 1e6},
        "trace_estimate_x": {"estimate": est, "standard_error": err, "exact": exact},
    }
    print(json.dumps(out))


def measured_peaks(torch, mpq):
    """What this chip sustains, measured in place: a plain device copy (HBM), the int8 matrix
    cores issuing from registers, on constant-byte and on uniformly random operands (the clock under
    matrix load depends on how much the operand bits toggle), and the vector ALUs on the error
    sweep's arithmetic."""
    n = mpq.diag_mfma_operand_bytes()
    g = torch.Generator(device="cuda").manual_seed(3)
    rnd = torch.randint(-127, 128, (n,), dtype=torch.int8, device="cuda", generator=g)
    const = torch.full((n,), 3, dtype=torch.int8, device="cuda")
    out = {"int8_mfma_tops_constant_bytes": round(mpq.diag_mfma_rate(const), 1),
           "int8_mfma_tops_random_bytes": round(mpq.diag_mfma_rate(rnd), 1),
           # the error sweep's own arithmetic on registers: the vector-ALU ceiling of the sweep kernels
           "sweep_arithmetic_t_lane_ops_per_s": round(mpq.diag_sweep_alu_rate(), 1)}
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB, more than the memory-side cache
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    out["copy_gbs_read_plus_write"] = round(2 * src.numel() * 4 * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    return out


def calibrate_copy(torch):
    """A plain device copy of known size (225792 KiB read, as many written), three times: what the
    FETCH_SIZE / WRITE_SIZE readings of a counter run are scaled by."""
    src = torch.empty(225792 * 256, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def run_gemm_shapes(torch, mpq, workloads, args):
    """mpq_qgemm on every configured GEMM shape (configurations 2, 3 and 5, int8 and packed int4
    weights, per-output-channel scales, fp32 output), operands rotated through more than the
    memory-side cache holds: time per launch, TOP/s, fraction of the int8 matrix peak, and
    fraction of the shape's own roofline min(matrix peak, arithmetic intensity x HBM peak)."""
    if args.calibrate_copy:
        calibrate_copy(torch)
    rows = gemm_shape_rows(workloads, only=args.shape)
    best = max(rows, key=lambda r: r["tops"])
    peaks = measured_peaks(torch, mpq)
    for r in rows:
        r["frac_of_measured_mfma_rate_random_bytes"] = round(r["tops"] / peaks["int8_mfma_tops_random_bytes"], 4)
    total_ops = sum(2.0 * r["M"] * r["N"] * r["K"] for r in rows)
    total_us = sum(r["us"] for r in rows)
    out = {
        "metric": "qgemm int8 TOPS over the configured shapes (W8 and W4, cold operands)",
        "value": total_ops / total_us / 1e6, "unit": "TOP/s", "n_gpus": 1, "steps": 30, "warmup": 4,
        "ms_per_step": total_us / 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8 x int8 -> int32, fp32 epilogue", "data": "synthetic",
        "config": {"workload": "gemm: the %d GEMM shapes of configurations 2, 3 and 5, int8 and packed int4 weights" % (len(rows) // 2)},
        "roofline": {"bound": "mfma", "achieved": best["tops"], "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                     "frac": best["tops"] / INT8_PEAK_TOPS,
                     "traffic": TRAFFIC_BYTES_PER_LAUNCH_GEMM.get((best["shape"], best["w_storage_bits"])),
                     "kernel": "qgemm %s W%d" % (best["shape"], best["w_storage_bits"]), "avg_launch_us": best["us"]},
        "measured_peaks": peaks,
        "shapes": rows,
    }
    print(json.dumps(out))


def run_kernels(torch, mpq, workloads, args):
    """Every streaming call of the path on ONE large tensor (16384 x 4096 fp32 = 268 MB, the hidden
    activation of configuration 5; five copies rotated so that the 256 MB memory-side cache is cold):
    microseconds per call (main kernel plus finishing kernel where there is one), algorithmic GB/s
    and the fraction of the HBM peak.  Best of three rounds of 20 back-to-back calls after six warm-up
    calls."""
    R, Cc, NBUF = 16384, 4096, 5
    n = R * Cc
    g = torch.Generator(device="cuda").manual_seed(11)
    xs = [torch.randn(R, Cc, device="cuda", generator=g) for _ in range(NBUF)]
    am_t = mpq.calibrate_absmax(xs[0])
    am_r = mpq.calibrate_absmax(xs[0], mpq.PER_ROW)
    y = torch.empty(R, Cc, device="cuda")
    codes = torch.empty(R, Cc, dtype=torch.int8, device="cuda")
    packed = torch.empty(R, Cc // 2, dtype=torch.uint8, device="cuda")
    out_t, out_r = torch.empty(1, device="cuda"), torch.empty(R, device="cuda")
    qe_t = torch.empty((1, 7), dtype=torch.float64, device="cuda")
    qe_r = torch.empty((R, 7), dtype=torch.float64, device="cuda")
    ws = mpq.Workspace()
    cases = [   # name, scope-table row, algorithmic bytes per element, call
        ("calibrate_absmax per tensor", "a1", 4.0, lambda i: mpq.calibrate_absmax(xs[i % NBUF], out=out_t, ws=ws)),
        ("calibrate_absmax per row", "a1", 4.0, lambda i: mpq.calibrate_absmax(xs[i % NBUF], mpq.PER_ROW, out=out_r, ws=ws)),
        ("fake_quant -> fp32", "a2", 8.0, lambda i: mpq.fake_quant(xs[i % NBUF], am_t, 8, y=y)),
        ("fake_quant -> int8 codes", "a2", 5.0,
         lambda i: mpq.fake_quant(xs[i % NBUF], am_t, 8, want_y=False, want_codes=True, codes=codes)),
        ("fake_quant -> packed int4", "a2", 4.5,
         lambda i: mpq.fake_quant(xs[i % NBUF], am_t, 4, want_y=False, want_packed4=True, packed4=packed)),
        ("fake_quant per row -> int8 codes", "a2", 5.0,
         lambda i: mpq.fake_quant(xs[i % NBUF], am_r, 8, mpq.PER_ROW, want_y=False, want_codes=True, codes=codes)),
        ("quant_error b = 2..8 per tensor", "a3", 4.0, lambda i: mpq.quant_error(xs[i % NBUF], am_t, out=qe_t, ws=ws)),
        ("quant_error b = 2..8 per row", "a3", 4.0,
         lambda i: mpq.quant_error(xs[i % NBUF], am_r, gran=mpq.PER_ROW, out=qe_r, ws=ws)),
        ("noise_inject, one level", "a4", 8.0, lambda i: mpq.noise_inject(xs[i % NBUF], am_t, 4, LAMBDA, 1, 2, out=y)),
        ("sse_pair", "a6", 8.0, lambda i: mpq.sse_pair(xs[i % NBUF], xs[(i + 1) % NBUF])),
    ]
    rows = []
    for name, row, bpe, fn in cases:
        for i in range(6):
            fn(i)
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(20):
                fn(i)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 20
            best = us if best is None or us < best else best
        rows.append({"call": name, "row": row, "us": round(best, 2), "bytes_per_element": bpe,
                     "gbs": round(bpe * n / best / 1e3, 1), "frac_of_hbm_peak": round(bpe * n / best / 1e3 / HBM_PEAK_GBS, 4)})
    slow = min(rows, key=lambda r: r["frac_of_hbm_peak"])
    total_bytes = sum(r["bytes_per_element"] for r in rows) * n
    total_us = sum(r["us"] for r in rows)
    print(json.dumps({
        "metric": "streaming calls of the path on one 268 MB tensor, algorithmic GB/s", "value": total_bytes / total_us / 1e3,
        "unit": "GB/s", "n_gpus": 1, "steps": 20, "warmup": 6, "ms_per_step": total_us / 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "kernels: a1, a2, a3, a4, a6 on one 16384 x 4096 fp32 tensor, five copies rotated (cold memory-side cache)"},
        "roofline": {"bound": "hbm", "achieved": slow["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": slow["frac_of_hbm_peak"], "traffic": None, "kernel": slow["call"], "bar": 0.70,
                     "algorithmic_per_launch": slow["bytes_per_element"] * n, "avg_launch_us": slow["us"]},
        "calls": rows}))


def run_latency(torch, mpq, workloads, args):
    """Kernel latency table of mpq_qgemm at inference batch size one (the configured ResNet-50 and
    BERT-base layer shapes with M divided by their batch of 32) and the relative latency /
    footprint it predicts for all-W4 against all-W8, the way the paper builds its latency columns."""
    from paper_2302_01382_amd import latency as lat
    groups = {"resnet50_batch1": [(g.M // 32, g.K, g.N) for g in workloads.CFG2],
              "bert_base_seq384_batch1": [(g.M // 32, g.K, g.N) for g in workloads.CFG3]}
    table = lat.LatencyTable()
    out_groups = {}
    for name, shapes in groups.items():
        table.measure(shapes)
        rows = [{"M": m, "K": k, "N": n, "w8_us": round(table.us[(m, k, n, 8)], 2), "w4_us": round(table.us[(m, k, n, 4)], 2)}
                for (m, k, n) in shapes]
        out_groups[name] = {"layers": rows,
                            "all_w8_us": round(table.estimate_us(shapes, [8] * len(shapes)), 2),
                            "all_w4_relative_latency": round(table.relative(shapes, [4] * len(shapes)), 4),
                            "all_w4_relative_footprint": lat.relative_footprint(shapes, [4] * len(shapes))}
    total = sum(v["all_w8_us"] for v in out_groups.values())
    print(json.dumps({
        "metric": "mpq_qgemm kernel latency table at batch 1 (microseconds) and the mixed-precision latency estimate",
        "value": total, "unit": "us (all layers W8A8, both models)", "n_gpus": 1, "steps": 40, "warmup": 5,
        "ms_per_step": total / 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8 x int8 -> int32 GEMM, fp32 epilogue", "data": "synthetic",
        "config": {"workload": "latency: qgemm per layer shape and weight storage (int8 / packed int4), cold operands"},
        "table": out_groups}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default: 100 for the sweep workloads, whose step is 0.7 ms; 20 otherwise)")
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed steps before them (default: 60 for the sweep workloads: from idle the chip needs "
                         "some 15 ms of work before its clocks are up, and the first 20 steps run 15 %% slower; 3 otherwise)")
    ap.add_argument("--workload", choices=["cfg2", "cfg3", "cfg4", "cfg4-1stream", "cfg4-unfused", "cfg5", "cfg5-twopass", "cfg5-unfused", "search", "latency", "hutchinson", "gemm", "headline", "sweep", "kernels"], default="headline")
    ap.add_argument("--shape", default=None, help="gemm: only this configured shape, as MxKxN (e.g. 16384x4096x1024)")
    ap.add_argument("--cpu-sample-rows", type=int, default=2048)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--streams", type=int, default=4,
                    help="cfg4: streams the independent tensors are dealt to (the box has 4 hardware queues per process)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain device copy of known size (225792 KiB) three times before the "
                         "warm-up: the reference that rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU only (the path has no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    sweep_like = args.workload in ("headline", "sweep")
    if args.steps is None:
        args.steps = 100 if sweep_like else 20
    if args.warmup is None:
        args.warmup = 60 if sweep_like else 3

    import torch
    from paper_2302_01382_amd import mpq, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; libmpq has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    mpq.lib()

    if args.workload == "headline":
        run_headline(torch, mpq, workloads, args)
        return
    if args.workload == "sweep":   # the sweep block of the default run alone (what the counter passes profile)
        if args.calibrate_copy:
            calibrate_copy(torch)
        sweep, _ = bench_sweep_cfg4(torch, mpq, workloads, args.steps, args.warmup)
        roof = sweep.pop("roofline")
        print(json.dumps({"metric": METRIC, "value": sweep["gbs"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
                          "warmup": args.warmup, "ms_per_step": sweep["ms_per_step"], "higher_is_better": True,
                          "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
                          "config": {"workload": "cfg4 sensitivity sweep, batched calls (the sweep block of the default run)"},
                          "sweep": sweep, "roofline": roof}))
        return
    if args.workload == "search":
        run_search(torch, mpq, workloads, args)
        return
    if args.workload == "latency":
        run_latency(torch, mpq, workloads, args)
        return
    if args.workload == "kernels":
        run_kernels(torch, mpq, workloads, args)
        return
    if args.workload == "hutchinson":
        run_hutchinson(torch, mpq, workloads, args)
        return
    if args.workload == "gemm":
        run_gemm_shapes(torch, mpq, workloads, args)
        return
    extra = {}
    traffic = None
    layers = None
    if args.workload in ("cfg2", "cfg3"):
        step, snapshot, nbytes, ops, label, layers = workload_layers(torch, mpq, workloads, args.workload)
        traffic = TRAFFIC_KIB_PER_LAUNCH_CFG2 if args.workload == "cfg2" else None
    elif args.workload in ("cfg4", "cfg4-unfused", "cfg4-1stream"):
        step, snapshot, nbytes, ops, label = workload_cfg4(torch, mpq, workloads, args.workload != "cfg4-unfused",
                                                           args.streams if args.workload == "cfg4" else 1)
    else:
        step, snapshot, nbytes, ops, label, ncand = workload_cfg5(torch, mpq, workloads, {"cfg5": "onepass", "cfg5-twopass": "twopass", "cfg5-unfused": "unfused"}[args.workload])
        extra["candidates_per_step"] = ncand
        args.steps = min(args.steps, 5)   # one step is 64 candidates (~20 ms); keep the GPU time bounded
    torch.cuda.synchronize()

    if args.calibrate_copy and layers is not None:
        dst = torch.empty_like(layers[0].a)
        for _ in range(3):
            dst.copy_(layers[0].a)   # plain copy: reads and writes layers[0].a.numel() * 4 bytes
        torch.cuda.synchronize()
        del dst

    m = measure(torch, step, snapshot, args.steps, args.warmup)
    ms = m["ms_per_step"]
    probe_ms = m["probe"].totals_ms()
    out = {
        "metric": METRIC,
        "value": nbytes / (ms * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 elementwise, int8 x int8 -> int32 GEMM",
        "data": "synthetic",
        "config": {"workload": label, "step_algorithmic_bytes": nbytes, "step_gemm_ops": ops},
        "launch": m["launch"],
        "qgemm": gemm_summary(m),
        "timed_call_ms_probe_step": {k: round(v, 4) for k, v in probe_ms.items()},
        "timed_call_gbs_probe_step": {k: round(m["probe"].bytes[k] / (v * 1e-3) / 1e9, 1)
                                      for k, v in probe_ms.items()},
        "roofline": roofline_of(m, traffic),
    }
    if "candidates_per_step" in extra:
        out["candidates_per_s"] = extra["candidates_per_step"] / (ms * 1e-3)
    out["measured_peaks"] = measured_peaks(torch, mpq)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(workloads, args.cpu_sample_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
