"""A stack of linear layers scored under a per-layer bit configuration: the evaluation step of
the paper's searches (Alg. 1, Alg. 2) built from libmpq calls only.

The model is y = W_L relu(... relu(W_1 x)): every layer's input is calibrated (max calibration,
Sec. 3.1), quantized to `act_bits` (Eq. 1) and multiplied with the layer's weight codes at the
width the configuration assigns to it; ReLU and the calibration of the next layer's input happen in
the GEMM's epilogue (mpq_qgemm_act), and the last layer takes the score against the fp32 output
of the unquantized model in its epilogue (mpq_qgemm_score).  The accuracy handed to the
searches is 1 - SSE / ||Y_ref||^2, a stand-in for the task accuracy the paper evaluates, which
needs its datasets and trained weights.  torch supplies device memory and the fp32 reference
output, nothing else.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

from . import mpq


class QuantStack:
    def __init__(self, x, weights: Sequence, bit_widths: Sequence[int], act_bits: int = 8,
                 w_gran: int = mpq.PER_ROW, use_graphs: bool = False):
        """x: fp32 device tensor [M, K_1]; weights: fp32 device tensors [N_l, K_l] with K_{l+1} = N_l;
        bit_widths: the widths (2..8) a layer may be given.
        use_graphs: in evaluate_by_calls, the launches of layer l at width b (quantize, step size,
        GEMM + ReLU + calibration) are captured into a HIP graph the first time that pair is
        evaluated and replayed from then on.  evaluate() itself issues everything from one native
        call and needs no graphs."""
        import torch
        self.torch = torch
        self.x = x.contiguous()
        self.weights = [w.contiguous() for w in weights]
        self.bit_widths = [int(b) for b in bit_widths]
        self.act_bits, self.w_gran = int(act_bits), w_gran
        for a, b in zip(self.weights[:-1], self.weights[1:]):
            if b.shape[1] != a.shape[0]:
                raise ValueError("layer shapes do not chain")
        if self.x.shape[1] != self.weights[0].shape[1]:
            raise ValueError("input width does not match the first layer")
        self.ws = mpq.Workspace()
        dev, f32 = self.x.device, torch.float32
        M = self.x.shape[0]
        # fp32 reference output of the unquantized model
        h = self.x
        for i, w in enumerate(self.weights):
            h = h @ w.t()
            if i + 1 < len(self.weights):
                h = torch.relu(h)
        self.y_ref = h.contiguous()
        self.ref_norm2 = float((self.y_ref.double() ** 2).sum().item())
        # every weight at every width, once: codes (int8, or packed nibbles up to 4 bits) and steps
        self.w_absmax = [mpq.calibrate_absmax(w, w_gran, ws=self.ws) for w in self.weights]
        self.w_q: List[Dict[int, Tuple[object, object, int]]] = []
        for w, am in zip(self.weights, self.w_absmax):
            per_b = {}
            for b in self.bit_widths:
                store = 4 if (b <= 4 and w.shape[1] % 2 == 0) else 8
                _, codes, packed = mpq.fake_quant(w, am, b, w_gran, want_y=False, want_codes=store == 8,
                                                  want_packed4=store == 4)
                per_b[b] = (codes if store == 8 else packed, mpq.scale_from_absmax(am, b), store)
            self.w_q.append(per_b)
        # buffers of one evaluation
        # one tensor for all layers' input maxima: the running maxima of layers 1.. are cleared by a
        # single fill at the start of an evaluation instead of one small kernel in front of every GEMM
        self.a_absmax_all = torch.zeros(len(self.weights), dtype=f32, device=dev)
        self.a_absmax = [self.a_absmax_all[l:l + 1] for l in range(len(self.weights))]
        self.a_scale_all = torch.empty(len(self.weights), dtype=f32, device=dev)
        self.a_scale = [self.a_scale_all[l:l + 1] for l in range(len(self.weights))]
        self.a_codes = [torch.empty((M, w.shape[1]), dtype=torch.int8, device=dev) for w in self.weights]
        self.h = [torch.empty((M, w.shape[0]), dtype=f32, device=dev) for w in self.weights[:-1]]
        self.sse = torch.empty(1, dtype=torch.float64, device=dev)
        # the model's input does not depend on the configuration: calibrated and quantized once
        mpq.calibrate_absmax(self.x, out=self.a_absmax[0], ws=self.ws)
        mpq.fake_quant(self.x, self.a_absmax[0], self.act_bits, want_y=False, codes=self.a_codes[0])
        mpq.scale_from_absmax(self.a_absmax[0], self.act_bits, out=self.a_scale[0])
        self.evaluations = 0
        self.repeats = 0
        self.scored: Dict[Tuple[int, ...], float] = {}
        self.use_graphs = use_graphs
        self.graphs = {}
        # the whole evaluation as one native call (mpq_stack_evaluate): the argument block is built once
        widths = self.bit_widths
        self.width_number = {b: i for i, b in enumerate(widths)}
        self.plan = mpq.StackPlan(
            M, [{"N": w.shape[0], "K": w.shape[1], "w_q": [self.w_q[l][b][0] for b in widths],
                 "w_scale": [self.w_q[l][b][1] for b in widths], "store": [self.w_q[l][b][2] for b in widths],
                 "a_codes": self.a_codes[l], "h": self.h[l] if l + 1 < len(self.weights) else None}
                for l, w in enumerate(self.weights)],
            self.a_absmax_all, self.a_scale_all, self.y_ref, self.act_bits, mpq.ACT_RELU, w_gran)

    def __len__(self):
        return len(self.weights)

    def evaluate(self, bits: Sequence[int]) -> float:
        """Accuracy 1 - SSE / ||Y_ref||^2 of the stack with layer l's weights at bits[l]: one native
        call enqueues every layer, then the one read-back of an evaluation."""
        self.plan.evaluate([self.width_number[int(b)] for b in bits], self.sse, self.ws)
        self.evaluations += 1
        return 1.0 - float(self.sse.item()) / self.ref_norm2

    def evaluate_once(self, bits: Sequence[int]) -> float:
        """evaluate() behind a table of the configurations already scored: the searches re-ask for a
        configuration they have seen whenever a trial changes nothing (the first width of the list
        equals the starting width, a rejected trial is followed by one that restores it), and the
        model is deterministic.  `evaluations` counts only the ones that ran on the device,
        `repeats` the ones answered from the table."""
        key = tuple(int(b) for b in bits)
        hit = self.scored.get(key)
        if hit is not None:
            self.repeats += 1
            return hit
        a = self.evaluate(bits)
        self.scored[key] = a
        return a

    def evaluate_by_calls(self, bits: Sequence[int]) -> float:
        """The same evaluation issued call by call from Python (optionally as one HIP graph per
        (layer, width)); kept as the reference the native call is checked against."""
        if len(self.weights) > 1:
            self.a_absmax_all[1:].zero_()   # a fill kernel; the epilogues below keep running maxima
        for l in range(len(self.weights)):
            b = int(bits[l])
            if not self.use_graphs:
                self._layer(l, b)
                continue
            g = self.graphs.get((l, b))
            if g is None:
                # once eagerly (sizes the workspace, so that nothing is allocated under capture),
                # then captured; both leave the layer's output in place like a replay does
                self._layer(l, b)
                self.torch.cuda.synchronize()
                g = self.torch.cuda.CUDAGraph()
                with self.torch.cuda.graph(g):
                    self._layer(l, b)
                self.graphs[(l, b)] = g
            g.replay()
        self.evaluations += 1
        return 1.0 - float(self.sse.item()) / self.ref_norm2   # the one read-back of an evaluation

    def _layer(self, l: int, b: int):
        """Layer l at weight width b: input h_{l-1} (x for the first layer) -> h_l, or the score."""
        P = mpq
        if l > 0:   # the input's maximum came out of the previous layer's epilogue; x is quantized once, at set-up
            P.fake_quant(self.h[l - 1], self.a_absmax[l], self.act_bits, want_y=False, codes=self.a_codes[l])
            P.scale_from_absmax(self.a_absmax[l], self.act_bits, out=self.a_scale[l])
        wq, sw, store = self.w_q[l][b]
        if l + 1 < len(self.weights):
            # ReLU and the max calibration of the next layer's input are taken in the epilogue
            P.qgemm_act(self.a_codes[l], wq, self.a_scale[l], sw, P.ACT_RELU, store, self.w_gran, y=self.h[l],
                        absmax=self.a_absmax[l + 1], accumulate=True)
        else:
            P.qgemm_score(self.a_codes[l], wq, self.a_scale[l], sw, self.y_ref, store, self.w_gran,
                          out=self.sse, ws=self.ws)

    def qe_sensitivity(self, b: int) -> List[float]:
        """E_QE of Eq. 2 for every weight tensor at width b (per-tensor scale)."""
        out = []
        for w in self.weights:
            am = mpq.calibrate_absmax(w, ws=self.ws)
            sse = mpq.quant_error(w, am, b_lo=b, b_hi=b, ws=self.ws)
            out.append(mpq.eqe(float(sse.item()), w.numel(), float(am.item())))
        return out

    def noise_sensitivity(self, b: int, lam: float = 0.28867513, seed: int = 0) -> List[float]:
        """E_N of Sec. 3.2.2 (Eq. 3-5) on this stack: for every layer, the drop of the score when
        Gaussian noise with the spread of b-bit rounding (sigma = lam * step_b, mpq_noise_inject) is
        added to that layer's weights alone, all layers otherwise at the widest listed width.  The
        noisy weights go through the same quantizer as the clean ones (widest width), into the
        layer's code buffer, which is restored afterwards; layer l draws from noise stream l."""
        top = max(self.bit_widths)
        base = self.evaluate([top] * len(self.weights))
        out = []
        for l, w in enumerate(self.weights):
            codes, scale, store = self.w_q[l][top]
            keep_codes, keep_scale = codes.clone(), scale.clone()
            noisy = mpq.noise_inject(w, self.w_absmax[l], b, lam, seed, l, self.w_gran)
            am = mpq.calibrate_absmax(noisy, self.w_gran, ws=self.ws)
            if store == 8:
                mpq.fake_quant(noisy, am, top, self.w_gran, want_y=False, codes=codes)
            else:
                mpq.fake_quant(noisy, am, top, self.w_gran, want_y=False, want_packed4=True, packed4=codes)
            mpq.scale_from_absmax(am, top, out=scale)
            out.append(base - self.evaluate([top] * len(self.weights)))
            codes.copy_(keep_codes)
            scale.copy_(keep_scale)
        return out

    def order_by(self, sensitivity: Sequence[float]) -> List[int]:
        """Layer ids in ascending order of sensitivity (ties: lower id first)."""
        return sorted(range(len(self.weights)), key=lambda l: (sensitivity[l], l))

    def bisection(self, order, target, ensure_target=True, evaluate=None):
        return mpq.search_bisection(order, sorted(self.bit_widths, reverse=True), target, evaluate or self.evaluate_once,
                                    ensure_target)

    def greedy(self, order, target, evaluate=None):
        return mpq.search_greedy(order, sorted(self.bit_widths, reverse=True), target, evaluate or self.evaluate_once)
