#!/usr/bin/env python3
"""Benchmark of the sparsified FFN training step (one pass of Alg. 1 + Alg. 2 = one "step") on one MI355X.

Prints ONE JSON line.  Headline (`value`, `ms_per_step`, `config.workload`, `roofline`, `cpu_baseline`): the largest
single-GPU configuration, the 70B-scale layer (T = 8192, d_model = 8192, d_ff = 28672) at ReLU zero fraction 0.90:
dense-equivalent TFLOP/s of ffn_sparse_step (12*T*D*F flop per step) and the speed-up over a dense bf16 FFN step built from
hipBLASLt GEMMs (torch.matmul) plus one-pass element-wise kernels, timed in the same process.  Under `configs` the same
figures for every other benchmark configuration (tiny, 1B, 7B, the 8-expert MoE layer, and the 70B layer at zero fractions
0.50 / 0.75 / 0.95); under `standalone_kernels` the two compressors alone at the 7B shape (HBM-bound, buffers rotated so
that no launch finds its input in the last-level cache); the 2:4 / V:N:M GEMM micro-benchmarks and the router's conversion
cost at the 1B shape.  `--workload W` makes W the headline instead (used for profiling one configuration).
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 matrix-core peak
HBM_PEAK_GBS = 8000.0
SPARSE_GEMM = "gemm_nt_v2_kernel<sparse A, smfmac_f32_32x32x32_bf16>"
DENSE_GEMM = "gemm_nt_v2_kernel<dense A, mfma_f32_32x32x16_bf16>"
WGRAD = "wgrad_vnm_kernel<compact V:N:M A, mfma_f32_32x32x16_bf16>"
VNM8_GEMM = "vnm8_gemm_kernel<V:2:8 A, smfmac_f32_32x32x32_bf16>"
ROUTER_GEMMS = ("router/y1c+sqrelu+2:4", "router/dy2c+dsqrelu", "router/y3", "router/dX", "router/dW2.T", "router/dW1")


def algorithmic_flops(stage, T, D, F, M=8):
    """Multiply-adds the method itself needs (non-zero products), times two, per launch."""
    tdf = float(T) * D * F
    act = 4.0 / M * tdf                                          # V:2:M activations: 2 of M survive (M = 8: a quarter)
    if stage.startswith("router/"):                              # neuron-level experts: every contraction covers 4 / M of the hidden units
        return act if stage in ROUTER_GEMMS else None
    return {"step/y1+sqrelu_vnm_compress": tdf, "step/dy2+dsqrelu_vnm": tdf, "step/y1": tdf, "step/dy2": tdf,   # 2:4 weights: half of K survives
            "step/y3": act, "step/dX": act, "step/dW2": act, "step/dW1": act}.get(stage)


def executed_flops(stage, T, D, F, M=8, gathered=True):
    """Flops the matrix cores are issued for (dense-equivalent of the instructions used)."""
    tdf = float(T) * D * F
    if stage.startswith("router/"):
        return 8.0 / M * tdf if stage in ROUTER_GEMMS else None
    act = (8.0 / M * tdf) if gathered else 2 * tdf              # eqs. (3), (7): only the kept columns are contracted / all F as plain 2:4
    return {"step/y1+sqrelu_vnm_compress": 2 * tdf, "step/dy2+dsqrelu_vnm": 2 * tdf, "step/y1": 2 * tdf, "step/dy2": 2 * tdf,
            "step/y3": act, "step/dX": act, "step/dW2": 2 * tdf, "step/dW1": 2 * tdf}.get(stage)


KERNEL_OF_STAGE = {"step/y1+sqrelu_vnm_compress": SPARSE_GEMM, "step/dy2+dsqrelu_vnm": SPARSE_GEMM, "step/y1": SPARSE_GEMM, "step/dy2": SPARSE_GEMM,
                   "step/y3": SPARSE_GEMM, "step/dX": SPARSE_GEMM, "step/dW2": WGRAD, "step/dW1": WGRAD,
                   "router/y1c+sqrelu+2:4": SPARSE_GEMM, "router/dy2c+dsqrelu": SPARSE_GEMM, "router/y3": SPARSE_GEMM, "router/dX": SPARSE_GEMM,
                   "router/dW2.T": DENSE_GEMM, "router/dW1": DENSE_GEMM}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="70b", help="headline workload: tiny | 1b | 7b | 70b | moe_expert | moe (8 experts, 16384 tokens routed top-2, grouped launches)")
    ap.add_argument("--zero-fraction", type=float, default=0.90)
    ap.add_argument("--mode", default="hard", choices=["hard", "soft"])
    ap.add_argument("--M", type=int, default=8, choices=[8, 16, 32, 64],
                    help="V:2:M block width of the activation format (Table 5); 8 is the headline configuration")
    ap.add_argument("--router", action="store_true",
                    help="time the neuron-level router's training step (Section 3.3: ffn_router_full_step = routing + grouped step, M / 4 experts) instead of the magnitude-based V:N:M step")
    ap.add_argument("--settle-s", type=float, default=None,
                    help="seconds of untimed work (both steps alternating) before the warm-up, so that the timed region sees steady-state clocks "
                         "(default 20; 0 with --headline-only, whose runs are traced by a profiler)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true", help="skip the other configurations, the stand-alone kernels and the micro-benchmarks (profiling runs)")
    ap.add_argument("--fp8", action="store_true", help="with --headline-only: also run the fp8 step (both weight-gradient variants) at the headline shape (profiling runs)")
    ap.add_argument("--micro-batches", action="store_true",
                    help="with --headline-only: also run the micro-batch variants (packed weights, separate forward / backward calls, float32 gradient accumulation; profiling runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy three times (reference kernel for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.settle_s is None:
        args.settle_s = 0.0 if args.headline_only else 20.0
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the step shards by tokens; no multi-GPU path is built). Use --gpus 1.")

    import numpy as np
    import torch
    import paper_2602_06183_amd as sffn
    from workload import CONFIGS, make_ffn_inputs, make_moe_inputs, make_router_inputs
    from workload.synth import neuron_std, bias_for_zero_fraction

    sffn.load()                     # fails loudly when the HIP library is missing
    mode = sffn.MODE_SOFT if args.mode == "soft" else sffn.MODE_HARD
    if args.workload == "moe" and (args.M != 8 or args.router):
        sys.exit("bench.py: the grouped (moe) step runs the magnitude-based M = 8 format")
    try:
        torch.backends.cuda.preferred_blas_library("hipblaslt")
    except Exception:
        pass

    def dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
        return torch.from_numpy(a).cuda()

    def bits(t):            # device bf16 tensor -> numpy bit patterns (for the CPU oracle leg)
        return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)

    def timed(fn, n):       # wall clock around n calls, synchronised on both sides
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    def ms_of(fn, n=10):    # events on torch's current stream, which is the stream the binding launches on
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / n

    def free():
        gc.collect()
        torch.cuda.empty_cache()

    class Workload:
        """Device tensors of one configuration, the sparse step and the dense baseline step on them."""

        def __init__(self, name, zero_fraction, M=8, router=False, host=None):
            self.name, self.zf, self.M, self.router, self.moe = name, zero_fraction, M, router, name == "moe"
            if self.moe:
                _, self.D, self.F = CONFIGS["moe_expert"]
                inp = host or make_moe_inputs(16384, 8, 2, self.D, self.F, seed=0, zero_fraction=zero_fraction)
                self.seg = [int(v) for v in inp["seg"]]
                self.T = int(inp["counts"].sum())           # flop are counted on routed tokens, not on the 64-row padding
            else:
                self.T, self.D, self.F = CONFIGS[name]
                inp = host or make_ffn_inputs(self.T, self.D, self.F, seed=0, zero_fraction=zero_fraction)
            self.host = inp
            self.X, self.W1, self.W2, self.b1, self.dY = (dev(inp[k]) for k in ("X", "W1", "W2", "b1", "dY"))
            T, D, F = self.T, self.D, self.F
            if router:
                self.means = dev(make_router_inputs(64, D, 4 * M, M, seed=0)["means"])
                self.step = sffn.FfnRouterStep(T, D, F, M, mode)
            else:
                # the timed configuration: no dense y1 / dy2 and no canonical copies of the packed tensors (inspection aids only)
                self.step = sffn.FfnStepGrouped(self.seg, D, F, mode, lean=True) if self.moe else sffn.FfnStep(T, D, F, mode, M=M, lean=True)
            self.flops = 12.0 * T * D * F
            # dense bf16 FFN step: six hipBLASLt GEMMs (torch.matmul) and the two element-wise equations, one pass each
            self.b1h = self.b1.to(torch.bfloat16)
            Tp = self.X.shape[0]                             # rows including padding
            bf = lambda *shape: torch.empty(shape, dtype=torch.bfloat16, device="cuda")
            self.y1, self.y2, self.dy2, self.dy1 = bf(Tp, F), bf(Tp, F), bf(Tp, F), bf(Tp, F)
            self.y3, self.dXd = bf(Tp, D), bf(Tp, D)
            self.dW1d, self.dW2d = torch.empty_like(self.W1), torch.empty_like(self.W2)
            if self.moe:
                self.parts = [tuple(t[self.seg[e]:self.seg[e + 1]] for t in (self.X, self.dY, self.y1, self.y2, self.y3, self.dy2, self.dy1, self.dXd))
                              for e in range(len(self.seg) - 1)]

        @staticmethod
        def _dense_ffn(X, W1, W2, b1h, dY, y1, y2, y3, dy2, dy1, dXd, dW1d, dW2d, elementwise=True):
            torch.addmm(b1h, X, W1.t(), out=y1)              # eq. (1)
            if elementwise:
                sffn.dense_sqrelu(y1, y2)                    # eq. (2), one pass
            torch.mm(y2, W2.t(), out=y3)                     # eq. (3)
            torch.mm(dY, W2, out=dy2)                        # eq. (4)
            torch.mm(dY.t(), y2, out=dW2d)                   # eq. (5)
            if elementwise:
                sffn.dense_dsqrelu(dy2, y1, dy1)             # eq. (6), one pass
            torch.mm(dy1, W1, out=dXd)                       # eq. (7)
            torch.mm(dy1.t(), X, out=dW1d)                   # eq. (8)

        def dense_step(self, elementwise=True):
            if self.moe:     # the dense MoE layer: the same eight calls per expert on its segment
                for e, (Xe, dYe, y1e, y2e, y3e, dy2e, dy1e, dXe) in enumerate(self.parts):
                    self._dense_ffn(Xe, self.W1[e], self.W2[e], self.b1h[e], dYe, y1e, y2e, y3e, dy2e, dy1e, dXe, self.dW1d[e], self.dW2d[e], elementwise)
            else:
                self._dense_ffn(self.X, self.W1, self.W2, self.b1h, self.dY, self.y1, self.y2, self.y3, self.dy2, self.dy1, self.dXd,
                                self.dW1d, self.dW2d, elementwise)

        def sparse_step(self):
            if self.router:      # Alg. 3 steps 1-2 and the grouped step in one call; the run offsets stay on the device
                self.step.full(self.means, self.X, self.W1, self.W2, self.b1, self.dY)
            else:
                self.step(self.X, self.W1, self.W2, self.b1, self.dY)

        def measure(self, steps, warmup):
            for _ in range(warmup):
                self.sparse_step()
                self.dense_step()
            r = {"ms_sparse": timed(self.sparse_step, steps), "ms_dense": timed(self.dense_step, steps)}      # the timed region: exactly `steps` steps
            r["ms_dense_gemms"] = timed(lambda: self.dense_step(False), steps)
            r["ms_sparse2"], r["ms_dense2"] = timed(self.sparse_step, steps), timed(self.dense_step, steps)  # second, interleaved pass: clock drift check
            return r

        def graph_replay_ms(self, steps):
            """The sparse step captured once in a HIP graph and replayed: what a training loop that captures its iteration pays
            (the entry points only enqueue kernels on the caller's stream, so they can be captured as they are)."""
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                self.sparse_step()
            graph.replay()
            return timed(graph.replay, steps)

        def retained_l1(self):
            """How much of the activation's L1 mass the V:N:M format keeps (sum of kept y2 / sum of all y2) and the ReLU zero
            fraction: one extra, untimed step that also stores the dense y1; plain torch reductions, measurement only."""
            if self.router or self.moe:
                return None, None
            self.y2 = self.dy2 = self.dy1 = None             # the dense baseline's buffers are no longer needed
            free()
            chk = sffn.FfnStep(self.T, self.D, self.F, mode, keep_dense=True, M=self.M)
            chk(self.X, self.W1, self.W2, self.b1, self.dY)
            sv = chk.saved()
            y2_all = torch.clamp_min(sv["y1"].float(), 0.0).square_().to(torch.bfloat16)        # eq. (2), rounded as the kernel does
            retained = round(float(sv["y2_vals"].float().sum() / y2_all.float().sum()), 4)
            zero_frac = round(float((y2_all == 0).float().mean()), 4)
            return retained, zero_frac

        def summary(self, r, with_l1=True):
            T, D, F = self.T, self.D, self.F
            tf = self.flops / (r["ms_sparse"] * 1e-3) / 1e12
            # speed-ups from both interleaved passes (sparse, dense, sparse, dense): the dense baseline slows by a few per cent while the
            # part warms up during the first passes, the sparse step hardly moves; the mean of the two passes cancels most of that drift
            sp, de = 0.5 * (r["ms_sparse"] + r["ms_sparse2"]), 0.5 * (r["ms_dense"] + r["ms_dense2"])
            out = {"T": T, "d_model": D, "d_ff": F, "zero_fraction": self.zf, "ms_per_step": round(r["ms_sparse"], 4),
                   "dense_ms_per_step": round(r["ms_dense"], 4), "dense_gemms_only_ms": round(r["ms_dense_gemms"], 4),
                   "speedup_vs_dense": round(de / sp, 4),
                   "speedup_vs_dense_gemms_only": round(r["ms_dense_gemms"] / r["ms_sparse"], 4),
                   "tflops_dense_equiv": round(tf, 2), "frac_of_mfma_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                   # the method's own non-zero multiply-adds: 4 T D F flop per step (eqs. (1), (4): T D F each; the four others T D F / 2)
                   # (V:2:M activations: eqs. (3), (5), (7), (8) shrink to 4 T D F / M flop each)
                   "algorithmic_frac_of_mfma_peak": round(tf * (2.0 + 16.0 / self.M) / 12.0 / MFMA_BF16_PEAK_TFLOPS, 4) if not self.router else None}
            if with_l1:
                out["retained_l1_fraction"], out["relu_zero_fraction"] = self.retained_l1()
            return out

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def fp8_section(hw, esteps, ewarm, ms16, msd):        # ms16, msd: the bf16-operand sparse step and the dense step of the same run
        # The same step with fp8 (E4M3) operands in eqs. (1), (3), (4), (7) (Section 3.4, closing paragraph), weight gradients in bf16.
        # Per-tensor scales as a delayed-scaling recipe would hold them: amax / 448 of each quantised tensor, from the step's own amax output.
        fp8_step = None
        if not hw.router and hw.M == 8 and hw.D % 128 == 0 and hw.F % 128 == 0:
            # one untimed call with provisional scales for the two inner tensors, then the maxima it reports (the delayed-scaling loop itself)
            amax = lambda t: max(float(t.float().abs().max()), 1e-12)
            sc = dict(x=amax(hw.X) / 448, w1=amax(hw.W1) / 448, w2=amax(hw.W2) / 448, y2=1.0, dy=amax(hw.dY) / 448, dy1=1.0)
            first = (sffn.FfnStepFp8Grouped(hw.seg, hw.D, hw.F, sc, mode) if hw.moe else sffn.FfnStepFp8(hw.T, hw.D, hw.F, sc, mode))
            first(hw.X, hw.W1, hw.W2, hw.b1, hw.dY)
            sc = {k: max(v, 1e-12) / 448 for k, v in first.amax_dict().items()}
            del first
            free()
            fp8_step = {"workload": hw.name, "bf16_sparse_ms_per_step": round(ms16, 4), "dense_bf16_ms_per_step": round(msd, 4),
                        "operands": "E4M3 codes in eqs. (1), (3), (4), (7), quantised inside the pruning passes and the V:N:M epilogues; "
                                    "six per-tensor scales = amax / 448; weight gradients (eqs. (5), (8)) in bf16, or on the same codes (fp8_weight_gradients)"}
            for name8, w8 in (("bf16_weight_gradients", False), ("fp8_weight_gradients", True)):
                st8 = (sffn.FfnStepFp8Grouped(hw.seg, hw.D, hw.F, sc, mode, wgrad_fp8=w8, lean=True) if hw.moe else
                       sffn.FfnStepFp8(hw.T, hw.D, hw.F, sc, mode, wgrad_fp8=w8, lean=True))
                run8 = lambda: st8(hw.X, hw.W1, hw.W2, hw.b1, hw.dY)
                for _ in range(ewarm):
                    run8()
                ms8 = timed(run8, esteps)
                fp8_step[name8] = {"ms_per_step": round(ms8, 4), "speedup_vs_dense_bf16": round(msd / ms8, 4), "speedup_vs_sparse_bf16": round(ms16 / ms8, 4),
                                   "tflops_dense_equiv": round(hw.flops / (ms8 * 1e-3) / 1e12, 2)}
                run8p = lambda: st8(hw.X, hw.W1, hw.W2, hw.b1, hw.dY, weights_packed=True)      # a micro-batch after the first: no weight passes
                run8p()
                ms8p = timed(run8p, esteps)
                fp8_step[name8]["weights_packed_ms_per_micro_batch"] = round(ms8p, 4)
                fp8_step[name8]["weights_packed_speedup_vs_dense_bf16"] = round(msd / ms8p, 4)
                del st8
                free()
            # Table 5's wider blocks with the same operands (fp8 weight gradients): eqs. (3), (7) on the gathered rows of the quantised weights
            wide8 = {}
            for m in (16, 32, 64):
                if hw.moe or (4 * hw.F // m) % 128:
                    continue
                first = sffn.FfnStepFp8(hw.T, hw.D, hw.F, sc, mode, M=m)
                first(hw.X, hw.W1, hw.W2, hw.b1, hw.dY)
                scm = {k: max(v, 1e-12) / 448 for k, v in first.amax_dict().items()}
                del first
                free()
                st8 = sffn.FfnStepFp8(hw.T, hw.D, hw.F, scm, mode, wgrad_fp8=True, lean=True, M=m)
                run8 = lambda: st8(hw.X, hw.W1, hw.W2, hw.b1, hw.dY)
                for _ in range(ewarm):
                    run8()
                ms8 = timed(run8, esteps)
                wide8["64:2:%d" % m] = {"ms_per_step": round(ms8, 4), "speedup_vs_dense_bf16": round(msd / ms8, 4), "tflops_dense_equiv": round(hw.flops / (ms8 * 1e-3) / 1e12, 2)}
                del st8
                free()
            if wide8:
                fp8_step["wide_blocks_fp8_weight_gradients"] = wide8
        return fp8_step

    def micro_section(hw, esteps, ewarm, sp_h, de_h):
        # Section 3.4: a weight is converted to 2:4 once per optimizer step and the cost is amortised over the micro-batches that pass through
        # the layer in between (pipeline parallelism / gradient accumulation).  SFFN_FLAG_WEIGHTS_PACKED = a micro-batch after the first: both
        # pruning passes skipped, same outputs.  Reported beside the headline, which always includes the pruning passes.
        if hw.router:
            return None
        run_packed = lambda: hw.step(hw.X, hw.W1, hw.W2, hw.b1, hw.dY, weights_packed=True)
        hw.sparse_step()
        for _ in range(ewarm):
            run_packed()
        ms_p = timed(run_packed, esteps)
        split_ms = None
        if not hw.moe:      # Alg. 1 and Alg. 2 as separate calls (ffn_sparse_forward / ffn_sparse_backward): the step's launches in two halves
            run_f = lambda: hw.step.forward(hw.X, hw.W1, hw.W2, hw.b1)
            run_b = lambda: hw.step.backward(hw.W1, hw.dY)
            run_f(); run_b()
            split_ms = {"forward_ms": round(timed(run_f, esteps), 4), "backward_ms": round(timed(run_b, esteps), 4)}
        accum = None
        if not hw.moe:      # weight gradients summed over the micro-batches in float32: inside the weight-gradient GEMMs' epilogues
                            # (SFFN_FLAG_DW_FP32_ACCUMULATE) against bf16 outputs + one add pass per weight in the framework
            acc_step = sffn.FfnStep(hw.T, hw.D, hw.F, mode, M=hw.M, lean=True, dw_fp32=True)
            main1, main2 = torch.zeros_like(acc_step.dW1), torch.zeros_like(acc_step.dW2)
            run_fused = lambda: acc_step(hw.X, hw.W1, hw.W2, hw.b1, hw.dY, weights_packed=True)

            def run_separate():
                _, _, g1, g2 = hw.step(hw.X, hw.W1, hw.W2, hw.b1, hw.dY, weights_packed=True)
                main1.add_(g1)
                main2.add_(g2)
            acc_step(hw.X, hw.W1, hw.W2, hw.b1, hw.dY)
            run_fused(); run_separate()
            accum = {"fused_into_the_weight_gradient_gemms_ms": round(timed(run_fused, esteps), 4),
                     "bf16_outputs_plus_add_passes_ms": round(timed(run_separate, esteps), 4)}
            del acc_step, main1, main2
            free()
        return {"weights_packed_ms_per_micro_batch": round(ms_p, 4), "speedup_vs_dense": round(de_h / ms_p, 4), "separate_calls": split_ms,
                "float32_gradient_accumulation": accum,
                "four_micro_batches_per_optimizer_step": {"ms_per_micro_batch": round((sp_h + 3 * ms_p) / 4, 4),
                                                          "speedup_vs_dense": round(de_h / ((sp_h + 3 * ms_p) / 4), 4)}}

    # ================= headline workload ===========================================================================
    M = args.M
    hw = Workload(args.workload, args.zero_fraction, M, args.router)
    T, D, F = hw.T, hw.D, hw.F
    # Before the warm-up the part is brought to the clocks it holds in a running job: a process that starts on an idle GPU sees the hipBLASLt
    # baseline 4-5 % faster for its first seconds (16.7 ms against 17.6 ms a few seconds later at `70b`; the sparse step moves by < 1 %), so a
    # speed-up taken there depends on how long the box had been idle.  Both steps alternate, untimed, for --settle-s seconds of wall clock.
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < args.settle_s:
        hw.sparse_step()
        hw.dense_step()
        torch.cuda.synchronize()
    res = hw.measure(args.steps, args.warmup)

    # ---- per-launch durations from HIP events on the stream the kernels run on --------------------
    sffn.profile_enable(True)
    acc = {}
    nprof = max(3, min(10, args.steps))
    for _ in range(nprof):
        hw.sparse_step()
        for name, ms in sffn.profile_read():
            acc[name] = acc.get(name, 0.0) + ms / nprof
    sffn.profile_enable(False)
    by_kernel = {}
    kos = dict(KERNEL_OF_STAGE)
    if M == 8 and not args.router:      # eqs. (3), (7) contract the V:2:8 activation as it is, kept rows picked at the fragment reads
        kos.update({"step/y3": VNM8_GEMM, "step/dX": VNM8_GEMM})
    if M != 8:      # wide blocks: eqs. (3), (7) gather rows, eqs. (5), (8) contract the dense transposed activation with the dense-operand tile kernel
        if "step/to24(y2)" not in acc:
            kos.update({"step/y3": "vnm_spmm_gather_kernel<smfmac_f32_32x32x32_bf16>", "step/dX": "vnm_spmm_gather_kernel<smfmac_f32_32x32x32_bf16>"})
        if "step/expand(y2)" in acc:    # the unfused path contracts the dense transposed activation; the fused one the compacted operand
            kos.update({"step/dW2": DENSE_GEMM, "step/dW1": DENSE_GEMM})
    for name, ms in acc.items():
        by_kernel.setdefault(kos.get(name, name), []).append((name, ms))
    dom_kernel = max(by_kernel, key=lambda k: sum(ms for _, ms in by_kernel[k]))
    launches = by_kernel[dom_kernel]
    avg_ms = sum(ms for _, ms in launches) / len(launches)
    alg = sum(algorithmic_flops(n, T, D, F, M) or 0.0 for n, _ in launches) / len(launches)
    gathered = "step/to24(y2)" not in acc
    exe = sum(executed_flops(n, T, D, F, M, gathered) or 0.0 for n, _ in launches) / len(launches)
    achieved = alg / (avg_ms * 1e-3) / 1e12
    # HBM bytes per launch of that kernel: from the rocprofv3 FETCH_SIZE / WRITE_SIZE passes of this same command, scaled by a
    # plain copy (the summaries and the scale factors are in profiles/; counters cannot be read from inside the timed process)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic_%s.json" % args.workload)
    if os.path.exists(tpath) and M == 8 and not args.router:
        traffic = json.load(open(tpath)).get(dom_kernel)
    roofline = {"bound": "mfma", "kernel": dom_kernel, "launches_per_step": len(launches), "launches": [n for n, _ in launches],
                "avg_launch_ms": round(avg_ms, 4), "algorithmic_flop_per_launch": alg,
                "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic,
                "issued": round(exe / (avg_ms * 1e-3) / 1e12, 2), "issued_frac": round(exe / (avg_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
    # the same figures for every contraction kernel of the step (the object above is the one with the largest share of the step)
    per_kernel = []
    for kname, ls in sorted(by_kernel.items(), key=lambda kv: -sum(ms for _, ms in kv[1])):
        a = sum(algorithmic_flops(n, T, D, F, M) or 0.0 for n, _ in ls) / len(ls)
        if a <= 0:
            continue
        e = sum(executed_flops(n, T, D, F, M, gathered) or 0.0 for n, _ in ls) / len(ls)
        ms = sum(v for _, v in ls) / len(ls)
        per_kernel.append({"kernel": kname, "launches": [n for n, _ in ls], "avg_launch_ms": round(ms, 4), "step_share": round(sum(v for _, v in ls) / sum(acc.values()), 3),
                           "achieved": round(a / (ms * 1e-3) / 1e12, 2), "frac": round(a / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                           "issued_frac": round(e / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)})
    roofline["kernels"] = per_kernel
    head = hw.summary(res)

    # ---- CPU oracle on the host cores: a bounded sample of the same workload -------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        # a narrower layer of the same d_model: the first Fs hidden units (whole V:N:M column blocks; hidden units only meet in
        # the sums of Y3 and dX) on the first Ts tokens, sized for roughly 10-30 s of numpy work
        Fs = F if F * D <= (1 << 25) else max(512, ((1 << 25) // D) // 64 * 64)
        Ts = min(T, max(64, (int(1.5e12 / (12.0 * D * Fs)) // 64) * 64))
        inp = hw.host
        w1o, w2o, b1o = (inp[k][0] if hw.moe else inp[k] for k in ("W1", "W2", "b1"))    # moe: expert 0 on its first tokens
        w1o, w2o, b1o = w1o[:Fs], np.ascontiguousarray(w2o[:, :Fs]), b1o[:Fs]
        t0 = time.perf_counter()
        if args.router:
            oracle.ffn_router_step_ref(inp["X"][:Ts], w1o, w2o, b1o, inp["dY"][:Ts], bits(hw.means), M, mode)
        else:
            oracle.ffn_sparse_step_ref(inp["X"][:Ts], w1o, w2o, b1o, inp["dY"][:Ts], mode, 64, M)
        dt = time.perf_counter() - t0
        cpu = {"value": round(12.0 * Ts * D * Fs / dt / 1e12, 5), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
               "sample": "oracle.%s on the first %d of %d tokens and the first %d of %d hidden units (same d_model, weights%s, bias), %.1f s"
                         % ("ffn_router_step_ref" if args.router else "ffn_sparse_step_ref", Ts, T, Fs, F, " of expert 0" if hw.moe else "", dt)}

    # ================= the other configurations, stand-alone kernels, micro-benchmarks =============================
    configs, kernels, gemm24, venom, router, fp8_bench, wide, router_step, fp8_step, other_mode = None, None, None, None, None, None, None, None, None, None
    micro = None
    if args.headline_only and args.micro_batches:
        micro = micro_section(hw, max(3, min(args.steps, 10)), max(1, min(args.warmup, 2)), 0.5 * (res["ms_sparse"] + res["ms_sparse2"]), 0.5 * (res["ms_dense"] + res["ms_dense2"]))
    if args.headline_only and args.fp8:
        fp8_step = fp8_section(hw, max(3, min(args.steps, 10)), max(1, min(args.warmup, 2)), 0.5 * (res["ms_sparse"] + res["ms_sparse2"]), 0.5 * (res["ms_dense"] + res["ms_dense2"]))
    if not args.headline_only and not args.router and M == 8:
        esteps, ewarm = max(3, min(args.steps, 10)), max(1, min(args.warmup, 2))
        configs = {}
        key = lambda name, zf: "%s@%.2f" % (name, zf)
        configs[key(hw.name, hw.zf)] = dict(head, headline=True)
        # the other mode of Section 2.2 on the same tensors (the paper's recipe prunes with soft-thresholding; positions, and so every GEMM, are the same)
        if not hw.moe:
            other = sffn.MODE_HARD if mode == sffn.MODE_SOFT else sffn.MODE_SOFT
            alt = sffn.FfnStep(hw.T, hw.D, hw.F, other, M=M, lean=True)
            run_alt = lambda: alt(hw.X, hw.W1, hw.W2, hw.b1, hw.dY)
            for _ in range(ewarm):
                run_alt()
            other_mode = {"mode": "hard" if other == sffn.MODE_HARD else "soft", "ms_per_step": round(timed(run_alt, esteps), 4)}
            del alt
            free()
        micro = micro_section(hw, esteps, ewarm, 0.5 * (res["ms_sparse"] + res["ms_sparse2"]), 0.5 * (res["ms_dense"] + res["ms_dense2"]))
        fp8_step = fp8_section(hw, esteps, ewarm, 0.5 * (res["ms_sparse"] + res["ms_sparse2"]), 0.5 * (res["ms_dense"] + res["ms_dense2"]))
        # configs[3]'s sweep of the ReLU zero fraction: same tensors, only the bias shifts
        if hw.name == "70b":
            std = neuron_std(hw.host["W1"])
            for zf in (0.50, 0.75, 0.90, 0.95):
                if abs(zf - hw.zf) < 1e-9:
                    continue
                hw.b1 = dev(bias_for_zero_fraction(std, zf))
                hw.b1h, hw.zf = hw.b1.to(torch.bfloat16), zf
                bf = lambda *shape: torch.empty(shape, dtype=torch.bfloat16, device="cuda")
                hw.y2, hw.dy2, hw.dy1 = bf(T, F), bf(T, F), bf(T, F)
                configs[key("70b", zf)] = hw.summary(hw.measure(esteps, ewarm))
        # Table 5's wider blocks at the headline shape (same tensors): the fused wide-block step, retained L1 mass included
        wide = {}
        if hw.name == "70b":
            host70, hw.y1 = hw.host, None
            del hw
            free()
            for m in (16, 32, 64):
                w = Workload("70b", 0.90, m, host=host70)
                wide["64:2:%d" % m] = w.summary(w.measure(esteps, ewarm))
                del w
                free()
            del host70
        else:
            del hw
            free()
        host_1b = None
        for name in ("tiny", "1b", "7b", "moe"):
            if key(name, 0.90) in configs:
                continue
            w = Workload(name, 0.90)
            r = w.measure(esteps if name != "tiny" else 50, ewarm)
            configs[key(name, 0.90)] = w.summary(r)
            if name == "moe":         # configs[4] with fp8 operands: grouped launches, scales shared by the experts
                configs[key(name, 0.90)]["fp8_step"] = fp8_section(w, esteps, ewarm, 0.5 * (r["ms_sparse"] + r["ms_sparse2"]), 0.5 * (r["ms_dense"] + r["ms_dense2"]))
            if name in ("tiny", "1b"):       # launch gaps are visible at these sizes: the same step replayed from a HIP graph
                configs[key(name, 0.90)]["graph_replay_ms_per_step"] = round(w.graph_replay_ms(50 if name == "tiny" else esteps), 4)
            if name == "1b":
                host_1b = w.host
            del w
            free()

        # the neuron-level router's whole training step (Section 3.3; routing + grouping inside the timed step) at the 1B shape
        router_step = {}
        for m in (8, 16, 32, 64):
            w = Workload("1b", 0.90, m, router=True, host=host_1b)
            r = w.measure(esteps, ewarm)
            run_rp = lambda: w.step.full(w.means, w.X, w.W1, w.W2, w.b1, w.dY, weights_packed=True)     # a later micro-batch: no weight preparation
            run_rp()
            ms_rp = timed(run_rp, esteps)
            router_step["64:2:%d" % m] = {"experts": m // 4, "ms_per_step": round(r["ms_sparse"], 4), "dense_ms_per_step": round(r["ms_dense"], 4),
                                          "speedup_vs_dense": round(r["ms_dense"] / r["ms_sparse"], 4),
                                          "weights_packed_ms_per_micro_batch": round(ms_rp, 4), "weights_packed_speedup_vs_dense": round(r["ms_dense"] / ms_rp, 4)}
            del w
            free()

        def gbs(fn, nbytes, n=12):
            return round(nbytes / (ms_of(fn, n) * 1e-3) / 1e9, 1)

        # ---- the two compressors alone at the 7B shape (HBM-bound; algorithmic bytes = input read once + packed outputs).
        #      Every launch reads a different copy of its input (4 weight copies = 512 MiB, 2 activation copies = 1 GiB, more
        #      than the 256 MB last-level cache), so the rate is an HBM rate and not a cache-resident one. --------------
        T7, D7, F7 = CONFIGS["7b"]
        wsrc = [(torch.randn((F7, D7), device="cuda") * 0.02).to(torch.bfloat16) for _ in range(4)]
        ysrc = [(torch.randn((T7, F7), device="cuda") - 1.2816).to(torch.bfloat16) for _ in range(2)]
        turn = [0]

        def rot(pool):
            turn[0] += 1
            return pool[turn[0] % len(pool)]
        kernels = {
            "shape": "7b: W [%d, %d], y1 [%d, %d]; inputs rotated through %d / %d copies" % (F7, D7, T7, F7, len(wsrc), len(ysrc)),
            "prune24_compress(W1) GB/s": gbs(lambda: sffn.prune24_compress(rot(wsrc), False, mode), 3.125 * F7 * D7),
            "prune24_compress(W2, trans) GB/s": gbs(lambda: sffn.prune24_compress(rot(wsrc), True, mode), 3.125 * F7 * D7),
            "sqrelu_vnm_compress GB/s": gbs(lambda: sffn.sqrelu_vnm_compress(rot(ysrc)), (2 + 0.5 + 0.0625 + 1.0 / 128) * T7 * F7),
            "hbm_peak GB/s": HBM_PEAK_GBS,
        }
        for m in (16, 32, 64):       # Table 5's block widths: bytes = input + packed values (2 of m) + metadata + column offsets
            kernels["sqrelu_vnm_compress 64:2:%d GB/s" % m] = gbs(lambda: sffn.sqrelu_vnm_compress(rot(ysrc), 64, m),
                                                                  (2 + 4.0 / m + 0.5 / m + 4.0 / (64 * m)) * T7 * F7)
        del wsrc, ysrc
        free()

        # ---- the paper's 2:4 micro-benchmark shape (Section 5.2.3): (m, n, k) = (4096, 16384, 4096), pruning included and excluded
        gx = torch.randn((4096, 4096), device="cuda").to(torch.bfloat16)
        gw = (torch.randn((16384, 4096), device="cuda") * 0.02).to(torch.bfloat16)
        gout = torch.empty((4096, 16384), dtype=torch.bfloat16, device="cuda")
        t_d = ms_of(lambda: torch.mm(gx, gw.t(), out=gout))
        gv, gm = sffn.prune24_compress(gw, False, mode)
        t_s = ms_of(lambda: sffn.spmm24_fwd(gx, gv, gm))
        t_p = ms_of(lambda: sffn.prune24_compress(gw, False, mode))
        _, _, gprep = sffn.prune24_compress_prepared(gw, mode)
        gws = torch.empty((sffn.load().sffn_spmm24_prepared_workspace_bytes(4096, 4096),), dtype=torch.uint8, device="cuda")
        t_sp = ms_of(lambda: sffn.spmm24_prepared(gx, gprep, 16384, workspace=gws))        # includes the pass that copies X into blocks
        t_pp = ms_of(lambda: sffn.prune24_compress_prepared(gw, mode))
        gemm24 = {"shape_mnk": [4096, 16384, 4096], "dense_ms": round(t_d, 4), "spmm24_ms": round(t_sp, 4), "prune24_ms": round(t_pp, 4),
                  "speedup_vs_dense": round(t_d / t_sp, 3), "speedup_with_pruning": round(t_d / (t_sp + t_pp), 3),
                  "operands": "weights prepared by the pruning pass (spmm24_prepared, X copied into blocks inside the timed call)",
                  "row_major_operands": {"spmm24_ms": round(t_s, 4), "prune24_ms": round(t_p, 4), "speedup_vs_dense": round(t_d / t_s, 3),
                                         "speedup_with_pruning": round(t_d / (t_s + t_p), 3)}}
        del gprep, gws
        # ---- the same contraction with fp8 (E4M3) operands (Section 3.4, closing paragraph): quantisation fused into the pruning pass,
        #      v_smfmac_f32_32x32x64_fp8_fp8; peak for this dtype is the dense fp8 matrix rate, 5.0 PFLOP/s ------------------------
        sx8, sw8 = float(gx.float().abs().max()) / 448.0, float(gw.float().abs().max()) / 448.0
        gxq = sffn.quantize_fp8(gx, sx8)
        gc8, gm8 = sffn.prune24_compress_fp8(gw, sw8, False, mode)
        t_s8 = ms_of(lambda: sffn.spmm24_fp8(gxq, sx8, gc8, gm8, sw8))
        t_p8 = ms_of(lambda: sffn.prune24_compress_fp8(gw, sw8, False, mode))
        t_q8 = ms_of(lambda: sffn.quantize_fp8(gx, sx8))
        alg8 = 4096.0 * 16384 * 4096                      # non-zero multiply-adds x 2 (half of k survives)
        fp8_bench = {"shape_mnk": [4096, 16384, 4096], "dense_bf16_ms": round(t_d, 4), "spmm24_bf16_ms": round(t_s, 4), "spmm24_fp8_ms": round(t_s8, 4),
                     "prune24_compress_fp8_ms": round(t_p8, 4), "quantize_fp8_X_ms": round(t_q8, 4),
                     "prune24_compress_fp8 GB/s": round((2 + 0.5 + 0.125) * 16384 * 4096 / (t_p8 * 1e-3) / 1e9, 1),
                     "speedup_vs_dense_bf16": round(t_d / t_s8, 3), "speedup_vs_dense_bf16_with_pruning_and_quantisation": round(t_d / (t_s8 + t_p8 + t_q8), 3),
                     "speedup_vs_sparse_bf16": round(t_s / t_s8, 3),
                     "roofline": {"bound": "mfma", "dtype": "fp8 (e4m3)", "peak": 5000.0, "unit": "TFLOP/s", "achieved": round(alg8 / (t_s8 * 1e-3) / 1e12, 2),
                                  "frac": round(alg8 / (t_s8 * 1e-3) / 1e12 / 5000.0, 4), "issued": round(2 * alg8 / (t_s8 * 1e-3) / 1e12, 2)}}
        del gx, gw, gout, gv, gm, gxq, gc8, gm8

        # ---- at the 1B shape: the activation GEMM alone for every block width of Table 5 against the dense GEMM of the same
        #      shape (Section 5.2.3's Venom micro-benchmark; out[T, D] = y2v[T, F] @ W1[F, D], eq. (7)'s orientation), and the
        #      conversion to V:N:M by the neuron-level router (Section 3.3; the three steps whose cost Section 3.4 discusses):
        #      routing (reads X once), stable grouping + gather of X, grouped matmul that emits V:N:M; E = M / 4 experts ----
        T1, D1, F1 = CONFIGS["1b"]
        h1 = host_1b or make_ffn_inputs(T1, D1, F1, seed=0)
        X1, W11, b11 = dev(h1["X"]), dev(h1["W1"]), dev(h1["b1"])
        y1_1 = torch.addmm(b11.to(torch.bfloat16), X1, W11.t())
        dense_out = torch.empty((T1, D1), dtype=torch.bfloat16, device="cuda")
        t_dense = ms_of(lambda: torch.mm(y1_1, W11, out=dense_out))
        venom = {"shape": "[%d, %d] x [%d, %d]" % (T1, F1, F1, D1), "dense_ms": round(t_dense, 4)}
        sy8, sw8v = float(y1_1.float().clamp_min(0).square().max()) / 448.0, float(W11.float().abs().max()) / 448.0
        w8v = sffn.quantize_fp8(W11, sw8v)
        for m in (8, 16, 32, 64):
            pack = sffn.sqrelu_vnm_compress(y1_1, 64, m)
            t = ms_of(lambda: sffn.vnm_spmm(pack[0], pack[1], pack[2], W11, 1, 64, m))
            pack8 = sffn.sqrelu_vnm_compress_fp8(y1_1, sy8, 64, m)          # the same contraction on E4M3 codes (Section 3.4, closing paragraph)
            t8 = ms_of(lambda: sffn.vnm_spmm_fp8(pack8[0], pack8[1], pack8[2], sy8, w8v, sw8v, 1, 64, m))
            venom["64:2:%d" % m] = {"ms": round(t, 4), "speedup_vs_dense": round(t_dense / t, 3), "fp8_ms": round(t8, 4),
                                    "fp8_speedup_vs_dense_bf16": round(t_dense / t8, 3)}
        del w8v
        del dense_out
        b1h1 = b11.to(torch.bfloat16)
        router = {"shape": "1b", "dense_y1_ms": round(ms_of(lambda: torch.addmm(b1h1, X1, W11.t(), out=y1_1)), 4)}
        for m in (8, 16, 32, 64):
            means_m = dev(make_router_inputs(64, D1, 4 * m, m, seed=0)["means"])
            t_route = ms_of(lambda: sffn.venom_route_launch(X1, means_m, m))
            rr = sffn.venom_route(X1, means_m, m)
            ws_r = torch.empty((sffn.load().sffn_venom_matmul_workspace_bytes(T1, D1, F1, m),), dtype=torch.uint8, device="cuda")
            t_mm = ms_of(lambda: sffn.venom_expert_matmul(X1, rr["perm"], rr["seg"], W11, b11, m, mode, keep_y1c=False, workspace=ws_r))
            router["64:2:%d" % m] = {"experts": m // 4, "rows": int(rr["perm"].shape[0]), "route_and_group_ms": round(t_route, 4),
                                     "route_and_group_GBs_of_X": round(T1 * D1 * 2 / (t_route * 1e-3) / 1e9, 1),
                                     "gather_prune_matmul_ms": round(t_mm, 4),
                                     "conversion_vs_dense_y1": round(router["dense_y1_ms"] / (t_route + t_mm), 3)}
            del ws_r, rr, means_m

    if args.workload == "moe":
        wl = ("moe: 8 experts, 16384 tokens routed top-2 = %d token slots in 64-row aligned segments, d_model=%d, d_ff=%d per expert, 2:4 weights (%s), "
              "V:N:M 64:2:8 SquaredReLU, zero fraction %.2f, seed 0; one grouped launch per stage" % (T, D, F, args.mode, args.zero_fraction))
    else:
        wl = ("%s: one FFN layer, T=%d tokens, d_model=%d, d_ff=%d, 2:4 weights (%s), V:N:M 64:2:%d SquaredReLU%s, zero fraction %.2f, seed 0"
              % (args.workload, T, D, F, args.mode, M,
                 " produced by the neuron-level router (%d experts, routing + grouping inside the timed step)" % (M // 4) if args.router else "",
                 args.zero_fraction))
    out = {
        "metric": "sparse FFN fwd+bwd TFLOP/s (dense-equiv) & speedup vs dense bf16, 1 MI355X",
        "value": head["tflops_dense_equiv"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl},
        "frac_of_mfma_peak": head["frac_of_mfma_peak"], "algorithmic_frac_of_mfma_peak": head["algorithmic_frac_of_mfma_peak"],
        "dense_ms_per_step": head["dense_ms_per_step"], "dense_gemms_only_ms": head["dense_gemms_only_ms"],
        "dense_baseline": "6 hipBLASLt bf16 GEMMs (torch.mm / addmm) + eq. (2) and eq. (6) as one-pass element-wise kernels; dense_gemms_only_ms leaves the two element-wise kernels out",
        "dense_tflops": round(12.0 * T * D * F / (head["dense_ms_per_step"] * 1e-3) / 1e12, 2),
        "dense_frac_of_mfma_peak": round(12.0 * T * D * F / (head["dense_ms_per_step"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
        "speedup_vs_dense": head["speedup_vs_dense"], "speedup_vs_dense_gemms_only": head["speedup_vs_dense_gemms_only"],
        "settle_s": args.settle_s,
        "second_pass": {"ms_per_step": round(res["ms_sparse2"], 4), "dense_ms_per_step": round(res["ms_dense2"], 4)},
        "stage_ms": {k: round(v, 4) for k, v in acc.items()},
        "retained_l1_fraction": head.get("retained_l1_fraction"), "relu_zero_fraction": head.get("relu_zero_fraction"),
        "configs": configs,
        "wide_blocks_70b": wide,
        "router_step_1b": router_step,
        "standalone_kernels": kernels,
        "venom_gemm_microbench": venom,
        "gemm24_microbench": gemm24,
        "fp8_microbench": fp8_bench,
        "fp8_step": fp8_step,
        "other_pruning_mode": other_mode,
        "micro_batches": micro,
        "router_conversion": router,
        "roofline": roofline, "cpu_baseline": cpu,
        "paper_context": "paper reports 1.4-1.5x for 2:4 GEMMs and 1.4-1.7x end-to-end on NVIDIA sparse tensor cores (Sections 1, 5.2.3); context, not a target",
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
