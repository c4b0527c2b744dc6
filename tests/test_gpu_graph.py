"""The training-step entry points under HIP graph capture: they only enqueue kernels on the caller's stream (no allocation,
no memset, no host read-back), so a captured step must replay to the same bits as the eager call.  Every replay is checked,
with new input contents and eager work in between (a graph that only worked on its first replay would pass a single check)."""
import numpy as np
import pytest
import torch

import paper_2602_06183_amd as sffn
from tests.util import to_dev, to_bits
from workload import make_ffn_inputs, make_moe_inputs, make_router_inputs

NAMES = ("Y3", "dX", "dW1", "dW2")


def _replay_against_eager(make_inputs, captured, eager, keys):
    """captured / eager: callables taking the dict of device inputs and returning the four outputs; `captured` is recorded
    once on static input buffers, then replayed three times, each time on fresh contents copied into those buffers."""
    static = {k: to_dev(v) for k, v in make_inputs(0).items() if k in keys}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up outside the capture (first-call set-up of the library)
        captured(static)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        outs = captured(static)
    for seed in (1, 2, 3):
        fresh = {k: to_dev(v) for k, v in make_inputs(seed).items() if k in keys}
        want = [to_bits(t).copy() for t in eager(fresh)]                # eager work between the replays
        torch.cuda.synchronize()
        for k in keys:
            static[k].copy_(fresh[k])
        for o in outs:
            o.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, ref in zip(NAMES, outs, want):
            assert np.array_equal(to_bits(got), ref), (name, seed)


@pytest.mark.gpu
@pytest.mark.parametrize("T,D,F,M,mode", [(512, 256, 1024, 8, sffn.MODE_HARD), (192, 320, 448, 8, sffn.MODE_SOFT), (256, 256, 1024, 16, sffn.MODE_HARD)])
def test_ffn_sparse_step_replays_in_a_graph(T, D, F, M, mode):
    a, b = sffn.FfnStep(T, D, F, mode, M=M), sffn.FfnStep(T, D, F, mode, M=M)
    call = lambda step: (lambda d: step(d["X"], d["W1"], d["W2"], d["b1"], d["dY"]))
    _replay_against_eager(lambda seed: make_ffn_inputs(T, D, F, seed=seed), call(a), call(b), ("X", "W1", "W2", "b1", "dY"))


@pytest.mark.gpu
def test_grouped_step_replays_in_a_graph():
    D, F = 256, 512
    first = make_moe_inputs(1024, 4, 2, D, F, seed=0)
    seg = [int(v) for v in first["seg"]]

    def inputs(seed):          # same segment table (it is a host argument of the call, frozen into the graph), new tensors
        inp = make_moe_inputs(1024, 4, 2, D, F, seed=0) if seed == 0 else None
        if inp is None:
            rng = np.random.default_rng(seed)
            inp = dict(first)
            for k in ("X", "dY"):
                inp[k] = rng.permutation(first[k].reshape(-1)).reshape(first[k].shape)
        return inp

    a, b = sffn.FfnStepGrouped(seg, D, F), sffn.FfnStepGrouped(seg, D, F)
    call = lambda step: (lambda d: step(d["X"], d["W1"], d["W2"], d["b1"], d["dY"]))
    _replay_against_eager(inputs, call(a), call(b), ("X", "W1", "W2", "b1", "dY"))


@pytest.mark.gpu
@pytest.mark.parametrize("M", [8, 32])
def test_router_full_step_replays_in_a_graph(M):
    """Routing, grouping and the six grouped contractions in one captured call: the run offsets never leave the device."""
    T, D, F = 1024, 256, 1024
    a, b = sffn.FfnRouterStep(T, D, F, M), sffn.FfnRouterStep(T, D, F, M)
    call = lambda step: (lambda d: step.full(d["means"], d["X"], d["W1"], d["W2"], d["b1"], d["dY"]))
    _replay_against_eager(lambda seed: make_router_inputs(T, D, F, M, seed=seed), call(a), call(b), ("means", "X", "W1", "W2", "b1", "dY"))


@pytest.mark.gpu
@pytest.mark.parametrize("wgrad_fp8,M", [(False, 8), (True, 8), (True, 16), (False, 64)])
def test_fp8_step_replays_in_a_graph(wgrad_fp8, M):
    T, D, F = 256, 256, 512 if M < 64 else 2048
    sc = dict(x=4.5 / 448, w1=0.1 / 448, w2=0.1 / 448, y2=2.0 / 448, dy=4.5 / 448, dy1=4.0 / 448)
    a, b = sffn.FfnStepFp8(T, D, F, sc, wgrad_fp8=wgrad_fp8, M=M), sffn.FfnStepFp8(T, D, F, sc, wgrad_fp8=wgrad_fp8, M=M)
    call = lambda step: (lambda d: step(d["X"], d["W1"], d["W2"], d["b1"], d["dY"]))
    _replay_against_eager(lambda seed: make_ffn_inputs(T, D, F, seed=seed), call(a), call(b), ("X", "W1", "W2", "b1", "dY"))


@pytest.mark.gpu
@pytest.mark.parametrize("M", [8, 16])
def test_split_calls_with_gradient_accumulation_replay_in_a_graph(M):
    """What a captured training iteration holds for one layer: the forward call, later the backward call that adds the weight gradients to
    float32 buffers (SFFN_FLAG_DW_FP32_ACCUMULATE), on a shared scratch buffer.  The helper zeroes the outputs before each replay, so every
    replay must leave exactly what an eager one-call step leaves in zeroed buffers."""
    T, D, F = 256, 256, 1024
    scratch = torch.empty((sffn.buffer_sizes(T, D, F, M=M)["scratch"],), dtype=torch.uint8, device="cuda")
    a, b = sffn.FfnStep(T, D, F, M=M, scratch=scratch, dw_fp32=True), sffn.FfnStep(T, D, F, M=M, dw_fp32=True)

    def captured(d):
        y3 = a.forward(d["X"], d["W1"], d["W2"], d["b1"])
        return (y3,) + tuple(a.backward(d["W1"], d["dY"]))

    def eager(d):
        b.dW1.zero_()
        b.dW2.zero_()
        return b(d["X"], d["W1"], d["W2"], d["b1"], d["dY"])
    _replay_against_eager(lambda seed: make_ffn_inputs(T, D, F, seed=seed), captured, eager, ("X", "W1", "W2", "b1", "dY"))
