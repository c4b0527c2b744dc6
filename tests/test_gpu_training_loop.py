"""The pieces a training loop uses, together and against the oracle: Alg. 1 and Alg. 2 as separate calls for a stack of layers that share
one scratch buffer, two micro-batches per optimizer step (the second on the packed weights of the first: Section 3.4's amortisation), weight
gradients summed in float32 inside the weight-gradient GEMMs.  Every contraction is checked teacher-forced against the oracle (eqs. (3), (5),
(7), (8) from the packed activations the GPU produced, which are checked bit for bit from the GPU's own y1 / dy2)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_06183_amd as sffn
from tests.util import to_dev, to_bits, assert_gemm_close
from workload import make_ffn_inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", [sffn.MODE_HARD, sffn.MODE_SOFT])
def test_layers_micro_batches_and_float32_gradient_accumulation(mode):
    T, D, F, L, MB = 256, 128, 512, 3, 2
    layers = [make_ffn_inputs(T, D, F, seed=100 + l) for l in range(L)]                 # weights and bias of layer l
    data = [[make_ffn_inputs(T, D, F, seed=200 + 10 * l + m) for m in range(MB)] for l in range(L)]      # X and dY of (layer, micro-batch)
    sz = sffn.buffer_sizes(T, D, F, mode, keep_dense=True)
    scratch = torch.empty((sz["scratch"],), dtype=torch.uint8, device="cuda")
    # one object per (layer, micro-batch in flight): its own saved buffer; the micro-batches of a layer share the layer's packed weights; the
    # float32 gradient buffers of a layer are shared too (both objects add to the first one's)
    steps = []
    for l in range(L):
        first = sffn.FfnStep(T, D, F, mode, keep_dense=True, scratch=scratch, dw_fp32=True)
        second = sffn.FfnStep(T, D, F, mode, keep_dense=True, scratch=scratch, weights_of=first, dw_fp32=True)
        second.dW1, second.dW2 = first.dW1, first.dW2
        steps.append([first, second])
    W = [dict(W1=to_dev(w["W1"]), W2=to_dev(w["W2"]), b1=to_dev(w["b1"])) for w in layers]
    packed, want_dw1, want_dw2 = {}, [0.0] * L, [0.0] * L
    # forward passes: micro-batch by micro-batch through the stack
    for m in range(MB):
        for l in range(L):
            st, d = steps[l][m], data[l][m]
            Y3 = to_bits(st.forward(to_dev(d["X"]), W[l]["W1"], W[l]["W2"], W[l]["b1"], weights_packed=(m > 0))).copy()
            sv = {k: to_bits(v).copy() for k, v in st.saved().items() if k in ("y1", "y2_vals", "y2_meta", "colidx", "w1_vals", "w1_meta")}
            rv, rm = oracle.prune24_compress(layers[l]["W1"], mode)
            assert np.array_equal(sv["w1_vals"], rv) and np.array_equal(sv["w1_meta"], rm)
            assert_gemm_close(sv["y1"], oracle.spmm24(d["X"], rv, rm, layers[l]["b1"]), "y1")
            yv, ym, yc = oracle.sqrelu_vnm_compress(sv["y1"])
            assert np.array_equal(sv["y2_vals"], yv) and np.array_equal(sv["y2_meta"], ym) and np.array_equal(sv["colidx"], yc)
            assert_gemm_close(Y3, oracle.vnm_spmm(yv, ym, yc, layers[l]["W2"], 0), "y3")
            packed[(l, m)] = (sv["y1"], yv, ym, yc)
            scratch.fill_(0xA5)
    # backward passes in reverse
    for m in reversed(range(MB)):
        for l in reversed(range(L)):
            st, d = steps[l][m], data[l][m]
            dX = to_bits(st.backward(W[l]["W1"], to_dev(d["dY"]))[0]).copy()
            sv = {k: to_bits(v).copy() for k, v in st.saved().items() if k in ("dy2", "dy1_vals")}
            y1, yv, ym, yc = packed[(l, m)]
            rv2, rm2 = oracle.prune24_compress(np.ascontiguousarray(layers[l]["W2"].T), mode)
            assert_gemm_close(sv["dy2"], oracle.spmm24(d["dY"], rv2, rm2, None), "dy2")
            dv = oracle.dsqrelu_vnm(sv["dy2"], y1, ym, yc)
            assert np.array_equal(sv["dy1_vals"], dv)
            assert_gemm_close(dX, oracle.vnm_spmm(dv, ym, yc, layers[l]["W1"], 1), "dX")
            want_dw2[l] = want_dw2[l] + oracle.bits_to_f64(oracle.vnm_wgrad(yv, ym, yc, d["dY"], 0))
            want_dw1[l] = want_dw1[l] + oracle.bits_to_f64(oracle.vnm_wgrad(dv, ym, yc, d["X"], 1))
            scratch.fill_(0x5A)
    for l in range(L):
        assert_gemm_close(to_bits(steps[l][0].dW1.to(torch.bfloat16)), oracle.f64_to_bits(want_dw1[l]), "dW1 summed over the micro-batches")
        assert_gemm_close(to_bits(steps[l][0].dW2.to(torch.bfloat16)), oracle.f64_to_bits(want_dw2[l]), "dW2 summed over the micro-batches")
