"""ffn_sparse_step_noalloc (the entry point for callers that cannot allocate: built-in workspace) against ffn_sparse_step on
the same inputs: same kernels, so every output must be the same bits.  Two calls in a row, the second on a smaller
shape (the built-in buffer then still holds the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2602_06183_amd as sffn
from paper_2602_06183_amd import binding
from tests.util import to_dev, to_bits
from workload import make_ffn_inputs


@pytest.mark.gpu
def test_noalloc_step_matches_the_workspace_entry_point_twice_in_a_row():
    for T, D, F, mode, seed in ((1024, 512, 2048, sffn.MODE_HARD, 0), (192, 320, 448, sffn.MODE_SOFT, 3), (1024, 512, 2048, sffn.MODE_SOFT, 1)):
        inp = make_ffn_inputs(T, D, F, seed=seed)
        dev = {k: to_dev(v) for k, v in inp.items()}
        ref_step = sffn.FfnStep(T, D, F, mode)
        ref = [to_bits(t).copy() for t in ref_step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])]
        out = (torch.zeros((T, D), dtype=torch.bfloat16, device="cuda"), torch.zeros((T, D), dtype=torch.bfloat16, device="cuda"),
               torch.zeros((F, D), dtype=torch.bfloat16, device="cuda"), torch.zeros((D, F), dtype=torch.bfloat16, device="cuda"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        sffn.ffn_sparse_step_noalloc(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"], out, mode)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before            # nothing came from torch's allocator either
        for name, got, want in zip(("Y3", "dX", "dW1", "dW2"), out, ref):
            assert np.array_equal(to_bits(got), want), (name, T, D, F)
        assert sffn.workspace_bytes(T, D, F, mode) <= sffn.NOALLOC_WORKSPACE_MAX


@pytest.mark.gpu
def test_noalloc_step_checked_against_the_oracle():
    """The same entry point, its outputs against the CPU oracle's contractions (teacher-forced on the packed operands of
    the workspace entry point, which produced the same bits above)."""
    import oracle
    from tests.util import assert_gemm_close
    T, D, F = 256, 128, 512
    inp = make_ffn_inputs(T, D, F, seed=5)
    dev = {k: to_dev(v) for k, v in inp.items()}
    out = tuple(torch.zeros(s, dtype=torch.bfloat16, device="cuda") for s in ((T, D), (T, D), (F, D), (D, F)))
    sffn.ffn_sparse_step_noalloc(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"], out)
    (_, _, _, _), step = sffn.ffn_sparse_step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])
    torch.cuda.synchronize()
    s = {k: to_bits(v) for k, v in step.saved().items()}
    yv, ym, yc = oracle.sqrelu_vnm_compress(s["y1"])
    assert np.array_equal(s["y2_vals"], yv)
    dv = oracle.dsqrelu_vnm(s["dy2"], s["y1"], ym, yc)
    assert_gemm_close(to_bits(out[0]), oracle.vnm_spmm(yv, ym, yc, inp["W2"], 0), "y3")
    assert_gemm_close(to_bits(out[1]), oracle.vnm_spmm(dv, ym, yc, inp["W1"], 1), "dX")
    assert_gemm_close(to_bits(out[2]), oracle.vnm_wgrad(dv, ym, yc, inp["X"], 1), "dW1")
    assert_gemm_close(to_bits(out[3]), oracle.vnm_wgrad(yv, ym, yc, inp["dY"], 0), "dW2")


def test_noalloc_step_refuses_shapes_beyond_its_buffer():
    """Host-side: a shape whose workspace exceeds the built-in buffer is refused before any HIP call (runs without a GPU)."""
    lib = sffn.load()
    fake = ctypes.c_void_p(0x1000)
    big = binding._Cfg(2048, 1024, 4096, 64, 8, 0, 0)
    assert lib.sffn_workspace_bytes(ctypes.byref(big)) > sffn.NOALLOC_WORKSPACE_MAX
    assert lib.ffn_sparse_step_noalloc(ctypes.byref(big), *([fake] * 9), None) == -3
    assert b"built-in buffer" in lib.sffn_last_error()
    bad = binding._Cfg(500, 256, 1024, 64, 8, 0, 0)
    assert lib.ffn_sparse_step_noalloc(ctypes.byref(bad), *([fake] * 9), None) == -1
    m12 = binding._Cfg(512, 256, 1024, 64, 12, 0, 0)
    assert lib.ffn_sparse_step_noalloc(ctypes.byref(m12), *([fake] * 9), None) == -1
