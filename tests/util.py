"""Helpers shared by the GPU parity tests: numpy bf16 bit patterns <-> torch device tensors, error metrics."""
import numpy as np
import torch

import oracle

REL_FRO_TOL = 5e-3          # relative Frobenius error bound for GEMM outputs
MAX_ELEM_TOL = 2e-2         # max elementwise error bound, times max|ref|


def to_dev(bits):
    """uint16 bf16 bit patterns (numpy) -> torch.bfloat16 tensor on cuda:0."""
    a = np.ascontiguousarray(bits)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


def to_bits(t):
    """torch tensor on device -> numpy (bf16 comes back as uint16 bit patterns)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def gemm_errors(got_bits, ref_bits):
    g, r = oracle.bits_to_f64(got_bits), oracle.bits_to_f64(ref_bits)
    fro = np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-300)
    mx = np.abs(g - r).max() / max(np.abs(r).max(), 1e-300)
    return fro, mx


def assert_gemm_close(got_bits, ref_bits, what=""):
    assert got_bits.shape == ref_bits.shape, (what, got_bits.shape, ref_bits.shape)
    assert np.all(np.isfinite(oracle.bits_to_f32(got_bits))), what
    fro, mx = gemm_errors(got_bits, ref_bits)
    assert fro <= REL_FRO_TOL, (what, "rel fro", fro)
    assert mx <= MAX_ELEM_TOL, (what, "max elem", mx)
