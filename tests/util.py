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


def assert_routing_matches_the_definition(expert_gpu, x_bits, means_bits, min_clear=0.98):
    """Order-free check of the router (paper Section 3.3 step 1): the GPU's expert ids against the plain definition,
    float64 x @ ExpertMeans -> argmax (ties low), on every token whose float64 top-2 gap exceeds the float32 rounding
    bound of the two scores.  Tokens inside the bound are counted and reported, not compared (there the stated summation
    order decides, which the bit-exact comparison with oracle.route_scores covers)."""
    clear = oracle.route_margin_is_clear(x_bits, means_bits)
    plain = oracle.route_top1(oracle.route_scores_plain(x_bits, means_bits))
    inside = int((~clear).sum())
    print("routing: %d of %d tokens inside the rounding bound (not compared with the float64 argmax)" % (inside, len(clear)))
    assert np.array_equal(np.asarray(expert_gpu)[clear], plain[clear])
    assert clear.mean() >= min_clear or len(clear) < 64, clear.mean()
