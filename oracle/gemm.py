"""The six contractions of the sparsified FFN step, each as a float64 matmul on the explicitly
masked dense matrix (CPU oracle, test infrastructure only).

Paper: eqs. (1), (3), (4), (5), (7), (8) with the operand choice of Alg. 1 / Alg. 2.  Inputs are
bf16 bit patterns; products are accumulated in float64 and rounded once (RNE) to bf16.
"""
import numpy as np
from .bf16 import bits_to_f64, f64_to_bits
from .sparse24 import prune24_decompress
from .vnm import vnm_decompress


def dense_nt(a_bits, b_bits, bias=None):
    """out[i, j] = bf16( sum_k a[i, k] * b[j, k] (+ bias[j]) )."""
    acc = bits_to_f64(a_bits) @ bits_to_f64(b_bits).T
    if bias is not None:
        acc = acc + np.asarray(bias, dtype=np.float32).astype(np.float64)[None, :]
    return f64_to_bits(acc)


def spmm24(x_bits, w_vals, w_meta, bias=None):
    """eq. (1) / eq. (4): out[t, n] = bf16( sum_k x[t, k] * Ws[n, k] (+ bias[n]) ), Ws given packed 2:4."""
    return dense_nt(x_bits, prune24_decompress(w_vals, w_meta), bias)


def vnm_spmm(a_vals, a_meta, a_colidx, w_bits, w_kmajor, V=64, M=8):
    """eq. (3) / eq. (7): out[t, n] = bf16( sum_f Av[t, f] * W(n, f) ); W stored [N, F] (w_kmajor=0) or [F, N] (1)."""
    a = vnm_decompress(a_vals, a_meta, a_colidx, V, M)
    w = np.asarray(w_bits, dtype=np.uint16)
    if w_kmajor:
        w = w.T
    return dense_nt(a, w)


def vnm_wgrad(a_vals, a_meta, a_colidx, g_bits, out_f_major, V=64, M=8):
    """eq. (5) / eq. (8): C[f, n] = sum_t Av[t, f] * G[t, n]; returned [F, N] if out_f_major else [N, F]."""
    a = bits_to_f64(vnm_decompress(a_vals, a_meta, a_colidx, V, M))
    c = a.T @ bits_to_f64(g_bits)
    return f64_to_bits(c if out_f_major else c.T)
