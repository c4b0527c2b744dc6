"""Whole sparsified FFN training step, stage by stage (CPU oracle, test infrastructure only).

Paper: Alg. 1 (forward) and Alg. 2 (backward) of Section 3, over eqs. (1)-(8) of Section 2.1.
Storage: X [T, D], W1 [F, D], W2 [D, F], dY [T, D] (bf16 bits, row-major), b1 [F] float32
(a workload device that sets the ReLU zero fraction; the paper's FFN has no bias).
"""
import numpy as np
from .sparse24 import prune24_compress, HARD
from .vnm import sqrelu_vnm_compress, dsqrelu_vnm
from .gemm import spmm24, vnm_spmm, vnm_wgrad, dense_nt
from .bf16 import bits_to_f32, f32_to_bits
from .vnm import sqrelu


def ffn_sparse_step_ref(X, W1, W2, b1, dY, mode=HARD, V=64, M=8):
    out = {}
    # Alg. 1 line 4: y1 = X @ sparsify24(W1), 2:4 along d_model
    w1_vals, w1_meta = prune24_compress(W1, mode)
    y1 = spmm24(X, w1_vals, w1_meta, b1)
    # Alg. 1 lines 5-6: SquaredReLU, then V:N:M
    y2_vals, y2_meta, colidx = sqrelu_vnm_compress(y1, V, M)
    # Alg. 1 line 7: y3 = y2 @ W2 (dense W2)
    y3 = vnm_spmm(y2_vals, y2_meta, colidx, W2, 0, V, M)
    # Alg. 2 line 2: dy2 = dy3 @ sparsify24(W2.T), 2:4 along d_model
    w2t_vals, w2t_meta = prune24_compress(np.ascontiguousarray(np.asarray(W2).T), mode)
    dy2 = spmm24(dY, w2t_vals, w2t_meta, None)
    # Alg. 2 line 3: dW2 = y2.T @ dy3, stored like W2: [D, F]
    dW2 = vnm_wgrad(y2_vals, y2_meta, colidx, dY, 0, V, M)
    # Alg. 2 line 4: dy1 = 2 dy2 ReLU(y1) on y2's mask
    dy1_vals = dsqrelu_vnm(dy2, y1, y2_meta, colidx, V, M)
    # Alg. 2 line 5: dX = dy1 @ W1.T (dense W1)
    dX = vnm_spmm(dy1_vals, y2_meta, colidx, W1, 1, V, M)
    # Alg. 2 line 6: dW1 = dy1.T @ X, stored like W1: [F, D]
    dW1 = vnm_wgrad(dy1_vals, y2_meta, colidx, X, 1, V, M)
    out.update(w1_vals=w1_vals, w1_meta=w1_meta, y1=y1, y2_vals=y2_vals, y2_meta=y2_meta,
               colidx=colidx, y3=y3, w2t_vals=w2t_vals, w2t_meta=w2t_meta, dy2=dy2,
               dy1_vals=dy1_vals, dW2=dW2, dX=dX, dW1=dW1)
    return out


def ffn_dense_ref(X, W1, W2, b1, dY):
    """eqs. (1)-(8) with nothing pruned (context for tests: the sparse step reduces to it when
    the masks keep everything that is non-zero)."""
    y1 = dense_nt(X, W1, b1)
    y2 = sqrelu(y1)
    y3 = dense_nt(y2, W2)
    dy2 = dense_nt(dY, np.ascontiguousarray(np.asarray(W2).T))
    y = bits_to_f32(y1)
    dy1 = f32_to_bits((np.float32(2.0) * bits_to_f32(dy2) * np.where(y > 0, y, np.float32(0))).astype(np.float32))
    dW2 = dense_nt(np.ascontiguousarray(np.asarray(dY).T), np.ascontiguousarray(y2.T))
    dX = dense_nt(dy1, np.ascontiguousarray(np.asarray(W1).T))
    dW1 = dense_nt(np.ascontiguousarray(dy1.T), np.ascontiguousarray(np.asarray(X).T))
    return dict(y1=y1, y2=y2, y3=y3, dy2=dy2, dy1=dy1, dW2=dW2, dX=dX, dW1=dW1)


def ffn_sparse_step_grouped_ref(X, W1, W2, b1, dY, seg_offsets, mode=HARD, V=64, M=8):
    """Mixture-of-experts form (Section 1: the method applies to MoE FFNs, each expert being one FFN of
    Alg. 1 / Alg. 2): expert e owns rows seg_offsets[e]..seg_offsets[e+1] of X and dY and its own
    W1[e] [F, D], W2[e] [D, F], b1[e] [F].  Returns a list with one ffn_sparse_step_ref result per expert
    (None for an expert without rows; its weight gradients are zero by the empty sum)."""
    res = []
    for e in range(len(seg_offsets) - 1):
        a, b = int(seg_offsets[e]), int(seg_offsets[e + 1])
        if b == a:
            res.append(None)
            continue
        res.append(ffn_sparse_step_ref(X[a:b], W1[e], W2[e], None if b1 is None else b1[e], dY[a:b], mode, V, M))
    return res
