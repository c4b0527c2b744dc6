"""SquaredReLU and the V:N:M (Venom) format with N = 2 (CPU oracle, test infrastructure only).

Paper: eq. (2) y2 = ReLU(y1)^2, eq. (6) dy1 = 2 * dy2 * ReLU(y1), Section 2.3 (blocks of V rows
by M columns; four columns survive per block; the surviving four are 2:4-pruned by magnitude),
Table 5 (sparsity = 1 - N/M).

Readings fixed here because the paper is silent or garbled:
  * a block is V rows x M columns (the printed "[nrows // V, M]" is the block count);
  * column score = sum over the block's rows of |y2|, accumulated in float32 starting from +0,
    rows added in ascending order, one RNE rounding per add; the four columns with the largest
    scores are kept, ties going to the lower column; kept offsets are stored ascending;
  * per row, the four kept columns (ascending) form one 2:4 group pruned by the rule of
    sparse24.prune24_positions;
  * dy1 inherits y2's mask: it is evaluated only where y2 was kept.
Packed layout: vals [T, 2F/M], meta [T, F/(2M)] (two blocks per byte, low nibble first),
colidx [T/V, F/M, 4] (uint8 offsets inside the block).
"""
import numpy as np
from .bf16 import bits_to_f32, f32_to_bits
from .sparse24 import prune24_compress, prune24_decompress, HARD


def sqrelu(y1_bits):
    """eq. (2): bf16(max(y1, 0)^2); the float32 product is rounded once (RNE) to bf16."""
    y = bits_to_f32(y1_bits)
    r = np.where(y > 0, y, np.float32(0.0)).astype(np.float32)
    with np.errstate(over="ignore"):
        return f32_to_bits(r * r)


def vnm_select_columns(y2_bits, V, M):
    """Returns (colidx uint8 [T/V, F/M, 4], scores float32 [T/V, F/M, M])."""
    y2_bits = np.asarray(y2_bits, dtype=np.uint16)
    T, F = y2_bits.shape
    assert T % V == 0 and F % M == 0 and M >= 4
    a = bits_to_f32(y2_bits & np.uint16(0x7FFF)).reshape(T // V, V, F // M, M)
    score = np.zeros((T // V, F // M, M), dtype=np.float32)
    for r in range(V):                                   # ascending rows, one float32 add each
        score = (score + a[:, r]).astype(np.float32)
    order = np.argsort(-score, axis=-1, kind="stable")   # score descending, column ascending on ties
    colidx = np.sort(order[..., :4], axis=-1).astype(np.uint8)
    return colidx, score


def _gather(y2_bits, colidx, V, M):
    T, F = y2_bits.shape
    blk = y2_bits.reshape(T // V, V, F // M, M)
    idx = np.broadcast_to(colidx[:, None, :, :].astype(np.int64), (T // V, V, F // M, 4))
    return np.take_along_axis(blk, idx, axis=-1).reshape(T, (F // M) * 4)


def vnm_compress(y2_bits, V=64, M=8):
    """y2 (bf16 bits [T, F]) -> (vals [T, 2F/M], meta [T, F/(2M)], colidx [T/V, F/M, 4])."""
    y2_bits = np.asarray(y2_bits, dtype=np.uint16)
    colidx, _ = vnm_select_columns(y2_bits, V, M)
    kept4 = _gather(y2_bits, colidx, V, M)                # logical 2:4 matrix [T, 4F/M]
    vals, meta = prune24_compress(kept4, HARD)
    return vals, meta, colidx


def vnm_decompress(vals, meta, colidx, V=64, M=8):
    """Packed V:N:M -> dense bf16 bits [T, F] with +0 everywhere that was dropped."""
    kept4 = prune24_decompress(vals, meta)                # [T, 4F/M]
    T = kept4.shape[0]
    nb = colidx.shape[1]
    dense = np.zeros((T // V, V, nb, M), dtype=np.uint16)
    idx = np.broadcast_to(colidx[:, None, :, :].astype(np.int64), (T // V, V, nb, 4))
    np.put_along_axis(dense, idx, kept4.reshape(T // V, V, nb, 4), axis=-1)
    return dense.reshape(T, nb * M)


def sqrelu_vnm_compress(y1_bits, V=64, M=8):
    """Alg. 1 lines 5-6 with the magnitude V:N:M rule of Section 2.3."""
    return vnm_compress(sqrelu(y1_bits), V, M)


def dsqrelu_vnm(dy2_bits, y1_bits, meta, colidx, V=64, M=8):
    """eq. (6) at y2's kept positions: dvals[t, s] = bf16(2 * dy2 * max(y1, 0)), same slots as y2's vals."""
    dy2_bits = np.asarray(dy2_bits, dtype=np.uint16)
    y1_bits = np.asarray(y1_bits, dtype=np.uint16)
    d = bits_to_f32(dy2_bits)
    y = bits_to_f32(y1_bits)
    with np.errstate(over="ignore", invalid="ignore"):
        full = f32_to_bits((np.float32(2.0) * d * np.where(y > 0, y, np.float32(0.0))).astype(np.float32))
    g4 = _gather(full, colidx, V, M)                      # values at the four kept columns
    T = g4.shape[0]
    G = g4.shape[1] // 4
    meta = np.asarray(meta, dtype=np.uint8)
    nib = np.empty((T, G), dtype=np.uint8)
    nib[:, 0::2] = meta & 0xF
    nib[:, 1::2] = meta >> 4
    p = np.stack([nib & 3, (nib >> 2) & 3], axis=-1).astype(np.int64)
    return np.take_along_axis(g4.reshape(T, G, 4), p, axis=-1).reshape(T, 2 * G)


def vnm_to_24(vals, meta, colidx, V=64, M=8):
    """Re-express a V:2:M matrix as a plain 2:4 matrix over all F columns (always possible for
    M % 4 == 0: two survivors per M >= 8 columns leave at most two per aligned group of four).
    Returns the dense bits; used only to state that equivalence in tests."""
    return vnm_decompress(vals, meta, colidx, V, M)
