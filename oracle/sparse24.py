"""2:4 magnitude pruning, soft-thresholding and the packed format (CPU oracle, test infrastructure only).

Paper: Section 2.2 (groups of four along the contraction axis, the two smallest magnitudes are
zeroed; soft-thresholding subtracts the second-smallest magnitude from the survivors) and
Section 3.2.1 (the matrix is stored packed, with sparsity metadata).

Readings fixed here because the paper is silent or garbled:
  * ties: rank the four entries by (magnitude descending, index ascending), keep the first two;
    magnitude is the bf16 bit pattern with the sign cleared, compared as an integer;
  * the threshold t of Section 2.2 is |t2|, the second-smallest magnitude of the group
    (the larger of the two dropped entries); a kept entry a becomes a - t (a >= 0) or
    a + t (a < 0), evaluated in float32 and rounded RNE to bf16;
  * packed layout: vals[r, 2g], vals[r, 2g+1] are the kept entries of group g in ascending
    position p0 < p1; nibble = p0 | p1 << 2; meta[r, g // 2] carries group 2j in bits 3:0 and
    group 2j+1 in bits 7:4.
"""
import numpy as np
from .bf16 import bits_to_f32, f32_to_bits

HARD, SOFT = 0, 1


def prune24_positions(bits):
    """bits: uint16 [R, K], K % 4 == 0.  Returns (kept [R, K/4, 2] ascending positions,
    third [R, K/4] position of the largest dropped entry)."""
    bits = np.asarray(bits, dtype=np.uint16)
    R, K = bits.shape
    assert K % 4 == 0
    mag = (bits.reshape(R, K // 4, 4) & np.uint16(0x7FFF)).astype(np.int32)
    order = np.argsort(-mag, axis=-1, kind="stable")   # magnitude descending, index ascending on ties
    kept = np.sort(order[..., :2], axis=-1)
    return kept, order[..., 2]


def prune24_compress(bits, mode=HARD):
    """Logical S[R, K] (bf16 bits) -> (vals uint16 [R, K/2], meta uint8 [R, K/8])."""
    bits = np.asarray(bits, dtype=np.uint16)
    R, K = bits.shape
    assert K % 8 == 0
    G = K // 4
    grp = bits.reshape(R, G, 4)
    kept, third = prune24_positions(bits)
    vals = np.take_along_axis(grp, kept, axis=-1)                       # [R, G, 2]
    if mode == SOFT:
        t_bits = np.take_along_axis(grp, third[..., None], axis=-1) & np.uint16(0x7FFF)
        t = bits_to_f32(t_bits)                                         # >= 0, [R, G, 1]
        a = bits_to_f32(vals)
        neg = (vals & np.uint16(0x8000)) != 0
        with np.errstate(invalid="ignore", over="ignore"):
            shrunk = np.where(neg, a + t, a - t).astype(np.float32)
        vals = f32_to_bits(shrunk)
    elif mode != HARD:
        raise ValueError("mode")
    nib = (kept[..., 0] | (kept[..., 1] << 2)).astype(np.uint8)          # [R, G]
    meta = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    return vals.reshape(R, K // 2).astype(np.uint16), meta


def prune24_decompress(vals, meta):
    """Inverse of the packing: (vals [R, K/2], meta [R, K/8]) -> dense bits [R, K] with +0 in dropped slots."""
    vals = np.asarray(vals, dtype=np.uint16)
    meta = np.asarray(meta, dtype=np.uint8)
    R, K2 = vals.shape
    G = K2 // 2
    nib = np.empty((R, G), dtype=np.uint8)
    nib[:, 0::2] = meta & 0xF
    nib[:, 1::2] = meta >> 4
    dense = np.zeros((R, G, 4), dtype=np.uint16)
    v = vals.reshape(R, G, 2)
    p0 = (nib & 3).astype(np.int64)
    p1 = ((nib >> 2) & 3).astype(np.int64)
    np.put_along_axis(dense, p0[..., None], v[..., 0:1], axis=-1)
    np.put_along_axis(dense, p1[..., None], v[..., 1:2], axis=-1)
    return dense.reshape(R, 4 * G)


def prune24_dense(bits, mode=HARD):
    """The masked (and, in SOFT mode, shrunk) matrix as dense bf16 bits: what the 2:4 GEMMs multiply by."""
    return prune24_decompress(*prune24_compress(bits, mode))
