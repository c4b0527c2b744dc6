"""Pins for the oracle's 2:4 pruning and packing (paper Section 2.2): brute force over pairs,
invariants, the hand-worked soft-threshold examples, packing round trips."""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle.sparse24 import HARD, SOFT

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def bf(x):
    return oracle.f32_to_bits(np.asarray(x, dtype=np.float32))


def test_selection_equals_pair_brute_force():
    """Kept pair = lexicographically smallest of the pairs with the largest |a_i| + |a_j|, over every
    4-tuple from an alphabet with repeats, +-0 and equal magnitudes of opposite sign."""
    alphabet = np.array([0.0, -0.0, 1.0, -1.0, 2.0, 0.5, -3.0], dtype=np.float32)
    tuples = np.array(list(itertools.product(range(len(alphabet)), repeat=4)))
    groups = alphabet[tuples]                                   # [N, 4]
    bits = bf(groups)
    kept, third = oracle.prune24_positions(bits)
    mag = np.abs(groups.astype(np.float64))
    pairs = list(itertools.combinations(range(4), 2))           # lexicographic order
    for n in range(len(groups)):
        best = max(mag[n, i] + mag[n, j] for i, j in pairs)
        want = next((i, j) for i, j in pairs if mag[n, i] + mag[n, j] == best)
        assert tuple(kept[n, 0]) == want, (groups[n], kept[n, 0], want)
        rest = [i for i in range(4) if i not in want]
        assert mag[n, third[n, 0]] == max(mag[n, rest])
        # ties among the dropped go to the lower index too
        assert third[n, 0] == min(i for i in rest if mag[n, i] == max(mag[n, rest]))


def test_hard_invariants_and_roundtrip():
    rng = np.random.default_rng(3)
    W = bf(rng.standard_normal((37, 64)) * 0.02)
    W[0, :8] = 0
    W[1, :4] = bf([1, 1, 1, 1])
    vals, meta = oracle.prune24_compress(W, HARD)
    assert vals.shape == (37, 32) and meta.shape == (37, 8) and meta.dtype == np.uint8
    dense = oracle.prune24_decompress(vals, meta)
    g = dense.reshape(37, 16, 4)
    assert ((g & 0x7FFF) != 0).sum(-1).max() <= 2
    w = W.reshape(37, 16, 4)
    keptmask = np.zeros_like(w, dtype=bool)
    kept, _ = oracle.prune24_positions(W)
    np.put_along_axis(keptmask, kept, True, axis=-1)
    assert keptmask.sum(-1).min() == 2 and keptmask.sum(-1).max() == 2
    # kept entries are bit copies, dropped are +0
    assert np.array_equal(g[keptmask], w[keptmask]) and np.all(g[~keptmask] == 0)
    mag = (w & 0x7FFF).astype(np.int32)
    assert np.all(np.where(keptmask, mag, 1 << 20).min(-1) >= np.where(~keptmask, mag, -1).max(-1))
    # nibbles are one of the six ascending pairs
    nibs = np.concatenate([(meta & 0xF).ravel(), (meta >> 4).ravel()])
    assert set(np.unique(nibs)) <= {0x4, 0x8, 0xC, 0x9, 0xD, 0xE}
    # all-zero group -> positions (0, 1); all-equal group -> positions (0, 1)
    assert meta[0, 0] == 0x44 and meta[1, 0] & 0xF == 0x4
    # compress(decompress(.)) is idempotent bit for bit
    v2, m2 = oracle.prune24_compress(dense, HARD)
    assert np.array_equal(v2, vals) and np.array_equal(m2, meta)


def test_meta_byte_layout_explicit():
    # one row, two groups: group 0 keeps positions (1, 3), group 1 keeps (0, 2)
    row = bf([[0.1, 5, 0.2, -6, 7, 0.1, -8, 0.2]])
    vals, meta = oracle.prune24_compress(row, HARD)
    assert list(oracle.bits_to_f32(vals[0])) == [5, -6, 7, -8]
    assert meta[0, 0] == ((1 | 3 << 2) | ((0 | 2 << 2) << 4))


def test_soft_threshold_golden_examples():
    rows = []
    for line in open(os.path.join(GOLD, "soft_threshold_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        a, o = line.split("->")
        rows.append(([float(v) for v in a.split()], [float(v) for v in o.split()]))
    A = bf([r[0] for r in rows])
    want = np.array([r[1] for r in rows], dtype=np.float32)
    got = oracle.bits_to_f32(oracle.prune24_dense(np.tile(A, (1, 2)), SOFT))[:, :4]
    assert np.array_equal(got, want)
    assert not np.any(np.signbit(got[want == 0]))          # shrunk-to-zero and dropped entries are +0


def test_soft_is_hard_shrunk_by_t_and_continuous():
    rng = np.random.default_rng(4)
    W = bf(rng.standard_normal((16, 32)))
    vh, mh = oracle.prune24_compress(W, HARD)
    vs, ms = oracle.prune24_compress(W, SOFT)
    assert np.array_equal(mh, ms)
    mag = np.sort(np.abs(oracle.bits_to_f64(W)).reshape(16, 8, 4), axis=-1)
    t = mag[..., 1]
    h = oracle.bits_to_f64(vh).reshape(16, 8, 2)
    want = np.sign(h) * (np.abs(h) - t[..., None])
    assert np.array_equal(oracle.bits_to_f64(vs).reshape(16, 8, 2), oracle.bits_to_f64(oracle.f64_to_bits(want)))
    # continuity across a rank swap: the 2nd and 3rd magnitudes trade places, SOFT moves by O(eps), HARD jumps
    eps = 2.0 ** -7
    a = bf([[4, 1 + eps, 1, 0.1, 0, 0, 0, 0]])
    b = bf([[4, 1, 1 + eps, 0.1, 0, 0, 0, 0]])
    sa = oracle.bits_to_f64(oracle.prune24_dense(a, SOFT))
    sb = oracle.bits_to_f64(oracle.prune24_dense(b, SOFT))
    ha = oracle.bits_to_f64(oracle.prune24_dense(a, HARD))
    hb = oracle.bits_to_f64(oracle.prune24_dense(b, HARD))
    assert np.abs(sa - sb).max() <= 2 * eps and np.abs(ha - hb).max() >= 1.0


def test_soft_rounding_is_float32_then_bf16():
    # |a| - t is not representable in bf16 here; the result is the RNE of the float32 difference
    a = bf([[1.0, 2.0 ** -9, 0, 0, 0, 0, 0, 0]])            # kept: 1.0 and 2^-9, t = 0
    a[0, 2] = bf([2.0 ** -9])[0]                                  # now t = 2^-9 (third largest), kept (0, 1)
    v, m = oracle.prune24_compress(a, SOFT)
    assert oracle.bits_to_f32(v[0, 0]) == np.float32(1.0)    # 1 - 2^-9 rounds (RNE, tie to even) to 1.0
    assert v[0, 1] == 0                                      # 2^-9 - 2^-9 = +0


@pytest.mark.parametrize("mode", [HARD, SOFT])
def test_special_values_are_deterministic(mode):
    sub = np.uint16(0x0001)                                  # smallest subnormal
    big = np.uint16(0x7F7F)                                  # largest finite
    row = np.array([[sub, 0x8000, 0x0000, sub | 0x8000, big, big | 0x8000, 0x3F80, 0xBF80]], dtype=np.uint16)
    v1, m1 = oracle.prune24_compress(row, mode)
    v2, m2 = oracle.prune24_compress(row.copy(), mode)
    assert np.array_equal(v1, v2) and np.array_equal(m1, m2)
    assert m1[0, 0] == ((0 | 3 << 2) | ((0 | 1 << 2) << 4))  # subnormals beat zeros; +-max beat +-1


def test_hard_pruning_is_total_on_bit_patterns():
    """Section 2.2 ranks magnitudes; read on bit patterns (sign cleared, compared as integers) the rule also orders what is not a number:
    NaN patterns above infinity above every finite value, ties to the lower index, and HARD mode hands the survivors on untouched."""
    row = np.array([[0x7F80, 0x3F80, 0x7FC1, 0x4000,          # inf, 1, NaN, 2        -> positions 0, 2
                     0xFF80, 0x7F80, 0x7F7F, 0xFF7F]],         # -inf, inf, max, -max  -> the two infinities (tie: lower index first)
                   dtype=np.uint16)
    v, m = oracle.prune24_compress(row, HARD)
    assert list(v[0]) == [0x7F80, 0x7FC1, 0xFF80, 0x7F80]
    assert m[0, 0] == ((0 | 2 << 2) | ((0 | 1 << 2) << 4))
