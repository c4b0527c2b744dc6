"""Pins for the oracle's SquaredReLU and V:N:M code (paper eq. (2), eq. (6), Section 2.3, Table 5)."""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def bf(x):
    return oracle.f32_to_bits(np.asarray(x, dtype=np.float32))


def test_sqrelu_values():
    y1 = bf([[-2.0, -0.0, 0.0, 0.5, 3.0, 1.0078125, 1e-30, -1e30]])
    y2 = oracle.sqrelu(y1)
    f = oracle.bits_to_f32(y2)[0]
    assert list(f[:5]) == [0.0, 0.0, 0.0, 0.25, 9.0] and not np.any(np.signbit(f[:3]))
    # 1.0078125^2 = 1.01568603515625 -> nearest bf16 (spacing 2^-7) is 1.015625
    assert f[5] == np.float32(1.015625)
    assert f[6] == 0.0 and f[7] == 0.0


@pytest.mark.parametrize("V", [1, 2, 4])
def test_column_choice_equals_subset_brute_force(V):
    """Kept columns = lexicographically smallest 4-subset among those of maximal total score, on
    small-integer blocks where float32 sums are exact; many ties on purpose."""
    rng = np.random.default_rng(10 + V)
    nblk = 300
    y2 = rng.integers(0, 4, size=(V, nblk * 8)).astype(np.float32)
    colidx, score = oracle.vnm_select_columns(bf(y2), V, 8)
    sums = y2.reshape(V, nblk, 8).sum(0)
    assert np.array_equal(score[0], sums)
    subsets = list(itertools.combinations(range(8), 4))
    for b in range(nblk):
        best = max(sums[b, list(s)].sum() for s in subsets)
        want = next(s for s in subsets if sums[b, list(s)].sum() == best)
        assert tuple(colidx[0, b]) == want


def test_score_is_sequential_float32_in_row_order():
    """2^24 + 1 + 1 + ... in float32, one add at a time, never leaves 2^24; any pairwise or wider
    accumulation would count the ones.  That decides which columns survive here."""
    V = 64
    y2 = np.zeros((V, 8), dtype=np.float32)
    y2[0, 0] = 2.0 ** 24
    y2[1:, 0] = 1.0          # column 0: sequential float32 sum stays 2^24 (exact sum 2^24 + 63)
    y2[0, 1] = 2.0 ** 24
    y2[1, 1] = 2.0           # column 1: 2^24 + 2 is representable -> beats column 0
    y2[:, 2] = 2.0 ** 18     # 64 * 2^18 = 2^24 exactly: ties with column 0, loses to it on index
    y2[0, 3] = 2.0 ** 24
    y2[0, 4] = 2.0 ** 24
    y2[0, 5] = 2.0 ** 24     # columns 3, 4, 5 tie with 0 and 2 at 2^24
    colidx, score = oracle.vnm_select_columns(bf(y2), V, 8)
    assert score[0, 0, 0] == np.float32(2.0 ** 24) and score[0, 0, 1] == np.float32(2.0 ** 24 + 2)
    assert list(colidx[0, 0]) == [0, 1, 2, 3]
    # descending row order would have given column 0 the score 2^24 + 64 (63 ones first: exact)
    assert np.float32(63.0) + np.float32(2.0 ** 24) != np.float32(2.0 ** 24)


def test_table5_sparsity_and_bytes():
    for line in open(os.path.join(GOLD, "table5_vnm_sparsity.txt")):
        if line.startswith("#") or not line.strip():
            continue
        V, N, M, pct = line.split()
        V, N, M, pct = int(V), int(N), int(M), float(pct)
        rng = np.random.default_rng(M)
        y2 = bf(np.abs(rng.standard_normal((2 * V, 4 * M))) + 0.5)     # no zeros going in
        vals, meta, colidx = oracle.vnm_compress(y2, V, M)
        dense = oracle.vnm_decompress(vals, meta, colidx, V, M)
        assert 100.0 * (1.0 - np.count_nonzero(dense) / dense.size) == pct == 100.0 * (1 - N / M)
        assert vals.shape == (2 * V, 4 * M * N // M) and meta.shape == (2 * V, 2) and colidx.shape == (2, 4, 4)


def test_m4_is_plain_24_and_v1_is_row_top2_of_8():
    rng = np.random.default_rng(5)
    y2 = bf(np.abs(rng.standard_normal((16, 64))) * (rng.random((16, 64)) < 0.4))
    vals, meta, colidx = oracle.vnm_compress(y2, 4, 4)
    v24, m24 = oracle.prune24_compress(y2)
    assert np.array_equal(vals, v24) and np.array_equal(meta, m24) and np.all(colidx == np.arange(4))
    vals, meta, colidx = oracle.vnm_compress(y2, 1, 8)
    dense = oracle.vnm_decompress(vals, meta, colidx, 1, 8).reshape(16, 8, 8)
    mag = (y2.reshape(16, 8, 8) & 0x7FFF).astype(np.int32)
    order = np.argsort(-mag, axis=-1, kind="stable")[..., :2]
    want = np.zeros_like(dense)
    np.put_along_axis(want, order, np.take_along_axis(y2.reshape(16, 8, 8), order, axis=-1), axis=-1)
    assert np.array_equal(dense, want)


def test_vnm_roundtrip_structure_and_24_view():
    rng = np.random.default_rng(6)
    y1 = bf(rng.standard_normal((128, 64)) - 1.0)
    vals, meta, colidx = oracle.sqrelu_vnm_compress(y1, 64, 8)
    assert vals.shape == (128, 16) and meta.shape == (128, 4) and colidx.shape == (2, 8, 4)
    assert np.all(np.diff(colidx.astype(int), axis=-1) > 0) and colidx.max() < 8
    dense = oracle.vnm_decompress(vals, meta, colidx, 64, 8)
    y2 = oracle.sqrelu(y1)
    nz = dense != 0
    assert np.array_equal(dense[nz], y2[nz])                       # survivors are bit copies of y2
    assert nz.reshape(128, 8, 8).sum(-1).max() <= 2                # N = 2 per M = 8
    assert nz.reshape(128, 16, 4).sum(-1).max() <= 2               # hence also a valid plain 2:4 matrix
    colmask = nz.reshape(2, 64, 8, 8).any(1)
    assert colmask.sum(-1).max() <= 4                              # at most 4 live columns per block
    # re-compressing the decompressed matrix reproduces values and metadata
    v2, m2, c2 = oracle.vnm_compress(dense, 64, 8)
    d2 = oracle.vnm_decompress(v2, m2, c2, 64, 8)
    assert np.array_equal(d2, dense)
    assert np.array_equal(oracle.vnm_to_24(vals, meta, colidx), dense)


def test_rows_with_fewer_than_two_nonzeros_fill_lowest_slots():
    y2 = np.zeros((64, 8), dtype=np.float32)
    y2[:, [1, 3, 4, 6]] = 1.0          # live columns
    y2[5] = 0
    y2[5, 4] = 9.0                     # one survivor in slot 2 of the kept four
    y2[6] = 0                          # no survivor at all
    vals, meta, colidx = oracle.vnm_compress(bf(np.tile(y2, (1, 2))), 64, 8)
    assert list(colidx[0, 0]) == [1, 3, 4, 6]
    assert (meta[5, 0] & 0xF) == (0 | 2 << 2) and list(oracle.bits_to_f32(vals[5, :2])) == [0.0, 9.0]
    assert (meta[6, 0] & 0xF) == (0 | 1 << 2) and list(vals[6, :2]) == [0, 0]


def test_dsqrelu_matches_elementwise_definition():
    rng = np.random.default_rng(7)
    y1 = bf(rng.standard_normal((64, 32)) - 0.5)
    dy2 = bf(rng.standard_normal((64, 32)))
    vals, meta, colidx = oracle.sqrelu_vnm_compress(y1)
    dvals = oracle.dsqrelu_vnm(dy2, y1, meta, colidx)
    dense = oracle.bits_to_f64(oracle.vnm_decompress(dvals, meta, colidx))
    mask_slots = np.zeros((64, 32), dtype=bool)
    ones = np.full_like(vals, 0x3F80)
    mask_slots = oracle.vnm_decompress(ones, meta, colidx) != 0        # every kept slot, also those holding 0
    want = 2.0 * oracle.bits_to_f64(dy2) * np.maximum(oracle.bits_to_f64(y1), 0.0)
    want = oracle.bits_to_f64(oracle.f64_to_bits(want)) * mask_slots
    assert np.array_equal(dense, want)
    assert mask_slots.reshape(64, 4, 8).sum(-1).min() == 2
