"""Property tests (hypothesis) of the oracle's packing rules: invariants that must hold for ANY input, drawn at random with
shrinking, next to the fixed-seed pins of the other test files.  Paper: Section 2.2 (2:4), Section 2.3 (V:N:M), Table 5,
Section 3.4's closing paragraph (fp8)."""
import numpy as np
from hypothesis import given, settings, strategies as st
from hypothesis.extra import numpy as hnp

import oracle
from oracle import fp8

# any finite bf16 bit pattern: sign, exponent below 255, any mantissa (zeros, subnormals and max-finite included)
finite_bf16 = st.integers(0, 0xFFFF).filter(lambda b: (b & 0x7F80) != 0x7F80)
# a small alphabet makes ties frequent
tie_heavy = st.sampled_from([0x0000, 0x8000, 0x3F80, 0xBF80, 0x4000, 0x3F00, 0x0001, 0x8001, 0x7F7F])


def matrix(elements, rows, cols):
    return hnp.arrays(np.uint16, (rows, cols), elements=elements)


@settings(max_examples=200, deadline=None)
@given(st.one_of(matrix(finite_bf16, 4, 16), matrix(tie_heavy, 4, 16)), st.sampled_from([oracle.sparse24.HARD, oracle.sparse24.SOFT]))
def test_prune24_invariants(w, mode):
    vals, meta = oracle.prune24_compress(w, mode)
    dense = oracle.prune24_decompress(vals, meta)
    grp, dg = w.reshape(4, 4, 4), dense.reshape(4, 4, 4)
    nib = np.stack([meta & 0xF, meta >> 4], axis=-1).reshape(4, 4)
    p0, p1 = nib & 3, nib >> 2
    assert np.all(p0 < p1)                                                     # two distinct positions, ascending
    mag = (grp & 0x7FFF).astype(np.int64)
    kept = np.zeros((4, 4, 4), dtype=bool)
    np.put_along_axis(kept, p0[..., None].astype(np.int64), True, axis=-1)
    np.put_along_axis(kept, p1[..., None].astype(np.int64), True, axis=-1)
    assert np.all(kept.sum(-1) == 2)
    # every kept magnitude >= every dropped one; among equal magnitudes the lower index is kept
    for r in range(4):
        for g in range(4):
            k, d = np.nonzero(kept[r, g])[0], np.nonzero(~kept[r, g])[0]
            assert mag[r, g, k].min() >= mag[r, g, d].max()
            for i in d:
                assert not np.any((mag[r, g, k] == mag[r, g, i]) & (k > i))
    assert np.all((dg != 0).sum(-1) <= 2) and np.all(dg[~kept] == 0)           # at most two non-zeros, dropped slots are +0
    if mode == oracle.sparse24.HARD:
        assert np.array_equal(dg[kept], grp[kept])                             # survivors are bit copies
        v2, m2 = oracle.prune24_compress(dense, mode)                          # packing the masked matrix again changes nothing
        assert np.array_equal(v2, vals) and np.array_equal(oracle.prune24_decompress(v2, m2), dense)
    else:
        t = oracle.bits_to_f32(np.sort(mag, axis=-1)[..., 1].astype(np.uint16))   # second-smallest magnitude
        a, h = oracle.bits_to_f32(dg), oracle.bits_to_f32(grp)
        with np.errstate(invalid="ignore", over="ignore"):
            want = oracle.f32_to_bits(np.where((grp & 0x8000) != 0, h + t[..., None], h - t[..., None]).astype(np.float32))
        assert np.array_equal(dg[kept], want[kept])                            # survivors move towards zero by t, one rounding
        assert np.all(np.abs(a[kept]) <= np.abs(h[kept]))


@settings(max_examples=60, deadline=None)
@given(st.integers(0, 2 ** 32 - 1), st.sampled_from([8, 16, 32, 64]), st.sampled_from([0.0, 0.8, 2.0]))
def test_vnm_invariants(seed, M, shift):
    rng = np.random.default_rng(seed)
    T, F = 128, 2 * M * 2
    y1 = oracle.f32_to_bits((rng.standard_normal((T, F)) - shift).astype(np.float32))
    y1[rng.random((T, F)) < 0.2] = 0x3F80                                      # frequent ties
    vals, meta, colidx = oracle.sqrelu_vnm_compress(y1, 64, M)
    assert vals.shape == (T, 2 * F // M) and meta.shape == (T, F // (2 * M)) and colidx.shape == (T // 64, F // M, 4)
    assert np.all(np.diff(colidx.astype(np.int64), axis=-1) > 0) and colidx.max() < M     # four distinct ascending offsets inside the block
    y2 = oracle.sqrelu(y1)
    dense = oracle.vnm_decompress(vals, meta, colidx, 64, M)
    blocks = dense.reshape(T // 64, 64, F // M, M)
    assert np.all((blocks != 0).any(axis=1).sum(axis=-1) <= 4)                 # at most four live columns per block
    assert np.all((blocks != 0).sum(axis=-1) <= 2)                             # at most two survivors per row of a block
    assert np.mean(dense != 0) <= 2.0 / M                                      # Table 5: sparsity >= 1 - N / M
    assert np.all((dense == 0) | (dense == y2))                                # survivors are y2's own values
    # kept columns carry at least the L1 mass of every dropped column (scores are exact here: sums of few bf16 squares may round,
    # so compare with the oracle's own float32 scores)
    _, score = oracle.vnm_select_columns(y2, 64, M)
    ks = np.take_along_axis(score, colidx.astype(np.int64), axis=-1)
    dropped = np.ones(score.shape, dtype=bool)
    np.put_along_axis(dropped, colidx.astype(np.int64), False, axis=-1)
    assert np.all(ks.min(axis=-1) >= np.where(dropped, score, -np.inf).max(axis=-1))
    # eq. (6) on the same mask lands in the same slots
    dy2 = oracle.f32_to_bits(rng.standard_normal((T, F)).astype(np.float32))
    dv = oracle.dsqrelu_vnm(dy2, y1, meta, colidx, 64, M)
    dd = oracle.vnm_decompress(dv, meta, colidx, 64, M)
    assert np.all((dd == 0) | (dense != 0) | (oracle.bits_to_f32(y1) <= 0))    # gradient only where y2 was kept (or y1 <= 0 kills it)


@settings(max_examples=300, deadline=None)
@given(st.floats(min_value=-500.0, max_value=500.0, allow_nan=False, width=32))
def test_e4m3_encode_is_monotone_and_nearest(x):
    c = int(fp8.e4m3_encode(np.float32(x)))
    v = float(fp8.e4m3_decode(np.uint8(c)))
    lo = float(fp8.e4m3_decode(np.uint8(max((c & 0x7F) - 1, 0) | (c & 0x80))))
    hi = float(fp8.e4m3_decode(np.uint8(min((c & 0x7F) + 1, 0x7E) | (c & 0x80))))
    xc = min(max(x, -448.0), 448.0)
    assert abs(xc - v) <= abs(xc - lo) and abs(xc - v) <= abs(xc - hi)
    y = np.nextafter(np.float32(x), np.float32(1e9))
    assert float(fp8.e4m3_decode(fp8.e4m3_encode(y))) >= v                      # monotone


@settings(max_examples=100, deadline=None)
@given(matrix(finite_bf16, 2, 16), st.sampled_from([2.0 ** -8, 0.013, 1.0, 5.0]), st.sampled_from([oracle.sparse24.HARD, oracle.sparse24.SOFT]))
def test_fp8_pruning_never_changes_the_selection(w, scale, mode):
    codes, meta = fp8.prune24_compress_fp8(w, scale, mode)
    _, meta16 = oracle.prune24_compress(w, mode)
    assert np.array_equal(meta, meta16)
    assert not np.any(codes == 0x7F) and not np.any(codes == 0xFF)              # finite input never encodes to NaN (saturating)
