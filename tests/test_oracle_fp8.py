"""Pins for the oracle's fp8 stage (paper Section 3.4, closing paragraph; format: OCP E4M3, finite-only variant)."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import fp8


def bf(x):
    return oracle.f32_to_bits(np.asarray(x, dtype=np.float32))


def test_e4m3_decode_all_256_codes():
    codes = np.arange(256, dtype=np.uint8)
    got = fp8.e4m3_decode(codes)
    ref = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float32).numpy()      # the library's table
    nan = np.isnan(ref)
    assert list(np.nonzero(nan)[0]) == [0x7F, 0xFF] and np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))                  # bit-equal, -0 included
    # anchors written out from the format's definition (bias 7, 3 mantissa bits, subnormals m * 2^-9, largest finite 448)
    for code, val in ((0x00, 0.0), (0x01, 2.0 ** -9), (0x07, 7 * 2.0 ** -9), (0x08, 2.0 ** -6), (0x38, 1.0), (0x39, 1.125), (0x40, 2.0),
                      (0x7E, 448.0), (0xB8, -1.0), (0xFE, -448.0), (0x77, 240.0), (0x78, 256.0)):
        assert got[code] == np.float32(val)
    assert np.signbit(got[0x80]) and got[0x80] == 0
    pos = got[:0x7F]
    assert np.all(np.diff(pos) > 0)                                                              # codes order like values


def test_e4m3_encode_round_trip_ties_and_saturation():
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    vals = fp8.e4m3_decode(codes)
    assert np.array_equal(fp8.e4m3_encode(vals), codes)                                          # every representable value is a fixed point
    # exact midpoints between neighbours go to the even code; one float32 ulp either side goes to the nearer one
    lo, hi = fp8.e4m3_decode(np.arange(0, 0x7E, dtype=np.uint8)), fp8.e4m3_decode(np.arange(1, 0x7F, dtype=np.uint8))
    for c in range(0x7E):
        mid = Fraction(float(lo[c])) + (Fraction(float(hi[c])) - Fraction(float(lo[c]))) / 2
        m32 = np.float32(float(mid))
        assert Fraction(float(m32)) == mid                                                       # midpoints are float32 numbers
        even = c if c % 2 == 0 else c + 1
        assert fp8.e4m3_encode(m32) == even and fp8.e4m3_encode(-m32) == (even | 0x80)
        assert fp8.e4m3_encode(np.nextafter(m32, np.float32(1e9))) == c + 1
        assert fp8.e4m3_encode(np.nextafter(m32, np.float32(-1e9))) == c
    for x, code in ((448.0, 0x7E), (449.0, 0x7E), (464.0, 0x7E), (465.0, 0x7E), (1e9, 0x7E), (-1e9, 0xFE), (3.0e38, 0x7E)):
        assert fp8.e4m3_encode(np.float32(x)) == code                                            # saturating, never NaN for finite input
    assert fp8.e4m3_encode(np.float32(2.0 ** -10)) == 0x00 and fp8.e4m3_encode(np.nextafter(np.float32(2.0 ** -10), np.float32(1))) == 0x01
    assert fp8.e4m3_encode(np.float32(-0.0)) == 0x80


def test_e4m3_encode_is_the_nearest_code_brute_force_and_matches_the_library():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4000).astype(np.float32) * s for s in (1e-3, 0.02, 1.0, 30.0, 200.0)])
    x = x[np.abs(x) <= 448]
    got = fp8.e4m3_encode(x)
    grid = fp8.e4m3_decode(np.arange(0x7F, dtype=np.uint8)).astype(np.float64)
    d = np.abs(np.abs(x.astype(np.float64))[:, None] - grid[None, :])
    best = d.min(axis=1)
    assert np.all(d[np.arange(len(x)), got & 0x7F] == best)                                      # a nearest grid point
    ties = (d == best[:, None]).sum(axis=1) > 1
    assert np.all((got[ties] & 1) == 0)                                                          # and the even one on a tie
    assert np.array_equal((got & 0x80) != 0, np.signbit(x))
    lib = torch.from_numpy(x.copy()).to(torch.float8_e4m3fn).view(torch.uint8).numpy()           # in range: the library rounds the same way
    assert np.array_equal(got, lib)


def test_quantize_scale_semantics():
    rng = np.random.default_rng(1)
    x = bf(rng.standard_normal((8, 64)) * 3)
    for k in (-5, 0, 3):                                                                         # a power-of-two scale is an exact shift
        assert np.array_equal(fp8.quantize_fp8(x, 2.0 ** k), fp8.e4m3_encode(oracle.bits_to_f32(x) * np.float32(2.0 ** -k)))
    assert np.array_equal(fp8.quantize_fp8(bf([1000.0, -1000.0]), 1.0), [0x7E, 0xFE])            # saturates instead of overflowing
    # the stated arithmetic is float32(x) * (float32(1) / scale), not x / scale in higher precision: scale = 7, x = 1.3671875 = 175/128:
    # x / 7 is exactly 25/128 = 0.1953125, the midpoint of two neighbouring codes -> tie -> the even code.  float32(1/7) is above
    # 1/7, so the float32 product lands just above the midpoint and takes the odd code above it instead.
    x = bf([1.3671875])
    exact = Fraction(175, 128) / 7
    assert exact == Fraction(25, 128)
    m32 = np.float32(1.3671875) * (np.float32(1.0) / np.float32(7.0))
    assert Fraction(float(m32)) > exact
    lo, hi = fp8.e4m3_encode(np.float32(24 / 128)), fp8.e4m3_encode(np.float32(26 / 128))
    assert hi == lo + 1 and lo % 2 == 0 and fp8.e4m3_encode(np.float32(float(exact))) == lo     # the exact quotient would tie to the even code
    assert fp8.quantize_fp8(x, 7.0)[0] == fp8.e4m3_encode(m32) == hi
    assert fp8.amax(bf([[0.5, -7.0], [3.0, -0.0]])) == np.float32(7.0) and fp8.amax(np.zeros((0, 4), dtype=np.uint16)) == 0


@pytest.mark.parametrize("mode", [oracle.sparse24.HARD, oracle.sparse24.SOFT])
def test_prune24_fp8_keeps_the_bf16_selection(mode):
    rng = np.random.default_rng(2 + mode)
    w = bf(rng.standard_normal((48, 128)) * 0.02)
    w[0, :8] = bf([0.0, -0.0, 0.0, 0.0, 1.0, 1.0, -1.0, 1.0])                                      # zero group, tied group
    scale = 0.02 * 4 / 448
    codes, meta = fp8.prune24_compress_fp8(w, scale, mode)
    vals, meta_bf16 = oracle.prune24_compress(w, mode)
    assert np.array_equal(meta, meta_bf16) and codes.shape == vals.shape and codes.dtype == np.uint8
    if mode == oracle.sparse24.HARD:                                                             # HARD: the survivors are bf16 bit copies, so this is their quantisation
        assert np.array_equal(codes, fp8.quantize_fp8(vals, scale))
    dense = oracle.prune24_decompress(fp8.codes_as_bf16_bits(codes), meta)
    assert np.all((dense.reshape(48, 32, 4) != 0).sum(axis=-1) <= 2)


def test_soft_threshold_goes_to_fp8_without_a_bf16_rounding_in_between():
    """a - t = 1.0703125 - 0.0068359375 = 1.0634765625, just above 1.0625, the midpoint of the fp8 neighbours 1.0 and 1.125:
    directly it rounds to 1.125; through bf16 it would first become 1.0625 and then tie to 1.0."""
    a, t = 1.0703125, 0.0068359375
    w = bf([[a, 2.0, t, 0.001, 0.0, 0.0, 0.0, 0.0]])
    assert oracle.bits_to_f32(w)[0, 0] == np.float32(a) and oracle.bits_to_f32(w)[0, 2] == np.float32(t)
    codes, meta = fp8.prune24_compress_fp8(w, 1.0, oracle.sparse24.SOFT)
    assert meta[0, 0] & 0xF == (0 | 1 << 2)
    assert fp8.e4m3_decode(codes[0, :2]).tolist() == [1.125, 2.0]
    vals, _ = oracle.prune24_compress(w, oracle.sparse24.SOFT)
    assert oracle.bits_to_f32(vals)[0, 0] == np.float32(1.0625) and fp8.quantize_fp8(vals, 1.0)[0, 0] == fp8.e4m3_encode(np.float32(1.0))


@pytest.mark.parametrize("M", [8, 32])
def test_vnm_fp8_keeps_the_bf16_selection(M):
    rng = np.random.default_rng(M)
    y1 = bf(rng.standard_normal((128, 256)) - 0.8)
    scale = 16.0 / 448
    codes, meta, colidx = fp8.sqrelu_vnm_compress_fp8(y1, scale, 64, M)
    vals, meta_b, colidx_b = oracle.sqrelu_vnm_compress(y1, 64, M)
    assert np.array_equal(meta, meta_b) and np.array_equal(colidx, colidx_b)
    assert np.array_equal(codes, fp8.quantize_fp8(vals, scale))
    assert np.all(fp8.e4m3_decode(codes) >= 0)


def test_fp8_contractions_exact_rationals_and_reduction_to_the_bf16_oracle():
    rng = np.random.default_rng(5)
    T, N, K = 6, 5, 16
    xq = rng.integers(0, 0x7F, size=(T, K)).astype(np.uint8) | (rng.integers(0, 2, size=(T, K)).astype(np.uint8) << 7)
    w = bf(rng.standard_normal((N, K)))
    wc, wm = fp8.prune24_compress_fp8(w, 1.0 / 64)
    sx, sw = np.float32(0.37), np.float32(1.0 / 64)
    bias = rng.standard_normal(N).astype(np.float32)
    got = fp8.spmm24_fp8(xq, sx, wc, wm, sw, bias)
    wd = oracle.prune24_decompress(fp8.codes_as_bf16_bits(wc), wm)
    s = Fraction(float(np.float32(sx) * np.float32(sw)))
    for t in range(T):
        for n in range(N):
            acc = sum(Fraction(float(fp8.e4m3_decode(xq[t, k]))) * Fraction(float(oracle.bits_to_f32(wd[n, k]))) for k in range(K))
            want = oracle.f64_to_bits(np.float64(float(acc * s + Fraction(float(bias[n])))))
            assert got[t, n] == want
    # operands that are exactly representable in fp8, scale 1: the fp8 contraction IS the bf16 one (already pinned)
    xi = bf(rng.integers(-4, 5, size=(8, 32)))
    wi = bf(rng.integers(-3, 4, size=(7, 32)))
    v16, m16 = oracle.prune24_compress(wi)
    c8, m8 = fp8.prune24_compress_fp8(wi, 1.0)
    assert np.array_equal(m8, m16)
    assert np.array_equal(fp8.spmm24_fp8(fp8.quantize_fp8(xi, 1.0), 1.0, c8, m8, 1.0), oracle.spmm24(xi, v16, m16))
    # power-of-two scales factor out exactly
    assert np.array_equal(oracle.bits_to_f32(fp8.spmm24_fp8(fp8.quantize_fp8(xi, 1.0), 4.0, c8, m8, 0.5)),
                          2 * oracle.bits_to_f32(oracle.spmm24(xi, v16, m16)))
    # V:N:M operand: same reduction, both orientations of the dense matrix
    y1 = bf(rng.integers(-2, 4, size=(64, 64)))
    wq = bf(rng.integers(-3, 4, size=(24, 64)))
    ac, am, aidx = fp8.sqrelu_vnm_compress_fp8(y1, 1.0)
    av, _, _ = oracle.sqrelu_vnm_compress(y1)
    for kmaj, wmat in ((0, wq), (1, np.ascontiguousarray(wq.T))):
        assert np.array_equal(fp8.vnm_spmm_fp8(ac, am, aidx, 1.0, fp8.quantize_fp8(wmat, 1.0), 1.0, kmaj), oracle.vnm_spmm(av, am, aidx, wmat, kmaj))


# ---- the whole step with fp8 operands (a stated reading: Section 3.4's closing paragraph applied to Alg. 1 / Alg. 2) ----------
def _step_inputs(T=64, D=32, F=64, seed=0):
    from workload import make_ffn_inputs
    return make_ffn_inputs(T, D, F, seed=seed)


def _amax(bits):
    return float(np.max(np.abs(oracle.bits_to_f32(bits))))


def _scales_for(inp, ref):
    """Per-tensor scales of a delayed-scaling recipe: amax / 448 of each quantised tensor, taken from the bf16 step."""
    y2 = oracle.sqrelu(ref["y1"])
    return dict(x=_amax(inp["X"]) / 448, w1=_amax(inp["W1"]) / 448, w2=_amax(inp["W2"]) / 448, y2=max(_amax(y2), 1e-6) / 448,
                dy=_amax(inp["dY"]) / 448, dy1=max(_amax(ref["dy1_vals"]), 1e-6) / 448)


def test_fp8_step_stays_within_the_quantisation_error_of_the_bf16_step():
    """Each fp8 operand carries a relative rounding error of at most 2^-4 (3 mantissa bits), so every contraction of the fp8 step
    must be close to the bf16 step's - and not equal to it."""
    inp = _step_inputs(128, 64, 128)
    ref = oracle.ffn_sparse_step_ref(inp["X"], inp["W1"], inp["W2"], inp["b1"], inp["dY"])
    got = oracle.ffn_sparse_step_fp8_ref(inp["X"], inp["W1"], inp["W2"], inp["b1"], inp["dY"], _scales_for(inp, ref))
    a, b = oracle.bits_to_f32(got["y1"]).astype(np.float64), oracle.bits_to_f32(ref["y1"]).astype(np.float64)
    rel = np.linalg.norm(a - b) / np.linalg.norm(b)
    assert 1e-4 < rel < 0.06, rel                     # two operands with <= 2^-4 relative error each, averaged over 32 / 2 products


def test_fp8_step_is_invariant_to_power_of_two_changes_of_any_single_scale():
    """code(x / (s / 2)) decodes to exactly twice code(x / s) while both stay normal numbers below 448, so halving ONE scale must
    leave every output bit-identical.  Using a tensor's scale on the wrong operand, or forgetting it in the product of the two
    scales after a contraction, breaks this for that scale.  Small-integer inputs keep every quantised tensor's dynamic range
    (largest / smallest non-zero magnitude) far below the 2^14 that the normal range of E4M3 spans."""
    rng = np.random.default_rng(11)
    T, D, F = 64, 32, 64
    ints = lambda shape: bf(rng.integers(-2, 3, shape).astype(np.float32))
    X, W1, W2, dY = ints((T, D)), ints((F, D)), ints((D, F)), ints((T, D))
    b1 = np.full(F, -2.0, dtype=np.float32)
    ref = oracle.ffn_sparse_step_ref(X, W1, W2, b1, dY)
    pow2 = lambda amax: float(2.0 ** np.ceil(np.log2(max(amax, 1.0) / 200.0)))       # largest code magnitude in (100, 200]
    base = dict(x=pow2(2), w1=pow2(2), w2=pow2(2), dy=pow2(2), y2=pow2(_amax(oracle.sqrelu(ref["y1"]))), dy1=pow2(_amax(ref["dy1_vals"])))
    want = oracle.ffn_sparse_step_fp8_ref(X, W1, W2, b1, dY, base)
    for name in ("xq", "w1_codes", "y2_codes", "dyq", "dy1_codes", "w2q", "w1q", "w2t_codes"):
        mag = np.abs(fp8.e4m3_decode(want[name]))
        assert mag.max() <= 224 and mag[mag > 0].min() >= 2.0 ** -6, name            # the premise: normal numbers, room to double
    assert np.count_nonzero(want["y2_codes"]) > 100 and np.count_nonzero(want["dy1_codes"]) > 100
    for k in base:
        s2 = dict(base)
        s2[k] = base[k] * 0.5
        got = oracle.ffn_sparse_step_fp8_ref(X, W1, W2, b1, dY, s2)
        for name in ("y1", "y3", "dy2", "dX", "dW1", "dW2", "dy1_vals", "y2_meta", "colidx"):
            assert np.array_equal(got[name], want[name]), (k, name)
    # and a scale used on the wrong tensor would show: the codes of the tensor whose scale changed double, the others do not move
    got = oracle.ffn_sparse_step_fp8_ref(X, W1, W2, b1, dY, dict(base, y2=base["y2"] * 0.5))
    assert np.array_equal(fp8.e4m3_decode(got["y2_codes"]), 2 * fp8.e4m3_decode(want["y2_codes"])) and np.array_equal(got["dy1_codes"], want["dy1_codes"])


def test_fp8_step_positions_are_those_of_the_bf16_rules_on_its_own_y1():
    """Selection looks at bf16 values only: on the fp8 step's own y1 the bf16 compressor gives the same metadata, column indices
    and survivors, and the survivors' codes are their quantisation; eq. (6) is the bf16 rule; weight gradients are the bf16 ones."""
    inp = _step_inputs(64, 32, 64, seed=5)
    ref = oracle.ffn_sparse_step_ref(inp["X"], inp["W1"], inp["W2"], inp["b1"], inp["dY"])
    sc = _scales_for(inp, ref)
    got = oracle.ffn_sparse_step_fp8_ref(inp["X"], inp["W1"], inp["W2"], inp["b1"], inp["dY"], sc)
    vals, meta, colidx = oracle.sqrelu_vnm_compress(got["y1"])
    assert np.array_equal(meta, got["y2_meta"]) and np.array_equal(colidx, got["colidx"]) and np.array_equal(vals, got["y2_vals"])
    assert np.array_equal(got["y2_codes"], fp8.quantize_fp8(vals, sc["y2"]))
    assert np.array_equal(got["dy1_vals"], oracle.dsqrelu_vnm(got["dy2"], got["y1"], meta, colidx))
    assert np.array_equal(got["dW2"], oracle.vnm_wgrad(vals, meta, colidx, inp["dY"], 0))
    assert np.array_equal(got["dW1"], oracle.vnm_wgrad(got["dy1_vals"], meta, colidx, inp["X"], 1))
    # weights: the pruned positions are those of the bf16 pruning
    _, m1 = oracle.prune24_compress(inp["W1"])
    assert np.array_equal(m1, got["w1_meta"])


@pytest.mark.parametrize("M", [16, 32])
def test_fp8_step_with_wide_blocks_keeps_the_bf16_rules_of_that_block_width(M):
    """Table 5's wider blocks: on its own y1 the fp8 step's metadata, column indices and survivors are those of the bf16 compressor for
    that M (so at most 2 of M entries survive), the codes are the survivors' quantisation, eq. (6) and the bf16 weight gradients are
    the bf16 rules for that M, and eq. (3) is the dense product of the decoded, decompressed codes times the two scales."""
    inp = _step_inputs(64, 32, 4 * M, seed=M)
    ref = oracle.ffn_sparse_step_ref(inp["X"], inp["W1"], inp["W2"], inp["b1"], inp["dY"], V=64, M=M)
    sc = _scales_for(inp, ref)
    got = oracle.ffn_sparse_step_fp8_ref(inp["X"], inp["W1"], inp["W2"], inp["b1"], inp["dY"], sc, V=64, M=M)
    vals, meta, colidx = oracle.sqrelu_vnm_compress(got["y1"], 64, M)
    assert np.array_equal(meta, got["y2_meta"]) and np.array_equal(colidx, got["colidx"]) and np.array_equal(vals, got["y2_vals"])
    assert np.array_equal(got["y2_codes"], fp8.quantize_fp8(vals, sc["y2"]))
    assert got["y2_codes"].shape == (64, 2 * 4 * M // M) and colidx.shape == (1, 4, 4)
    assert np.array_equal(got["dy1_vals"], oracle.dsqrelu_vnm(got["dy2"], got["y1"], meta, colidx, 64, M))
    assert np.array_equal(got["dW2"], oracle.vnm_wgrad(vals, meta, colidx, inp["dY"], 0, 64, M))
    assert np.array_equal(got["dW1"], oracle.vnm_wgrad(got["dy1_vals"], meta, colidx, inp["X"], 1, 64, M))
    # eq. (3) on codes = the dense product of the decoded, decompressed codes
    a = fp8.e4m3_decode(oracle.vnm_decompress(got["y2_codes"], meta, colidx, 64, M)).astype(np.float64)
    w = fp8.e4m3_decode(got["w2q"]).astype(np.float64)
    want = oracle.f64_to_bits(a @ w.T * np.float64(np.float32(sc["y2"]) * np.float32(sc["w2"])))
    assert np.array_equal(got["y3"], want)
    assert np.mean(a != 0) <= 2.0 / M


def test_fp8_step_saturates_instead_of_overflowing():
    inp = _step_inputs(64, 32, 64, seed=7)
    ref = oracle.ffn_sparse_step_ref(inp["X"], inp["W1"], inp["W2"], inp["b1"], inp["dY"])
    sc = _scales_for(inp, ref)
    sc["x"] = sc["x"] / 64                         # X / scale reaches 64 x 448: every large entry clamps to +-448
    got = oracle.ffn_sparse_step_fp8_ref(inp["X"], inp["W1"], inp["W2"], inp["b1"], inp["dY"], sc)
    dec = fp8.e4m3_decode(got["xq"])
    assert np.all(np.isfinite(dec)) and np.max(np.abs(dec)) == 448.0 and np.mean(np.abs(dec) == 448.0) > 0.5
    assert np.all(np.isfinite(oracle.bits_to_f32(got["y3"])))


def test_fp8_weight_gradients_contract_the_codes_of_the_other_contractions():
    """wgrad_fp8: eq. (5) / eq. (8) as a plain triple loop over the decoded codes (exact rationals), orientation and scales included;
    and with every quantised value exactly representable the fp8 weight gradients equal the bf16 ones."""
    rng = np.random.default_rng(5)
    T, F, N = 64, 16, 8
    y1 = bf(rng.integers(-2, 4, (T, F)).astype(np.float32))                                          # y2 in {0, 1, 4, 9}: codes are exact at scale 1/2
    codes, meta, cix = fp8.sqrelu_vnm_compress_fp8(y1, 0.5)
    g = bf(rng.integers(-3, 4, (T, N)).astype(np.float32))
    gq = fp8.quantize_fp8(g, 0.25)
    dense = oracle.bits_to_f32(oracle.vnm_decompress(fp8.codes_as_bf16_bits(codes), meta, cix)).astype(np.float64)
    gd = fp8.e4m3_decode(gq).astype(np.float64)
    for fmaj in (0, 1):
        got = oracle.bits_to_f32(fp8.vnm_wgrad_fp8(codes, meta, cix, 0.5, gq, 0.25, fmaj))
        for f in range(F):
            for n in range(N):
                want = sum(Fraction(dense[t, f]) * Fraction(gd[t, n]) for t in range(T)) * Fraction(0.5) * Fraction(0.25)
                assert Fraction(float(got[f, n] if fmaj else got[n, f])) == want          # small integers: the bf16 rounding is exact
    # all values representable (integers / scale = integers <= 16): the fp8 contraction is the bf16 contraction
    vals, meta_b, cix_b = oracle.sqrelu_vnm_compress(y1)
    assert np.array_equal(fp8.vnm_wgrad_fp8(codes, meta, cix, 0.5, gq, 0.25, 1), oracle.vnm_wgrad(vals, meta_b, cix_b, g, 1))
    inp = _step_inputs(64, 32, 64, seed=9)
    ref = oracle.ffn_sparse_step_ref(inp["X"], inp["W1"], inp["W2"], inp["b1"], inp["dY"])
    sc = _scales_for(inp, ref)
    a = oracle.ffn_sparse_step_fp8_ref(inp["X"], inp["W1"], inp["W2"], inp["b1"], inp["dY"], sc)
    b = oracle.ffn_sparse_step_fp8_ref(inp["X"], inp["W1"], inp["W2"], inp["b1"], inp["dY"], sc, wgrad_fp8=True)
    for k in a:                                   # the flag changes the weight gradients and nothing else
        if k != "amax":
            assert np.array_equal(a[k], b[k]) == (k not in ("dW1", "dW2")), k
    assert a["amax"] == b["amax"] and a["amax"]["x"] == np.float32(np.abs(oracle.bits_to_f32(inp["X"])).max()) \
        and a["amax"]["y2"] == np.float32(oracle.bits_to_f32(a["y2_vals"]).max()) and a["amax"]["dy1"] == np.float32(np.abs(oracle.bits_to_f32(a["dy1_vals"])).max())
    assert np.array_equal(b["dW2"], fp8.vnm_wgrad_fp8(b["y2_codes"], b["y2_meta"], b["colidx"], sc["y2"], b["dyq"], sc["dy"], 0))
    assert np.array_equal(b["dW1"], fp8.vnm_wgrad_fp8(b["dy1_codes"], b["y2_meta"], b["colidx"], sc["dy1"], b["xq"], sc["x"], 1))
