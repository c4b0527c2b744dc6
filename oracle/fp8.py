"""fp8 operands for the sparsified FFN step (CPU oracle, test infrastructure only).

Paper: Section 3.4, closing paragraph: fp8 quantisation is orthogonal to 2:4 / V:N:M sparsity and can be fused with
the sparsification pass (an element-wise scan); Section 1: the 2:4 hardware covers bf16 and fp8 operands.  The paper
gives that one statement and no recipe, so everything below is a stated reading:

  * Format: OCP 8-bit float E4M3 (finite-only variant: bias 7, 3 mantissa bits, subnormals, largest finite 448, no
    infinities, S.1111.111 = NaN) - the fp8 type of the target's matrix instructions.  Codes are uint8.
  * Scale: one float32 scale per tensor, GIVEN by the caller (delayed scaling: taken from an earlier step's amax);
    real value ~ decode(code) * scale.  Quantisation of a real x: m = float32(x) * inv, inv = float32(1) / scale, one
    float32 rounding; clamped to [-448, 448] (saturating); then ONE round-to-nearest-even to E4M3.
  * What is quantised: the survivors of the 2:4 weight pruning (in the same pass), the survivors of the V:N:M
    activation compressor (in the same pass), and the dense operand of eqs. (1), (3), (4), (7) (a plain scan).
    SELECTION COMES FIRST and looks at the bf16 magnitudes only, so positions, metadata and column indices are
    bit-identical to the bf16 path; only the stored values change.  A soft-thresholded survivor a -/+ t goes from its
    float32 value straight to fp8 (no bf16 rounding in between: that is what fusing the two passes means).
  * Contractions: out = bf16( (sum_k decode(qa) * decode(qb)) * (scale_a * scale_b) + bias ), the sum exact here
    (float64); scale_a * scale_b is ONE float32 product.  The weight gradients (contraction over tokens) stay bf16.
"""
import numpy as np
from .bf16 import bits_to_f32, f64_to_bits
from .sparse24 import prune24_positions, prune24_decompress, HARD, SOFT
from .vnm import sqrelu, vnm_select_columns, vnm_decompress, _gather, sqrelu_vnm_compress, dsqrelu_vnm
from .gemm import vnm_wgrad

E4M3_MAX = 448.0


def e4m3_decode(codes):
    """uint8 codes -> float32 values (exact).  Written from the format's definition: sign, 4 exponent bits (bias 7),
    3 mantissa bits; exponent 0 = subnormal m * 2^-9; S.1111.111 = NaN."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int32)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e, m = (c >> 3) & 0xF, c & 7
    mag = np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    out = (sign * mag).astype(np.float32)
    return np.where((e == 15) & (m == 7), np.float32(np.nan), out)


def e4m3_encode(x):
    """float32 -> uint8 codes: saturate to +-448, then one round-to-nearest-even (ties to the even mantissa).  Finite
    inputs only (the callers' inputs are finite by contract); -0 keeps its sign."""
    f = np.clip(np.asarray(x, dtype=np.float32), np.float32(-E4M3_MAX), np.float32(E4M3_MAX))
    a = np.abs(f).astype(np.float64)
    # spacing of the target grid at |x|: 2^(e-3) for |x| in [2^e, 2^(e+1)), e clamped to [-6, 8]; 2^-9 below 2^-6
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    e = np.clip(e, -6, 8)
    q = np.exp2(e - 3)
    n = np.rint(a / q)                                   # numpy rounds halves to even; a / q is exact (power of two)
    r = n * q                                            # may carry to the next binade (n = 16): still on the grid
    # back to the code: r = (1 + m/8) 2^(E-7) or m 2^-9
    with np.errstate(divide="ignore"):
        e2 = np.floor(np.log2(np.where(r > 0, r, 1.0)))
    sub = r < 2.0 ** -6
    E = np.where(sub, 0, e2 + 7).astype(np.int32)
    m = np.where(sub, np.rint(r * 2.0 ** 9), np.rint((r / np.exp2(e2) - 1.0) * 8.0)).astype(np.int32)
    code = (E << 3) | m
    sign = np.signbit(f).astype(np.int32) << 7
    return (code | sign).astype(np.uint8)


def inv_scale(scale):
    """float32(1) / float32(scale): the factor applied before rounding (one float32 division)."""
    return np.float32(1.0) / np.float32(scale)


def quantize_f32(x32, scale):
    """Real values given as float32 -> codes: one float32 product with 1 / scale, saturate, RNE to E4M3."""
    with np.errstate(over="ignore"):
        m = (np.asarray(x32, dtype=np.float32) * inv_scale(scale)).astype(np.float32)
    return e4m3_encode(m)


def quantize_fp8(x_bits, scale):
    """bf16 bit patterns -> fp8 codes of the same shape (the dense operand of eqs. (1), (3), (4), (7))."""
    return quantize_f32(bits_to_f32(x_bits), scale)


def amax(x_bits):
    """Largest magnitude of a bf16 tensor as float32 (what a delayed-scaling recipe records for the next step)."""
    return np.float32(np.max(bits_to_f32(np.asarray(x_bits, dtype=np.uint16) & np.uint16(0x7FFF)), initial=0.0))


def prune24_compress_fp8(bits, scale, mode=HARD):
    """Section 2.2 + quantisation in one pass: logical S[R, K] (bf16 bits) -> (codes uint8 [R, K/2], meta uint8 [R, K/8]).
    Positions and metadata are those of sparse24.prune24_compress; a survivor's value (in SOFT mode the float32
    a -/+ t) is quantised with `scale`."""
    bits = np.asarray(bits, dtype=np.uint16)
    R, K = bits.shape
    assert K % 8 == 0
    G = K // 4
    grp = bits.reshape(R, G, 4)
    kept, third = prune24_positions(bits)
    vals = np.take_along_axis(grp, kept, axis=-1)
    a = bits_to_f32(vals)
    if mode == SOFT:
        t = bits_to_f32(np.take_along_axis(grp, third[..., None], axis=-1) & np.uint16(0x7FFF))
        neg = (vals & np.uint16(0x8000)) != 0
        with np.errstate(invalid="ignore", over="ignore"):
            a = np.where(neg, a + t, a - t).astype(np.float32)
    elif mode != HARD:
        raise ValueError("mode")
    nib = (kept[..., 0] | (kept[..., 1] << 2)).astype(np.uint8)
    meta = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    return quantize_f32(a, scale).reshape(R, K // 2), meta


def codes_as_bf16_bits(codes):
    """decode(codes) as bf16 bit patterns (exact: an E4M3 value has 4 significant bits and an exponent inside bf16's
    range), so that the bf16 decompressors can place them."""
    f = e4m3_decode(codes)
    return (np.ascontiguousarray(f).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def sqrelu_vnm_compress_fp8(y1_bits, scale, V=64, M=8):
    """Alg. 1 lines 5-6 with fp8 values: y2 = bf16(max(y1, 0)^2) exactly as in the bf16 path (the column scores, the
    column choice and the per-row 2:4 choice all look at the bf16 y2), then the two survivors of every block are
    quantised with `scale`.  -> (codes uint8 [T, 2F/M], meta [T, F/(2M)], colidx [T/V, F/M, 4])."""
    y2 = sqrelu(y1_bits)
    colidx, _ = vnm_select_columns(y2, V, M)
    kept4 = _gather(y2, colidx, V, M)
    T, K4 = kept4.shape
    kept, _ = prune24_positions(kept4)
    vals = np.take_along_axis(kept4.reshape(T, K4 // 4, 4), kept, axis=-1)
    nib = (kept[..., 0] | (kept[..., 1] << 2)).astype(np.uint8)
    meta = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    return quantize_fp8(vals, scale).reshape(T, K4 // 2), meta, colidx


def _finish(acc, scale_a, scale_b, bias):
    s = np.float32(scale_a) * np.float32(scale_b)                        # ONE float32 product
    acc = acc * np.float64(s)
    if bias is not None:
        acc = acc + np.asarray(bias, dtype=np.float32).astype(np.float64)[None, :]
    return f64_to_bits(acc)


def spmm24_fp8(xq, scale_x, w_codes, w_meta, scale_w, bias=None):
    """eq. (1) / eq. (4) on fp8 operands: out[t, n] = bf16( (sum_k dec(xq[t, k]) dec(Ws[n, k])) scale_x scale_w + bias[n] ),
    Ws packed 2:4 fp8 ([N, K/2] codes, [N, K/8] metadata).  The sum is exact (float64 on exactly decoded values)."""
    w = prune24_decompress(codes_as_bf16_bits(w_codes), w_meta)
    acc = e4m3_decode(xq).astype(np.float64) @ bits_to_f32(w).astype(np.float64).T
    return _finish(acc, scale_x, scale_w, bias)


def vnm_spmm_fp8(a_codes, a_meta, a_colidx, scale_a, wq, scale_w, w_kmajor, V=64, M=8):
    """eq. (3) / eq. (7) on fp8 operands: out[t, n] = bf16( (sum_f dec(Av[t, f]) dec(W(n, f))) scale_a scale_w ); the
    V:N:M activation carries fp8 codes, W (codes) is stored [N, F] (w_kmajor = 0) or [F, N] (1)."""
    a = vnm_decompress(codes_as_bf16_bits(a_codes), a_meta, a_colidx, V, M)
    w = e4m3_decode(wq).astype(np.float64)
    if w_kmajor:
        w = w.T
    return _finish(bits_to_f32(a).astype(np.float64) @ w.T, scale_a, scale_w, None)


def vnm_wgrad_fp8(a_codes, a_meta, a_colidx, scale_a, gq, scale_g, out_f_major, V=64, M=8):
    """eq. (5) / eq. (8) on fp8 operands: out[f, n] (out_f_major = 1) or out[n, f] (0) = bf16( (sum_t dec(Av[t, f]) dec(G[t, n])) scale_a scale_g ),
    Av = the V:N:M code matrix, gq = codes of G [T, N].  The sum is exact (float64 on exactly decoded values)."""
    a = bits_to_f32(vnm_decompress(codes_as_bf16_bits(a_codes), a_meta, a_colidx, V, M)).astype(np.float64)       # [T, F]
    acc = a.T @ e4m3_decode(gq).astype(np.float64)                                                                # [F, N]
    if not out_f_major:
        acc = acc.T
    return f64_to_bits(acc * np.float64(np.float32(scale_a) * np.float32(scale_g)))


def ffn_sparse_step_fp8_ref(X, W1, W2, b1, dY, scales, mode=HARD, V=64, M=8, wgrad_fp8=False):
    """Alg. 1 + Alg. 2 with fp8 operands in the four contractions whose sparse operand is 2:4 along the contraction
    (eqs. (1), (3), (4), (7)); a stated reading built from the functions above, in the paper's order.

    scales: dict of six per-tensor float32 scales given by the caller (delayed scaling):
      x, w1, w2, y2, dy, dy1.  Both uses of a weight share its scale (W1: pruned in eq. (1), dense in eq. (7); W2: dense
      in eq. (3), pruned transposed in eq. (4)).
    Everything that decides a position stays bf16: y1 is the bf16 output of eq. (1), y2 = bf16(max(y1, 0)^2) picks the
    columns and the per-row survivors, eq. (6) is evaluated in bf16 arithmetic on the bf16 dy2 and y1 exactly as in the
    bf16 step, and only then are the survivors quantised for the next contraction.  The weight gradients (eqs. (5), (8),
    contraction over tokens) stay bf16 on the bf16 survivors and the bf16 dY / X, unless wgrad_fp8: then they contract the
    codes that eqs. (3) / (7) and eqs. (4) / (1) already use (y2 and dY for eq. (5), dy1 and X for eq. (8)), with those tensors' scales."""
    s = {k: np.float32(v) for k, v in scales.items()}
    xq = quantize_fp8(X, s["x"])
    w1_codes, w1_meta = prune24_compress_fp8(W1, s["w1"], mode)
    y1 = spmm24_fp8(xq, s["x"], w1_codes, w1_meta, s["w1"], b1)                       # Alg. 1 line 4
    y2_codes, y2_meta, colidx = sqrelu_vnm_compress_fp8(y1, s["y2"], V, M)           # Alg. 1 lines 5-6
    y2_vals, meta_b, colidx_b = sqrelu_vnm_compress(y1, V, M)                         # the bf16 survivors (weight gradients)
    assert np.array_equal(meta_b, y2_meta) and np.array_equal(colidx_b, colidx)
    w2q = quantize_fp8(W2, s["w2"])
    y3 = vnm_spmm_fp8(y2_codes, y2_meta, colidx, s["y2"], w2q, s["w2"], 0, V, M)      # Alg. 1 line 7
    dyq = quantize_fp8(dY, s["dy"])
    w2t_codes, w2t_meta = prune24_compress_fp8(np.ascontiguousarray(np.asarray(W2).T), s["w2"], mode)
    dy2 = spmm24_fp8(dyq, s["dy"], w2t_codes, w2t_meta, s["w2"], None)                # Alg. 2 line 2
    dW2 = vnm_wgrad(y2_vals, y2_meta, colidx, dY, 0, V, M)                            # Alg. 2 line 3 (bf16)
    dy1_vals = dsqrelu_vnm(dy2, y1, y2_meta, colidx, V, M)                            # Alg. 2 line 4 (bf16 arithmetic)
    dy1_codes = quantize_fp8(dy1_vals, s["dy1"])
    w1q = quantize_fp8(W1, s["w1"])
    dX = vnm_spmm_fp8(dy1_codes, y2_meta, colidx, s["dy1"], w1q, s["w1"], 1, V, M)    # Alg. 2 line 5
    dW1 = vnm_wgrad(dy1_vals, y2_meta, colidx, X, 1, V, M)                            # Alg. 2 line 6 (bf16)
    if wgrad_fp8:
        dW2 = vnm_wgrad_fp8(y2_codes, y2_meta, colidx, s["y2"], dyq, s["dy"], 0, V, M)
        dW1 = vnm_wgrad_fp8(dy1_codes, y2_meta, colidx, s["dy1"], xq, s["x"], 1, V, M)
    amax_of = dict(x=amax(X), w1=amax(W1), w2=amax(W2), y2=amax(y2_vals), dy=amax(dY), dy1=amax(dy1_vals))     # what the next step's scales come from
    return dict(amax=amax_of, xq=xq, w1_codes=w1_codes, w1_meta=w1_meta, y1=y1, y2_codes=y2_codes, y2_vals=y2_vals, y2_meta=y2_meta, colidx=colidx,
                w2q=w2q, y3=y3, dyq=dyq, w2t_codes=w2t_codes, w2t_meta=w2t_meta, dy2=dy2, dW2=dW2, dy1_vals=dy1_vals,
                dy1_codes=dy1_codes, w1q=w1q, dX=dX, dW1=dW1)


def ffn_sparse_step_fp8_grouped_ref(X, W1, W2, b1, dY, seg_offsets, scales, mode=HARD, V=64, M=8, wgrad_fp8=False):
    """Mixture-of-experts form of the fp8 step (Section 1: the method applies to MoE FFNs, each expert being one FFN of Alg. 1 /
    Alg. 2): expert e owns rows seg_offsets[e]..seg_offsets[e+1] of X and dY and its own W1[e], W2[e], b1[e]; the six scales are
    shared by all experts.  Returns one ffn_sparse_step_fp8_ref result per expert (None for an expert without rows; its weight
    gradients are zero by the empty sum)."""
    res = []
    for e in range(len(seg_offsets) - 1):
        a, b = int(seg_offsets[e]), int(seg_offsets[e + 1])
        if b == a:
            res.append(None)
            continue
        res.append(ffn_sparse_step_fp8_ref(X[a:b], W1[e], W2[e], None if b1 is None else b1[e], dY[a:b], scales, mode, V, M, wgrad_fp8))
    return res
