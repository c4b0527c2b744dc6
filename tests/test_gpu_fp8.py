"""GPU parity of the fp8 entry points (paper Section 3.4, closing paragraph) against oracle/fp8.py on identical seeded inputs:
codes, metadata and column indices bit-exact; contractions within the GEMM tolerance of the oracle's exact sum over the same codes."""
import numpy as np
import pytest
import torch

import oracle
from oracle import fp8
import paper_2602_06183_amd as sffn
from tests.util import to_dev, to_bits, assert_gemm_close, gemm_errors
from workload import bf16_bits_from_f32, make_ffn_inputs

pytestmark = pytest.mark.gpu


def rnd_bits(rng, shape, scale=1.0):
    return bf16_bits_from_f32(rng.standard_normal(shape, dtype=np.float32) * np.float32(scale))


def u8(t):
    return t.detach().cpu().numpy()


def test_quantize_fp8_every_bf16_pattern_and_scales():
    """All 65536 bf16 bit patterns that are finite, at several scales (powers of two and not), saturation included."""
    allbits = np.arange(65536, dtype=np.uint16)
    finite = (allbits & 0x7F80) != 0x7F80
    x = np.ascontiguousarray(allbits[finite][: (finite.sum() // 8) * 8])
    for scale in (1.0, 0.02 * 4 / 448, 7.0, 2.0 ** -12, 3.1e-3, 1000.0):
        got, amax = sffn.quantize_fp8(to_dev(x), scale, want_amax=True)
        assert np.array_equal(u8(got), fp8.quantize_fp8(x, scale)), scale
        assert float(amax.cpu()[0]) == float(fp8.amax(x))


@pytest.mark.parametrize("mode", [sffn.MODE_HARD, sffn.MODE_SOFT])
@pytest.mark.parametrize("R,K,trans", [(64, 64, 0), (192, 320, 0), (448, 2048, 0), (64, 64, 1), (192, 320, 1), (1024, 256, 1)])
def test_prune24_compress_fp8(R, K, trans, mode):
    from tests.test_gpu_kernels import adversarial_rows
    rng = np.random.default_rng(R + 3 * K + trans)
    S = rnd_bits(rng, (R, K), 0.02)
    adv = adversarial_rows(K)
    S[: adv.shape[0]] = adv
    S[20, :8] = bf16_bits_from_f32(np.array([1.0703125, 2.0, 0.0068359375, 0.001, 30.0, -30.0, 29.0, 1.0], dtype=np.float32))
    scale = 0.05 / 448
    stored = np.ascontiguousarray(S.T) if trans else S
    codes, meta, amax = sffn.prune24_compress_fp8(to_dev(stored), scale, bool(trans), mode, want_amax=True)
    rc, rm = fp8.prune24_compress_fp8(S, scale, mode)
    assert np.array_equal(u8(meta), rm)
    assert np.array_equal(u8(codes), rc)
    _, rm16 = oracle.prune24_compress(S, mode)
    assert np.array_equal(u8(meta), rm16)                          # same selection as the bf16 path
    if mode == sffn.MODE_HARD:
        rv, _ = oracle.prune24_compress(S, mode)
        finite = rv[(rv & 0x7F80) != 0x7F80]
        assert float(amax.cpu()[0]) == float(fp8.amax(finite))


@pytest.mark.parametrize("M", [8, 16, 32, 64])
@pytest.mark.parametrize("T,F", [(64, 256), (192, 1152)])
def test_sqrelu_vnm_compress_fp8(T, F, M):
    rng = np.random.default_rng(T + F + M)
    y1 = bf16_bits_from_f32(rng.standard_normal((T, F), dtype=np.float32) - np.float32(0.8))
    y1[:64, 0:M] = 0xBF80
    y1[:64, M:2 * M] = 0x3F80
    y1[:64, 2 * M:2 * M + 4] = 0x4580                              # 4096^2 = 2^24: saturates the fp8 range at this scale
    scale = 12.0 / 448
    codes, meta, colidx = sffn.sqrelu_vnm_compress_fp8(to_dev(y1), scale, 64, M)
    rc, rm, ri = fp8.sqrelu_vnm_compress_fp8(y1, scale, 64, M)
    assert np.array_equal(u8(colidx), ri) and np.array_equal(u8(meta), rm)
    assert np.array_equal(u8(codes), rc)
    _, m16, c16 = oracle.sqrelu_vnm_compress(y1, 64, M)
    assert np.array_equal(u8(meta), m16) and np.array_equal(u8(colidx), c16)


@pytest.mark.parametrize("T,N,K", [(64, 64, 128), (192, 320, 384), (512, 1024, 256), (384, 256, 2048)])
def test_spmm24_fp8(T, N, K):
    rng = np.random.default_rng(T + 3 * N + 7 * K)
    X = rnd_bits(rng, (T, K))
    W = rnd_bits(rng, (N, K), 0.02)
    bias = rng.standard_normal(N).astype(np.float32)
    sx, sw = 4.0 / 448, 0.08 / 448
    xq = fp8.quantize_fp8(X, sx)
    wc, wm = fp8.prune24_compress_fp8(W, sw, oracle.sparse24.SOFT)
    dxq, dwc, dwm = torch.from_numpy(xq).cuda(), torch.from_numpy(wc).cuda(), torch.from_numpy(wm).cuda()
    assert_gemm_close(to_bits(sffn.spmm24_fp8(dxq, sx, dwc, dwm, sw, to_dev(bias))), fp8.spmm24_fp8(xq, sx, wc, wm, sw, bias), "fp8 fwd+bias")
    assert_gemm_close(to_bits(sffn.spmm24_fp8(dxq, sx, dwc, dwm, sw, None)), fp8.spmm24_fp8(xq, sx, wc, wm, sw, None), "fp8 fwd")
    # how far the quantised contraction is from the bf16 one on the same inputs (reported; 3 mantissa bits per factor)
    v16, m16 = oracle.prune24_compress(W, oracle.sparse24.SOFT)
    fro, _ = gemm_errors(fp8.spmm24_fp8(xq, sx, wc, wm, sw, None), oracle.spmm24(X, v16, m16, None))
    print("fp8 vs bf16 contraction, relative Frobenius distance: %.4f" % fro)
    assert fro < 0.08


def test_spmm24_fp8_exact_on_small_integers():
    """Small integers are exact in E4M3 (scale 1) and their products and sums exact in fp32: the fp8 matrix cores must then
    reproduce the bf16 oracle bit for bit, which pins the operand / metadata layout of the fp8 instruction."""
    rng = np.random.default_rng(7)
    T, N, K = 128, 192, 256
    X = bf16_bits_from_f32(rng.integers(-3, 4, (T, K)).astype(np.float32))
    W = bf16_bits_from_f32(rng.integers(-3, 4, (N, K)).astype(np.float32))
    wc, wm = sffn.prune24_compress_fp8(to_dev(W), 1.0)
    got = to_bits(sffn.spmm24_fp8(sffn.quantize_fp8(to_dev(X), 1.0), 1.0, wc, wm, 1.0))
    v16, m16 = oracle.prune24_compress(W)
    assert np.array_equal(oracle.bits_to_f32(got), oracle.bits_to_f32(oracle.spmm24(X, v16, m16, None)))
    y1 = bf16_bits_from_f32(rng.integers(-2, 4, (T, K)).astype(np.float32))
    for M in (8, 32):
        ac, am, ai = sffn.sqrelu_vnm_compress_fp8(to_dev(y1), 1.0, 64, M)
        av, _, _ = oracle.sqrelu_vnm_compress(y1, 64, M)
        Wd = bf16_bits_from_f32(rng.integers(-3, 4, (N, K)).astype(np.float32))
        for kmaj, w in ((0, Wd), (1, np.ascontiguousarray(Wd.T))):
            got = to_bits(sffn.vnm_spmm_fp8(ac, am, ai, 1.0, sffn.quantize_fp8(to_dev(w), 1.0), 1.0, kmaj, 64, M))
            assert np.array_equal(oracle.bits_to_f32(got), oracle.bits_to_f32(oracle.vnm_spmm(av, u8(am), u8(ai), w, kmaj, 64, M)))


@pytest.mark.parametrize("M", [8, 16, 32, 64])
@pytest.mark.parametrize("T,F,D", [(64, 128, 64), (192, 384, 320), (256, 2048, 192), (576, 4096, 320)])
def test_vnm_spmm_fp8(T, F, D, M):
    rng = np.random.default_rng(T + 3 * F + 7 * D + M)
    y1 = bf16_bits_from_f32(rng.standard_normal((T, F), dtype=np.float32) - np.float32(0.8))
    W2 = rnd_bits(rng, (D, F), 0.02)
    W1 = rnd_bits(rng, (F, D), 0.02)
    sa, sw = 12.0 / 448, 0.08 / 448
    ac, am, ai = fp8.sqrelu_vnm_compress_fp8(y1, sa, 64, M)
    dac, dam, dai = (torch.from_numpy(a).cuda() for a in (ac, am, ai))
    for kmaj, w in ((0, W2), (1, W1)):
        wq = fp8.quantize_fp8(w, sw)
        got = sffn.vnm_spmm_fp8(dac, dam, dai, sa, torch.from_numpy(wq).cuda(), sw, kmaj, 64, M)
        assert_gemm_close(to_bits(got), fp8.vnm_spmm_fp8(ac, am, ai, sa, wq, sw, kmaj, 64, M), "fp8 vnm_spmm kmajor=%d" % kmaj)


def test_fp8_forward_chain_at_the_1b_shape():
    """eq. (1) -> eq. (2) + V:N:M -> eq. (3) with fp8 operands at the 1B layer shape, scales from the tensors' own amax (as a
    delayed-scaling recipe would carry them over), teacher-forced on sampled rows / token blocks."""
    T, D, F = 8192, 2048, 8192
    inp = make_ffn_inputs(T, D, F, seed=0)
    dev = {k: to_dev(v) for k, v in inp.items()}
    sx = float(fp8.amax(inp["X"])) / 448
    sw1 = float(fp8.amax(inp["W1"])) / 448
    sw2 = float(fp8.amax(inp["W2"])) / 448
    xq = sffn.quantize_fp8(dev["X"], sx)
    wc, wm = sffn.prune24_compress_fp8(dev["W1"], sw1)
    y1 = sffn.spmm24_fp8(xq, sx, wc, wm, sw1, dev["b1"])
    sy = 16.0 / 448
    ac, am, ai, amax = sffn.sqrelu_vnm_compress_fp8(y1, sy, 64, 8, want_amax=True)
    w2q = sffn.quantize_fp8(dev["W2"], sw2)
    y3 = sffn.vnm_spmm_fp8(ac, am, ai, sy, w2q, sw2, 0)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    rows = np.sort(rng.choice(T, 32, replace=False))
    rc, rm = fp8.prune24_compress_fp8(inp["W1"], sw1)
    assert np.array_equal(u8(wc), rc) and np.array_equal(u8(wm), rm)
    xq_ref = fp8.quantize_fp8(inp["X"][rows], sx)
    assert np.array_equal(u8(xq)[rows], xq_ref)
    y1b = to_bits(y1)
    assert_gemm_close(y1b[rows], fp8.spmm24_fp8(xq_ref, sx, rc, rm, sw1, inp["b1"]), "fp8 y1 rows")
    for tb in (0, 57, 127):
        r = slice(64 * tb, 64 * tb + 64)
        oc, om, oi = fp8.sqrelu_vnm_compress_fp8(y1b[r], sy)
        assert np.array_equal(u8(ai)[tb:tb + 1], oi) and np.array_equal(u8(am)[r], om) and np.array_equal(u8(ac)[r], oc)
        w2q_ref = fp8.quantize_fp8(inp["W2"], sw2)
        assert_gemm_close(to_bits(y3)[r], fp8.vnm_spmm_fp8(oc, om, oi, sy, w2q_ref, sw2, 0), "fp8 y3 block")
    assert 0 < float(amax.cpu()[0]) < 1e4


# ---- the whole step with fp8 operands (ffn_sparse_step_fp8) --------------------------------------------------------------------
def _fp8_step_scales(inp):
    """Delayed-scaling stand-in: amax / 448 of each quantised tensor, taken from the oracle's bf16 step on the same inputs."""
    ref = oracle.ffn_sparse_step_ref(inp["X"], inp["W1"], inp["W2"], inp["b1"], inp["dY"])
    amax = lambda b: float(np.max(np.abs(oracle.bits_to_f32(b))))
    return dict(x=amax(inp["X"]) / 448, w1=amax(inp["W1"]) / 448, w2=amax(inp["W2"]) / 448, y2=max(amax(oracle.sqrelu(ref["y1"])), 1e-6) / 448,
                dy=amax(inp["dY"]) / 448, dy1=max(amax(ref["dy1_vals"]), 1e-6) / 448)


def _check_fp8_step_against_oracle(inp, sc, s, outs, mode, wgrad_fp8=False, M=8):
    """Teacher-forced: every oracle stage consumes the GPU's output of the stage before it.  Returns dy1's survivors (bf16 bits)."""
    f8 = oracle.fp8
    T, F = s["y1"].shape
    c1, m1 = f8.prune24_compress_fp8(inp["W1"], sc["w1"], mode)
    assert np.array_equal(s["w1_meta"], m1) and np.array_equal(s["w1_codes"], c1)
    xq = f8.quantize_fp8(inp["X"], sc["x"])
    assert_gemm_close(s["y1"], f8.spmm24_fp8(xq, sc["x"], c1, m1, sc["w1"], inp["b1"]), "y1")
    yc, ym, cix = f8.sqrelu_vnm_compress_fp8(s["y1"], sc["y2"], 64, M)
    assert np.array_equal(s["colidx"], cix) and np.array_equal(s["y2_meta"], ym) and np.array_equal(s["y2_codes"], yc)
    yv, ym_b, cix_b = oracle.sqrelu_vnm_compress(s["y1"], 64, M)          # the bf16 survivors (weight gradients, y1_kept)
    assert np.array_equal(ym_b, ym) and np.array_equal(cix_b, cix)
    if M == 8:
        ones = np.arange(1, yv.size + 1, dtype=np.uint32).reshape(yv.shape)
        slot_of = oracle.vnm_decompress((ones & 0xFFFF).astype(np.uint16), ym, cix).astype(np.int64) \
            + (oracle.vnm_decompress((ones >> 16).astype(np.uint16), ym, cix).astype(np.int64) << 16)
        want_kept = np.zeros(yv.size, dtype=np.uint16)
        tt, ff = np.nonzero(slot_of)
        want_kept[slot_of[tt, ff] - 1] = s["y1"][tt, ff]
        want_kept = want_kept.reshape(T // 64, 64, F // 64, 8, 2).transpose(0, 2, 1, 3, 4)
        assert np.array_equal(s["y1_kept"].reshape(-1), want_kept.reshape(-1))
    assert_gemm_close(outs["Y3"], f8.vnm_spmm_fp8(yc, ym, cix, sc["y2"], f8.quantize_fp8(inp["W2"], sc["w2"]), sc["w2"], 0, 64, M), "y3")
    c2, m2 = f8.prune24_compress_fp8(np.ascontiguousarray(inp["W2"].T), sc["w2"], mode)
    assert np.array_equal(s["w2t_meta"], m2) and np.array_equal(s["w2t_codes"], c2)
    assert_gemm_close(s["dy2"], f8.spmm24_fp8(f8.quantize_fp8(inp["dY"], sc["dy"]), sc["dy"], c2, m2, sc["w2"], None), "dy2")
    dv = oracle.dsqrelu_vnm(s["dy2"], s["y1"], ym, cix, 64, M)
    dq = f8.quantize_fp8(dv, sc["dy1"])
    if M == 8:
        assert np.array_equal(s["dy1_vals"], dv)
    else:           # wide blocks: dy1's survivors leave as codes only (y1 at the kept slots is checked through them)
        assert np.array_equal(s["dy1_codes"], dq)
    assert_gemm_close(outs["dX"], f8.vnm_spmm_fp8(dq, ym, cix, sc["dy1"], f8.quantize_fp8(inp["W1"], sc["w1"]), sc["w1"], 1, 64, M), "dX")
    if wgrad_fp8:
        assert_gemm_close(outs["dW2"], f8.vnm_wgrad_fp8(yc, ym, cix, sc["y2"], f8.quantize_fp8(inp["dY"], sc["dy"]), sc["dy"], 0, 64, M), "dW2")
        assert_gemm_close(outs["dW1"], f8.vnm_wgrad_fp8(dq, ym, cix, sc["dy1"], xq, sc["x"], 1, 64, M), "dW1")
    else:
        assert_gemm_close(outs["dW2"], oracle.vnm_wgrad(yv, ym, cix, inp["dY"], 0, 64, M), "dW2")
        assert_gemm_close(outs["dW1"], oracle.vnm_wgrad(dv, ym, cix, inp["X"], 1, 64, M), "dW1")
    return dv


@pytest.mark.parametrize("wgrad_fp8", [False, True])
@pytest.mark.parametrize("T,D,F,mode,seed", [(64, 128, 128, sffn.MODE_HARD, 0), (512, 256, 1024, sffn.MODE_HARD, 0), (512, 256, 1024, sffn.MODE_SOFT, 1),
                                             (192, 384, 640, sffn.MODE_SOFT, 2), (448, 256, 512, sffn.MODE_HARD, 3)])
def test_ffn_sparse_step_fp8(T, D, F, mode, seed, wgrad_fp8):
    """The fused fp8 step, teacher-forced stage by stage; then the timed configuration (no dense y1 / dy2) must give the same bits."""
    from workload import make_ffn_inputs
    inp = make_ffn_inputs(T, D, F, seed=seed)
    sc = _fp8_step_scales(inp)
    dev = {k: to_dev(v) for k, v in inp.items()}
    step = sffn.FfnStepFp8(T, D, F, sc, mode, keep_dense=True, wgrad_fp8=wgrad_fp8)
    outs = step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])
    torch.cuda.synchronize()
    s = {k: to_bits(v) if v.dtype == torch.bfloat16 else v.cpu().numpy() for k, v in step.saved().items()}
    o = {k: to_bits(v) for k, v in zip(("Y3", "dX", "dW1", "dW2"), outs)}
    _check_fp8_step_against_oracle(inp, sc, s, o, mode, wgrad_fp8)
    # the six maxima for the next step's scales: exact, whatever order the atomics arrive in
    yv = oracle.sqrelu_vnm_compress(s["y1"])[0]
    amax = lambda b: float(np.float32(np.abs(oracle.bits_to_f32(b)).max()))
    want = dict(x=amax(inp["X"]), w1=amax(inp["W1"]), w2=amax(inp["W2"]), y2=amax(yv), dy=amax(inp["dY"]), dy1=amax(s["dy1_vals"]))
    assert step.amax_dict() == want
    lean = sffn.FfnStepFp8(T, D, F, sc, mode, wgrad_fp8=wgrad_fp8, lean=True)           # no canonical copies: same outputs
    for k, v in zip(("Y3", "dX", "dW1", "dW2"), lean(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])):
        assert np.array_equal(to_bits(v), o[k]), ("lean", k)
    assert lean.amax_dict() == want
    fast = sffn.FfnStepFp8(T, D, F, sc, mode, wgrad_fp8=wgrad_fp8)
    outs2 = fast(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])
    torch.cuda.synchronize()
    for k, v in zip(("Y3", "dX", "dW1", "dW2"), outs2):
        assert np.array_equal(to_bits(v), o[k]), k
    assert fast.amax_dict() == want
    fast(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])            # a second call clears the maxima first
    assert fast.amax_dict() == want
    s2 = fast.saved()
    for k in ("y2_codes", "y2_meta", "colidx", "w1_codes", "w2t_codes"):
        assert np.array_equal(s2[k].cpu().numpy(), s[k]), k
    assert np.array_equal(to_bits(s2["dy1_vals"]), s["dy1_vals"]) and np.array_equal(to_bits(s2["y1_kept"]), s["y1_kept"])


@pytest.mark.parametrize("wgrad_fp8", [False, True])
@pytest.mark.parametrize("M,T,D,F,mode,seed", [(16, 192, 256, 512, sffn.MODE_HARD, 0), (32, 192, 256, 1024, sffn.MODE_SOFT, 1), (64, 256, 384, 2048, sffn.MODE_HARD, 2),
                                               (16, 512, 256, 1536, sffn.MODE_SOFT, 3), (64, 128, 128, 6144, sffn.MODE_HARD, 4)])
def test_ffn_sparse_step_fp8_wide_blocks(M, T, D, F, mode, seed, wgrad_fp8):
    """The fp8 step with V:2:M blocks of 16 / 32 / 64 columns (Table 5): general-M epilogues on codes, eqs. (3), (7) on the gathered rows of
    the quantised weights.  Teacher-forced stage by stage; then the timed configurations must give the same bits."""
    from workload import make_ffn_inputs
    inp = make_ffn_inputs(T, D, F, seed=seed)
    sc = _fp8_step_scales(inp)
    dev = {k: to_dev(v) for k, v in inp.items()}
    step = sffn.FfnStepFp8(T, D, F, sc, mode, keep_dense=True, wgrad_fp8=wgrad_fp8, M=M)
    outs = step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])
    torch.cuda.synchronize()
    s = {k: to_bits(v) if v.dtype == torch.bfloat16 else v.cpu().numpy() for k, v in step.saved().items()}
    o = {k: to_bits(v) for k, v in zip(("Y3", "dX", "dW1", "dW2"), outs)}
    dv = _check_fp8_step_against_oracle(inp, sc, s, o, mode, wgrad_fp8, M)
    density = np.mean(oracle.vnm_decompress(oracle.fp8.codes_as_bf16_bits(s["y2_codes"]), s["y2_meta"], s["colidx"], 64, M) != 0)
    assert density <= 2.0 / M + 1e-9                       # Table 5: sparsity at least 1 - N / M
    yv = oracle.sqrelu_vnm_compress(s["y1"], 64, M)[0]
    amax = lambda b: float(np.float32(np.abs(oracle.bits_to_f32(b)).max()))
    want = dict(x=amax(inp["X"]), w1=amax(inp["W1"]), w2=amax(inp["W2"]), y2=amax(yv), dy=amax(inp["dY"]), dy1=amax(dv))
    assert step.amax_dict() == want
    for kw in (dict(lean=True), dict()):
        other = sffn.FfnStepFp8(T, D, F, sc, mode, wgrad_fp8=wgrad_fp8, M=M, **kw)
        for k, v in zip(("Y3", "dX", "dW1", "dW2"), other(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])):
            assert np.array_equal(to_bits(v), o[k]), (kw, k)
        assert other.amax_dict() == want
        s2 = other.saved()
        for k in ("y2_codes", "y2_meta", "colidx", "dy1_codes"):
            assert np.array_equal(s2[k].cpu().numpy(), s[k]), (kw, k)


def test_grouped_fp8_step_wide_blocks_matches_oracle_per_expert():
    """The grouped fp8 step at M = 32 (uneven segments, one of them empty), every expert's share teacher-forced like the plain step."""
    from workload import make_moe_inputs
    D, F, M = 256, 1024, 32
    m = make_moe_inputs(n_tokens=600, n_experts=3, top_k=2, D=D, F=F, seed=6)
    seg = np.concatenate([m["seg"][:1], m["seg"][:1], m["seg"][1:]]).astype(np.int64)          # an empty segment in first place
    extra = make_ffn_inputs(64, D, F, seed=98)
    W1 = np.concatenate([extra["W1"][None], m["W1"]])
    W2 = np.concatenate([extra["W2"][None], m["W2"]])
    b1 = np.concatenate([extra["b1"][None], m["b1"]])
    mm = dict(X=m["X"], dY=m["dY"], W1=W1, W2=W2, b1=b1)
    amax = lambda b: float(np.float32(np.abs(oracle.bits_to_f32(b)).max()))
    sc = dict(x=amax(mm["X"]) / 448, w1=amax(W1) / 448, w2=amax(W2) / 448, y2=20.0 / 448, dy=amax(mm["dY"]) / 448, dy1=30.0 / 448)
    dev = {k: to_dev(v) for k, v in mm.items()}
    step = sffn.FfnStepFp8Grouped(seg, D, F, sc, sffn.MODE_HARD, keep_dense=True, wgrad_fp8=True, M=M)
    outs = step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])
    torch.cuda.synchronize()
    s = {k: (to_bits(v) if v.dtype == torch.bfloat16 else v.cpu().numpy()) for k, v in step.saved().items()}
    o = {k: to_bits(v) for k, v in zip(("Y3", "dX", "dW1", "dW2"), outs)}
    assert not o["dW1"][0].any() and not o["dW2"][0].any()
    y2max = dy1max = 0.0
    for e in (1, 2, 3):
        a, b = int(seg[e]), int(seg[e + 1])
        inp = dict(X=mm["X"][a:b], W1=W1[e], W2=W2[e], b1=b1[e], dY=mm["dY"][a:b])
        se = {k: s[k][e] for k in ("w1_codes", "w1_meta", "w2t_codes", "w2t_meta")}
        se.update({k: s[k][a:b] for k in ("y1", "y2_codes", "y2_meta", "dy2", "dy1_codes")})
        se["colidx"] = s["colidx"][a // 64:b // 64]
        oe = dict(Y3=o["Y3"][a:b], dX=o["dX"][a:b], dW1=o["dW1"][e], dW2=o["dW2"][e])
        dv = _check_fp8_step_against_oracle(inp, sc, se, oe, sffn.MODE_HARD, True, M)
        y2max = max(y2max, amax(oracle.sqrelu_vnm_compress(se["y1"], 64, M)[0]))
        dy1max = max(dy1max, amax(dv))
    got = step.amax_dict()
    assert got["x"] == amax(mm["X"]) and got["w1"] == amax(W1) and got["w2"] == amax(W2) and got["dy"] == amax(mm["dY"])
    assert got["y2"] == y2max and got["dy1"] == dy1max


def test_ffn_sparse_step_fp8_rejects_what_it_does_not_cover():
    from paper_2602_06183_amd import binding
    with pytest.raises(sffn.SffnError):
        sffn.FfnStepFp8(64, 64, 128, dict(x=1, w1=1, w2=1, y2=1, dy=1, dy1=1))               # D not a multiple of 128
    with pytest.raises(sffn.SffnError):
        sffn.FfnStepFp8(64, 128, 1280, dict(x=1, w1=1, w2=1, y2=1, dy=1, dy1=1), M=64)       # 4 F / M = 80 is not a multiple of 128
    step = sffn.FfnStepFp8(64, 128, 128, dict(x=1, w1=1, w2=1, y2=0.0, dy=1, dy1=1))
    z = lambda *shape: torch.zeros(shape, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sffn.SffnError):
        step(z(64, 128), z(128, 128), z(128, 128), None, z(64, 128))                          # a zero scale


def test_fp8_weight_gradient_kernel_exact_on_small_integers():
    """Pins the operand layout of the dense fp8 matrix instruction and the token-block ring: with integer activations and gradients every
    product and sum is exact, so eqs. (5), (8) on codes must equal the oracle bit for bit (scales are powers of two)."""
    rng = np.random.default_rng(2)
    T, D, F = 448, 128, 256
    ints = lambda shape, lo, hi: bf16_bits_from_f32(rng.integers(lo, hi, shape).astype(np.float32))
    inp = dict(X=ints((T, D), -2, 3), W1=ints((F, D), -2, 3), W2=ints((D, F), -2, 3), dY=ints((T, D), -2, 3), b1=np.full(F, -3.0, dtype=np.float32))
    sc = dict(x=2.0 ** -4, w1=2.0 ** -4, w2=2.0 ** -4, y2=8.0, dy=2.0 ** -4, dy1=64.0)
    dev = {k: to_dev(v) for k, v in inp.items()}
    step = sffn.FfnStepFp8(T, D, F, sc, keep_dense=True, wgrad_fp8=True)
    Y3, dX, dW1, dW2 = (to_bits(t) for t in step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"]))
    ref = oracle.ffn_sparse_step_fp8_ref(inp["X"], inp["W1"], inp["W2"], inp["b1"], inp["dY"], sc, wgrad_fp8=True)
    s = step.saved()
    assert np.array_equal(to_bits(s["y1"]), ref["y1"])                       # integer sums: eq. (1) is exact on both sides
    assert np.array_equal(s["y2_codes"].cpu().numpy(), ref["y2_codes"]) and np.array_equal(to_bits(s["dy1_vals"]), ref["dy1_vals"])
    f32 = oracle.bits_to_f32
    assert np.array_equal(f32(dW2), f32(ref["dW2"])) and np.array_equal(f32(dW1), f32(ref["dW1"]))
    assert np.count_nonzero(f32(dW2)) > 1000 and np.count_nonzero(f32(dW1)) > 1000


def test_fp8_step_delayed_scaling_round_trip():
    """The maxima one call leaves behind, turned into the next call's scales (amax / 448), put every tensor's largest code at the
    top of the E4M3 range without saturating anything else - the loop a delayed-scaling recipe runs."""
    T, D, F = 256, 256, 512
    inp = make_ffn_inputs(T, D, F, seed=4)
    dev = {k: to_dev(v) for k, v in inp.items()}
    step = sffn.FfnStepFp8(T, D, F, dict(x=1.0, w1=1.0, w2=1.0, y2=1.0, dy=1.0, dy1=1.0))      # first call: scales unknown
    step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])
    a = step.amax_dict()
    assert all(v > 0 for v in a.values())
    step.set_scales({k: v / 448.0 for k, v in a.items()})
    step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])
    s = step.saved()
    for name in ("w1_codes", "w2t_codes", "y2_codes"):
        top = np.abs(fp8.e4m3_decode(s[name].cpu().numpy())).max()
        assert 416.0 <= top <= 448.0, (name, top)              # the largest survivor lands in the top binade (exactly 448 when it is the tensor's maximum)
    assert np.abs(fp8.e4m3_decode(s["y2_codes"].cpu().numpy())).max() == 448.0


@pytest.mark.parametrize("M,wgrad_fp8,lean", [(8, False, False), (8, True, True), (16, True, False)])
def test_fp8_step_on_packed_weights_is_bit_identical(M, wgrad_fp8, lean):
    """SFFN_FLAG_WEIGHTS_PACKED for the fp8 step (Section 3.4: conversion once per optimizer step): the second micro-batch runs neither
    weight pass - the weights handed to it are garbage and go unread - and gives the bits of a full call; the weights' maxima come back 0."""
    T, D, F = 320, 256, 1024
    a, b = make_ffn_inputs(T, D, F, seed=31), make_ffn_inputs(T, D, F, seed=32)
    sc = dict(x=5.0 / 448, w1=0.1 / 448, w2=0.1 / 448, y2=8.0 / 448, dy=5.0 / 448, dy1=2.0 / 448)
    W1, W2, b1 = to_dev(a["W1"]), to_dev(a["W2"]), to_dev(a["b1"])
    step = sffn.FfnStepFp8(T, D, F, sc, sffn.MODE_SOFT, wgrad_fp8=wgrad_fp8, lean=lean, M=M)
    fresh = sffn.FfnStepFp8(T, D, F, sc, sffn.MODE_SOFT, wgrad_fp8=wgrad_fp8, lean=lean, M=M)
    step(to_dev(a["X"]), W1, W2, b1, to_dev(a["dY"]))
    junk = torch.full_like(W1, 7.0)
    got = [to_bits(t).copy() for t in step(to_dev(b["X"]), junk, junk.view(D, F), b1, to_dev(b["dY"]), weights_packed=True)]
    want = [to_bits(t).copy() for t in fresh(to_dev(b["X"]), W1, W2, b1, to_dev(b["dY"]))]
    for name, x, y in zip(("Y3", "dX", "dW1", "dW2"), got, want):
        assert np.array_equal(x, y), name
    ga, wa = step.amax_dict(), fresh.amax_dict()
    assert ga["w1"] == 0.0 and ga["w2"] == 0.0 and wa["w1"] > 0.0
    for k in ("x", "y2", "dy", "dy1"):
        assert ga[k] == wa[k], k


@pytest.mark.parametrize("M,wgrad_fp8", [(8, False), (8, True), (32, True)])
def test_fp8_forward_and_backward_as_separate_calls_are_bit_identical(M, wgrad_fp8):
    """ffn_sparse_forward_fp8 + ffn_sparse_backward_fp8 against the one-call fp8 step: outputs and the six maxima (the forward call owns
    x, w1, w2, y2, the backward call dy, dy1)."""
    T, D, F = 320, 256, 1024
    inp = make_ffn_inputs(T, D, F, seed=51)
    dev = {k: to_dev(v) for k, v in inp.items()}
    sc = dict(x=5.0 / 448, w1=0.1 / 448, w2=0.1 / 448, y2=8.0 / 448, dy=5.0 / 448, dy1=2.0 / 448)
    sz = sffn.buffer_sizes(T, D, F, sffn.MODE_HARD, M=M, fp8=True, wgrad_fp8=wgrad_fp8)
    scratch = torch.empty((sz["scratch"],), dtype=torch.uint8, device="cuda")           # a buffer that other layers would use in between
    split = sffn.FfnStepFp8(T, D, F, sc, sffn.MODE_HARD, wgrad_fp8=wgrad_fp8, M=M, scratch=scratch)
    whole = sffn.FfnStepFp8(T, D, F, sc, sffn.MODE_HARD, wgrad_fp8=wgrad_fp8, M=M)
    assert sz["scratch"] + sz["saved"] + sz["weights"] == whole.layout["total"]
    split.amax.fill_(-1.0)
    y3 = to_bits(split.forward(dev["X"], dev["W1"], dev["W2"], dev["b1"])).copy()
    scratch.fill_(0xA5)
    mid = split.amax_dict()
    assert mid["dy"] == -1.0 and mid["dy1"] == -1.0 and mid["x"] > 0 and mid["y2"] > 0       # the forward call leaves the backward pass's maxima alone
    want = [to_bits(t).copy() for t in whole(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])]
    got = [y3] + [to_bits(t).copy() for t in split.backward(dev["dY"])]
    for name, x, y in zip(("Y3", "dX", "dW1", "dW2"), got, want):
        assert np.array_equal(x, y), name
    assert split.amax_dict() == whole.amax_dict()


def test_fp8_grouped_forward_and_backward_as_separate_calls_are_bit_identical():
    from workload import make_moe_inputs
    D, F = 256, 384
    m = make_moe_inputs(n_tokens=700, n_experts=3, top_k=2, D=D, F=F, seed=6)
    dev = {k: to_dev(m[k]) for k in ("X", "W1", "W2", "b1", "dY")}
    sc = dict(x=5.0 / 448, w1=0.1 / 448, w2=0.1 / 448, y2=8.0 / 448, dy=5.0 / 448, dy1=2.0 / 448)
    sz = sffn.buffer_sizes(int(m["seg"][-1]), D, F, n_experts=3, fp8=True, wgrad_fp8=True)
    scratch = torch.empty((sz["scratch"],), dtype=torch.uint8, device="cuda")
    split, whole = sffn.FfnStepFp8Grouped(m["seg"], D, F, sc, wgrad_fp8=True, scratch=scratch), sffn.FfnStepFp8Grouped(m["seg"], D, F, sc, wgrad_fp8=True)
    assert sz["scratch"] + sz["saved"] + sz["weights"] == whole.layout["total"]
    y3 = to_bits(split.forward(dev["X"], dev["W1"], dev["W2"], dev["b1"])).copy()
    scratch.fill_(0x5A)
    want = [to_bits(t).copy() for t in whole(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])]
    got = [y3] + [to_bits(t).copy() for t in split.backward(dev["dY"])]
    for name, x, y in zip(("Y3", "dX", "dW1", "dW2"), got, want):
        assert np.array_equal(x, y), name
    assert split.amax_dict() == whole.amax_dict()


@pytest.mark.parametrize("M,wgrad_fp8", [(8, True), (8, False), (16, True)])
def test_fp8_step_weight_gradients_accumulate_in_float32(M, wgrad_fp8):
    from tests.test_gpu_kernels import _check_fp32_accumulation
    T, D, F = 320, 256, 1024
    inp = [make_ffn_inputs(T, D, F, seed=71 + i) for i in range(2)]
    sc = dict(x=5.0 / 448, w1=0.1 / 448, w2=0.1 / 448, y2=8.0 / 448, dy=5.0 / 448, dy1=2.0 / 448)
    W1, W2, b1 = to_dev(inp[0]["W1"]), to_dev(inp[0]["W2"]), to_dev(inp[0]["b1"])
    batches = [(to_dev(i["X"]), W1, W2, b1, to_dev(i["dY"])) for i in inp]
    _check_fp32_accumulation(lambda f32: sffn.FfnStepFp8(T, D, F, sc, sffn.MODE_HARD, wgrad_fp8=wgrad_fp8, M=M, dw_fp32=f32), batches)


@pytest.mark.parametrize("wgrad_fp8", [False, True])
def test_grouped_fp8_step_matches_oracle_per_expert(wgrad_fp8):
    """The mixture-of-experts form of the fp8 step (uneven segments, one of them empty): every expert's share is checked
    teacher-forced like the plain fp8 step, with the scales shared by all experts; the empty expert gets zero weight gradients."""
    from workload import make_moe_inputs
    D, F = 256, 384
    m = make_moe_inputs(n_tokens=700, n_experts=3, top_k=2, D=D, F=F, seed=5)
    seg = np.concatenate([m["seg"][:2], m["seg"][1:]]).astype(np.int64)          # an empty segment in second place
    extra = make_ffn_inputs(64, D, F, seed=99)
    W1 = np.concatenate([m["W1"][:1], extra["W1"][None], m["W1"][1:]])
    W2 = np.concatenate([m["W2"][:1], extra["W2"][None], m["W2"][1:]])
    b1 = np.concatenate([m["b1"][:1], extra["b1"][None], m["b1"][1:]])
    mm = dict(X=m["X"], dY=m["dY"], W1=W1, W2=W2, b1=b1)
    amax = lambda b: float(np.float32(np.abs(oracle.bits_to_f32(b)).max()))
    sc = dict(x=amax(mm["X"]) / 448, w1=amax(W1) / 448, w2=amax(W2) / 448, y2=20.0 / 448, dy=amax(mm["dY"]) / 448, dy1=30.0 / 448)
    dev = {k: to_dev(v) for k, v in mm.items()}
    step = sffn.FfnStepFp8Grouped(seg, D, F, sc, sffn.MODE_SOFT, keep_dense=True, wgrad_fp8=wgrad_fp8)
    outs = step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])
    torch.cuda.synchronize()
    s = {k: (to_bits(v) if v.dtype == torch.bfloat16 else v.cpu().numpy()) for k, v in step.saved().items()}
    o = {k: to_bits(v) for k, v in zip(("Y3", "dX", "dW1", "dW2"), outs)}
    assert not o["dW1"][1].any() and not o["dW2"][1].any()
    y2max = dy1max = 0.0
    for e in (0, 2, 3):
        a, b = int(seg[e]), int(seg[e + 1])
        inp = dict(X=mm["X"][a:b], W1=W1[e], W2=W2[e], b1=b1[e], dY=mm["dY"][a:b])
        se = {k: s[k][e] for k in ("w1_codes", "w1_meta", "w2t_codes", "w2t_meta")}
        se.update({k: s[k][a:b] for k in ("y1", "y2_codes", "y2_meta", "dy2", "dy1_vals")})
        se["colidx"] = s["colidx"][a // 64:b // 64]
        se["y1_kept"] = s["y1_kept"].reshape(-1)[a * F // 4:b * F // 4]
        oe = dict(Y3=o["Y3"][a:b], dX=o["dX"][a:b], dW1=o["dW1"][e], dW2=o["dW2"][e])
        _check_fp8_step_against_oracle(inp, sc, se, oe, sffn.MODE_SOFT, wgrad_fp8)
        y2max = max(y2max, amax(oracle.sqrelu_vnm_compress(se["y1"])[0]))
        dy1max = max(dy1max, amax(se["dy1_vals"]))
    got = step.amax_dict()
    assert got["x"] == amax(mm["X"]) and got["w1"] == amax(W1) and got["w2"] == amax(W2) and got["dy"] == amax(mm["dY"])
    assert got["y2"] == y2max and got["dy1"] == dy1max
