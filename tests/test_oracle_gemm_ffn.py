"""Pins for the oracle's contractions and the whole step: exact rational triple loops on tiny
shapes, the masked-dense identity, finite differences of the masked FFN, workload statistics."""
from fractions import Fraction

import numpy as np

import oracle
from oracle.sparse24 import HARD, SOFT
from workload import make_ffn_inputs, make_moe_segments


def bf(x):
    return oracle.f32_to_bits(np.asarray(x, dtype=np.float32))


def _frac(bits):
    return [[Fraction(float(v)) for v in row] for row in oracle.bits_to_f64(bits)]


def test_spmm24_triple_loop_exact():
    rng = np.random.default_rng(8)
    T, N, K = 5, 6, 16
    X = bf(rng.integers(-8, 9, (T, K)) / 4.0)
    W = bf(rng.integers(-8, 9, (N, K)) / 8.0)
    bias = (rng.integers(-4, 5, N) / 2.0).astype(np.float32)
    vals, meta = oracle.prune24_compress(W)
    out = oracle.bits_to_f64(oracle.spmm24(X, vals, meta, bias))
    Ws = _frac(oracle.prune24_dense(W))
    Xf = _frac(X)
    for t in range(T):
        for n in range(N):
            acc = Fraction(float(bias[n]))
            for k in range(K):
                acc += Xf[t][k] * Ws[n][k]
            assert out[t, n] == oracle.bits_to_f64(oracle.f64_to_bits(np.float64(float(acc))))


def test_vnm_gemms_triple_loop_exact():
    rng = np.random.default_rng(9)
    T, F, D = 8, 16, 5
    y2 = bf(rng.integers(0, 5, (T, F)) / 2.0)
    vals, meta, colidx = oracle.vnm_compress(y2, 4, 8)
    A = _frac(oracle.vnm_decompress(vals, meta, colidx, 4, 8))
    W2 = bf(rng.integers(-8, 9, (D, F)) / 8.0)         # [N, F]
    W1 = bf(rng.integers(-8, 9, (F, D)) / 8.0)         # [F, N]  (k-major)
    G = bf(rng.integers(-8, 9, (T, D)) / 4.0)
    y3 = oracle.bits_to_f64(oracle.vnm_spmm(vals, meta, colidx, W2, 0, 4, 8))
    dx = oracle.bits_to_f64(oracle.vnm_spmm(vals, meta, colidx, W1, 1, 4, 8))
    cf = oracle.bits_to_f64(oracle.vnm_wgrad(vals, meta, colidx, G, 1, 4, 8))
    cn = oracle.bits_to_f64(oracle.vnm_wgrad(vals, meta, colidx, G, 0, 4, 8))
    W2f, W1f, Gf = _frac(W2), _frac(W1), _frac(G)
    rnd = lambda fr: oracle.bits_to_f64(oracle.f64_to_bits(np.float64(float(fr))))
    for t in range(T):
        for d in range(D):
            assert y3[t, d] == rnd(sum(A[t][f] * W2f[d][f] for f in range(F)))
            assert dx[t, d] == rnd(sum(A[t][f] * W1f[f][d] for f in range(F)))
    for f in range(F):
        for d in range(D):
            w = rnd(sum(A[t][f] * Gf[t][d] for t in range(T)))
            assert cf[f, d] == w and cn[d, f] == w
    assert cf.shape == (F, D) and cn.shape == (D, F)


def test_sparse_gemm_is_dense_gemm_on_masked_matrix():
    inp = make_ffn_inputs(128, 64, 128, seed=1)
    vals, meta = oracle.prune24_compress(inp["W1"])
    masked = oracle.bits_to_f64(oracle.prune24_dense(inp["W1"]))
    want = oracle.bits_to_f64(inp["X"]) @ masked.T + inp["b1"].astype(np.float64)
    got = oracle.bits_to_f64(oracle.spmm24(inp["X"], vals, meta, inp["b1"]))
    assert np.abs(got - want).max() <= np.abs(want).max() * 2.0 ** -8   # one bf16 rounding


def _masked_ffn_loss(X, W1, W2, b1, dY, mask):
    y1 = X @ W1.T + b1
    y2 = np.maximum(y1, 0.0) ** 2 * mask
    return float(np.sum((y2 @ W2.T) * dY))


def test_backward_is_gradient_of_masked_forward():
    """With W1 and W2.T already 2:4 along d_model (so HARD pruning changes nothing) and the V:N:M
    mask frozen, Alg. 2 is the exact gradient of <dY, y3>; check against central differences."""
    rng = np.random.default_rng(11)
    T, D, F = 64, 16, 32
    X = bf(rng.standard_normal((T, D)))
    dY = bf(rng.standard_normal((T, D)))
    W1 = oracle.prune24_dense(bf(rng.standard_normal((F, D)) * 0.3))
    W2 = np.ascontiguousarray(oracle.prune24_dense(bf(rng.standard_normal((F, D)) * 0.3)).T)
    b1 = (rng.standard_normal(F) * 0.1 - 0.3).astype(np.float32)
    ref = oracle.ffn_sparse_step_ref(X, W1, W2, b1, dY, HARD)
    ones = np.full_like(ref["y2_vals"], 0x3F80)
    mask = (oracle.vnm_decompress(ones, ref["y2_meta"], ref["colidx"]) != 0).astype(np.float64)
    Xf, W1f, W2f, dYf = (oracle.bits_to_f64(a) for a in (X, W1, W2, dY))
    b = b1.astype(np.float64)

    def num_grad(which, shape, n=60):
        g = np.zeros(shape)
        idx = [tuple(rng.integers(0, s) for s in shape) for _ in range(n)]
        h = 1e-5
        for ij in idx:
            args = dict(X=Xf.copy(), W1=W1f.copy(), W2=W2f.copy())
            args[which][ij] += h
            lp = _masked_ffn_loss(args["X"], args["W1"], args["W2"], b, dYf, mask)
            args[which][ij] -= 2 * h
            lm = _masked_ffn_loss(args["X"], args["W1"], args["W2"], b, dYf, mask)
            g[ij] = (lp - lm) / (2 * h)
        return g, idx

    for which, key in (("X", "dX"), ("W1", "dW1"), ("W2", "dW2")):
        got = oracle.bits_to_f64(ref[key])
        g, idx = num_grad(which, got.shape)
        a = np.array([got[ij] for ij in idx])
        w = np.array([g[ij] for ij in idx])
        scale = np.abs(oracle.bits_to_f64(ref[key])).max()
        assert np.abs(a - w).max() <= 0.03 * scale, (key, np.abs(a - w).max(), scale)
        assert np.linalg.norm(a - w) <= 0.03 * np.linalg.norm(w) + 1e-9, key


def test_step_stage_shapes_and_soft_mode_differs_only_through_weights():
    inp = make_ffn_inputs(128, 64, 128, seed=2)
    r0 = oracle.ffn_sparse_step_ref(mode=HARD, **inp)
    r1 = oracle.ffn_sparse_step_ref(mode=SOFT, **inp)
    assert r0["y1"].shape == (128, 128) and r0["y3"].shape == (128, 64) and r0["dW1"].shape == (128, 64)
    assert r0["dW2"].shape == (64, 128) and r0["dX"].shape == (128, 64) and r0["colidx"].shape == (2, 16, 4)
    assert np.array_equal(r0["w1_meta"], r1["w1_meta"]) and not np.array_equal(r0["w1_vals"], r1["w1_vals"])
    # dX uses the dense, unpruned W1 (Alg. 2 line 5): recompute it that way
    dense_dy1 = oracle.vnm_decompress(r0["dy1_vals"], r0["y2_meta"], r0["colidx"])
    assert np.array_equal(r0["dX"], oracle.dense_nt(dense_dy1, np.ascontiguousarray(inp["W1"].T)))


def test_dense_limit():
    """When nothing is pruned away (weights already 2:4, at most two live hidden units per block of 8 sharing
    4 live columns), the sparse step equals the dense FFN of eqs. (1)-(8) bit for bit."""
    rng = np.random.default_rng(12)
    T, D, F = 64, 16, 16
    X = bf(np.abs(rng.standard_normal((T, D))))
    dY = bf(rng.standard_normal((T, D)))
    W1f = np.zeros((F, D), dtype=np.float32)
    live = [1, 6, 8, 13]                                    # one or two live neurons per group of 4
    W1f[live] = np.abs(rng.standard_normal((len(live), D))) * 0.3
    W1 = oracle.prune24_dense(bf(W1f))
    W2 = np.ascontiguousarray(oracle.prune24_dense(bf(rng.standard_normal((F, D)) * 0.3)).T)
    b1 = np.full(F, -0.01, dtype=np.float32)
    s = oracle.ffn_sparse_step_ref(X, W1, W2, b1, dY, HARD)
    d = oracle.ffn_dense_ref(X, W1, W2, b1, dY)
    assert np.array_equal(oracle.vnm_decompress(s["y2_vals"], s["y2_meta"], s["colidx"]), d["y2"])
    for k in ("y1", "y3", "dy2", "dX", "dW1", "dW2"):
        assert np.array_equal(s[k], d[k]), k


def test_workload_zero_fraction_and_moe_segments():
    for frac in (0.5, 0.75, 0.9, 0.95):
        inp = make_ffn_inputs(512, 256, 1024, seed=0, zero_fraction=frac)
        v, m = oracle.prune24_compress(inp["W1"])
        y1 = oracle.spmm24(inp["X"], v, m, inp["b1"])
        zf = np.mean(oracle.sqrelu(y1) == 0)
        assert abs(zf - frac) < 0.01, (frac, zf)
    counts, offs = make_moe_segments()
    assert counts.sum() == 16384 * 2 and np.all(offs % 64 == 0) and np.all(np.diff(offs) >= counts)
    assert len(set(counts.tolist())) > 1


def test_grouped_step_is_the_plain_step_per_segment_and_ignores_zero_padding():
    """Mixture-of-experts form: one expert over all rows is the plain step; rows of zeros appended to a
    segment (the 64-row padding) change nothing the expert returns for its real rows or its weights:
    a zero row gives y1 = b1 < 0, so y2 = 0 there, which adds nothing to the column scores, and its
    dY row is zero, which adds nothing to either weight gradient."""
    from workload import make_moe_inputs
    m = make_moe_inputs(n_tokens=150, n_experts=3, top_k=2, D=64, F=128, seed=5)
    seg, counts = m["seg"], m["counts"]
    assert int(counts.sum()) == 300 and all(int(v) % 64 == 0 for v in seg) and int(seg[-1]) >= 300
    res = oracle.ffn_sparse_step_grouped_ref(m["X"], m["W1"], m["W2"], m["b1"], m["dY"], seg)
    for e in range(3):
        a, n = int(seg[e]), int(counts[e])
        assert n % 64 != 0                                   # the case is only a test if there is padding
        assert not m["X"][a + n:int(seg[e + 1])].any() and not m["dY"][a + n:int(seg[e + 1])].any()
        r = res[e]
        # weight gradients recomputed from the real rows alone, as dense fp64 sums over the masked activations
        y2d = oracle.bits_to_f64(oracle.vnm_decompress(r["y2_vals"], r["y2_meta"], r["colidx"]))
        dy1d = oracle.bits_to_f64(oracle.vnm_decompress(r["dy1_vals"], r["y2_meta"], r["colidx"]))
        assert not y2d[n:].any() and not dy1d[n:].any()      # padded rows carry no activation and no gradient
        assert np.array_equal(r["dW2"], oracle.f64_to_bits(oracle.bits_to_f64(m["dY"][a:a + n]).T @ y2d[:n]))
        assert np.array_equal(r["dW1"], oracle.f64_to_bits(dy1d[:n].T @ oracle.bits_to_f64(m["X"][a:a + n])))
    one = oracle.ffn_sparse_step_grouped_ref(m["X"], m["W1"][:1], m["W2"][:1], m["b1"][:1], m["dY"], [0, int(seg[-1])])
    ref = oracle.ffn_sparse_step_ref(m["X"], m["W1"][0], m["W2"][0], m["b1"][0], m["dY"])
    for k in ref:
        assert np.array_equal(one[0][k], ref[k]), k
    assert oracle.ffn_sparse_step_grouped_ref(m["X"], m["W1"], m["W2"], m["b1"], m["dY"], [0, 0, 64, int(seg[-1])])[0] is None
