"""Pins for the oracle's neuron-level router (paper Section 3.3, Alg. 3, the three conversion steps of Section 3.4)."""
import numpy as np
import pytest

import oracle
from workload import make_router_inputs


def bf(x):
    return oracle.f32_to_bits(np.asarray(x, dtype=np.float32))


def test_route_scores_exact_on_small_integers_and_close_to_float64():
    rng = np.random.default_rng(0)
    x = rng.integers(-4, 5, size=(37, 192)).astype(np.float32)
    m = rng.integers(-3, 4, size=(5, 192)).astype(np.float32)
    s = oracle.route_scores(bf(x), bf(m))
    assert s.dtype == np.float32 and np.array_equal(s, (x.astype(np.float64) @ m.astype(np.float64).T).astype(np.float32))
    xr, mr = bf(rng.standard_normal((64, 512))), bf(rng.standard_normal((4, 512)))
    ref = oracle.bits_to_f64(xr) @ oracle.bits_to_f64(mr).T
    mag = np.abs(oracle.bits_to_f64(xr)) @ np.abs(oracle.bits_to_f64(mr)).T
    # 8 sequential + 6 tree additions, each within half an ulp of a partial sum bounded by the sum of magnitudes
    assert np.all(np.abs(oracle.route_scores(xr, mr) - ref) <= 14 * 2.0 ** -24 * mag)


def test_route_scores_summation_order():
    """A vector on which the stated order (64 partial sums over 8-element chunks taken round-robin, then folding by 32,
    16, ...) and the plain left-to-right order give different float32 results: products 2^24 at d = 0 (chunk 0, lane
    0), -2^24 at d = 256 (chunk 32, lane 32), 1 at d = 512 (chunk 64, lane 0 again).  Stated order: lane 0 holds
    2^24 + 1 -> 2^24 (tie to even), lane 32 holds -2^24, the fold gives 0.  Left to right (or exact) gives 1."""
    x = np.zeros((1, 1024), dtype=np.float32)
    m = np.zeros((1, 1024), dtype=np.float32)
    x[0, 0], m[0, 0] = 4096.0, 4096.0
    x[0, 256], m[0, 256] = -4096.0, 4096.0
    x[0, 512], m[0, 512] = 1.0, 1.0
    assert (x.astype(np.float64) @ m.astype(np.float64).T)[0, 0] == 1.0
    assert oracle.route_scores(bf(x), bf(m))[0, 0] == 0.0
    # the same 1 in the next chunk belongs to lane 1 and survives the folds
    x[0, 512], m[0, 512] = 0.0, 0.0
    x[0, 520], m[0, 520] = 1.0, 1.0
    assert oracle.route_scores(bf(x), bf(m))[0, 0] == 1.0
    # inside a chunk the eight products are added in ascending d: 2^24, 1, 1 -> 2^24 (each 1 is lost), -2^24 last -> 0;
    # with the two 1s first the sum would be 2
    x[:], m[:] = 0.0, 0.0
    x[0, 0], m[0, 0] = 4096.0, 4096.0
    x[0, 1], m[0, 1] = 1.0, 1.0
    x[0, 2], m[0, 2] = 1.0, 1.0
    x[0, 3], m[0, 3] = -4096.0, 4096.0
    assert oracle.route_scores(bf(x), bf(m))[0, 0] == 0.0


def test_route_top1_brute_force_ties_and_cosine():
    s = np.array([[1.0, 3.0, 3.0, -1.0], [2.0, 2.0, 2.0, 2.0], [-5.0, -4.0, -4.5, -4.0], [0.0, -0.0, 0.0, 0.0]], dtype=np.float32)
    assert list(oracle.route_top1(s)) == [1, 0, 1, 0]
    rng = np.random.default_rng(1)
    s = rng.integers(-3, 4, size=(500, 6)).astype(np.float32)
    want = [min(e for e in range(6) if row[e] == max(row)) for row in s]
    assert list(oracle.route_top1(s)) == want
    # unit-length means: the dot product ranks experts as the cosine similarity does (Section 3.3 names both)
    inp = make_router_inputs(256, 128, 256, 32, seed=5)
    x, m = oracle.bits_to_f64(inp["X"]), oracle.bits_to_f64(inp["means"])
    assert np.allclose(np.linalg.norm(m, axis=1), 1.0, atol=4e-3)           # bf16 storage of a unit vector
    cos = (x @ m.T) / (np.linalg.norm(x, axis=1)[:, None] * np.linalg.norm(m, axis=1)[None, :])
    got = oracle.route_top1(oracle.route_scores(inp["X"], inp["means"]))
    top2 = np.sort(cos, axis=1)[:, -2:]
    clear = (top2[:, 1] - top2[:, 0]) > 1e-2                                # margins far above bf16 norm error and fp32 rounding
    assert clear.sum() > 128 and np.array_equal(got[clear], np.argmax(cos, axis=1)[clear])


def test_stated_order_agrees_with_the_plain_definition_on_clear_margins():
    """Section 3.3 step 1 is x @ ExpertMeans; the stated float32 order only settles near-ties.  Wherever the float64 gap
    between the two best experts exceeds the rounding bound of both scores, the ordered float32 argmax must be the
    definition's, and such tokens must be the overwhelming majority on the router workload."""
    for T, D, M, seed in ((700, 256, 8, 1), (1500, 1024, 32, 2), (900, 520, 64, 3)):
        inp = make_router_inputs(T, D, 256, M, seed=seed)
        clear = oracle.route_margin_is_clear(inp["X"], inp["means"])
        plain = oracle.route_top1(oracle.route_scores_plain(inp["X"], inp["means"]))
        got = oracle.route_top1(oracle.route_scores(inp["X"], inp["means"]))
        assert clear.mean() > 0.99 and np.array_equal(got[clear], plain[clear])
    # a constructed near-tie: the definition's gap is below the bound, so the token is reported as undecided
    x = bf(np.ones((1, 64)))
    m = bf(np.stack([np.full(64, 0.5), np.full(64, 0.5)]))
    assert not oracle.route_margin_is_clear(x, m)[0]
    assert oracle.route_margin_is_clear(x, bf(np.stack([np.full(64, 0.5), np.full(64, 0.25)])))[0]


@pytest.mark.parametrize("T,E", [(0, 2), (1, 2), (200, 4), (777, 16), (640, 8)])
def test_expert_permutation_properties(T, E):
    rng = np.random.default_rng(T + E)
    expert = rng.integers(0, E, size=T)
    if T == 640:
        expert[:] = 3                                                       # one expert takes everything
    perm, seg = oracle.expert_permutation(expert, E)
    assert len(perm) == (T + 63) // 64 * 64 + 64 * E and seg[0] == 0 and np.all(seg % 64 == 0)
    real = perm[perm >= 0]
    assert sorted(real) == list(range(T))                                   # every token exactly once
    for e in range(E):
        run = perm[seg[e]:seg[e + 1]]
        tok = run[run >= 0]
        n = int((expert == e).sum())
        assert len(tok) == n and np.all(expert[tok] == e) and np.all(np.diff(tok) > 0)      # stable
        assert np.all(run[:n] >= 0) and np.all(run[n:] < 0) and seg[e + 1] - seg[e] == (n + 63) // 64 * 64
    assert np.all(perm[seg[E]:] < 0)


def _literal_alg3(inp, M, expert, mode):
    """Alg. 3 as printed: out = zeros; for every token, out[i] += x[i] @ W[expert] with W[expert] = the (2:4-pruned)
    W1 restricted to the expert's hidden units; then eq. (2).  Dense [T, F] result, python loop over tokens."""
    X, W1, b1 = oracle.bits_to_f64(inp["X"]), oracle.bits_to_f64(oracle.prune24_dense(inp["W1"], mode)), inp["b1"].astype(np.float64)
    T, F = X.shape[0], W1.shape[0]
    owner = (np.arange(F) % M) // 4
    y2 = np.zeros((T, F), dtype=np.uint16)
    for i in range(T):
        We = np.where((owner == expert[i])[:, None], W1, 0.0)
        out = X[i] @ We.T + np.where(owner == expert[i], b1, 0.0)
        y2[i] = oracle.sqrelu(oracle.f64_to_bits(out[None, :]))[0]
    return y2


@pytest.mark.parametrize("M,mode", [(8, oracle.sparse24.HARD), (16, oracle.sparse24.SOFT), (32, oracle.sparse24.HARD)])
def test_moe_to_venom_equals_literal_algorithm_then_24(M, mode):
    T, D, F = 150, 64, 128
    inp = make_router_inputs(T, D, F, M, seed=11, zero_fraction=0.5)
    r = oracle.moe_to_venom(inp["X"], inp["W1"], inp["b1"], inp["means"], M, mode)
    y2 = _literal_alg3(inp, M, r["expert"], mode)
    dense = oracle.vnm_decompress(r["vals"], r["meta"], r["colidx"], 64, M)            # [Tcap, F]
    real = r["perm"] >= 0
    assert not dense[~real].any()
    # brute-force 2:4 inside the expert's four columns of every block: keep the two largest, ties to the lower column
    want = np.zeros_like(y2)
    for i in range(T):
        cols0 = 4 * r["expert"][i]
        for g in range(F // M):
            c = g * M + cols0 + np.arange(4)
            v = y2[i, c]
            order = sorted(range(4), key=lambda k: (-int(v[k] & 0x7FFF), k))[:2]
            want[i, c[order]] = v[order]
    assert np.array_equal(dense[real], want[r["perm"][real]])
    assert (dense != 0).mean() <= 2.0 / M                                           # Table 5: sparsity at least 1 - N / M


def test_router_output_is_what_section_2_3_would_select():
    """The matrix Alg. 3 produces, written out densely in permuted row order, is V:N:M by construction: the magnitude
    rule of Section 2.3 applied to it picks the expert's columns back (wherever each of them carries mass) and the same
    packed values."""
    M = 16
    inp = make_router_inputs(1024, 64, 256, M, seed=2, zero_fraction=0.5)
    r = oracle.moe_to_venom(inp["X"], inp["W1"], inp["b1"], inp["means"], M)
    dense = oracle.vnm_decompress(r["vals"], r["meta"], r["colidx"], 64, M)
    # the dense y2 before the per-row 2:4: scatter the compact y2 to its hidden units
    y2c = oracle.sqrelu(r["y1c"])
    y2c[r["perm"] < 0] = 0
    full = np.zeros_like(dense)
    for e in range(M // 4):
        rows = slice(int(r["seg"][e]), int(r["seg"][e + 1]))
        full[rows][:, oracle.cluster_rows(e, M, 256)] = y2c[rows]
    vals, meta, colidx = oracle.vnm_compress(full, 64, M)
    mass = oracle.bits_to_f64(full).reshape(-1, 64, 256 // M, M).sum(axis=1)            # [blocks, F / M, M]
    ok = (np.take_along_axis(mass, r["colidx"].astype(np.int64), axis=-1) > 0).all(axis=-1)   # all four expert columns carry mass
    assert ok.mean() > 0.5
    assert np.array_equal(colidx[ok], r["colidx"][ok])
    okr = np.repeat(ok, 64, axis=0)                                                      # [Tcap, F / M]
    assert np.array_equal(vals.reshape(-1, 256 // M, 2)[okr], r["vals"].reshape(-1, 256 // M, 2)[okr])
    # and the activation GEMM on it is the dense product with the masked matrix
    y3 = oracle.vnm_spmm(r["vals"], r["meta"], r["colidx"], inp["W2"], 0, 64, M)
    assert np.array_equal(y3, oracle.dense_nt(dense, inp["W2"]))


def test_router_step_backward_is_the_gradient_of_its_forward():
    """With W1 and W2.T already 2:4 along d_model and the routing and 2:4 masks frozen, the router step's backward is the
    exact gradient of <dY, y3> of a forward in which every token only sees its expert's hidden units; central
    differences in float64 on sampled entries.  Hidden units of experts that got no token have zero weight gradients."""
    rng = np.random.default_rng(21)
    T, D, F, M = 96, 16, 64, 16
    inp = make_router_inputs(T, D, F, M, seed=9, zero_fraction=0.5)
    X, dY = inp["X"], inp["dY"]
    W1 = oracle.prune24_dense(bf(rng.standard_normal((F, D)) * 0.3))
    W2 = np.ascontiguousarray(oracle.prune24_dense(bf(rng.standard_normal((F, D)) * 0.3)).T)
    b1 = (rng.standard_normal(F) * 0.1).astype(np.float32)
    means = inp["means"].copy()
    means[3] = bf(-oracle.bits_to_f32(means[0]))                 # expert 3 mirrors expert 0: few tokens prefer it; fine either way
    ref = oracle.ffn_router_step_ref(X, W1, W2, b1, dY, means, M)
    ones = np.full_like(ref["vals"], 0x3F80)
    maskp = (oracle.vnm_decompress(ones, ref["meta"], ref["colidx"], 64, M) != 0)
    mask = maskp[ref["row_of_token"]].astype(np.float64)          # token order [T, F]
    Xf, W1f, W2f, dYf = (oracle.bits_to_f64(a) for a in (X, W1, W2, dY))
    b = b1.astype(np.float64)

    def loss(Xa, W1a, W2a):
        y1 = Xa @ W1a.T + b[None, :]
        y2 = mask * np.maximum(y1, 0.0) ** 2
        return float(((y2 @ W2a.T) * dYf).sum())

    for which, key in (("X", "dX"), ("W1", "dW1"), ("W2", "dW2")):
        got = oracle.bits_to_f64(ref[key])
        scale = np.abs(got).max()
        for _ in range(60):
            args = dict(X=Xf.copy(), W1=W1f.copy(), W2=W2f.copy())
            ij = tuple(rng.integers(0, n) for n in got.shape)
            h = 1e-5
            args[which][ij] += h
            lp = loss(args["X"], args["W1"], args["W2"])
            args[which][ij] -= 2 * h
            lm = loss(args["X"], args["W1"], args["W2"])
            assert abs(got[ij] - (lp - lm) / (2 * h)) <= 0.03 * scale, (key, ij)
    # forward value, token order
    y3 = oracle.bits_to_f64(ref["y3"])
    y1 = oracle.bits_to_f64(oracle.f64_to_bits(Xf @ W1f.T + b[None, :]))
    y2 = mask * oracle.bits_to_f64(oracle.sqrelu(oracle.f64_to_bits(y1)))
    assert np.abs(y3 - y2 @ W2f.T).max() <= 0.02 * np.abs(y3).max()
    unused = [e for e in range(M // 4) if ref["seg"][e + 1] == ref["seg"][e]]
    for e in unused:
        assert not ref["dW1"][oracle.cluster_rows(e, M, F)].any() and not ref["dW2"][:, oracle.cluster_rows(e, M, F)].any()


@pytest.mark.parametrize("M,F", [(8, 64), (16, 128), (32, 256), (64, 1024)])
def test_cluster_rows_partition_the_hidden_units(M, F):
    """The experts' hidden units are non-overlapping and cover all of them (Section 3.3: non-overlapping subsets), four
    consecutive units of every M-block each, and scatter_compact puts compact column j of expert e exactly there."""
    E = M // 4
    allrows = np.concatenate([oracle.cluster_rows(e, M, F) for e in range(E)])
    assert sorted(allrows) == list(range(F))
    for e in range(E):
        r = oracle.cluster_rows(e, M, F)
        assert len(r) == 4 * F // M and np.all((r % M) // 4 == e) and np.all(np.diff(r.reshape(-1, 4), axis=1) == 1)
    seg = np.arange(E + 1) * 64
    c = (np.arange(64 * E * (4 * F // M)).reshape(64 * E, 4 * F // M) % 65000 + 1).astype(np.uint16)
    full = oracle.scatter_compact(c, seg, M, F)
    for e in range(E):
        rows = slice(64 * e, 64 * e + 64)
        assert np.array_equal(full[rows][:, oracle.cluster_rows(e, M, F)], c[rows])
        assert np.count_nonzero(full[rows]) == c[rows].size
