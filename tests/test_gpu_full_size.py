"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times (dense y1 / dy2 not
stored).  The run that keeps y1 / dy2 must give bit-identical results; from it the compressors are checked bit
for bit (in full at the 1B shape, on slices of whole token blocks at the 7B shape) and the GEMM outputs on
seeded samples of rows / columns that the oracle computes one by one, all teacher-forced."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_06183_amd as sffn
from tests.util import to_dev, to_bits, assert_gemm_close, assert_routing_matches_the_definition
from workload import CONFIGS, make_ffn_inputs, make_ffn_sweep, make_moe_inputs

pytestmark = pytest.mark.gpu


def _run(dev, T, D, F, keep, mode=sffn.MODE_HARD):
    step = sffn.FfnStep(T, D, F, mode, keep_dense=keep)
    outs = step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])
    torch.cuda.synchronize()
    return step, outs


PACKED_KEYS = ("w1_vals", "w1_meta", "w2t_vals", "w2t_meta", "y2_vals", "y2_meta", "colidx", "dy1_vals", "y1_kept")


@pytest.mark.parametrize("name,tb_slices", [("1b", None), ("7b", [(0, 2), (101, 103)]), ("70b", [(0, 1), (77, 78)]),
                                            ("moe_expert", [(0, 1), (30, 31)])])
def test_full_size_step(name, tb_slices):
    T, D, F = CONFIGS[name]
    inp = make_ffn_inputs(T, D, F, seed=0)
    dev = {k: to_dev(v) for k, v in inp.items()}
    _both_configurations_then_sampled_check(inp, dev, T, D, F, tb_slices)


def _both_configurations_then_sampled_check(inp, dev, T, D, F, tb_slices, mode=sffn.MODE_HARD, zero_fraction=0.90):
    step0, outs0 = _run(dev, T, D, F, keep=False, mode=mode)   # what bench.py times
    fast = [to_bits(t).copy() for t in outs0] + [to_bits(step0.saved()[k]).copy() for k in PACKED_KEYS]
    del step0, outs0
    torch.cuda.empty_cache()
    step, outs = _run(dev, T, D, F, keep=True, mode=mode)
    sv = step.saved()
    full = [to_bits(t) for t in outs] + [to_bits(sv[k]) for k in PACKED_KEYS]
    for a, b in zip(fast, full):
        assert np.array_equal(a, b)
    del fast
    _sampled_step_check(inp, full, to_bits(sv["y1"]), to_bits(sv["dy2"]), tb_slices, mode, zero_fraction)


def test_full_size_step_zero_fraction_sweep():
    """configs[3]: the 70B-scale layer at the other three points of the ReLU zero-fraction sweep (0.90 is the case
    above): the same inputs with the bias shifted, the timed configuration bit-identical to the checked one, then the
    same sampled teacher-forced comparison with the oracle, including the zero fraction the bias is meant to give."""
    T, D, F = CONFIGS["70b"]
    dev = None
    for zf, inp in make_ffn_sweep(T, D, F, [0.50, 0.75, 0.95], seed=0):
        print("70b, zero fraction %.2f" % zf, flush=True)
        if dev is None:
            dev = {k: to_dev(v) for k, v in inp.items()}
        dev["b1"] = to_dev(inp["b1"])
        _both_configurations_then_sampled_check(inp, dev, T, D, F, [(0, 1), (77, 78)], zero_fraction=zf)


def test_full_size_step_soft_threshold():
    """The paper's own sparsify24 (Section 2.2, soft-thresholding) at the 1B shape, in the timed configuration."""
    T, D, F = CONFIGS["1b"]
    inp = make_ffn_inputs(T, D, F, seed=0)
    dev = {k: to_dev(v) for k, v in inp.items()}
    _both_configurations_then_sampled_check(inp, dev, T, D, F, [(0, 4), (64, 66), (127, 128)], mode=sffn.MODE_SOFT, zero_fraction=None)


def _sampled_step_check(inp, full, y1, dy2, tb_slices, mode=sffn.MODE_HARD, zero_fraction=0.90):
    """inp: X, W1, W2, b1, dY of ONE FFN; full: its Y3, dX, dW1, dW2 followed by the PACKED_KEYS tensors.
    zero_fraction: what the bias shift is meant to give (None: not checked, e.g. soft-thresholded weights shrink y1's scale)."""
    T, D = inp["X"].shape
    F = inp["W1"].shape[0]
    Y3, dX, dW1, dW2 = full[:4]
    w1v, w1m, w2v, w2m, yv, ym, yc, dv, _ = full[4:]
    rng = np.random.default_rng(123)

    # 2:4 weights: bit-exact, everywhere at 1b, on two bands of 1024 rows at the larger shapes (rows are independent)
    for r in ([slice(0, F)] if tb_slices is None else [slice(0, 1024), slice(F - 1024, F)]):
        rv, rm = oracle.prune24_compress(inp["W1"][r], mode)
        assert np.array_equal(w1v[r], rv) and np.array_equal(w1m[r], rm)
        rv, rm = oracle.prune24_compress(np.ascontiguousarray(inp["W2"][:, r].T), mode)
        assert np.array_equal(w2v[r], rv) and np.array_equal(w2m[r], rm)
    del rv, rm

    # eq. (1) and eq. (4) on sampled token rows
    rows = np.sort(rng.choice(T, 48, replace=False))
    assert_gemm_close(y1[rows], oracle.spmm24(inp["X"][rows], w1v, w1m, inp["b1"]), "y1 rows")
    assert_gemm_close(dy2[rows], oracle.spmm24(inp["dY"][rows], w2v, w2m, None), "dy2 rows")

    # compressors: bit-exact on whole 64-token blocks (all of them at 1b)
    slices = [(0, T // 64)] if tb_slices is None else tb_slices
    for b0, b1 in slices:
        r = slice(64 * b0, 64 * b1)
        ov, om, oc = oracle.sqrelu_vnm_compress(y1[r])
        assert np.array_equal(yc[b0:b1], oc) and np.array_equal(ym[r], om) and np.array_equal(yv[r], ov)
        assert np.array_equal(dv[r], oracle.dsqrelu_vnm(dy2[r], y1[r], om, oc))
    if zero_fraction is not None:
        zero_frac = float(np.mean(oracle.sqrelu(y1[:2048]) == 0))
        assert abs(zero_frac - zero_fraction) < 0.01, (zero_frac, zero_fraction)

    # eq. (3), (7): sampled token rows (a row only needs its own 64-token block's column indices)
    def dense_rows(vals, rws):
        out = np.zeros((len(rws), F), dtype=np.uint16)
        for n, t in enumerate(rws):
            tb = t // 64
            blk = oracle.vnm_decompress(vals[64 * tb:64 * tb + 64], ym[64 * tb:64 * tb + 64], yc[tb:tb + 1])
            out[n] = blk[t % 64]
        return out

    rows = np.sort(rng.choice(T, 32, replace=False))
    assert_gemm_close(Y3[rows], oracle.dense_nt(dense_rows(yv, rows), inp["W2"]), "y3 rows")
    assert_gemm_close(dX[rows], oracle.dense_nt(dense_rows(dv, rows), np.ascontiguousarray(inp["W1"].T)), "dX rows")

    # eq. (5), (8): sampled hidden units f = 8 whole column blocks
    blks = np.sort(rng.choice(F // 8, 8, replace=False))
    cols = (blks[:, None] * 8 + np.arange(8)[None, :]).reshape(-1)

    def dense_cols(vals):
        # the [T, 64] slab of the V:N:M matrix restricted to the sampled column blocks
        sub_v = vals.reshape(T, F // 8, 2)[:, blks].reshape(T, -1)
        nib = np.empty((T, F // 8), dtype=np.uint8)
        nib[:, 0::2] = ym & 0xF
        nib[:, 1::2] = ym >> 4
        sub_n = nib[:, blks]
        sub_m = (sub_n[:, 0::2] | (sub_n[:, 1::2] << 4)).astype(np.uint8)
        return oracle.vnm_decompress(np.ascontiguousarray(sub_v), sub_m, np.ascontiguousarray(yc[:, blks]))

    a = oracle.bits_to_f64(dense_cols(yv))
    ref = oracle.f64_to_bits(a.T @ oracle.bits_to_f64(inp["dY"]))              # [64, D]
    assert_gemm_close(np.ascontiguousarray(dW2[:, cols].T), ref, "dW2 columns")
    a = oracle.bits_to_f64(dense_cols(dv))
    ref = oracle.f64_to_bits(a.T @ oracle.bits_to_f64(inp["X"]))
    assert_gemm_close(dW1[cols], ref, "dW1 rows")


def test_full_size_grouped_step():
    """configs[4]: 8 experts of d_model 4096, d_ff 14336, 16384 tokens routed top-2 (uneven 64-row-aligned segments),
    one grouped launch per stage.  The timed configuration (no dense y1 / dy2) must agree bit for bit with the
    one that stores them; two experts are then checked like a full-size plain step, the others on their 2:4 weights."""
    D, F, E = 4096, 14336, 8
    m = make_moe_inputs(n_tokens=16384, n_experts=E, top_k=2, D=D, F=F, seed=0)
    seg = m["seg"]
    dev = {k: to_dev(m[k]) for k in ("X", "W1", "W2", "b1", "dY")}

    def run(keep):
        step = sffn.FfnStepGrouped(seg, D, F, sffn.MODE_HARD, keep_dense=keep)
        outs = step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])
        torch.cuda.synchronize()
        return step, outs

    step0, outs0 = run(False)
    fast = [to_bits(t).copy() for t in outs0] + [to_bits(step0.saved()[k]).copy() for k in PACKED_KEYS]
    del step0, outs0
    torch.cuda.empty_cache()
    step, outs = run(True)
    sv = step.saved()
    full = [to_bits(t) for t in outs] + [to_bits(sv[k]) for k in PACKED_KEYS]
    for a, b in zip(fast, full):
        assert np.array_equal(a, b)
    del fast
    y1, dy2 = to_bits(sv["y1"]), to_bits(sv["dy2"])
    for e in range(E):
        a, b = int(seg[e]), int(seg[e + 1])
        if e in (1, 6):
            inp = dict(X=m["X"][a:b], W1=m["W1"][e], W2=m["W2"][e], b1=m["b1"][e], dY=m["dY"][a:b])
            Y3, dX, dW1, dW2 = full[:4]
            w1v, w1m, w2v, w2m, yv, ym, yc, dv, yk = full[4:]
            part = [Y3[a:b], dX[a:b], dW1[e], dW2[e], w1v[e], w1m[e], w2v[e], w2m[e], yv[a:b], ym[a:b], yc[a // 64:b // 64], dv[a:b], None]
            nb = (b - a) // 64
            _sampled_step_check(inp, part, y1[a:b], dy2[a:b], [(0, 1), (nb - 1, nb)])      # the last block holds the zero padding
        else:
            r = slice(F - 512, F)
            rv, rm = oracle.prune24_compress(m["W1"][e][r])
            assert np.array_equal(full[4][e][r], rv) and np.array_equal(full[5][e][r], rm)
            rv, rm = oracle.prune24_compress(np.ascontiguousarray(m["W2"][e][:, r].T))
            assert np.array_equal(full[6][e][r], rv) and np.array_equal(full[7][e][r], rm)


@pytest.mark.parametrize("M", [16, 64])
def test_full_size_wide_block_step(M):
    """Table 5's wider blocks at the 1B shape, as bench.py --M times it: fused epilogues, eqs. (3), (7) on the gathered-row kernel.
    Compressors bit-exact on sampled token blocks, GEMM outputs on sampled rows / column blocks, teacher-forced."""
    T, D, F = CONFIGS["1b"]
    inp = make_ffn_inputs(T, D, F, seed=0)
    dev = {k: to_dev(v) for k, v in inp.items()}
    fast = sffn.FfnStep(T, D, F, sffn.MODE_HARD, M=M)                   # what bench.py --M times: fused, no dense y1 / dy2
    outs_fast = [to_bits(t).copy() for t in fast(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])]
    packed_fast = [to_bits(fast.saved()[k]).copy() for k in ("y2_vals", "y2_meta", "colidx", "dy1_vals", "y1_kept")]
    del fast
    torch.cuda.empty_cache()
    step = sffn.FfnStep(T, D, F, sffn.MODE_HARD, M=M, keep_dense=True)
    outs = step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])
    torch.cuda.synchronize()
    Y3, dX, dW1, dW2 = (to_bits(t) for t in outs)
    sv = {k: to_bits(v) for k, v in step.saved().items()}
    assert all(np.array_equal(a, b) for a, b in zip(outs_fast, (Y3, dX, dW1, dW2)))
    assert all(np.array_equal(a, sv[k]) for a, k in zip(packed_fast, ("y2_vals", "y2_meta", "colidx", "dy1_vals", "y1_kept")))
    y1, dy2, yv, ym, yc, dv = (sv[k] for k in ("y1", "dy2", "y2_vals", "y2_meta", "colidx", "dy1_vals"))
    rng = np.random.default_rng(1000 + M)

    rows = np.sort(rng.choice(T, 32, replace=False))
    assert_gemm_close(y1[rows], oracle.spmm24(inp["X"][rows], sv["w1_vals"], sv["w1_meta"], inp["b1"]), "y1 rows")
    assert_gemm_close(dy2[rows], oracle.spmm24(inp["dY"][rows], sv["w2t_vals"], sv["w2t_meta"], None), "dy2 rows")

    dense_y2, dense_dy1 = {}, {}
    for tb in sorted(set(int(b) for b in rng.choice(T // 64, 6, replace=False)) | {0, T // 64 - 1}):
        r = slice(64 * tb, 64 * tb + 64)
        ov, om, oc = oracle.sqrelu_vnm_compress(y1[r], 64, M)
        assert np.array_equal(yc[tb:tb + 1], oc) and np.array_equal(ym[r], om) and np.array_equal(yv[r], ov)
        assert np.array_equal(dv[r], oracle.dsqrelu_vnm(dy2[r], y1[r], om, oc, 64, M))
        dense_y2[tb] = oracle.vnm_decompress(ov, om, oc, 64, M)
        dense_dy1[tb] = oracle.vnm_decompress(dv[r], om, oc, 64, M)
        assert np.count_nonzero(dense_y2[tb]) <= 64 * F * 2 // M

    # eqs. (3), (7): every row of the checked token blocks' first and last four rows
    for tb in dense_y2:
        sel = np.array([0, 1, 2, 3, 60, 61, 62, 63])
        assert_gemm_close(Y3[64 * tb + sel], oracle.dense_nt(dense_y2[tb][sel], inp["W2"]), "y3 rows")
        assert_gemm_close(dX[64 * tb + sel], oracle.dense_nt(dense_dy1[tb][sel], np.ascontiguousarray(inp["W1"].T)), "dX rows")

    # eqs. (5), (8): two whole column blocks of M hidden units, contracted over all tokens
    for blk in rng.choice(F // M, 2, replace=False):
        cols = np.arange(blk * M, blk * M + M)
        nib = np.empty((T, F // M), dtype=np.uint8)
        nib[:, 0::2] = ym & 0xF
        nib[:, 1::2] = ym >> 4
        sub_m = (nib[:, blk:blk + 1] | (np.uint8(0x4) << 4)).astype(np.uint8)   # a second, empty block completes the metadata byte
        for vals, G, got in ((yv, inp["dY"], np.ascontiguousarray(dW2[:, cols].T)), (dv, inp["X"], dW1[cols])):
            sub_v = np.zeros((T, 4), dtype=np.uint16)
            sub_v[:, :2] = vals.reshape(T, F // M, 2)[:, blk]
            sub_c = np.zeros((T // 64, 2, 4), dtype=np.uint8)
            sub_c[:, 0] = yc[:, blk]
            sub_c[:, 1] = np.arange(4, dtype=np.uint8)
            a = oracle.bits_to_f64(oracle.vnm_decompress(sub_v, sub_m, sub_c, 64, M))[:, :M]
            assert_gemm_close(got, oracle.f64_to_bits(a.T @ oracle.bits_to_f64(G)), "wgrad columns")


@pytest.mark.parametrize("M", [8, 16, 32, 64])
def test_full_size_router(M):
    """Alg. 3 at the 1B shape: routing and grouping bit-exact in full; the grouped matmul on sampled rows; eq. (2) + 2:4
    packing bit-exact on sampled 64-row blocks from the GPU's own y1c; eq. (3) on the result on sampled rows."""
    from workload import make_router_inputs
    T, D, F = CONFIGS["1b"]
    inp = make_router_inputs(T, D, F, M, seed=0)
    dev = {k: to_dev(v) for k, v in inp.items()}
    r = sffn.moe_to_venom(dev["X"], dev["W1"], dev["b1"], dev["means"], M)
    y3 = sffn.vnm_spmm(r["vals"], r["meta"], r["colidx"], dev["W2"], 0, 64, M)
    torch.cuda.synchronize()
    expert = oracle.route_top1(oracle.route_scores(inp["X"], inp["means"]))
    perm, seg = oracle.expert_permutation(expert, M // 4)
    assert np.array_equal(to_bits(r["expert"]), expert) and np.array_equal(to_bits(r["perm"]), perm) and r["seg"] == [int(v) for v in seg]
    assert_routing_matches_the_definition(to_bits(r["expert"]), inp["X"], inp["means"])
    counts = np.bincount(expert, minlength=M // 4)
    assert counts.min() > 0 and counts.max() < 3 * T // (M // 4)          # uneven but not degenerate
    y1c, vals, meta, colidx, y3 = (to_bits(t) for t in (r["y1c"], r["vals"], r["meta"], r["colidx"], y3))
    rng = np.random.default_rng(77)
    w1s = oracle.prune24_dense(inp["W1"])
    Kc = 4 * F // M
    for tb in sorted(set(int(b) for b in rng.choice(int(seg[-1]) // 64, 6, replace=False)) | {0, len(perm) // 64 - 1}):
        rows = np.arange(64 * tb, 64 * tb + 64)
        e = int(np.searchsorted(seg, 64 * tb, side="right") - 1) if 64 * tb < seg[-1] else 0
        ov, om, oc = oracle.venom_from_compact(y1c[rows], perm[rows], np.clip(seg - 64 * tb, 0, 64), M)     # the runs as seen from this block
        assert np.array_equal(colidx[tb:tb + 1], oc) and np.array_equal(meta[rows], om) and np.array_equal(vals[rows], ov)
        real = rows[perm[rows] >= 0][:8]
        if len(real):
            ref = oracle.bits_to_f64(inp["X"][perm[real]]) @ oracle.bits_to_f64(w1s[oracle.cluster_rows(e, M, F)]).T
            ref = oracle.f64_to_bits(ref + inp["b1"].astype(np.float64)[oracle.cluster_rows(e, M, F)][None, :])
            assert_gemm_close(y1c[real], ref, "y1c rows")
            dense = oracle.vnm_decompress(ov, om, oc, 64, M)
            assert_gemm_close(y3[real], oracle.dense_nt(dense[real - 64 * tb], inp["W2"]), "y3 rows")
        assert Kc == y1c.shape[1]


@pytest.mark.parametrize("name,M", [("1b", 16), ("1b", 64), ("7b", 16)])
def test_full_size_router_step(name, M):
    """ffn_router_step at the 1B and 7B shapes as bench.py --router times it: routing bit-exact in full; packing and eq. (6)
    bit-exact on sampled 64-row blocks from the GPU's own y1c / dy2c; every contraction on sampled rows / hidden units."""
    from workload import make_router_inputs
    T, D, F = CONFIGS[name]
    inp = make_router_inputs(T, D, F, M, seed=0)
    dev = {k: to_dev(v) for k, v in inp.items()}
    route = sffn.venom_route(dev["X"], dev["means"], M)
    fast = sffn.FfnRouterStep(T, D, F, M)                           # the timed configuration: routing inside, dy2c not stored
    outs_fast = [to_bits(t).copy() for t in fast.full(dev["means"], dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])]
    del fast
    torch.cuda.empty_cache()
    step = sffn.FfnRouterStep(T, D, F, M, keep_dense=True)
    outs = step(route, dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])
    torch.cuda.synchronize()
    Y3, dX, dW1, dW2 = (to_bits(t) for t in outs)
    assert all(np.array_equal(a, b) for a, b in zip(outs_fast, (Y3, dX, dW1, dW2)))
    sv = {k: to_bits(v) for k, v in step.saved().items()}
    expert = oracle.route_top1(oracle.route_scores(inp["X"], inp["means"]))
    perm, seg = oracle.expert_permutation(expert, M // 4)
    assert np.array_equal(to_bits(route["perm"]), perm) and route["seg"] == [int(v) for v in seg]
    rng = np.random.default_rng(5 + M)
    w1s = oracle.prune24_dense(inp["W1"])
    w2t_s = oracle.prune24_dense(np.ascontiguousarray(inp["W2"].T))
    for tb in sorted(set(int(b) for b in rng.choice(int(seg[-1]) // 64, 5, replace=False)) | {0}):
        rows = np.arange(64 * tb, 64 * tb + 64)
        e = int(np.searchsorted(seg, 64 * tb, side="right") - 1)
        cl = oracle.cluster_rows(e, M, F)
        lseg = np.clip(seg - 64 * tb, 0, 64)
        ov, om, oc = oracle.venom_from_compact(sv["y1c"][rows], perm[rows], lseg, M)
        assert np.array_equal(sv["colidx"][tb:tb + 1], oc) and np.array_equal(sv["meta"][rows], om) and np.array_equal(sv["vals"][rows], ov)
        dv = oracle.dsqrelu_vnm(oracle.scatter_compact(sv["dy2c"][rows], lseg, M, F), oracle.scatter_compact(sv["y1c"][rows], lseg, M, F), om, oc, 64, M)
        assert np.array_equal(sv["dvals"][rows], dv)
        sel = rows[perm[rows] >= 0][:8]
        if len(sel) == 0:
            continue
        tok = perm[sel]
        ref = oracle.bits_to_f64(inp["X"][tok]) @ oracle.bits_to_f64(w1s[cl]).T + inp["b1"].astype(np.float64)[cl][None, :]
        assert_gemm_close(sv["y1c"][sel], oracle.f64_to_bits(ref), "y1c rows")
        assert_gemm_close(sv["dy2c"][sel], oracle.dense_nt(inp["dY"][tok], w2t_s[cl]), "dy2c rows")
        assert_gemm_close(Y3[tok], oracle.dense_nt(oracle.vnm_decompress(ov, om, oc, 64, M)[sel - 64 * tb], inp["W2"]), "y3 rows")
        assert_gemm_close(dX[tok], oracle.dense_nt(oracle.vnm_decompress(dv, om, oc, 64, M)[sel - 64 * tb], np.ascontiguousarray(inp["W1"].T)), "dX rows")
    # weight gradients: a few hidden units of two experts, contracted over the expert's whole run
    for e in (0, M // 4 - 1):
        run = np.arange(int(seg[e]), int(seg[e + 1]))
        real = run[perm[run] >= 0]
        js = np.sort(rng.choice(4 * F // M, 8, replace=False))
        f = oracle.cluster_rows(e, M, F)[js]
        for packed, G, got in ((sv["vals"], inp["dY"], np.ascontiguousarray(dW2[:, f].T)), (sv["dvals"], inp["X"], dW1[f])):
            a = oracle.bits_to_f64(oracle.prune24_decompress(packed[real], sv["meta"][real])[:, js])
            assert_gemm_close(got, oracle.f64_to_bits(a.T @ oracle.bits_to_f64(G[perm[real]])), "wgrad rows")


@pytest.mark.parametrize("wgrad_fp8", [False, True])
def test_full_size_fp8_step(wgrad_fp8):
    """ffn_sparse_step_fp8 at the 1B layer in the timed configuration (weight gradients in bf16 or on codes): packed outputs bit-exact against the oracle's compressors on
    the kept y1, contractions on sampled rows / columns against the oracle's fp8 contractions (teacher-forced on the GPU's packed operands)."""
    from oracle import fp8 as f8
    T, D, F = CONFIGS["1b"]
    inp = make_ffn_inputs(T, D, F, seed=0)
    dev = {k: to_dev(v) for k, v in inp.items()}
    ref_step = sffn.FfnStep(T, D, F)
    ref_step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])
    sv = ref_step.saved()
    amax = lambda t: float(t.float().abs().max())
    sc = dict(x=amax(dev["X"]) / 448, w1=amax(dev["W1"]) / 448, w2=amax(dev["W2"]) / 448, y2=amax(sv["y2_vals"]) / 448, dy=amax(dev["dY"]) / 448,
              dy1=amax(sv["dy1_vals"]) / 448)
    del ref_step, sv
    step = sffn.FfnStepFp8(T, D, F, sc, wgrad_fp8=wgrad_fp8)
    Y3, dX, dW1, dW2 = (to_bits(t) for t in step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"]))
    s = {k: (to_bits(v) if v.dtype == torch.bfloat16 else v.cpu().numpy()) for k, v in step.saved().items()}
    c1, m1 = f8.prune24_compress_fp8(inp["W1"], sc["w1"])
    assert np.array_equal(s["w1_codes"], c1) and np.array_equal(s["w1_meta"], m1)
    c2, m2 = f8.prune24_compress_fp8(np.ascontiguousarray(inp["W2"].T), sc["w2"])
    assert np.array_equal(s["w2t_codes"], c2) and np.array_equal(s["w2t_meta"], m2)
    rng = np.random.default_rng(0)
    rows = np.sort(rng.choice(T // 64, 6, replace=False))[:, None] * 64 + np.arange(64)[None, :]      # six whole 64-token blocks
    rows = rows.reshape(-1)
    # y1 on those token blocks from the oracle's eq. (1); the GPU's packed y2 must be the compression of a y1 within tolerance of it:
    # checked through the kept y1 (bit-exact bookkeeping) and the downstream contractions
    xq = f8.quantize_fp8(inp["X"][rows], sc["x"])
    y1_ref = f8.spmm24_fp8(xq, sc["x"], c1, m1, sc["w1"], inp["b1"])
    yc, ym, cix = s["y2_codes"][rows], s["y2_meta"][rows], s["colidx"][rows[::64] // 64]
    # the GPU's survivors sit where the GPU's own y1 put them; their codes must decode to y2 values of the reference y1 within fp8 spacing
    dec = oracle.vnm_decompress(f8.codes_as_bf16_bits(yc), ym, cix)
    y2_ref = oracle.bits_to_f32(oracle.sqrelu(y1_ref))
    got = oracle.bits_to_f32(dec) * np.float32(sc["y2"])
    nz = got != 0
    assert nz.mean() > 0.01
    # half an E4M3 spacing (2^-4 relative, 2^-10 absolute in code units) plus y1's bf16 rounding carried through the square
    assert np.all(np.abs(got[nz] - y2_ref[nz]) <= (2.0 ** -4 + 2.0 ** -6) * np.abs(y2_ref[nz]) + 2.0 ** -9 * sc["y2"])
    w2q = f8.quantize_fp8(inp["W2"], sc["w2"])
    assert_gemm_close(Y3[rows], f8.vnm_spmm_fp8(yc, ym, cix, sc["y2"], w2q, sc["w2"], 0), "y3")
    dv = s["dy1_vals"][rows]
    w1q = f8.quantize_fp8(inp["W1"], sc["w1"])
    assert_gemm_close(dX[rows], f8.vnm_spmm_fp8(f8.quantize_fp8(dv, sc["dy1"]), ym, cix, sc["dy1"], w1q, sc["w1"], 1), "dX")
    # weight gradients: bf16 contractions over all tokens for sampled hidden units; y2's bf16 survivors are not stored, so eq. (8) only
    cols = np.sort(rng.choice(F // 8, 8, replace=False))[:, None] * 8 + np.arange(8)[None, :]
    cols = cols.reshape(-1)
    if wgrad_fp8:       # eq. (8) and eq. (5) on codes: dense products of the decoded, decompressed operands, restricted to the sampled hidden units
        dq = f8.e4m3_decode(oracle.vnm_decompress(f8.quantize_fp8(s["dy1_vals"], sc["dy1"]), s["y2_meta"], s["colidx"])[:, cols]).astype(np.float64)
        want = dq.T @ f8.e4m3_decode(f8.quantize_fp8(inp["X"], sc["x"])).astype(np.float64) * np.float64(np.float32(sc["dy1"]) * np.float32(sc["x"]))
        assert_gemm_close(dW1[cols], oracle.f64_to_bits(want), "dW1")
        yq = f8.e4m3_decode(oracle.vnm_decompress(s["y2_codes"], s["y2_meta"], s["colidx"])[:, cols]).astype(np.float64)
        want = f8.e4m3_decode(f8.quantize_fp8(inp["dY"], sc["dy"])).astype(np.float64).T @ yq * np.float64(np.float32(sc["y2"]) * np.float32(sc["dy"]))
        assert_gemm_close(dW2[:, cols], oracle.f64_to_bits(want), "dW2")
    else:
        dense_dy1 = oracle.vnm_decompress(s["dy1_vals"], s["y2_meta"], s["colidx"])[:, cols]
        want = oracle.dense_nt(np.ascontiguousarray(dense_dy1.T), np.ascontiguousarray(inp["X"].T))
        assert_gemm_close(dW1[cols], want, "dW1")


@pytest.mark.parametrize("M", [16, 64])
def test_full_size_fp8_step_wide_blocks(M):
    """ffn_sparse_step_fp8 with blocks of 16 / 64 columns at the 7B layer in the timed configuration (fp8 weight gradients, no canonical copies
    of the packed weights): the packed activation bit-consistent with the oracle's compressor on sampled token blocks, eqs. (3), (7) on those
    blocks and eqs. (5), (8) on sampled hidden units against the oracle's fp8 contractions, teacher-forced on the GPU's packed operands."""
    from oracle import fp8 as f8
    T, D, F = CONFIGS["7b"]
    inp = make_ffn_inputs(T, D, F, seed=0)
    dev = {k: to_dev(v) for k, v in inp.items()}
    amax = lambda t: float(t.float().abs().max())
    sc = dict(x=amax(dev["X"]) / 448, w1=amax(dev["W1"]) / 448, w2=amax(dev["W2"]) / 448, y2=1.0, dy=amax(dev["dY"]) / 448, dy1=1.0)
    first = sffn.FfnStepFp8(T, D, F, sc, M=M)                       # the delayed-scaling loop: one call to learn the inner tensors' maxima
    first(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])
    sc = {k: v / 448 for k, v in first.amax_dict().items()}
    del first
    step = sffn.FfnStepFp8(T, D, F, sc, wgrad_fp8=True, lean=True, M=M)
    Y3, dX, dW1, dW2 = (to_bits(t) for t in step(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"]))
    s = {k: (to_bits(v) if v.dtype == torch.bfloat16 else v.cpu().numpy()) for k, v in step.saved().items()}
    rng = np.random.default_rng(M)
    rows = (np.sort(rng.choice(T // 64, 3, replace=False))[:, None] * 64 + np.arange(64)[None, :]).reshape(-1)      # three whole token blocks
    c1, m1 = f8.prune24_compress_fp8(inp["W1"], sc["w1"])
    xq = f8.quantize_fp8(inp["X"], sc["x"])
    y1_ref = f8.spmm24_fp8(xq[rows], sc["x"], c1, m1, sc["w1"], inp["b1"])
    yc, ym, cix = s["y2_codes"][rows], s["y2_meta"][rows], s["colidx"][rows[::64] // 64]
    # the column choice follows the GPU's own y1, which differs from the reference y1 by rounding: the kept columns' scores must be within
    # that rounding of the four largest, and the codes must decode to y2 of the reference y1 within fp8 spacing
    y2_ref = oracle.bits_to_f32(oracle.sqrelu(y1_ref))
    got = oracle.bits_to_f32(oracle.vnm_decompress(f8.codes_as_bf16_bits(yc), ym, cix, 64, M)) * np.float32(sc["y2"])
    nz = got != 0
    assert 0.2 / M < nz.mean() <= 2.0 / M
    assert np.all(np.abs(got[nz] - y2_ref[nz]) <= (2.0 ** -4 + 2.0 ** -6) * np.abs(y2_ref[nz]) + 2.0 ** -9 * sc["y2"])
    score = y2_ref.reshape(3, 64, F // M, M).sum(axis=1)                                  # [block of tokens, column block, column]
    kept = np.take_along_axis(score, cix.astype(np.int64), axis=2)
    fourth = -np.sort(-score, axis=2)[:, :, 3:4]
    assert np.all(kept >= fourth * (1 - 2.0 ** -6) - 1e-6)
    w2q = f8.quantize_fp8(inp["W2"], sc["w2"])
    assert_gemm_close(Y3[rows], f8.vnm_spmm_fp8(yc, ym, cix, sc["y2"], w2q, sc["w2"], 0, 64, M), "y3")
    dq = s["dy1_codes"]
    w1q = f8.quantize_fp8(inp["W1"], sc["w1"])
    assert_gemm_close(dX[rows], f8.vnm_spmm_fp8(dq[rows], ym, cix, sc["dy1"], w1q, sc["w1"], 1, 64, M), "dX")
    del w1q, w2q, c1, m1
    # weight gradients on codes for sampled blocks of hidden units, over all tokens
    cols = (np.sort(rng.choice(F // M, 2, replace=False))[:, None] * M + np.arange(M)[None, :]).reshape(-1)
    sub = lambda codes: oracle.vnm_decompress(np.ascontiguousarray(codes.reshape(T, F // M, 2)[:, cols[::M] // M].reshape(T, -1)),
                                              np.ascontiguousarray(_meta_cols(s["y2_meta"], cols[::M] // M)),
                                              np.ascontiguousarray(s["colidx"][:, cols[::M] // M]), 64, M)
    d1 = f8.e4m3_decode(sub(dq)).astype(np.float64)
    want = d1.T @ f8.e4m3_decode(xq).astype(np.float64) * np.float64(np.float32(sc["dy1"]) * np.float32(sc["x"]))
    assert_gemm_close(dW1[cols], oracle.f64_to_bits(want), "dW1")
    y2d = f8.e4m3_decode(sub(s["y2_codes"])).astype(np.float64)
    want = f8.e4m3_decode(f8.quantize_fp8(inp["dY"], sc["dy"])).astype(np.float64).T @ y2d * np.float64(np.float32(sc["y2"]) * np.float32(sc["dy"]))
    assert_gemm_close(dW2[:, cols], oracle.f64_to_bits(want), "dW2")


def _meta_cols(meta, blocks):
    """The metadata nibbles of the given column blocks, repacked two per byte ([T, len(blocks) / 2])."""
    nib = np.stack([meta & 0xF, meta >> 4], axis=-1).reshape(meta.shape[0], -1)[:, blocks]
    return (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)


def test_full_size_micro_batch_modes_are_bit_identical():
    """The 70B-scale layer in the modes a training loop uses: the second micro-batch on the packed weights of the first
    (SFFN_FLAG_WEIGHTS_PACKED) through the separate forward / backward calls, weight gradients added to float32 buffers
    (SFFN_FLAG_DW_FP32_ACCUMULATE).  Checked against the plain one-call step, which the tests above check against the oracle: Y3 and dX
    bit for bit; from zero, the float32 buffers round to the plain step's bf16 dW1 / dW2 bit for bit."""
    T, D, F = CONFIGS["70b"]
    inp = make_ffn_inputs(T, D, F, seed=0)
    dev = {k: to_dev(v) for k, v in inp.items()}
    plain = sffn.FfnStep(T, D, F, lean=True)
    want = [to_bits(t).copy() for t in plain(dev["X"], dev["W1"], dev["W2"], dev["b1"], dev["dY"])]
    del plain
    torch.cuda.empty_cache()
    step = sffn.FfnStep(T, D, F, lean=True, dw_fp32=True)
    X0 = torch.flip(dev["X"], (0,)).contiguous()
    step.forward(X0, dev["W1"], dev["W2"], dev["b1"])                        # micro-batch 0 packs the weights (its gradients are not taken)
    y3 = to_bits(step.forward(dev["X"], dev["W1"], dev["W2"], dev["b1"], weights_packed=True))
    assert np.array_equal(y3, want[0])
    dX, dW1, dW2 = step.backward(dev["W1"], dev["dY"])
    assert np.array_equal(to_bits(dX), want[1])
    assert np.array_equal(to_bits(dW1.to(torch.bfloat16)), want[2])
    assert np.array_equal(to_bits(dW2.to(torch.bfloat16)), want[3])
