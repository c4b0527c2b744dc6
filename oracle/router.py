"""Neuron-level experts that produce the V:N:M format directly (CPU oracle, test infrastructure only).

Paper: Section 3.3 and Alg. 3 ("Convert Activation to Venom"): W1's hidden units are clustered offline into
non-overlapping subsets ("experts"); per step (1) every token picks its experts from x @ ExpertMeans, (2) tokens
are permuted so that tokens of one expert are adjacent, (3) a batched matmul multiplies each token group with its
expert's slice of W1; the result is a V:N:M matrix.  Section 3.4 lists the same three steps as the conversion cost.

Readings fixed here because the paper is silent, garbled or at odds with itself:
  * Experts and the format.  A V:N:M block keeps 4 of its M columns, so the format holds exactly one expert's
    columns per block: there are E = M / 4 experts, expert e owns the hidden units f with (f mod M) / 4 == e
    (the offline clustering is a fixed re-ordering of W1's rows that puts them there), and a token goes to ONE
    expert (Alg. 3's inner loop over "expertids" has one iteration).
  * Similarity.  The text says cosine distance in one place and the product x @ ExpertMeans in another.  The means
    are taken unit-normalised (an offline step), which makes the dot product rank experts exactly as the cosine
    does; expert(t) = argmax_e s[t, e], ties to the lower e.
  * Arithmetic of s (it decides an integer, so it is part of the contract): float32; the D products x[t, d] *
    mean[e, d] (exact in float32 for bf16 factors) are cut into chunks of 8 consecutive d; partial sum p_l,
    l = 0..63, accumulates the chunks l, l + 64, l + 128, ... in ascending d (start +0, one rounding per add); the
    64 partials are then folded p_l + p_(l + 32) for l < 32, then + 16, 8, 4, 2, 1.
  * Permutation.  Stable: inside an expert's run tokens keep ascending order; every run is padded to a multiple of
    V = 64 rows; perm[r] is the token of row r or -1 for a padding row; the row capacity is ceil64(T) + 64 E, rows
    past the last run are padding too.
  * Batched matmul.  Row r of expert e's run holds, for compact column j, hidden unit row(e, j) = (j / 4) M + 4 e +
    j % 4: y1c[r, j] = bf16(x[perm[r]] . W1s[row(e, j)] + b1[row(e, j)]) with W1s the 2:4-pruned W1 of Alg. 1 line 4.
    Then eq. (2) and the 2:4 rule of Section 2.3 on each group of four consecutive compact columns (they are the four
    kept columns of one block).  Padding rows are all +0.  colidx of every block in expert e's run is (4e, ..., 4e+3).
"""
import numpy as np
from .bf16 import bits_to_f32, bits_to_f64, f64_to_bits
from .sparse24 import prune24_compress, prune24_dense, HARD
from .vnm import sqrelu, vnm_decompress, dsqrelu_vnm
from .gemm import vnm_spmm, vnm_wgrad, dense_nt


def route_scores_plain(x_bits, means_bits):
    """THE DEFINITION (Section 3.3, step 1; Alg. 3's similarity): s = x @ ExpertMeans, here in float64 through the
    library matmul, no summation order implied.  route_top1 of it is the expert the paper's rule picks."""
    return bits_to_f64(np.asarray(x_bits, dtype=np.uint16)) @ bits_to_f64(np.asarray(means_bits, dtype=np.uint16)).T


def route_margin_is_clear(x_bits, means_bits):
    """Per token: does the definition decide the expert whatever the order of the float32 summation?  True where the
    float64 gap between the best and the second-best score exceeds the sum of the two experts' rounding bounds
    14 * 2^-24 * sum_d |x||mean| (8 sequential + 6 tree additions of the stated order; any order with as few
    roundings per term stays inside it)."""
    x, m = bits_to_f64(np.asarray(x_bits, dtype=np.uint16)), bits_to_f64(np.asarray(means_bits, dtype=np.uint16))
    s, bound = x @ m.T, 14 * 2.0 ** -24 * (np.abs(x) @ np.abs(m).T)
    if s.shape[1] < 2:
        return np.ones(s.shape[0], dtype=bool)
    order = np.argsort(-s, axis=1, kind="stable")
    t = np.arange(s.shape[0])
    e1, e2 = order[:, 0], order[:, 1]
    return (s[t, e1] - s[t, e2]) > (bound[t, e1] + bound[t, e2])


def route_scores(x_bits, means_bits):
    """s[t, e] in float32.  NOT part of the definition but the contract's choice of ONE summation order (the paper fixes
    none), needed because the score decides an integer: everything from here to the end of this function restates the
    order given in the module header, so that near-ties resolve identically on both sides.  Away from near-ties the
    order is immaterial: route_top1(route_scores) == route_top1(route_scores_plain) wherever route_margin_is_clear.
    D must be a multiple of 8."""
    x = bits_to_f32(np.asarray(x_bits, dtype=np.uint16))
    m = bits_to_f32(np.asarray(means_bits, dtype=np.uint16))
    T, D = x.shape
    E = m.shape[0]
    assert D % 8 == 0 and m.shape[1] == D
    p = np.zeros((T, E, 64), dtype=np.float32)
    lane_d = 8 * np.arange(64)
    for base in range(0, D, 512):                        # chunks base / 8 + l, l = 0..63, of this round
        for k in range(8):
            d = base + lane_d + k
            live = d < D                                 # a lane whose chunk does not exist adds nothing
            prod = np.zeros((T, E, 64), dtype=np.float32)
            prod[:, :, live] = x[:, None, d[live]] * m[None, :, d[live]]           # exact in float32
            p = np.where(live[None, None, :], (p + prod).astype(np.float32), p)
    w = 32
    while w >= 1:
        p = (p[..., :w] + p[..., w:2 * w]).astype(np.float32)
        w //= 2
    return p[..., 0]


def route_top1(scores):
    """expert[t] = argmax_e scores[t, e], ties to the lower e."""
    return np.argmax(scores, axis=1).astype(np.int32)          # numpy returns the first maximum


def expert_permutation(expert, E, V=64):
    """Returns (perm int32 [Tcap], seg int64 [E + 1]): stable grouping of tokens by expert, runs padded to V rows."""
    expert = np.asarray(expert)
    T = expert.shape[0]
    cap = (T + V - 1) // V * V + V * E
    perm = np.full(cap, -1, dtype=np.int32)
    seg = np.zeros(E + 1, dtype=np.int64)
    for e in range(E):
        tok = np.nonzero(expert == e)[0]                        # ascending
        perm[seg[e]:seg[e] + len(tok)] = tok
        seg[e + 1] = seg[e] + (len(tok) + V - 1) // V * V
    return perm, seg


def cluster_rows(e, M, F):
    """Hidden units of expert e in compact-column order: row(e, j) = (j / 4) M + 4 e + j % 4."""
    j = np.arange(4 * F // M)
    return (j // 4) * M + 4 * e + j % 4


def expert_matmul(x_bits, perm, seg, w1_bits, b1, M, mode=HARD):
    """Step 3: y1c [Tcap, 4F/M] bf16 bits (padding rows: +0)."""
    x_bits = np.asarray(x_bits, dtype=np.uint16)
    F = w1_bits.shape[0]
    w1s = prune24_dense(w1_bits, mode)
    y1c = np.zeros((len(perm), 4 * F // M), dtype=np.uint16)
    for e in range(len(seg) - 1):
        rows = cluster_rows(e, M, F)
        r = np.arange(seg[e], seg[e + 1])
        r = r[perm[r] >= 0]
        acc = bits_to_f64(x_bits[perm[r]]) @ bits_to_f64(w1s[rows]).T
        if b1 is not None:
            acc = acc + np.asarray(b1, dtype=np.float32).astype(np.float64)[rows][None, :]
        y1c[r] = f64_to_bits(acc)
    return y1c


def venom_from_compact(y1c_bits, perm, seg, M, V=64):
    """eq. (2) + 2:4 on every group of four compact columns -> (vals [Tcap, 2F/M], meta [Tcap, F/(2M)],
    colidx [Tcap/V, F/M, 4]).  Padding rows are +0 with the metadata of an all-zero group."""
    y1c_bits = np.asarray(y1c_bits, dtype=np.uint16)
    cap, Kc = y1c_bits.shape
    y2 = sqrelu(y1c_bits)
    y2[np.asarray(perm) < 0] = 0
    vals, meta = prune24_compress(y2, HARD)
    colidx = np.zeros((cap // V, Kc // 4, 4), dtype=np.uint8)
    colidx[:] = np.arange(4, dtype=np.uint8)                    # rows past the last run: expert 0's columns, all-zero values
    for e in range(len(seg) - 1):
        colidx[seg[e] // V:seg[e + 1] // V] = (4 * e + np.arange(4)).astype(np.uint8)
    return vals, meta, colidx


def moe_to_venom(x_bits, w1_bits, b1, means_bits, M, mode=HARD, V=64):
    """Alg. 3 end to end.  Returns dict(expert, perm, seg, y1c, vals, meta, colidx)."""
    E = M // 4
    assert means_bits.shape[0] == E
    expert = route_top1(route_scores(x_bits, means_bits))
    perm, seg = expert_permutation(expert, E, V)
    y1c = expert_matmul(x_bits, perm, seg, w1_bits, b1, M, mode)
    vals, meta, colidx = venom_from_compact(y1c, perm, seg, M, V)
    return dict(expert=expert, perm=perm, seg=seg, y1c=y1c, vals=vals, meta=meta, colidx=colidx)


def scatter_compact(c_bits, seg, M, F):
    """[rows, 4F/M] in compact-column order -> [rows, F] with every run's columns at its expert's hidden units."""
    full = np.zeros((c_bits.shape[0], F), dtype=np.uint16)
    for e in range(len(seg) - 1):
        rows = slice(int(seg[e]), int(seg[e + 1]))
        full[rows][:, cluster_rows(e, M, F)] = c_bits[rows]
    return full


def ffn_router_step_ref(x_bits, w1_bits, w2_bits, b1, dy_bits, means_bits, M, mode=HARD, V=64):
    """Alg. 1 + Alg. 2 with Alg. 3 as the activation sparsifier: the forward computes only the routed expert's hidden
    units, and every later contraction sees the resulting V:N:M matrix (in permuted row order, padding rows zero).
    The backward is Alg. 2 on that matrix: dy2 = dY @ sparsify24(W2.T) (needed only at the kept slots), eq. (6) on
    y2's mask, dX with the dense W1, both weight gradients (rows of hidden units no token was routed to get exact
    zeros from the empty sum).  Y3 and dX are returned in token order."""
    r = moe_to_venom(x_bits, w1_bits, b1, means_bits, M, mode, V)
    perm, seg = r["perm"], r["seg"]
    T, D = np.asarray(x_bits).shape
    F = np.asarray(w1_bits).shape[0]
    real = perm >= 0
    xp = np.zeros((len(perm), D), dtype=np.uint16)
    dyp = np.zeros((len(perm), D), dtype=np.uint16)
    xp[real], dyp[real] = np.asarray(x_bits)[perm[real]], np.asarray(dy_bits)[perm[real]]
    y3p = vnm_spmm(r["vals"], r["meta"], r["colidx"], w2_bits, 0, V, M)                       # eq. (3), dense W2
    w2t_s = prune24_dense(np.ascontiguousarray(np.asarray(w2_bits).T), mode)                   # sparsify24(W2.T), 2:4 along d_model
    dy2 = dense_nt(dyp, w2t_s)                                                                 # eq. (4) [rows, F]
    y1_full = scatter_compact(r["y1c"], seg, M, F)
    dvals = dsqrelu_vnm(dy2, y1_full, r["meta"], r["colidx"], V, M)                            # eq. (6) on y2's mask
    dxp = vnm_spmm(dvals, r["meta"], r["colidx"], w1_bits, 1, V, M)                            # eq. (7), dense W1
    dW2 = vnm_wgrad(r["vals"], r["meta"], r["colidx"], dyp, 0, V, M)                           # eq. (5)
    dW1 = vnm_wgrad(dvals, r["meta"], r["colidx"], xp, 1, V, M)                                # eq. (8)
    row_of_token = np.empty(T, dtype=np.int64)
    row_of_token[perm[real]] = np.nonzero(real)[0]
    dy2c = np.zeros_like(r["y1c"])
    for e in range(len(seg) - 1):
        rows = slice(int(seg[e]), int(seg[e + 1]))
        dy2c[rows] = dy2[rows][:, cluster_rows(e, M, F)]
    r.update(row_of_token=row_of_token, y3p=y3p, dy2c=dy2c, dvals=dvals, dxp=dxp,
             y3=y3p[row_of_token], dX=dxp[row_of_token], dW1=dW1, dW2=dW2)
    return r
