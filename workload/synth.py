"""Seeded synthetic FFN workloads.

These stand in for the Llama-style FFN activations and weights of the paper's experiments
(Table 1 gives d_model / d_ffn for the 1B and 7B models), which need datasets and trained
weights.  What is reproduced: shapes, bf16 storage, Gaussian statistics and the fraction of
SquaredReLU outputs that are zero (the paper reports more than 90 %), set through a per-neuron
pre-activation bias.  Tensors are returned as numpy uint16 bf16 bit patterns.
"""
import numpy as np

# name -> (tokens T, d_model D, d_ff F)
CONFIGS = {
    "tiny": (512, 256, 1024),        # single small layer; the CPU oracle finishes in well under a second
    "1b": (8192, 2048, 8192),        # Table 1, Llama 1B FFN; batch 4 x seq 2048
    "7b": (16384, 4096, 16384),      # Table 1, Llama 7B FFN; batch 4 x seq 4096
    "70b": (8192, 8192, 28672),      # 70B-scale layer
    "moe_expert": (16384 * 2 // 8, 4096, 14336),  # one expert's mean share of 16384 tokens routed top-2 over 8
}

# standard-normal quantiles: P(N(0,1) < z) = zero fraction of the SquaredReLU output
Z_FOR_ZERO_FRACTION = {0.50: 0.0, 0.75: 0.6744897501960817, 0.90: 1.2815515655446004, 0.95: 1.6448536269514722}


def bf16_bits_from_f32(x):
    """float32 -> bf16 bit pattern, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(np.asarray(x, dtype=np.float32)).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def _bits_to_f64(b):
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def neuron_std(W1):
    """Standard deviation of every neuron's pre-activation under X ~ N(0, 1) once the two smallest magnitudes of every
    four consecutive weights are dropped: the root of the sum, over groups, of the two largest squares (float64).
    (Closed form of the workload's statistics, not the sparsifier: no positions, no packing, no tie rule.)"""
    F, D = W1.shape
    out = np.empty(F, dtype=np.float64)
    step = max(1, (1 << 24) // D)
    for r in range(0, F, step):                   # row chunks keep the float64 temporaries small
        q = _bits_to_f64(W1[r:r + step]) ** 2
        a, b, c, d = q[:, 0::4], q[:, 1::4], q[:, 2::4], q[:, 3::4]
        hi1, lo1, hi2, lo2 = np.maximum(a, b), np.minimum(a, b), np.maximum(c, d), np.minimum(c, d)
        top = np.stack([np.maximum(np.minimum(hi1, hi2), np.maximum(lo1, lo2)), np.maximum(hi1, hi2)], axis=-1)   # 2nd largest, largest
        out[r:r + step] = np.sqrt(top.sum(axis=(1, 2)))
    return out


def bias_for_zero_fraction(std, zero_fraction):
    """b1 [F] float32 = -z * std with z the standard-normal quantile of the wanted SquaredReLU zero fraction."""
    z = Z_FOR_ZERO_FRACTION[zero_fraction] if zero_fraction in Z_FOR_ZERO_FRACTION else float(zero_fraction)
    return (-z * std).astype(np.float32)


def make_ffn_inputs(T, D, F, seed=0, zero_fraction=0.90, w_std=0.02):
    """X [T, D] ~ N(0,1), W1 [F, D] and W2 [D, F] ~ N(0, w_std^2), dY [T, D] ~ N(0,1), all bf16 bits;
    b1 [F] float32 = -z * s_f where s_f is the standard deviation of neuron f's pre-activation
    under X ~ N(0,1) once W1's two smallest magnitudes of every four along D are dropped, i.e.
    the root of the sum, over groups, of the two largest squares."""
    rng = np.random.default_rng(seed)
    X = bf16_bits_from_f32(rng.standard_normal((T, D), dtype=np.float32))
    W1 = bf16_bits_from_f32(rng.standard_normal((F, D), dtype=np.float32) * np.float32(w_std))
    W2 = bf16_bits_from_f32(rng.standard_normal((D, F), dtype=np.float32) * np.float32(w_std))
    dY = bf16_bits_from_f32(rng.standard_normal((T, D), dtype=np.float32))
    b1 = bias_for_zero_fraction(neuron_std(W1), zero_fraction)
    return dict(X=X, W1=W1, W2=W2, b1=b1, dY=dY)


def make_ffn_sweep(T, D, F, zero_fractions, seed=0, w_std=0.02):
    """The inputs of make_ffn_inputs for several zero fractions: X, W1, W2, dY are the same arrays (same seed), only the
    bias shift differs.  Yields (zero_fraction, inputs)."""
    base = make_ffn_inputs(T, D, F, seed, zero_fractions[0], w_std)
    std = neuron_std(base["W1"])
    for zf in zero_fractions:
        yield zf, dict(base, b1=bias_for_zero_fraction(std, zf))


def make_moe_segments(n_tokens=16384, n_experts=8, top_k=2, seed=0, align=64):
    """Top-k routing from N(0,1) logits: per-expert token counts and 64-row-aligned segment offsets."""
    rng = np.random.default_rng(seed)
    logits = rng.standard_normal((n_tokens, n_experts), dtype=np.float32)
    top = np.argsort(-logits, axis=1, kind="stable")[:, :top_k]
    counts = np.bincount(top.reshape(-1), minlength=n_experts).astype(np.int64)
    padded = (counts + align - 1) // align * align
    offsets = np.concatenate([[0], np.cumsum(padded)]).astype(np.int64)
    return counts, offsets


def make_moe_inputs(n_tokens, n_experts, top_k, D, F, seed=0, zero_fraction=0.90, w_std=0.02, align=64):
    """Grouped-FFN workload: `n_tokens` tokens routed top-k over `n_experts` experts by N(0,1) logits (uneven
    counts from the seed).  Each expert's slots are consecutive rows, padded with zero rows to a multiple of
    `align`; expert e's weights and bias come from make_ffn_inputs' recipe with seed + e, its rows from a
    generator of their own.  Returns X, dY [T, D], W1 [E, F, D], W2 [E, D, F], b1 [E, F], counts, seg (offsets)."""
    counts, seg = make_moe_segments(n_tokens, n_experts, top_k, seed, align)
    T = int(seg[-1])
    X = np.zeros((T, D), dtype=np.uint16)
    dY = np.zeros((T, D), dtype=np.uint16)
    W1 = np.empty((n_experts, F, D), dtype=np.uint16)
    W2 = np.empty((n_experts, D, F), dtype=np.uint16)
    b1 = np.empty((n_experts, F), dtype=np.float32)
    for e in range(n_experts):
        part = make_ffn_inputs(int(counts[e]), D, F, seed + e, zero_fraction, w_std)
        a = int(seg[e])
        X[a:a + int(counts[e])] = part["X"]
        dY[a:a + int(counts[e])] = part["dY"]
        W1[e], W2[e], b1[e] = part["W1"], part["W2"], part["b1"]
    return dict(X=X, W1=W1, W2=W2, b1=b1, dY=dY, counts=counts, seg=seg)


def make_router_inputs(T, D, F, M, seed=0, zero_fraction=0.90, w_std=0.02):
    """Workload of the neuron-level router (Section 3.3): make_ffn_inputs plus the E = M / 4 expert means.
    Expert e owns the hidden units f with (f mod M) / 4 == e (the offline clustering, taken as already applied to
    the row order of W1); its mean is the average of those rows of W1 plus a random direction of comparable
    size (random weights have no cluster structure of their own), normalised to unit length and stored as bf16.
    Tokens then split unevenly but not degenerately over the experts."""
    inp = make_ffn_inputs(T, D, F, seed, zero_fraction, w_std)
    rng = np.random.default_rng(seed + 1000)
    E = M // 4
    w = _bits_to_f64(inp["W1"])
    f = np.arange(F)
    means = np.empty((E, D), dtype=np.float64)
    for e in range(E):
        m = w[(f % M) // 4 == e].mean(axis=0)
        m = m + rng.standard_normal(D) * np.linalg.norm(m) / np.sqrt(D) * (1.0 + 0.5 * e / max(E - 1, 1))
        means[e] = m / np.linalg.norm(m)
    inp["means"] = bf16_bits_from_f32(means.astype(np.float32))
    return inp
