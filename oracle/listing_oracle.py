"""Blocked fp64 evaluation of the paper's FUSED block programs (numpy).

TEST INFRASTRUCTURE ONLY (same rule as oracle.py).  This is the second,
independent check of the definition oracle: it evaluates the fully fused loop
nests that the paper's fusion algorithm ends with,

  * Example 3, last step (Flash-RMSNorm+FFN-SwiGLU): per (m, n) output block a
    serial loop over hidden blocks k, inside it a serial loop over model-dim
    blocks d that accumulates the row sum of squares and both products with
    the transposed weight blocks; the inverse norm is applied to the two
    products AFTER the dots (Rule 4, swap scale/dot), then Swish, Hadamard
    product and the dot with the transposed down-projection block;
  * Example 2, last step (Flash-LayerNorm+Matmul): per (m, n) one loop over k
    accumulating row sums, row sums of squares, the row sums of the transposed
    weight block and the dot; afterwards the rank-one correction
    outer(-mean, column sums) is added (Rule 5, swap shift/dot) and the rows
    are scaled by the inverse standard deviation (Rule 4);
  * Example 3's first snapshot (taken before any map extension), where the
    hidden is produced block by block and then consumed by the N-map,

using only the block operators of the paper's Table 1, for arbitrary block
counts.  The extensions the paper does not have (1/D in the mean, eps, the
gain vectors) are placed where linearity allows them to go:

  xh W   = diag(r) ((X diag(g)) W)
  LN(X)W = diag(r) ((X diag(gamma)) W - mu (gamma^T W)) + 1 (beta^T W)

Agreement of these nests with the unfused definition for every block
splitting is the paper's claim that the rules are logic preserving and that
block shapes do not change the result.
"""
from __future__ import annotations

import numpy as np


# --- Table 1: functional block operators -----------------------------------
def row_sum(a):            # sum of each row of a block -> vector of length rows
    return a.sum(axis=1)


def row_scale(a, c):       # multiply row i by c[i]
    return a * c[:, None]


def dot(a, b):             # a times the transpose of b
    return a @ b.T


def outer(a, b):
    return np.outer(a, b)


def add(a, b):
    return a + b


def mul(a, b):
    return a * b


def _splits(n: int, parts: int):
    """parts contiguous index ranges covering range(n) (sizes differ by <= 1)."""
    edges = np.linspace(0, n, parts + 1).round().astype(int)
    return [slice(int(edges[i]), int(edges[i + 1])) for i in range(parts)]


def bf16_bits_to_f64(a) -> np.ndarray:
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


# --- building blocks of the fused nests (each is one stage of a nest, evaluated block by block) ----------
def _prepared_ffn(X, g, W1, W3, W2):
    """fp64 operands; the gain is folded into the transposed up-projections: (X diag(g)) W = X (diag(g) W)"""
    X, g, W1, W3, W2 = (bf16_bits_to_f64(t) for t in (X, g, W1, W3, W2))
    return X, (g[:, None] * W1).T, (g[:, None] * W3).T, W2.T       # X [M,D], WT, VT [F,D], UT [D,F]


def _sum_of_squares(X, m, dblocks):
    """row sums of squares of the row block, accumulated over the model-dimension blocks"""
    return sum(row_sum(X[m, d] ** 2) for d in dblocks)


def _products(X, WT, VT, m, k, dblocks):
    """the two contractions of row block m with the transposed weight blocks of hidden block k,
    accumulated over the model-dimension blocks (one pass over X[m, :] serves both)"""
    p = sum(dot(X[m, d], WT[k, d]) for d in dblocks)
    q = sum(dot(X[m, d], VT[k, d]) for d in dblocks)
    return p, q


def _hidden_block(p, q, r):
    """inverse norm applied to the finished products (Rule 4), Swish on one, Hadamard product with the other"""
    ps, qs = row_scale(p, r), row_scale(q, r)
    return mul(ps / (1.0 + np.exp(-ps)), qs)


def fused_rmsnorm_swiglu_ffn(X, g, W1, W3, W2, eps, nM=1, nN=1, nK=1, nD=1):
    """Example 3, final fused nest, with block counts (nM, nN, nK, nD) for the row, output-column,
    hidden and model dimensions.  Everything lives under the (m, n) maps: for every hidden block the
    statistics and both products are recomputed from X (the replicated work of the extended maps),
    and the output block accumulates the hidden blocks' contributions one after the other."""
    X, WT, VT, UT = _prepared_ffn(X, g, W1, W3, W2)
    M, D = X.shape
    F = WT.shape[0]
    dblocks = _splits(D, nD)
    O = np.zeros((M, D))
    for m in _splits(M, nM):
        for n in _splits(D, nN):
            out = 0.0
            for k in _splits(F, nK):
                # (in the nest the statistics ride along in the products' loop over d: same sums)
                r = 1.0 / np.sqrt(_sum_of_squares(X, m, dblocks) / D + eps)
                h = _hidden_block(*_products(X, WT, VT, m, k, dblocks), r)
                out = out + dot(h, UT[n, k])
            O[m, n] = out
    return O


def snapshot1_rmsnorm_swiglu_ffn(X, g, W1, W3, W2, eps, nM=1, nN=1, nK=1, nD=1):
    """Example 3, first snapshot (before the N-map is extended): statistics once per row block, a
    K-map that writes the hidden blocks to a list in global memory, then an N-map that reduces over it."""
    X, WT, VT, UT = _prepared_ffn(X, g, W1, W3, W2)
    M, D = X.shape
    F = WT.shape[0]
    dblocks, kblocks = _splits(D, nD), _splits(F, nK)
    O = np.zeros((M, D))
    for m in _splits(M, nM):
        r = 1.0 / np.sqrt(_sum_of_squares(X, m, dblocks) / D + eps)
        hidden = [_hidden_block(*_products(X, WT, VT, m, k, dblocks), r) for k in kblocks]   # the buffered list
        for n in _splits(D, nN):
            O[m, n] = sum(dot(h, UT[n, k]) for h, k in zip(hidden, kblocks))
    return O


def fused_layernorm_matmul(X, gamma, beta, W, eps, nM=1, nN=1, nK=1):
    """Example 2, final fused nest, with block counts (nM, nN, nK) for rows, output columns and the
    contraction dimension: under the (m, n) maps ONE loop over k gathers the row sums and row sums of
    squares of X, the column sums of the gain-scaled and of the bias-scaled weight block, and the
    product; mean and deviation are applied to the finished product (Rules 5 and 4)."""
    X, gamma, beta, W = (bf16_bits_to_f64(t) for t in (X, gamma, beta, W))
    M, KK = X.shape
    N = W.shape[1]
    YT = (gamma[:, None] * W).T          # [N, KK]  gain folded into the weights
    BT = (beta[:, None] * W).T           # [N, KK]  its column sums are the bias row beta^T W
    kblocks = _splits(KK, nK)
    Z = np.zeros((M, N))
    for m in _splits(M, nM):
        for n in _splits(N, nN):
            sums = {"x": 0.0, "xx": 0.0, "colw": 0.0, "colb": 0.0, "xw": 0.0}
            for k in kblocks:
                x, yt = X[m, k], YT[n, k]
                for name, term in (("x", row_sum(x)), ("xx", row_sum(x ** 2)), ("colw", row_sum(yt)),
                                   ("colb", row_sum(BT[n, k])), ("xw", dot(x, yt))):
                    sums[name] = sums[name] + term
            mean = sums["x"] / KK
            rstd = (sums["xx"] / KK - mean ** 2 + eps) ** (-0.5)
            centred = add(outer(-mean, sums["colw"]), sums["xw"])      # (x - mean) gamma W without forming x - mean
            Z[m, n] = row_scale(centred, rstd) + sums["colb"][None, :]
    return Z


# ============================================================ Example 1
def fused_attention(Q, K, V, nM=1, nN=1, nD=1, nL=1):
    """Example 1's final fused nest (the "unsafe" Flash Attention the fusion algorithm ends with):
    under the (m, l) maps a serial loop over key blocks; the score block of a key block is a
    contraction over the feature blocks, its plain exponential (no stabilisation) feeds both running
    sums - the row sums and the product with the transposed value block - and the rows are divided
    by the row sums at the very end.  Q [M,d], K [N,d], V [N,L] float64."""
    Mt, dt = Q.shape
    Nt, Lt = V.shape
    rows, keys = np.array_split(np.arange(Mt), nM), np.array_split(np.arange(Nt), nN)
    feats, vals = np.array_split(np.arange(dt), nD), np.array_split(np.arange(Lt), nL)
    VT = V.T
    O = np.empty((Mt, Lt))

    def exp_scores(m, n):
        return np.exp(sum(dot(Q[np.ix_(m, d)], K[np.ix_(n, d)]) for d in feats) * (dt ** -0.5))

    for m in rows:
        for l in vals:
            denominator = np.zeros(len(m))
            numerator = np.zeros((len(m), len(l)))
            for n in keys:
                e = exp_scores(m, n)
                denominator = add(denominator, row_sum(e))
                numerator = add(numerator, dot(e, VT[np.ix_(l, n)]))
            O[np.ix_(m, l)] = row_scale(numerator, 1.0 / denominator)
    return O


# --- the Appendix: numbers as significand-exponent pairs (s, t) = s * e^t ---
# Here in its row-wise form: a block carries one exponent per row.
def se_exp(X):
    """elementwise exp of a block as (significands, row exponents)"""
    z = X.max(axis=1)
    return np.exp(X - z[:, None]), z


def se_add(a, b):
    """(S1,t1) + (S2,t2) with a common exponent z = max(t1,t2) per row; S may be
    a block or a vector of per-row values"""
    (S1, t1), (S2, t2) = a, b
    z = np.maximum(t1, t2)
    w1, w2 = np.exp(t1 - z), np.exp(t2 - z)
    if S1.ndim == 2:
        return S1 * w1[:, None] + S2 * w2[:, None], z
    return S1 * w1 + S2 * w2, z


def safe_attention(Q, K, V, nM=1, nN=1):
    """The same nest with the Appendix's numerical safety: every exponentiated
    block is a (significand block, per-row exponent) pair, sums of pairs are
    brought to the larger exponent, the final division is a division of pairs.
    This is the form the GPU kernel follows (row-wise shared exponents)."""
    Mt, dt = Q.shape
    Nt, Lt = V.shape
    O = np.empty((Mt, Lt))
    for m in np.array_split(np.arange(Mt), nM):
        den = (np.zeros(len(m)), np.full(len(m), -np.inf))        # the number 0
        num = (np.zeros((len(m), Lt)), np.full(len(m), -np.inf))
        for n in np.array_split(np.arange(Nt), nN):
            S, t = se_exp(dot(Q[m], K[n]) * (dt ** -0.5))
            den = se_add(den, (row_sum(S), t))
            num = se_add(num, (dot(S, V[n].T), t))
        # (num_S e^{num_t}) / (den_S e^{den_t}): both carry the same exponent history
        O[m] = row_scale(num[0], 1.0 / den[0]) * np.exp(num[1] - den[1])[:, None]
    return O
