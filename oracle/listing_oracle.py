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


def fused_rmsnorm_swiglu_ffn(X, g, W1, W3, W2, eps, nM=1, nN=1, nK=1, nD=1):
    """Example 3, final fused nest, with block counts (nM, nN, nK, nD) for the
    row, output-column, hidden and model dimensions."""
    X, g, W1, W3, W2 = (bf16_bits_to_f64(t) for t in (X, g, W1, W3, W2))
    M, D = X.shape
    F = W1.shape[1]
    WT = (g[:, None] * W1).T              # [F, D]  gain folded: (X diag(g)) W
    VT = (g[:, None] * W3).T              # [F, D]
    UT = W2.T                             # [D_out, F]
    O = np.zeros((M, D))
    for m in _splits(M, nM):                       # forall m
        for n in _splits(D, nN):                   # forall n
            acc_o = 0.0
            for k in _splits(F, nK):               # for k (serial reduction)
                ssq = 0.0
                p = 0.0
                q = 0.0
                for d in _splits(D, nD):           # for d (serial reduction)
                    x = X[m, d]
                    ssq = ssq + row_sum(x ** 2)
                    p = p + dot(x, WT[k, d])
                    q = q + dot(x, VT[k, d])
                r = 1.0 / np.sqrt(ssq / D + eps)
                ps = row_scale(p, r)
                sw = ps / (1.0 + np.exp(-ps))
                qs = row_scale(q, r)
                h = mul(sw, qs)
                acc_o = acc_o + dot(h, UT[n, k])
            O[m, n] = acc_o
    return O


def snapshot1_rmsnorm_swiglu_ffn(X, g, W1, W3, W2, eps, nM=1, nN=1, nK=1, nD=1):
    """Example 3, first snapshot (before the N-map is extended): statistics
    once per row block, a K-map that writes the hidden blocks to a global
    buffer, then an N-map that reduces over them."""
    X, g, W1, W3, W2 = (bf16_bits_to_f64(t) for t in (X, g, W1, W3, W2))
    M, D = X.shape
    F = W1.shape[1]
    WT = (g[:, None] * W1).T
    VT = (g[:, None] * W3).T
    UT = W2.T
    O = np.zeros((M, D))
    for m in _splits(M, nM):
        ssq = 0.0
        for d in _splits(D, nD):
            ssq = ssq + row_sum(X[m, d] ** 2)
        r = 1.0 / np.sqrt(ssq / D + eps)
        hidden = {}                                 # the buffered edge I1[m, k]
        for ki, k in enumerate(_splits(F, nK)):
            p = 0.0
            q = 0.0
            for d in _splits(D, nD):
                x = X[m, d]
                p = p + dot(x, WT[k, d])
                q = q + dot(x, VT[k, d])
            ps = row_scale(p, r)
            hidden[ki] = mul(ps / (1.0 + np.exp(-ps)), row_scale(q, r))
        for n in _splits(D, nN):
            acc = 0.0
            for ki, k in enumerate(_splits(F, nK)):
                acc = acc + dot(hidden[ki], UT[n, k])
            O[m, n] = acc
    return O


def fused_layernorm_matmul(X, gamma, beta, W, eps, nM=1, nN=1, nK=1):
    """Example 2, final fused nest, with block counts (nM, nN, nK) for rows,
    output columns and the contraction dimension."""
    X, gamma, beta, W = (bf16_bits_to_f64(t) for t in (X, gamma, beta, W))
    M, KK = X.shape
    N = W.shape[1]
    YT = (gamma[:, None] * W).T          # [N, KK]  gain folded into the weights
    BT = (beta[:, None] * W).T           # [N, KK]  bias row: beta^T W after row_sum
    Z = np.zeros((M, N))
    for m in _splits(M, nM):
        for n in _splits(N, nN):
            s1 = 0.0
            s2 = 0.0
            col = 0.0
            bia = 0.0
            acc = 0.0
            for k in _splits(KK, nK):
                x = X[m, k]
                s1 = s1 + row_sum(x)
                s2 = s2 + row_sum(x ** 2)
                yt = YT[n, k]
                col = col + row_sum(yt)
                bia = bia + row_sum(BT[n, k])
                acc = acc + dot(x, yt)
            negmu = -s1 / KK
            rstd = (s2 / KK - negmu ** 2 + eps) ** (-0.5)
            t = add(outer(negmu, col), acc)
            t = row_scale(t, rstd)
            Z[m, n] = t + bia[None, :]
    return Z


# ============================================================ Example 1
def fused_attention(Q, K, V, nM=1, nN=1, nD=1, nL=1):
    """Example 1's final fused nest (the "unsafe" Flash Attention the fusion
    algorithm ends with): per (m, l) output block a serial loop over key blocks
    n; inside it a serial loop over feature blocks d accumulates the dot of the
    query block with the key block; the scaled scores are exponentiated block by
    block, their row sums and the dot with the transposed value block are
    accumulated, and the rows are divided by the accumulated row sums at the
    end.  No stabilisation: plain exp.  Q [M,d], K [N,d], V [N,L] float64."""
    Mt, dt = Q.shape
    Nt, Lt = V.shape
    mb, nb = np.array_split(np.arange(Mt), nM), np.array_split(np.arange(Nt), nN)
    db, lb = np.array_split(np.arange(dt), nD), np.array_split(np.arange(Lt), nL)
    O = np.empty((Mt, Lt))
    VT = V.T
    for m in mb:
        for l in lb:
            t5 = np.zeros(len(m))
            t7 = np.zeros((len(m), len(l)))
            for n in nb:
                t3 = np.zeros((len(m), len(n)))
                for d in db:
                    t3 = add(t3, dot(Q[np.ix_(m, d)], K[np.ix_(n, d)]))
                t4 = np.exp(t3 * (dt ** -0.5))
                t5 = add(t5, row_sum(t4))
                t7 = add(t7, dot(t4, VT[np.ix_(l, n)]))
            O[np.ix_(m, l)] = row_scale(t7, 1.0 / t5)
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
