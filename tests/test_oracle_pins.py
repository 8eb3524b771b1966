"""Pins of the fp64 definition oracle against things other than itself.

Nothing here needs a GPU.  The oracle (oracle/bb_oracle.c) is checked against
  * hand-derived closed forms stored in tests/golden/closed_forms.txt,
  * an exact-rational brute force on tiny shapes (fractions + 50-digit decimal
    for sqrt/exp), written in a different loop order,
  * invariants the operator definitions fix,
  * an unfused torch fp64 composition (library routines),
  * the paper's fused loop nests evaluated block by block
    (oracle/listing_oracle.py) for many block splittings -- Rule 4 and Rule 5.
"""
import math
import os
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest
import torch

import bb_inputs
from oracle import listing_oracle as lo
from oracle import oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


def bf16(a):
    """numpy float -> uint16 bf16 bit patterns (round to nearest even)."""
    t = torch.as_tensor(np.asarray(a, dtype=np.float64)).to(torch.float32).to(torch.bfloat16)
    return t.contiguous().view(torch.uint16).numpy().copy()


def f64(bits):
    return lo.bf16_bits_to_f64(bits)


def small_ffn(M, D, F, seed):
    return tuple(bb_inputs.bits(t) for t in bb_inputs.make_ffn(M, D, F, seed))


def small_ln(M, D, N, seed):
    return tuple(bb_inputs.bits(t) for t in bb_inputs.make_ln(M, D, N, seed))


def golden():
    out = {}
    with open(os.path.join(HERE, "golden", "closed_forms.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, *vals = line.split()
            out[name] = np.array([float(v) for v in vals])
    return out


# --------------------------------------------------------------------------
# closed forms
# --------------------------------------------------------------------------
def test_closed_form_onehot():
    X = bf16([[2, 0, 0, 0]])
    g = bf16([1, 1, 1, 1])
    W1 = bf16([[0.5, -1], [7, 7], [7, 7], [7, 7]])     # rows 1..3 must not matter
    W3 = bf16([[3, 2], [5, 5], [5, 5], [5, 5]])
    W2 = bf16([[1, 0, 2, 0], [0, 1, 0, -1]])
    Y = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 0.0)
    np.testing.assert_allclose(Y[0], golden()["ffn_onehot"], rtol=1e-14)


def test_closed_form_eps_inside_sqrt_added_to_mean():
    X = bf16([[2.0 ** -8]])
    Y = orc.rmsnorm_swiglu_ffn(X, bf16([1.5]), bf16([[2]]), bf16([[1]]), bf16([[1]]), 2.0 ** -16)
    np.testing.assert_allclose(Y[0], golden()["ffn_eps"], rtol=1e-14)


def test_closed_form_layernorm_biased_variance():
    Y = orc.layernorm_matmul(bf16([[1, 3]]), bf16([2, 0.5]), bf16([0.25, -1]),
                             bf16([[1, 2], [4, -2]]), 0.0)
    np.testing.assert_allclose(Y[0], golden()["ln_biased"], rtol=1e-14)


def test_onehot_general_scalar_formula():
    # x = c e_j  =>  xh = g_j c / sqrt(c^2/D + eps) e_j ; Y is a few scalars
    D, F, j, c, eps = 8, 5, 3, -3.0, 1e-3
    _, g, W1, W3, W2 = small_ffn(1, D, F, 5)
    x = np.zeros((1, D)); x[0, j] = c
    Y = orc.rmsnorm_swiglu_ffn(bf16(x), g, W1, W3, W2, eps)
    e = orc.float32_eps(eps)
    xh = f64(g)[j] * c / math.sqrt(c * c / D + e)
    a = xh * f64(W1)[j]; b = xh * f64(W3)[j]
    want = (a / (1 + np.exp(-a)) * b) @ f64(W2)
    np.testing.assert_allclose(Y[0], want, rtol=1e-13)


def test_w2_identity_gives_hidden():
    D = F = 6
    X, g, W1, W3, _ = small_ffn(3, D, F, 2)
    Y = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, bf16(np.eye(F)), 1e-6)
    x = f64(X); r = 1 / np.sqrt((x ** 2).mean(1, keepdims=True) + orc.float32_eps(1e-6))
    xh = x * r * f64(g)
    a = xh @ f64(W1); b = xh @ f64(W3)
    np.testing.assert_allclose(Y, a / (1 + np.exp(-a)) * b, rtol=1e-12)


def test_ln_identity_weight_rows_have_mean0_var_v_over_v_plus_eps():
    M, D, eps = 4, 16, 0.25
    X, _, _, _ = small_ln(M, D, D, 3)
    Y = orc.layernorm_matmul(X, bf16(np.ones(D)), bf16(np.zeros(D)), bf16(np.eye(D)), eps)
    v = f64(X).var(axis=1)            # biased
    np.testing.assert_allclose(Y.mean(axis=1), 0, atol=1e-14)
    np.testing.assert_allclose(Y.var(axis=1), v / (v + eps), rtol=1e-12)


# --------------------------------------------------------------------------
# exact brute force on tiny shapes
# --------------------------------------------------------------------------
getcontext().prec = 50


def _frac(bits):
    return [[Fraction(float(v)) for v in row] for row in np.atleast_2d(f64(bits))]


def _dec(fr):
    return Decimal(fr.numerator) / Decimal(fr.denominator)


def brute_ffn(X, g, W1, W3, W2, eps):
    X_, W1_, W3_, W2_ = _frac(X), _frac(W1), _frac(W3), _frac(W2)
    g_ = _frac(g)[0]
    M, D, F = len(X_), len(X_[0]), len(W1_[0])
    epsd = _dec(Fraction(orc.float32_eps(eps)))
    Y = np.zeros((M, D))
    for i in range(M):
        ms = sum(v * v for v in X_[i]) / D
        rms = (_dec(ms) + epsd).sqrt()
        for n in reversed(range(D)):                 # output-column outermost
            tot = Decimal(0)
            for f in reversed(range(F)):
                a = sum(g_[d] * X_[i][d] * W1_[d][f] for d in range(D))
                b = sum(g_[d] * X_[i][d] * W3_[d][f] for d in range(D))
                ad, bd = _dec(a) / rms, _dec(b) / rms
                tot += ad / (1 + (-ad).exp()) * bd * _dec(W2_[f][n])
            Y[i, n] = float(tot)
    return Y


def brute_ln(X, gamma, beta, W, eps):
    X_, W_ = _frac(X), _frac(W)
    ga, be = _frac(gamma)[0], _frac(beta)[0]
    M, D, N = len(X_), len(X_[0]), len(W_[0])
    epsd = _dec(Fraction(orc.float32_eps(eps)))
    Y = np.zeros((M, N))
    for i in range(M):
        s1 = sum(X_[i]); s2 = sum(v * v for v in X_[i])
        mu = s1 / D
        var = s2 / D - mu * mu                      # the paper's one-pass sigma formula
        sd = (_dec(var) + epsd).sqrt()
        for n in range(N):
            lin = sum(ga[d] * (X_[i][d] - mu) * W_[d][n] for d in range(D))
            bias = sum(be[d] * W_[d][n] for d in range(D))
            Y[i, n] = float(_dec(lin) / sd + _dec(bias))
    return Y


@pytest.mark.parametrize("M,D,F", [(1, 1, 1), (2, 3, 4), (3, 4, 2), (1, 5, 1), (4, 1, 3)])
def test_bruteforce_ffn(M, D, F):
    X, g, W1, W3, W2 = small_ffn(M, D, F, 10 * M + D + F)
    want = brute_ffn(X, g, W1, W3, W2, 1e-6)
    got = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 1e-6)
    np.testing.assert_allclose(got, want, rtol=2e-13, atol=1e-300)


@pytest.mark.parametrize("M,D,N", [(1, 2, 1), (2, 3, 4), (3, 4, 2), (2, 5, 1)])
def test_bruteforce_ln(M, D, N):
    X, ga, be, W = small_ln(M, D, N, 7 * M + D + N)
    want = brute_ln(X, ga, be, W, 1e-5)
    got = orc.layernorm_matmul(X, ga, be, W, 1e-5)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)


# --------------------------------------------------------------------------
# invariants fixed by the definitions
# --------------------------------------------------------------------------
M0, D0, F0 = 5, 24, 40


@pytest.fixture(scope="module")
def base():
    t = small_ffn(M0, D0, F0, 1)
    return t, orc.rmsnorm_swiglu_ffn(*t, 1e-6)


def test_row_scaling_invariance_up_to_eps(base):
    (X, g, W1, W3, W2), Y = base
    alpha = np.array([[2.0], [0.5], [8.0], [4.0], [0.25]])   # powers of two: exact in bf16
    Xs = bf16(f64(X) * alpha)
    Y0 = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 0.0)
    Ys = orc.rmsnorm_swiglu_ffn(Xs, g, W1, W3, W2, 0.0)
    np.testing.assert_allclose(Ys, Y0, rtol=1e-12)
    # with eps the change is O(eps / mean(x^2))
    Ye = orc.rmsnorm_swiglu_ffn(Xs, g, W1, W3, W2, 1e-6)
    assert np.abs(Ye - Y).max() < 1e-4 * np.abs(Y).max()
    assert np.abs(Ye - Y).max() > 0


def test_negative_row_scaling_is_not_invariant(base):
    (X, g, W1, W3, W2), Y = base
    Yn = orc.rmsnorm_swiglu_ffn(bf16(-f64(X)), g, W1, W3, W2, 1e-6)
    assert np.abs(Yn - Y).max() > 1e-3          # Swish is not odd


@pytest.mark.parametrize("which", ["g", "W1", "W3", "W2"])
def test_zero_operand_gives_zero(base, which):
    (X, g, W1, W3, W2), _ = base
    args = dict(g=g, W1=W1, W3=W3, W2=W2)
    args[which] = np.zeros_like(args[which])
    Y = orc.rmsnorm_swiglu_ffn(X, args["g"], args["W1"], args["W3"], args["W2"], 1e-6)
    assert np.all(Y == 0)


def test_linear_in_w2_and_w3(base):
    (X, g, W1, W3, W2), Y = base
    Y2 = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, bf16(2 * f64(W2)), 1e-6)
    np.testing.assert_allclose(Y2, 2 * Y, rtol=1e-13)
    Y3 = orc.rmsnorm_swiglu_ffn(X, g, W1, bf16(-4 * f64(W3)), W2, 1e-6)
    np.testing.assert_allclose(Y3, -4 * Y, rtol=1e-13)
    # but NOT linear in W1 (that is the Swish branch)
    Y1 = orc.rmsnorm_swiglu_ffn(X, g, bf16(2 * f64(W1)), W3, W2, 1e-6)
    assert np.abs(Y1 - 2 * Y).max() > 1e-3 * np.abs(Y).max()


def test_swapping_w1_w3_changes_result(base):
    (X, g, W1, W3, W2), Y = base
    Ys = orc.rmsnorm_swiglu_ffn(X, g, W3, W1, W2, 1e-6)
    assert np.abs(Ys - Y).max() > 1e-3 * np.abs(Y).max()


def test_hidden_unit_permutation(base):
    (X, g, W1, W3, W2), Y = base
    p = np.random.default_rng(0).permutation(F0)
    Yp = orc.rmsnorm_swiglu_ffn(X, g, W1[:, p].copy(), W3[:, p].copy(), W2[p].copy(), 1e-6)
    np.testing.assert_allclose(Yp, Y, rtol=1e-10, atol=1e-13)


def test_model_channel_permutation(base):
    (X, g, W1, W3, W2), Y = base
    p = np.random.default_rng(1).permutation(D0)
    Yp = orc.rmsnorm_swiglu_ffn(X[:, p].copy(), g[p].copy(), W1[p].copy(), W3[p].copy(), W2, 1e-6)
    np.testing.assert_allclose(Yp, Y, rtol=1e-10, atol=1e-13)


def test_output_channel_permutation_and_transposed_w2_detected(base):
    (X, g, W1, W3, W2), Y = base
    p = np.random.default_rng(2).permutation(D0)
    Yp = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2[:, p].copy(), 1e-6)
    np.testing.assert_array_equal(Yp, Y[:, p])


def test_row_independence_and_row_list(base):
    (X, g, W1, W3, W2), Y = base
    rows = [4, 0, 2, 2]
    Ys = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 1e-6, rows=rows)
    np.testing.assert_array_equal(Ys, Y[rows])
    Yr = orc.rmsnorm_swiglu_ffn(X[rows].copy(), g, W1, W3, W2, 1e-6)
    np.testing.assert_array_equal(Yr, Y[rows])


def test_empty():
    X, g, W1, W3, W2 = small_ffn(1, 4, 4, 0)
    assert orc.rmsnorm_swiglu_ffn(X[:0], g, W1, W3, W2, 1e-6).shape == (0, 4)


def test_ln_shift_invariance_and_gamma_zero():
    M, D, N = 4, 32, 12
    X, ga, be, W = small_ln(M, D, N, 4)
    Y = orc.layernorm_matmul(X, ga, be, W, 1e-5)
    # integers + 8: exactly representable shift on small-integer data
    Xi = np.round(f64(X) * 4)
    Y0 = orc.layernorm_matmul(bf16(Xi), ga, be, W, 1e-5)
    Y8 = orc.layernorm_matmul(bf16(Xi + 8), ga, be, W, 1e-5)
    np.testing.assert_allclose(Y8, Y0, rtol=1e-12, atol=1e-13)
    # gamma = 0: every row equals beta^T W
    Yz = orc.layernorm_matmul(X, np.zeros_like(ga), be, W, 1e-5)
    want = f64(be) @ f64(W)
    np.testing.assert_allclose(Yz, np.tile(want, (M, 1)), rtol=1e-13, atol=1e-15)
    # beta enters only through the row-independent vector beta^T W
    Yb = orc.layernorm_matmul(X, ga, np.zeros_like(be), W, 1e-5)
    np.testing.assert_allclose(Y - Yb, np.tile(want, (M, 1)), rtol=1e-9, atol=1e-12)


def test_cross_link_zero_mean_rows_ln_equals_rmsnorm():
    # rows with exactly zero mean: LN(X; gamma, beta=0) = RMSNorm(X; g=gamma)
    M, D, F = 3, 16, 10
    X, g, W1, W3, W2 = small_ffn(M, D, F, 6)
    x = np.round(f64(X) * 8) / 8
    x[:, D // 2:] = -x[:, :D // 2]                    # exact zero mean
    Xz = bf16(x)
    W13 = np.concatenate([W1, W3], axis=1).copy()
    Z = orc.layernorm_matmul(Xz, g, np.zeros_like(g), W13, 1e-6)
    a, b = Z[:, :F], Z[:, F:]
    want = (a / (1 + np.exp(-a)) * b) @ f64(W2)
    got = orc.rmsnorm_swiglu_ffn(Xz, g, W1, W3, W2, 1e-6)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-14)


# --------------------------------------------------------------------------
# library composition (torch fp64, unfused)
# --------------------------------------------------------------------------
def test_against_torch_fp64_composition():
    M, D, F = 7, 48, 80
    Xt, gt, W1t, W3t, W2t = bb_inputs.make_ffn(M, D, F, 9, "student4")
    eps = 1e-6
    X, g, W1, W3, W2 = (t.double() for t in (Xt, gt, W1t, W3t, W2t))
    xh = torch.nn.functional.rms_norm(X, (D,), weight=g, eps=orc.float32_eps(eps))
    want = (torch.nn.functional.silu(xh @ W1) * (xh @ W3)) @ W2
    got = orc.rmsnorm_swiglu_ffn(Xt, gt, W1t, W3t, W2t, eps)
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-10, atol=1e-13)


def test_ln_against_torch_fp64_composition():
    M, D, N = 6, 40, 24
    Xt, gat, bet, Wt = bb_inputs.make_ln(M, D, N, 11)
    X, ga, be, W = (t.double() for t in (Xt, gat, bet, Wt))
    want = torch.nn.functional.layer_norm(X, (D,), ga, be, eps=orc.float32_eps(1e-5)) @ W
    got = orc.layernorm_matmul(Xt, gat, bet, Wt, 1e-5)
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-10, atol=1e-13)


# --------------------------------------------------------------------------
# the paper's fused nests, block by block (Rule 4 / Rule 5 algebra,
# independence of the result from the block counts)
# --------------------------------------------------------------------------
SPLITS = [(1, 1, 1, 1), (2, 1, 1, 1), (1, 3, 1, 1), (1, 1, 4, 1), (1, 1, 1, 5),
          (3, 2, 5, 4), (6, 12, 20, 12), (2, 1, 7, 3)]


@pytest.mark.parametrize("nM,nN,nK,nD", SPLITS)
def test_fused_nest_example3_matches_definition(nM, nN, nK, nD):
    X, g, W1, W3, W2 = small_ffn(6, 12, 20, 3)
    want = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 1e-6)
    e = orc.float32_eps(1e-6)
    got = lo.fused_rmsnorm_swiglu_ffn(X, g, W1, W3, W2, e, nM, nN, nK, nD)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-14)
    snap = lo.snapshot1_rmsnorm_swiglu_ffn(X, g, W1, W3, W2, e, nM, nN, nK, nD)
    np.testing.assert_allclose(snap, want, rtol=1e-11, atol=1e-14)


@pytest.mark.parametrize("nM,nN,nK", [(1, 1, 1), (2, 3, 1), (1, 1, 6), (4, 2, 5), (8, 9, 12)])
def test_fused_nest_example2_matches_definition(nM, nN, nK):
    X, ga, be, W = small_ln(8, 12, 9, 5)
    want = orc.layernorm_matmul(X, ga, be, W, 1e-5)
    got = lo.fused_layernorm_matmul(X, ga, be, W, orc.float32_eps(1e-5), nM, nN, nK)
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)


# --------------------------------------------------------------------------
# regression fixture written by tests/golden/make_golden.py (oracle only)
# --------------------------------------------------------------------------
def test_c1_regression_fixture():
    path = os.path.join(HERE, "golden", "c1_oracle_samples.txt")
    X, g, W1, W3, W2 = (bb_inputs.bits(t) for t in bb_inputs.make_config("c1"))
    rows, cols, vals = [], [], []
    with open(path) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            r, c, v = line.split()
            rows.append(int(r)); cols.append(int(c)); vals.append(float.fromhex(v))
    ur = sorted(set(rows))
    Y = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 1e-6, rows=ur)
    got = np.array([Y[ur.index(r), c] for r, c in zip(rows, cols)])
    np.testing.assert_allclose(got, np.array(vals), rtol=1e-12)


# --------------------------------------------------------------------------
# Attention (Example 1): softmax(Q K^T / sqrt(d)) V
# --------------------------------------------------------------------------
def small_attn(B, M, N, d, dv, seed):
    return tuple(bb_inputs.bits(t) for t in bb_inputs.make_attn(B, M, N, d, dv, seed))


def attn_ref64(Qb, Kb, Vb):
    """plain numpy fp64 composition per batch entry (library matmul / exp)"""
    Q, K, V = f64(Qb), f64(Kb), f64(Vb)
    out = []
    for b in range(Q.shape[0]):
        S = Q[b] @ K[b].T / math.sqrt(Q.shape[2])
        P = np.exp(S - S.max(axis=1, keepdims=True))
        out.append((P / P.sum(axis=1, keepdims=True)) @ V[b])
    return np.concatenate(out, axis=0)


def test_attention_closed_form_two_keys():
    O = orc.attention(bf16([[[2, 0, 0, 0]]]), bf16([[[1, 0, 0, 0], [-1, 0, 0, 0]]]), bf16([[[1, 0], [0, 1]]]))
    np.testing.assert_allclose(O[0], golden()["attn_two_keys"], rtol=1e-14)


def test_attention_closed_form_scale_is_inverse_sqrt_d():
    q = np.zeros((1, 1, 16)); q[0, 0, 0] = 4
    K = np.zeros((1, 3, 16)); K[0, :, 0] = [1, 0, -1]
    O = orc.attention(bf16(q), bf16(K), bf16([[[1, 2], [3, -1], [0, 4]]]))
    np.testing.assert_allclose(O[0], golden()["attn_scale"], rtol=1e-14)


def test_attention_zero_queries_average_the_values():
    Q, K, V = small_attn(2, 5, 9, 8, 6, 1)
    O = orc.attention(np.zeros_like(Q), K, V)
    for b in range(2):
        np.testing.assert_allclose(O[5 * b:5 * b + 5], np.tile(f64(V)[b].mean(axis=0), (5, 1)), rtol=1e-13)


def test_attention_single_key_returns_its_value_row():
    Q, K, V = small_attn(1, 4, 1, 8, 5, 2)
    np.testing.assert_allclose(orc.attention(Q, K, V), np.tile(f64(V)[0, 0], (4, 1)), rtol=1e-15)


def test_attention_brute_force_decimal():
    """independent scalar evaluation with 50-digit decimals, different loop order"""
    getcontext().prec = 50
    Qb, Kb, Vb = small_attn(1, 3, 4, 2, 3, 3)
    Q, K, V = f64(Qb)[0], f64(Kb)[0], f64(Vb)[0]
    O = orc.attention(Qb, Kb, Vb)
    rd = Decimal(2).sqrt()
    for i in range(3):
        e = []
        for j in range(4):
            s = sum(Decimal(float(Q[i, c])) * Decimal(float(K[j, c])) for c in reversed(range(2))) / rd
            e.append(s.exp())
        den = sum(e)
        for c in range(3):
            want = sum(e[j] * Decimal(float(V[j, c])) for j in range(4)) / den
            assert abs(Decimal(float(O[i, c])) - want) <= Decimal(10) ** -14 * (1 + abs(want))


def test_attention_matches_library_composition_and_torch():
    Qb, Kb, Vb = small_attn(3, 17, 33, 16, 24, 4)
    O = orc.attention(Qb, Kb, Vb)
    np.testing.assert_allclose(O, attn_ref64(Qb, Kb, Vb), rtol=1e-12, atol=1e-14)
    t = lambda a: torch.as_tensor(f64(a))
    want = torch.nn.functional.scaled_dot_product_attention(t(Qb), t(Kb), t(Vb)).reshape(-1, 24).numpy()
    np.testing.assert_allclose(O, want, rtol=1e-11, atol=1e-13)


def test_attention_invariants():
    Qb, Kb, Vb = small_attn(2, 6, 10, 8, 4, 5)
    O = orc.attention(Qb, Kb, Vb)
    # permuting the keys together with their values changes nothing
    perm = np.random.default_rng(0).permutation(10)
    np.testing.assert_allclose(orc.attention(Qb, Kb[:, perm], Vb[:, perm]), O, rtol=1e-12, atol=1e-15)
    # linear in V; rows are convex combinations of value rows
    np.testing.assert_allclose(orc.attention(Qb, Kb, bf16(2 * f64(Vb))), 2 * O, rtol=1e-13)
    V = f64(Vb)
    for b in range(2):
        blk = O[6 * b:6 * b + 6]
        assert np.all(blk <= V[b].max(axis=0) + 1e-12) and np.all(blk >= V[b].min(axis=0) - 1e-12)
    # adding the same vector to every key shifts all scores of a query equally: softmax unchanged
    # (keys on a 1/16 grid so that the shifted keys are exactly representable in bf16)
    Kq = np.clip(np.round(f64(Kb) * 16) / 16, -2, 2)
    c = np.zeros(8); c[3] = 1.0
    np.testing.assert_allclose(orc.attention(Qb, bf16(Kq + c), Vb), orc.attention(Qb, bf16(Kq), Vb),
                               rtol=1e-11, atol=1e-13)
    # row subset / batch independence
    rows = [11, 0, 7]
    np.testing.assert_allclose(orc.attention(Qb, Kb, Vb, rows=rows), O[rows], rtol=0, atol=0)
    np.testing.assert_allclose(orc.attention(Qb[1:], Kb[1:], Vb[1:]), O[6:], rtol=0, atol=0)


@pytest.mark.parametrize("split", [dict(), dict(nM=2, nN=3, nD=4, nL=2), dict(nM=5, nN=11, nD=8, nL=3)])
def test_attention_fused_nest_agrees_for_every_block_splitting(split):
    Qb, Kb, Vb = small_attn(1, 5, 11, 8, 3, 6)
    O = orc.attention(Qb, Kb, Vb)
    np.testing.assert_allclose(lo.fused_attention(f64(Qb)[0], f64(Kb)[0], f64(Vb)[0], **split), O, rtol=1e-12)


@pytest.mark.parametrize("split", [dict(), dict(nM=2, nN=4), dict(nM=5, nN=11)])
def test_attention_significand_exponent_pairs_agree_and_do_not_overflow(split):
    Qb, Kb, Vb = small_attn(1, 5, 11, 8, 3, 7)
    O = orc.attention(Qb, Kb, Vb)
    np.testing.assert_allclose(lo.safe_attention(f64(Qb)[0], f64(Kb)[0], f64(Vb)[0], **split), O, rtol=1e-12)
    # scores of several hundred: plain exp overflows, the pairs and the oracle do not
    big = bf16(f64(Qb) * 256)
    Ob = orc.attention(big, Kb, Vb)
    assert np.all(np.isfinite(Ob))
    np.testing.assert_allclose(lo.safe_attention(f64(big)[0], f64(Kb)[0], f64(Vb)[0], **split), Ob, rtol=1e-11, atol=1e-14)
    with np.errstate(over="ignore", invalid="ignore"):
        assert not np.all(np.isfinite(lo.fused_attention(f64(big)[0] * 8, f64(Kb)[0], f64(Vb)[0])))


# ---------------------------------------------------------------- residual connection
def test_residual_is_the_operator_plus_r_and_exact_for_zero_w2():
    X, g, W1, W3, W2 = bb_inputs.make_ffn(6, 64, 96, seed=12)
    R = bb_inputs.make_ffn(6, 64, 96, seed=13)[0]
    base = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 1e-6)
    got = orc.rmsnorm_swiglu_ffn_residual(X, g, W1, W3, W2, R, 1e-6)
    assert np.array_equal(got - base, R.double().numpy() + 0 * base) or np.allclose(got - base, R.double().numpy(), rtol=0, atol=1e-12)
    zero = torch.zeros_like(W2)
    assert np.array_equal(orc.rmsnorm_swiglu_ffn_residual(X, g, W1, W3, zero, R, 1e-6), R.double().numpy())
    rows = [4, 1]
    assert np.array_equal(orc.rmsnorm_swiglu_ffn_residual(X, g, W1, W3, W2, R, 1e-6, rows=rows), got[rows])
