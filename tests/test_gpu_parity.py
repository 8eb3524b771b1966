"""GPU parity: the HIP library (through its C ABI) against the fp64 oracle on
the same seeded inputs.  Gates (both operators; bb_parity.py derives the second):

    max_i  || Ygpu[i,:] - Yref[i,:] ||_2 / || Yref[i,:] ||_2                   <=  2e-2
    max_ij | Ygpu[i,j] - Yref[i,j] | / ( || Yref[i,:] ||_2 / sqrt(columns) )   <=  3e-2

bf16 operands, fp32 accumulation; the oracle sees the same bf16-rounded inputs.
"""
import numpy as np
import pytest
import torch

import bb_inputs
import bb_parity
import paper_2505_07829_amd as bb
from oracle import oracle as orc

pytestmark = pytest.mark.gpu
TOL = 2e-2


def dev(ts):
    return [t.cuda() for t in ts]


def row_rel_err(Y_gpu, Y_ref):
    """the row figure; the element-wise gate is asserted on the way (every comparison in this file passes here)"""
    row, elem = bb_parity.errors(Y_gpu, Y_ref)
    assert elem <= bb_parity.TOL_ELEM, f"element error {elem:.3e} > {bb_parity.TOL_ELEM} (row error {row:.3e})"
    return row


def sample_rows(M, tile=128, extra=6, seed=0):
    """first/last row of every row tile of the kernels (128 rows: every 256-row tile's edges are among them)
    plus a few random rows"""
    rows = set()
    for t0 in range(0, M, tile):
        rows.add(t0); rows.add(min(M, t0 + tile) - 1)
    rng = np.random.default_rng(seed)
    rows.update(int(r) for r in rng.integers(0, M, size=extra))
    return sorted(rows)


def ffn_case(cpu, eps, rows=None, variant=bb.VARIANT_AUTO, unfused=False):
    X, g, W1, W3, W2 = cpu
    bb.bb_set_variant(variant)
    try:
        Y = bb.bb_rmsnorm_swiglu_ffn(*dev(cpu), eps, unfused=unfused)
        torch.cuda.synchronize()
    finally:
        bb.bb_set_variant(bb.VARIANT_AUTO)
    ref = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, eps, rows=rows)
    got = Y if rows is None else Y[rows]
    return row_rel_err(got, ref)


@pytest.fixture(scope="module", autouse=True)
def _lib():
    bb.load()
    yield
    bb.bb_shutdown()


# ---------------------------------------------------------------- small shapes
@pytest.mark.parametrize("variant", [bb.VARIANT_SNAPSHOT1, bb.VARIANT_NEST, bb.VARIANT_AUTO])
def test_c1_full(variant):
    c = bb_inputs.CONFIGS["c1"]
    err = ffn_case(bb_inputs.make_config("c1"), c.eps, variant=variant)
    print("c1 rel err", err)
    assert err <= TOL


@pytest.mark.parametrize("M,D,F", [(1, 64, 64), (5, 264, 712), (16, 256, 704), (17, 72, 136),
                                   (130, 264, 712), (300, 520, 1032), (257, 128, 256)])
def test_ragged_shapes_snapshot1(M, D, F):
    err = ffn_case(bb_inputs.make_ffn(M, D, F, seed=M + D), 1e-6, variant=bb.VARIANT_SNAPSHOT1)
    assert err <= TOL


@pytest.mark.parametrize("M,D,F", [(1, 64, 64), (5, 264, 712), (16, 256, 704), (9, 72, 136), (16, 520, 1032),
                                   # two groups of 16 rows
                                   (17, 72, 136), (32, 520, 1032), (25, 264, 712), (31, 1032, 2056)])
def test_ragged_shapes_stream(M, D, F):
    err = ffn_case(bb_inputs.make_ffn(M, D, F, seed=M + F), 1e-6, variant=bb.VARIANT_STREAM)
    assert err <= TOL


# the fully fused nest (last snapshot of Example 3 with one block of output columns): one launch, D <= 512
@pytest.mark.parametrize("M,D,F", [(1, 64, 64), (16, 256, 704), (17, 72, 136), (64, 256, 704), (130, 264, 712),
                                   (300, 512, 1032), (33, 392, 200), (250, 512, 2816)])
def test_ragged_shapes_nest(M, D, F):
    err = ffn_case(bb_inputs.make_ffn(M, D, F, seed=M + D + 1), 1e-6, variant=bb.VARIANT_NEST)
    assert err <= TOL


def test_nest_is_one_launch_on_c1():
    c = bb_inputs.CONFIGS["c1"]
    cpu = bb_inputs.make_config("c1")
    bb.bb_set_variant(bb.VARIANT_NEST)
    bb.bb_profile_enable(True)
    try:
        Y = bb.bb_rmsnorm_swiglu_ffn(*dev(cpu), c.eps)
        names = [k for k, _ in bb.bb_profile_last()]
    finally:
        bb.bb_profile_enable(False)
        bb.bb_set_variant(bb.VARIANT_AUTO)
    assert names == ["ffn_nest"]
    assert row_rel_err(Y, orc.rmsnorm_swiglu_ffn(*cpu, c.eps)) <= TOL


def launches_of_auto(M, D, F):
    d = dev(bb_inputs.make_ffn(M, D, F, seed=3))
    bb.bb_profile_enable(True)
    try:
        bb.bb_rmsnorm_swiglu_ffn(*d, 1e-6)
        return [k for k, _ in bb.bb_profile_last()]
    finally:
        bb.bb_profile_enable(False)


def test_auto_runs_the_nest_where_its_wavefront_pairs_take_all_hidden_blocks_at_once():
    # D <= 256 and F <= 768, any number of rows (also those the streaming kernel would take)
    for M, D, F in [(64, 256, 704), (8, 128, 768), (1500, 200, 696)]:
        assert launches_of_auto(M, D, F) == ["ffn_nest"], (M, D, F)
    # one more hidden block, a wider model, or more blocks of 16 rows than compute units: the other programs
    for M, D, F in [(64, 256, 776), (64, 264, 704), (8, 256, 1408), (4112, 64, 128)]:
        assert "ffn_nest" not in launches_of_auto(M, D, F), (M, D, F)


def test_nest_refuses_a_model_dimension_whose_output_block_does_not_fit():
    cpu = bb_inputs.make_ffn(32, 520, 256, seed=2)
    bb.bb_set_variant(bb.VARIANT_NEST)
    try:
        with pytest.raises(bb.BBError) as e:
            bb.bb_rmsnorm_swiglu_ffn(*dev(cpu), 1e-6)
        assert e.value.status == bb.BB_ERR_VARIANT
    finally:
        bb.bb_set_variant(bb.VARIANT_AUTO)


def test_stream_repeated_calls_keep_scratch_clean():
    cpu = bb_inputs.make_ffn(16, 256, 704, seed=3)
    X, g, W1, W3, W2 = cpu
    ref = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 1e-6)
    d = dev(cpu)
    bb.bb_set_variant(bb.VARIANT_STREAM)
    try:
        outs = []
        for _ in range(5):
            outs.append(bb.bb_rmsnorm_swiglu_ffn(*d, 1e-6))
        # a different shape in between forces a new scratch layout
        other = bb_inputs.make_ffn(7, 128, 384, seed=4)
        Yo = bb.bb_rmsnorm_swiglu_ffn(*dev(other), 1e-6)
        outs.append(bb.bb_rmsnorm_swiglu_ffn(*d, 1e-6))
        torch.cuda.synchronize()
    finally:
        bb.bb_set_variant(bb.VARIANT_AUTO)
    for Y in outs:
        assert row_rel_err(Y, ref) <= TOL
    refo = orc.rmsnorm_swiglu_ffn(*other, 1e-6)
    assert row_rel_err(Yo, refo) <= TOL


def test_variant_switching_shares_workspace():
    cpu = bb_inputs.make_ffn(16, 256, 704, seed=5)
    ref = orc.rmsnorm_swiglu_ffn(*cpu, 1e-6)
    d = dev(cpu)
    for v in (bb.VARIANT_STREAM, bb.VARIANT_SNAPSHOT1, bb.VARIANT_STREAM, bb.VARIANT_STREAM):
        bb.bb_set_variant(v)
        Y = bb.bb_rmsnorm_swiglu_ffn(*d, 1e-6)
        torch.cuda.synchronize()
        bb.bb_set_variant(bb.VARIANT_AUTO)
        assert row_rel_err(Y, ref) <= TOL


@pytest.mark.parametrize("which", [1, 2, 3, 4])
@pytest.mark.parametrize("variant", [bb.VARIANT_STREAM, bb.VARIANT_SNAPSHOT1, bb.VARIANT_NEST])
def test_zero_operand_gives_exact_zero(which, variant):
    cpu = list(bb_inputs.make_ffn(16, 128, 256, seed=6))
    cpu[which] = torch.zeros_like(cpu[which])           # g, W1, W3 or W2
    bb.bb_set_variant(variant)
    try:
        Y = bb.bb_rmsnorm_swiglu_ffn(*dev(cpu), 1e-6)
        torch.cuda.synchronize()
    finally:
        bb.bb_set_variant(bb.VARIANT_AUTO)
    assert torch.all(Y.float() == 0)


def test_eps_matters_when_rows_are_tiny():
    # mean(x^2) ~ eps: the output must follow the oracle, which a kernel that
    # drops eps or puts it outside the root would miss by tens of percent
    cpu = list(bb_inputs.make_ffn(16, 256, 512, seed=8))
    cpu[0] = (cpu[0].float() * 1e-3).to(torch.bfloat16)
    for v in (bb.VARIANT_STREAM, bb.VARIANT_SNAPSHOT1, bb.VARIANT_NEST):
        assert ffn_case(cpu, 1e-6, variant=v) <= TOL


def test_unfused_small():
    assert ffn_case(bb_inputs.make_config("c1"), 1e-6, unfused=True) <= TOL
    assert ffn_case(bb_inputs.make_ffn(130, 264, 712, seed=1), 1e-6, unfused=True) <= TOL


@pytest.mark.parametrize("M,D,N", [(1, 64, 64), (64, 256, 512), (130, 264, 712), (300, 520, 1032)])
@pytest.mark.parametrize("unfused", [False, True])
def test_ln_small(M, D, N, unfused):
    cpu = bb_inputs.make_ln(M, D, N, seed=M)
    Y = bb.bb_layernorm_matmul(*dev(cpu), 1e-5, unfused=unfused)
    torch.cuda.synchronize()
    ref = orc.layernorm_matmul(*cpu, 1e-5)
    assert row_rel_err(Y, ref) <= TOL


def test_ln_gamma_zero_gives_bias_row():
    X, ga, be, W = bb_inputs.make_ln(40, 128, 256, seed=2)
    ga = torch.zeros_like(ga)
    Y = bb.bb_layernorm_matmul(*dev((X, ga, be, W)), 1e-5)
    torch.cuda.synchronize()
    ref = orc.layernorm_matmul(X, ga, be, W, 1e-5)
    assert row_rel_err(Y, ref) <= TOL
    assert torch.all(Y == Y[0:1])                        # every row identical


# Complete-tile kernels (no bounds checks) with an odd and an even number of
# contraction steps, and the shortest contractions (one and two steps): the
# rotated main loop has a prologue, paired steps and a parity-dependent tail.
@pytest.mark.parametrize("M,D,F", [(256, 256, 384), (256, 192, 384), (128, 256, 448), (128, 64, 128),
                                   (128, 128, 64), (384, 320, 640), (512, 64, 192)])
@pytest.mark.parametrize("unfused", [False, True])
def test_complete_tiles_and_step_parities_ffn(M, D, F, unfused):
    err = ffn_case(bb_inputs.make_ffn(M, D, F, seed=M + D + F), 1e-6, variant=bb.VARIANT_SNAPSHOT1, unfused=unfused)
    assert err <= TOL


@pytest.mark.parametrize("M,D,N", [(256, 192, 512), (256, 256, 512), (128, 64, 256), (128, 128, 768), (384, 448, 256)])
@pytest.mark.parametrize("unfused", [False, True])
def test_complete_tiles_and_step_parities_ln(M, D, N, unfused):
    cpu = bb_inputs.make_ln(M, D, N, seed=M + D + N)
    Y = bb.bb_layernorm_matmul(*dev(cpu), 1e-5, unfused=unfused)
    torch.cuda.synchronize()
    ref = orc.layernorm_matmul(*cpu, 1e-5)
    assert row_rel_err(Y, ref) <= TOL


# Few rows, long contractions: fewer tiles than compute units, so the
# contraction range of a tile is split over several workgroups (fp32 partial
# results + a reduce kernel), for the gate/up product and for the down product.
@pytest.mark.parametrize("M,D,F", [(17, 4096, 11008), (48, 4096, 11008), (130, 2048, 5632), (300, 1024, 2816),
                                   (64, 520, 1416), (33, 264, 2056)])
def test_split_contraction_few_rows(M, D, F):
    cpu = bb_inputs.make_ffn(M, D, F, seed=M + 7)
    assert ffn_case(cpu, 1e-6, variant=bb.VARIANT_SNAPSHOT1) <= TOL
    if D <= 2048:
        assert ffn_case(cpu, 1e-6, unfused=True) <= TOL


# Transposed-weight entry points (W1t [F,D], W3t [F,D], W2t [D,F]; Wt [N,D]):
# the oracle takes the logical matrices, the library their transposes.
def tr(w):
    return w.t().contiguous()


@pytest.mark.parametrize("M,D,F", [(1, 64, 64), (16, 256, 704), (130, 264, 712), (300, 520, 1032), (256, 256, 384),
                                   (256, 192, 384), (128, 64, 128), (48, 2048, 5632), (17, 4096, 11008)])
def test_transposed_weights_ffn(M, D, F):
    X, g, W1, W3, W2 = bb_inputs.make_ffn(M, D, F, seed=M + D)
    Y = bb.bb_rmsnorm_swiglu_ffn_t(*dev((X, g, tr(W1), tr(W3), tr(W2))), 1e-6)
    torch.cuda.synchronize()
    assert row_rel_err(Y, orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 1e-6)) <= TOL


@pytest.mark.parametrize("M,D,N", [(1, 64, 64), (64, 256, 512), (130, 264, 712), (256, 192, 512), (384, 448, 256)])
def test_transposed_weights_ln(M, D, N):
    X, ga, be, W = bb_inputs.make_ln(M, D, N, seed=M + N)
    Y = bb.bb_layernorm_matmul_t(*dev((X, ga, be, tr(W))), 1e-5)
    torch.cuda.synchronize()
    assert row_rel_err(Y, orc.layernorm_matmul(X, ga, be, W, 1e-5)) <= TOL


def test_c3_transposed_weights_sampled_rows():
    c = bb_inputs.CONFIGS["c3"]
    X, g, W1, W3, W2 = bb_inputs.make_config("c3")
    rows = sample_rows(c.M)
    Y = bb.bb_rmsnorm_swiglu_ffn_t(*dev((X, g, tr(W1), tr(W3), tr(W2))), c.eps)
    torch.cuda.synchronize()
    err = row_rel_err(Y[rows], orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, c.eps, rows=rows))
    print("c3 transposed rel err", err)
    assert err <= TOL


# ------------------------------------------------------------ full-size configs
def test_c2_decode_full():
    c = bb_inputs.CONFIGS["c2"]
    cpu = bb_inputs.make_config("c2")
    for v in (bb.VARIANT_AUTO, bb.VARIANT_SNAPSHOT1):
        err = ffn_case(cpu, c.eps, variant=v)
        print("c2 variant", v, "rel err", err)
        assert err <= TOL


def test_c3_prefill_sampled_rows():
    c = bb_inputs.CONFIGS["c3"]
    cpu = bb_inputs.make_config("c3")
    rows = sample_rows(c.M)
    err = ffn_case(cpu, c.eps, rows=rows)
    print("c3 rel err", err, "rows", len(rows))
    assert err <= TOL


def test_c4_large_sampled_rows():
    c = bb_inputs.CONFIGS["c4"]
    cpu = bb_inputs.make_config("c4")
    rows = sample_rows(c.M, extra=2)
    err = ffn_case(cpu, c.eps, rows=rows)
    print("c4 rel err", err, "rows", len(rows))
    assert err <= TOL


def test_c5_ln_sampled_rows():
    c = bb_inputs.CONFIGS["c5"]
    cpu = bb_inputs.make_config("c5")
    rows = sample_rows(c.M, extra=4)
    Y = bb.bb_layernorm_matmul(*dev(cpu), c.eps)
    torch.cuda.synchronize()
    ref = orc.layernorm_matmul(*cpu, c.eps, rows=rows)
    err = row_rel_err(Y[rows], ref)
    print("c5 rel err", err, "rows", len(rows))
    assert err <= TOL


# ---------------------------------------------------------------- measured selection
def test_tune_records_fastest_candidate_and_auto_follows():
    bb.bb_tune_clear()
    cpu = bb_inputs.make_ffn(96, 512, 1408, seed=4)
    d = dev(cpu)
    M, D, F = 96, 512, 1408
    assert bb.bb_tuned_variant(bb.OP_FFN, M, D, F) == bb.VARIANT_AUTO
    chosen, ms = bb.bb_rmsnorm_swiglu_ffn_tune(*d, 1e-6, reps=3)
    # (STREAM is no candidate above 16 rows; the fully fused nest is one up to a model dimension of 512)
    assert set(ms) == {bb.VARIANT_SNAPSHOT1, bb.VARIANT_UNFUSED, bb.VARIANT_PRESCALE, bb.VARIANT_NEST}
    assert chosen == min(ms, key=ms.get) and all(v > 0 for v in ms.values())
    assert bb.bb_tuned_variant(bb.OP_FFN, M, D, F) == chosen
    assert bb.bb_tuned_variant(bb.OP_FFN, M + 1, D, F) == bb.VARIANT_AUTO  # exact shapes only
    # AUTO now runs the recorded program: its kernel list is that program's
    bb.bb_profile_enable(True)
    Y = bb.bb_rmsnorm_swiglu_ffn(*d, 1e-6)
    names = [k for k, _ in bb.bb_profile_last()]
    bb.bb_profile_enable(False)
    assert ("rmsnorm_rows" in names) == (chosen == bb.VARIANT_UNFUSED)
    assert ("rms_gain_rows" in names) == (chosen == bb.VARIANT_PRESCALE)
    assert ("ffn_nest" in names) == (chosen == bb.VARIANT_NEST)
    ref = orc.rmsnorm_swiglu_ffn(*cpu, 1e-6)
    assert row_rel_err(Y, ref) <= TOL
    bb.bb_tune_clear()
    assert bb.bb_tuned_variant(bb.OP_FFN, M, D, F) == bb.VARIANT_AUTO


def test_tune_decode_shape_has_three_candidates():
    bb.bb_tune_clear()
    cpu = bb_inputs.make_ffn(8, 512, 1408, seed=5)
    chosen, ms = bb.bb_rmsnorm_swiglu_ffn_tune(*dev(cpu), 1e-6, reps=3)
    assert set(ms) == {bb.VARIANT_STREAM, bb.VARIANT_SNAPSHOT1, bb.VARIANT_UNFUSED, bb.VARIANT_NEST}
    Y = bb.bb_rmsnorm_swiglu_ffn(*dev(cpu), 1e-6)
    assert row_rel_err(Y, orc.rmsnorm_swiglu_ffn(*cpu, 1e-6)) <= TOL
    bb.bb_tune_clear()


def test_tune_layernorm_and_forced_unfused_variant():
    bb.bb_tune_clear()
    cpu = bb_inputs.make_ln(200, 512, 768, seed=6)
    ref = orc.layernorm_matmul(*cpu, 1e-5)
    chosen, ms = bb.bb_layernorm_matmul_tune(*dev(cpu), 1e-5, reps=3)
    assert set(ms) == {bb.VARIANT_SNAPSHOT1, bb.VARIANT_UNFUSED, bb.VARIANT_PRESCALE} and chosen in ms
    assert row_rel_err(bb.bb_layernorm_matmul(*dev(cpu), 1e-5), ref) <= TOL
    bb.bb_tune_clear()
    # the unfused program through the main entry points when forced
    bb.bb_set_variant(bb.VARIANT_UNFUSED)
    try:
        bb.bb_profile_enable(True)
        Y = bb.bb_layernorm_matmul(*dev(cpu), 1e-5)
        names = [k for k, _ in bb.bb_profile_last()]
        bb.bb_profile_enable(False)
        assert "layernorm_rows" in names and row_rel_err(Y, ref) <= TOL
    finally:
        bb.bb_set_variant(bb.VARIANT_AUTO)


# ---------------------------------------------------------------- residual epilogue
def residual_case(M, D, F, seed, transposed=False, in_place=None):
    X, g, W1, W3, W2 = bb_inputs.make_ffn(M, D, F, seed=seed)
    R = X if in_place == "x" else bb_inputs.make_ffn(M, D, F, seed=seed + 100)[0]
    ref = orc.rmsnorm_swiglu_ffn_residual(X, g, W1, W3, W2, R, 1e-6)
    ws = [w.t().contiguous() for w in (W1, W3, W2)] if transposed else [W1, W3, W2]
    Xd, gd = X.cuda(), g.cuda()
    Rd = Xd if in_place == "x" else R.cuda()
    Yd = Rd if in_place else None
    Y = bb.bb_rmsnorm_swiglu_ffn_residual(Xd, gd, *[w.cuda() for w in ws], Rd, 1e-6, Y=Yd, transposed=transposed)
    torch.cuda.synchronize()
    return row_rel_err(Y, ref)


@pytest.mark.parametrize("M,D,F", [(1, 64, 64), (9, 264, 712), (16, 512, 1408),        # streaming kernel
                                   (17, 72, 136), (96, 512, 1408), (130, 264, 712),     # split contraction / ragged tiles
                                   (256, 512, 1024), (512, 1024, 2816), (300, 520, 1032)])
def test_residual_epilogue(M, D, F):
    assert residual_case(M, D, F, seed=M + F) <= TOL


@pytest.mark.parametrize("M,D,F", [(17, 72, 136), (96, 512, 1408), (130, 264, 712)])
def test_residual_epilogue_fully_fused_nest(M, D, F):
    bb.bb_set_variant(bb.VARIANT_NEST)
    try:
        assert residual_case(M, D, F, seed=M + F) <= TOL
        assert residual_case(M, D, F, seed=5, in_place="x") <= TOL
    finally:
        bb.bb_set_variant(bb.VARIANT_AUTO)


@pytest.mark.parametrize("M,D,F", [(130, 264, 712), (512, 1024, 2816), (16, 256, 704)])
def test_residual_epilogue_transposed_weights(M, D, F):
    assert residual_case(M, D, F, seed=7, transposed=True) <= TOL


@pytest.mark.parametrize("M,D,F", [(8, 256, 704), (200, 512, 1408), (2048, 1024, 2816)])
@pytest.mark.parametrize("mode", ["r", "x"])
def test_residual_in_place(M, D, F, mode):
    # Y written over R; in mode "x" R is X itself: y = x + FFN(norm(x)) in place
    assert residual_case(M, D, F, seed=3, in_place=mode) <= TOL


def test_residual_dominates_small_ffn_output():
    # a residual 1000 times larger than the FFN output: the sum is rounded once, so the result is
    # within half a bf16 step of the exact sum (a second rounding would show as up to a full step)
    X, g, W1, W3, W2 = bb_inputs.make_ffn(64, 256, 704, seed=21)
    R = (1000.0 * bb_inputs.make_ffn(64, 256, 704, seed=22)[0].float()).to(torch.bfloat16)
    ref = orc.rmsnorm_swiglu_ffn_residual(X, g, W1, W3, W2, R, 1e-6)
    Y = bb.bb_rmsnorm_swiglu_ffn_residual(*dev((X, g, W1, W3, W2, R)), 1e-6).float().cpu().numpy().astype(np.float64)
    step = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - 7)       # bf16 spacing at |ref|
    ffn = ref - R.double().numpy()
    slack = 2e-2 * np.sqrt((ffn ** 2).mean(axis=1, keepdims=True))               # error of the FFN part itself
    assert np.all(np.abs(Y - ref) <= 0.5 * step + slack)


# ---------------------------------------------------------------- split contraction with 256-row tiles
@pytest.mark.parametrize("M,D,F", [(520, 1032, 4104),     # ragged rows, columns and contraction; odd steps per workgroup
                                   (520, 1032, 6144),     # even steps per workgroup
                                   (512, 1024, 8192),     # complete tiles: the variant without bounds checks
                                   (768, 768, 4096)])
def test_split_contraction_256_row_tiles(M, D, F):
    # the down projection of these shapes has few 256-row tiles and a long contraction: 256-row
    # tiles with the contraction split over workgroups (also through the transposed layout and
    # with the residual added by the reduce kernel)
    cpu = bb_inputs.make_ffn(M, D, F, seed=M + F)
    rows = sample_rows(M, extra=10, seed=1)
    X, g, W1, W3, W2 = cpu
    ref = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 1e-6, rows=rows)
    d = dev(cpu)
    Y = bb.bb_rmsnorm_swiglu_ffn(*d, 1e-6)
    assert row_rel_err(Y[rows], ref) <= TOL
    Yt = bb.bb_rmsnorm_swiglu_ffn_t(d[0], d[1], *[w.t().contiguous() for w in d[2:]], 1e-6)
    assert row_rel_err(Yt[rows], ref) <= TOL
    Yr = bb.bb_rmsnorm_swiglu_ffn_residual(*d, d[0], 1e-6)
    assert row_rel_err(Yr[rows], ref + X[rows].double().numpy()) <= TOL


# ---------------------------------------------------------------- tile order
# The tiles are walked in groups of row tiles (four 256-row tiles or eight 128-row tiles); shapes whose number of row
# tiles is no multiple of the group: 6 = 4 + 2 tiles of 256 rows (the last one ragged), 11 = 8 + 3 tiles of 128 rows.
@pytest.mark.parametrize("M,D,F", [(1300, 128, 3072), (1408, 128, 384), (1330, 72, 3080)])
@pytest.mark.parametrize("variant", [bb.VARIANT_SNAPSHOT1, bb.VARIANT_PRESCALE])
def test_tile_order_with_a_short_last_group_ffn(M, D, F, variant):
    cpu = bb_inputs.make_ffn(M, D, F, seed=M + F)
    assert ffn_case(cpu, 1e-6, variant=variant) <= TOL
    assert ffn_case(cpu, 1e-6, unfused=True) <= TOL


@pytest.mark.parametrize("M,D,N", [(1300, 128, 6144), (1408, 64, 768)])
def test_tile_order_with_a_short_last_group_ln(M, D, N):
    cpu = bb_inputs.make_ln(M, D, N, seed=M + N)
    ref = orc.layernorm_matmul(*cpu, 1e-5)
    for variant in (bb.VARIANT_PRESCALE, bb.VARIANT_SNAPSHOT1):
        bb.bb_set_variant(variant)
        try:
            Y = bb.bb_layernorm_matmul(*dev(cpu), 1e-5)
            torch.cuda.synchronize()
        finally:
            bb.bb_set_variant(bb.VARIANT_AUTO)
        assert row_rel_err(Y, ref) <= TOL


# Any number of rows runs through the kernels without bounds checks as long as the columns and the contraction
# are complete tiles: the ragged last row tile reads its last valid row in place of the missing ones and stores
# only the valid ones.  (In place over the residual a stored row past M would be visible as a changed R.)
@pytest.mark.parametrize("M,D,F", [(1, 64, 128), (257, 128, 256), (300, 256, 512), (1000, 512, 1024), (2047, 1024, 2816)])
def test_ragged_rows_on_complete_columns_ffn(M, D, F):
    cpu = bb_inputs.make_ffn(M, D, F, seed=M + F)
    for variant in (bb.VARIANT_SNAPSHOT1, bb.VARIANT_PRESCALE):
        if variant == bb.VARIANT_PRESCALE and M <= 16:
            continue
        assert ffn_case(cpu, 1e-6, variant=variant) <= TOL
    assert ffn_case(cpu, 1e-6, unfused=True) <= TOL
    bb.bb_set_variant(bb.VARIANT_SNAPSHOT1)
    try:
        assert residual_case(M, D, F, seed=M) <= TOL
        assert residual_case(M, D, F, seed=M, in_place="x") <= TOL
        assert residual_case(M, D, F, seed=M, transposed=True) <= TOL
    finally:
        bb.bb_set_variant(bb.VARIANT_AUTO)


# ... and any number of columns: a ragged last column tile reads its last valid chunk of columns in place of the
# missing ones.  Gate/up with 712 = 5 x 128 + 72 hidden units, down projections with 320 = 256 + 64 and
# 896 = 3 x 256 + 128 columns (contractions of 768 and 4864: complete steps), ragged rows on top.
@pytest.mark.parametrize("M,D,F", [(300, 256, 712), (300, 320, 768), (1000, 320, 1352), (700, 896, 4864)])
def test_ragged_columns_on_complete_contractions_ffn(M, D, F):
    cpu = bb_inputs.make_ffn(M, D, F, seed=M + F)
    rows = sample_rows(M, extra=10, seed=2)
    for variant in (bb.VARIANT_SNAPSHOT1, bb.VARIANT_PRESCALE):
        assert ffn_case(cpu, 1e-6, rows=rows, variant=variant) <= TOL
    assert ffn_case(cpu, 1e-6, rows=rows, unfused=True) <= TOL
    X, g, W1, W3, W2 = cpu
    ref = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 1e-6, rows=rows)
    d = dev(cpu)
    bb.bb_set_variant(bb.VARIANT_SNAPSHOT1)
    try:
        Yt = bb.bb_rmsnorm_swiglu_ffn_t(d[0], d[1], *[w.t().contiguous() for w in d[2:]], 1e-6)
        Yr = bb.bb_rmsnorm_swiglu_ffn_residual(*d, d[0], 1e-6)
        torch.cuda.synchronize()
    finally:
        bb.bb_set_variant(bb.VARIANT_AUTO)
    assert row_rel_err(Yt[rows], ref) <= TOL
    assert row_rel_err(Yr[rows], ref + X[rows].double().numpy()) <= TOL


@pytest.mark.parametrize("M,D,N", [(300, 256, 712), (1000, 320, 1352), (2047, 1024, 2056)])
def test_ragged_columns_on_complete_contractions_ln(M, D, N):
    cpu = bb_inputs.make_ln(M, D, N, seed=M + N)
    ref = orc.layernorm_matmul(*cpu, 1e-5)
    for variant in (bb.VARIANT_PRESCALE, bb.VARIANT_SNAPSHOT1, bb.VARIANT_UNFUSED):
        bb.bb_set_variant(variant)
        try:
            Y = bb.bb_layernorm_matmul(*dev(cpu), 1e-5)
            torch.cuda.synchronize()
        finally:
            bb.bb_set_variant(bb.VARIANT_AUTO)
        assert row_rel_err(Y, ref) <= TOL
    d = dev(cpu)
    Yt = bb.bb_layernorm_matmul_t(d[0], d[1], d[2], d[3].t().contiguous(), 1e-5)
    torch.cuda.synchronize()
    assert row_rel_err(Yt, ref) <= TOL


@pytest.mark.parametrize("M,D,N", [(1, 64, 256), (300, 256, 512), (1000, 512, 1024), (2047, 1024, 2048)])
def test_ragged_rows_on_complete_columns_ln(M, D, N):
    cpu = bb_inputs.make_ln(M, D, N, seed=M + N)
    ref = orc.layernorm_matmul(*cpu, 1e-5)
    for variant in (bb.VARIANT_PRESCALE, bb.VARIANT_SNAPSHOT1, bb.VARIANT_UNFUSED):
        bb.bb_set_variant(variant)
        try:
            Y = bb.bb_layernorm_matmul(*dev(cpu), 1e-5)
            torch.cuda.synchronize()
        finally:
            bb.bb_set_variant(bb.VARIANT_AUTO)
        assert row_rel_err(Y, ref) <= TOL
    d = dev(cpu)
    Yt = bb.bb_layernorm_matmul_t(d[0], d[1], d[2], d[3].t().contiguous(), 1e-5)
    torch.cuda.synchronize()
    assert row_rel_err(Yt, ref) <= TOL


# ---------------------------------------------------------------- statistics loop as its own kernel
@pytest.mark.parametrize("M,D,F", [(17, 72, 136), (130, 264, 712), (300, 520, 1032), (512, 1024, 2816),
                                   (2048, 1024, 2816)])
def test_prescale_variant(M, D, F):
    cpu = bb_inputs.make_ffn(M, D, F, seed=M + 1)
    err = ffn_case(cpu, 1e-6, variant=bb.VARIANT_PRESCALE)
    assert err <= TOL
    # same arithmetic as the fused prologue: bf16(x g) operands, inverse norm after the dots
    bb.bb_set_variant(bb.VARIANT_PRESCALE)
    try:
        Y1 = bb.bb_rmsnorm_swiglu_ffn(*dev(cpu), 1e-6)
    finally:
        bb.bb_set_variant(bb.VARIANT_AUTO)
    Y2 = bb.bb_rmsnorm_swiglu_ffn(*dev(cpu), 1e-6)
    diff = (Y1.float() - Y2.float()).abs().max().item()
    assert diff <= 2e-2 * Y2.float().abs().max().item()


def test_prescale_variant_refused_for_few_rows():
    cpu = bb_inputs.make_ffn(8, 256, 704, seed=2)
    bb.bb_set_variant(bb.VARIANT_PRESCALE)
    try:
        with pytest.raises(bb.BBError) as e:
            bb.bb_rmsnorm_swiglu_ffn(*dev(cpu), 1e-6)
        assert e.value.status == -9
    finally:
        bb.bb_set_variant(bb.VARIANT_AUTO)


@pytest.mark.parametrize("M,D,N", [(5, 72, 136), (200, 512, 768), (257, 264, 520), (1024, 1024, 2048)])
@pytest.mark.parametrize("variant", [bb.VARIANT_PRESCALE, bb.VARIANT_SNAPSHOT1])
def test_layernorm_variants(M, D, N, variant):
    # statistics by a row kernel (PRESCALE, what AUTO runs from 256 rows on) and inside the product
    # loop (SNAPSHOT1), untransposed and transposed weights
    cpu = bb_inputs.make_ln(M, D, N, seed=M + N)
    ref = orc.layernorm_matmul(*cpu, 1e-5)
    bb.bb_set_variant(variant)
    try:
        Y = bb.bb_layernorm_matmul(*dev(cpu), 1e-5)
    finally:
        bb.bb_set_variant(bb.VARIANT_AUTO)
    assert row_rel_err(Y, ref) <= TOL
    X, ga, be, W = dev(cpu)
    assert row_rel_err(bb.bb_layernorm_matmul_t(X, ga, be, W.t().contiguous(), 1e-5), ref) <= TOL


# ------------------------------------------------ few rows on transposed weights: the streaming kernel of that layout
@pytest.mark.parametrize("M,D,F", [(1, 8, 8), (2, 64, 64), (16, 256, 704), (3, 520, 1000), (16, 2048, 8192),
                                   (5, 4104, 11016), (7, 8192, 8192), (16, 512, 32768), (9, 1024, 40000)])
def test_transposed_stream_shapes(M, D, F):
    # ragged unit and column ranges per workgroup, idle workgroups (fewer units than workgroups), several
    # blocks of the model dimension in LDS (D > 4096), the widest plan (128 units per workgroup), and a
    # hidden size past the plan (falls back to the tiled kernels)
    X, g, W1, W3, W2 = bb_inputs.make_ffn(M, D, F, seed=M + D + F)
    ref = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 1e-6)
    d = dev((X, g, tr(W1), tr(W3), tr(W2)))
    Y = bb.bb_rmsnorm_swiglu_ffn_t(*d, 1e-6)
    torch.cuda.synchronize()
    assert row_rel_err(Y, ref) <= TOL
    # a second call reuses the barrier words and the hidden-block scratch
    Y2 = bb.bb_rmsnorm_swiglu_ffn_t(*d, 1e-6)
    torch.cuda.synchronize()
    assert torch.equal(Y.view(torch.uint16), Y2.view(torch.uint16))


def test_transposed_stream_c2_all_rows_and_layouts_agree():
    c = bb_inputs.CONFIGS["c2"]
    X, g, W1, W3, W2 = bb_inputs.make_config("c2")
    ref = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, c.eps)
    d = dev((X, g, W1, W3, W2))
    Yt = bb.bb_rmsnorm_swiglu_ffn_t(d[0], d[1], tr(d[2]), tr(d[3]), tr(d[4]), c.eps)
    Y = bb.bb_rmsnorm_swiglu_ffn(*d, c.eps)
    torch.cuda.synchronize()
    err = row_rel_err(Yt, ref)
    print("c2 transposed stream rel err", err)
    assert err <= TOL
    assert row_rel_err(Y, ref) <= TOL
    # interleaving the two streaming kernels (they share the barrier words) keeps both correct
    Yt2 = bb.bb_rmsnorm_swiglu_ffn_t(d[0], d[1], tr(d[2]), tr(d[3]), tr(d[4]), c.eps)
    torch.cuda.synchronize()
    assert torch.equal(Yt.view(torch.uint16), Yt2.view(torch.uint16))


def test_transposed_stream_residual_and_forced_tiled_variant():
    M, D, F = 11, 1024, 2816
    X, g, W1, W3, W2 = bb_inputs.make_ffn(M, D, F, seed=77)
    ref = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 1e-6)
    d = dev((X, g, tr(W1), tr(W3), tr(W2)))
    Yr = bb.bb_rmsnorm_swiglu_ffn_residual(*d, d[0], 1e-6, transposed=True)
    torch.cuda.synchronize()
    assert row_rel_err(Yr, ref + X.double().numpy()) <= TOL
    # in place: Y = R = X
    Xc = d[0].clone()
    bb.bb_rmsnorm_swiglu_ffn_residual(Xc, d[1], d[2], d[3], d[4], Xc, 1e-6, Y=Xc, transposed=True)
    torch.cuda.synchronize()
    assert torch.equal(Xc.view(torch.uint16), Yr.view(torch.uint16))
    bb.bb_set_variant(bb.VARIANT_SNAPSHOT1)           # the tiled kernels on the same operands
    try:
        Ys = bb.bb_rmsnorm_swiglu_ffn_t(*d, 1e-6)
        torch.cuda.synchronize()
    finally:
        bb.bb_set_variant(bb.VARIANT_AUTO)
    assert row_rel_err(Ys, ref) <= TOL


def test_transposed_stream_large_activations():
    # |x| ~ 1e3 with heavy tails: the statistics are fp32 sums of squares, the inverse norm comes after the dots
    M, D, F = 16, 4096, 1024
    X, g, W1, W3, W2 = bb_inputs.make_ffn(M, D, F, seed=5)
    X = (X.float() * 1000.0).to(torch.bfloat16)
    ref = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 1e-6)
    Y = bb.bb_rmsnorm_swiglu_ffn_t(*dev((X, g, tr(W1), tr(W3), tr(W2))), 1e-6)
    torch.cuda.synchronize()
    assert row_rel_err(Y, ref) <= TOL


# ------------------------------------------------ the streaming kernels keep no host-side state per launch
@pytest.mark.parametrize("transposed", [False, True])
def test_stream_kernels_replay_from_a_captured_graph(transposed):
    # the grid barriers' epoch lives in device memory, so a captured launch can be replayed: several
    # replays, with eager calls of both streaming kernels and new inputs in between, each compared with
    # the eager result on the same inputs
    M, D, F = 16, 1024, 2816
    X, g, W1, W3, W2 = bb_inputs.make_ffn(M, D, F, seed=31)
    d = dev((X, g, W1, W3, W2))
    dt = [d[0], d[1], tr(d[2]), tr(d[3]), tr(d[4])]
    call = (lambda Y: bb.bb_rmsnorm_swiglu_ffn_t(*dt, 1e-6, Y=Y)) if transposed else \
           (lambda Y: bb.bb_rmsnorm_swiglu_ffn(*d, 1e-6, Y=Y))
    out_g = torch.empty((M, D), dtype=torch.bfloat16, device="cuda")
    out_e = torch.empty_like(out_g)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(out_g)                                    # warm-up: workspace, kernel attributes
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(out_g)
    for rep in range(4):
        newX = bb_inputs.make_ffn(M, D, F, seed=40 + rep)[0].cuda()
        d[0].copy_(newX)
        graph.replay()
        torch.cuda.synchronize()
        call(out_e)                                    # eager, same inputs
        bb.bb_rmsnorm_swiglu_ffn(*d, 1e-6)             # and the other layout's kernel shares the barrier words
        bb.bb_rmsnorm_swiglu_ffn_t(*dt, 1e-6)
        torch.cuda.synchronize()
        assert torch.equal(out_g.view(torch.uint16), out_e.view(torch.uint16)), rep
    ref = orc.rmsnorm_swiglu_ffn(d[0].cpu(), g, W1, W3, W2, 1e-6)
    assert row_rel_err(out_g, ref) <= TOL
