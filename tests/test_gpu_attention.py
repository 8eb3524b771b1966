"""GPU parity of bb_attention (Example 1 with the Appendix's numerics) against
the fp64 oracle's definition softmax(Q K^T / sqrt(d)) V on the same seeded
bf16 inputs.  Gate, per query row:

    || O_gpu[i,:] - O_ref[i,:] ||_2 / || O_ref[i,:] ||_2  <=  2e-2

(scores and sums in fp32; the exponentiated scores are rounded to bf16 before
the second product, relative error 2^-9 each, and the output once more.)
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


def rel_err(O_gpu, O_ref):
    """the row figure; the element-wise gate (bb_parity.py) is asserted on the way"""
    row, elem = bb_parity.errors(O_gpu, O_ref)
    assert elem <= bb_parity.TOL_ELEM, f"element error {elem:.3e} > {bb_parity.TOL_ELEM} (row error {row:.3e})"
    return row


def run(Q, K, V, rows=None):
    O = bb.bb_attention(Q.cuda(), K.cuda(), V.cuda())
    torch.cuda.synchronize()
    ref = orc.attention(Q, K, V, rows=rows)
    flat = O.reshape(-1, O.shape[-1])
    return rel_err(flat if rows is None else flat[rows], ref)


@pytest.fixture(scope="module", autouse=True)
def _lib():
    bb.load()
    yield
    bb.bb_shutdown()


@pytest.mark.parametrize("d,dv", [(64, 64), (64, 128), (128, 64), (128, 128)])
def test_head_dimensions(d, dv):
    # several query blocks and key blocks, complete tiles
    err = run(*bb_inputs.make_attn(2, 256, 320, d, dv, seed=d + dv))
    print("attention", d, dv, "rel err", err)
    assert err <= TOL


@pytest.mark.parametrize("B,M,N", [(1, 1, 1), (1, 1, 7), (3, 5, 64), (2, 33, 65), (1, 128, 63), (2, 129, 127),
                                   (1, 300, 200), (5, 17, 449), (1, 64, 1)])
@pytest.mark.parametrize("d,dv", [(64, 64), (128, 128)])
def test_ragged_queries_and_keys(B, M, N, d, dv):
    err = run(*bb_inputs.make_attn(B, M, N, d, dv, seed=B + M + N))
    assert err <= TOL


def test_one_key_returns_its_value_row():
    # softmax over one key is 1: O[b, m, :] = V[b, 0, :] exactly (bf16 in, bf16 out)
    Q, K, V = bb_inputs.make_attn(2, 70, 1, 128, 128, seed=3)
    O = bb.bb_attention(Q.cuda(), K.cuda(), V.cuda()).cpu()
    assert torch.equal(O.view(torch.uint16), V.expand(2, 70, 128).contiguous().view(torch.uint16))


@pytest.mark.parametrize("q_scale", [8.0, 64.0, 400.0])
def test_large_scores_stay_finite_and_correct(q_scale):
    # scaled scores of size q_scale * N(0,1): exp overflows fp32 from about 89
    # without the row exponents; with them the result matches the definition.
    # (At the largest scale a row's softmax is close to one-hot.)
    Q, K, V = bb_inputs.make_attn(2, 130, 300, 128, 128, seed=11, q_scale=q_scale)
    assert run(Q, K, V) <= TOL


def test_maximum_moves_late_and_early():
    # the key with the largest score sits in the last block for half of the
    # queries and in the first block for the others: the accumulators are
    # rescaled by a tiny factor at the last step / never after the first
    Q, K, V = bb_inputs.make_attn(1, 128, 256, 64, 64, seed=5)
    K = K.float()
    Qf = Q.float()
    K[0, 250] = 3.0 * Qf[0, :64].mean(0) * 8     # aligned with the first 64 queries
    K[0, 3] = 3.0 * Qf[0, 64:].mean(0) * 8       # aligned with the others
    K = K.to(torch.bfloat16)
    assert run(Q, K, V) <= TOL


def test_constant_rows_uniform_softmax():
    # all keys equal: uniform weights, O = mean of V rows for every query
    Q, _, V = bb_inputs.make_attn(1, 40, 192, 64, 128, seed=9)
    K = torch.ones(1, 192, 64, dtype=torch.bfloat16)
    O = bb.bb_attention(Q.cuda(), K.cuda(), V.cuda()).float().cpu().numpy().astype(np.float64)
    want = V.double().numpy().mean(axis=1)                       # [1, dv]
    err = np.linalg.norm(O[0] - want, axis=1) / np.linalg.norm(want)
    assert err.max() <= TOL


def test_problems_are_independent():
    # one call with B problems equals B calls with one problem each, bit for bit
    Q, K, V = bb_inputs.make_attn(3, 150, 130, 128, 128, seed=21)
    Qd, Kd, Vd = Q.cuda(), K.cuda(), V.cuda()
    O = bb.bb_attention(Qd, Kd, Vd)
    for b in range(3):
        Ob = bb.bb_attention(Qd[b:b + 1].contiguous(), Kd[b:b + 1].contiguous(), Vd[b:b + 1].contiguous())
        assert torch.equal(O[b].view(torch.uint16), Ob[0].view(torch.uint16))


def test_output_buffer_tail_untouched():
    # M not a multiple of the query block: rows past M are not written
    Q, K, V = bb_inputs.make_attn(1, 100, 100, 64, 64, seed=2)
    buf = torch.full((1, 128, 64), 7.0, dtype=torch.bfloat16, device="cuda")
    lib = bb.load()
    from paper_2505_07829_amd.binding import _ptr, _stream
    Qd, Kd, Vd = Q.cuda(), K.cuda(), V.cuda()
    rc = lib.bb_attention(_ptr(Qd), _ptr(Kd), _ptr(Vd), _ptr(buf), 1, 100, 100, 64, 64, _stream())
    assert rc == 0
    torch.cuda.synchronize()
    assert torch.all(buf[0, 100:] == 7.0)
    ref = orc.attention(Q, K, V)
    assert rel_err(buf[0, :100], ref) <= TOL


def test_empty_batches_are_noops():
    Q, K, V = bb_inputs.make_attn(1, 8, 8, 64, 64, seed=1)
    O = bb.bb_attention(Q[:0].cuda(), K[:0].cuda(), V[:0].cuda())
    assert O.shape == (0, 8, 64)
    O = bb.bb_attention(Q[:, :0].cuda(), K.cuda(), V.cuda())
    assert O.shape == (1, 0, 64)


def test_bench_size_sampled_rows():
    # the workload bench.py times for attention: 32 heads x 4096 x 4096, d = dv = 128;
    # the oracle computes sampled query rows (first/last of query blocks, random ones)
    B, M, N, d = 32, 4096, 4096, 128
    Q, K, V = bb_inputs.make_attn(B, M, N, d, d, seed=0)
    rng = np.random.default_rng(0)
    rows = sorted(set([0, 127, 128, M - 1, (B - 1) * M, B * M - 1, 17 * M + 2047, 17 * M + 2048]
                      + [int(r) for r in rng.integers(0, B * M, size=24)]))
    err = run(Q, K, V, rows=rows)
    print("attention bench size rel err", err)
    assert err <= TOL


def test_eight_wavefront_workgroups_on_the_shape_that_selects_them():
    # head dimension 128, M a multiple of 256 and enough query blocks for every compute unit:
    # 256 queries per workgroup; parity as everywhere else
    Q, K, V = bb_inputs.make_attn(64, 1024, 384, 128, 128, seed=8)
    assert run(Q, K, V, rows=list(range(0, 64 * 1024, 997))) <= TOL


# ---------------------------------------------------------------- few queries: keys split over workgroups
@pytest.mark.parametrize("B,M,N", [(32, 1, 4096), (8, 1, 8192), (4, 16, 2048), (2, 130, 4096), (1, 1, 777),
                                   (3, 5, 64 * 13), (16, 1, 4096 + 17), (3, 1, 1), (2, 1, 63), (5, 1, 257),
                                   (1, 1, 70000), (600, 1, 1100), (2, 2, 8192)])
@pytest.mark.parametrize("d,dv", [(128, 128), (64, 128), (128, 64), (64, 64)])
def test_split_keys_decode_shapes(B, M, N, d, dv):
    # (several of these split the keys, the ones whose block count has no suitable divisor or that
    # are short do not; bb_attention_workspace_bytes says which)
    err = run(*bb_inputs.make_attn(B, M, N, d, dv, seed=B + N))
    assert err <= TOL


def test_split_keys_is_taken_and_needs_workspace():
    assert bb.bb_attention_workspace_bytes(32, 1, 4096, 128, 128) > 0
    assert bb.bb_attention_workspace_bytes(32, 2, 4096, 128, 128) > 0
    assert bb.bb_attention_workspace_bytes(1, 1, 1, 128, 128) > 0              # one query: always (slots + counters)
    assert bb.bb_attention_workspace_bytes(32, 4096, 4096, 128, 128) == 0      # enough query blocks
    assert bb.bb_attention_workspace_bytes(32, 2, 256, 128, 128) == 0          # short sequence
    assert bb.bb_attention_workspace_bytes(1, 2, 64 * 13, 128, 128) == 0       # 13 blocks: no divisor
    assert bb.bb_attention_workspace_bytes(2, 2, 4096, 96, 128) == 0           # invalid head dimension


def test_split_keys_large_scores_and_late_maximum():
    # the maximum of a row sits in the last split for some queries and in the first for others, and
    # the scores are large: the partial results carry very different exponents
    Q, K, V = bb_inputs.make_attn(2, 8, 4096, 128, 128, seed=4, q_scale=30.0)
    K = K.float()
    K[0, 4090] = 4.0 * Q[0, 0].float()
    K[1, 5] = 4.0 * Q[1, 3].float()
    assert run(Q, K.to(torch.bfloat16), V) <= TOL


def test_split_keys_with_caller_workspace_too_small_is_an_error():
    Q, K, V = [t.cuda() for t in bb_inputs.make_attn(32, 1, 4096, 128, 128, seed=1)]
    need = bb.bb_attention_workspace_bytes(32, 1, 4096, 128, 128)
    ws = torch.zeros(need // 2 // 256 * 256, dtype=torch.uint8, device="cuda")
    bb.bb_set_workspace(ws)
    try:
        with pytest.raises(bb.BBError) as e:
            bb.bb_attention(Q, K, V)
        assert e.value.status == -7
        big = torch.zeros(need, dtype=torch.uint8, device="cuda")
        bb.bb_set_workspace(big)
        O = bb.bb_attention(Q, K, V)
        torch.cuda.synchronize()
        assert torch.isfinite(O.float()).all()
    finally:
        bb.bb_set_workspace(None)


def test_split_keys_arrival_counters_survive_other_calls():
    # few query rows: the last workgroup of a (problem, query block) to finish adds the partial
    # results; its counters sit at the start of the workspace that the other entry points also use.
    # Calls in a row, with other batch sizes and with a streaming FFN call between them, must each
    # give the oracle's result (a counter left non-zero would leave rows of O unwritten).
    cases = [bb_inputs.make_attn(B, M, 4096, 128, 128, seed=40 + B) for B, M in [(32, 1), (4, 3), (32, 1), (9, 16)]]
    refs = [orc.attention(*c) for c in cases]
    X, g, W1, W3, W2 = [t.cuda() for t in bb_inputs.make_ffn(8, 512, 1024, seed=3)]
    for rep in range(3):
        for (Q, K, V), ref in zip(cases, refs):
            O = bb.bb_attention(Q.cuda(), K.cuda(), V.cuda())
            O2 = bb.bb_attention(Q.cuda(), K.cuda(), V.cuda())
            torch.cuda.synchronize()
            assert rel_err(O.reshape(-1, 128), ref) <= TOL
            assert torch.equal(O, O2)                          # fixed order of addition: the same bits
            if rep == 1:
                bb.bb_rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 1e-6)


@pytest.mark.parametrize("pos", [5, 2000, 4090])
def test_one_query_large_scores_maximum_early_middle_late(pos):
    # one query per problem (the streaming kernel): a dominant key in the first, a middle or the last
    # workgroup's range; the other slots' exponents are far below it
    Q, K, V = bb_inputs.make_attn(3, 1, 4096, 128, 128, seed=6, q_scale=30.0)
    K = K.float()
    K[1, pos] = 4.0 * Q[1, 0].float()
    assert run(Q, K.to(torch.bfloat16), V) <= TOL


def test_one_query_constant_keys_give_the_mean_of_the_values():
    # closed form: equal scores -> uniform weights -> O = mean of V's rows (ragged N: masked keys weigh 0)
    B, N = 2, 1000
    Q = torch.ones(B, 1, 128, dtype=torch.bfloat16)
    K = torch.full((B, N, 128), 0.5, dtype=torch.bfloat16)
    V = bb_inputs.make_attn(B, 1, N, 128, 128, seed=2)[2]
    O = bb.bb_attention(Q.cuda(), K.cuda(), V.cuda())
    torch.cuda.synchronize()
    mean = V.double().mean(dim=1).numpy()
    assert rel_err(O.reshape(B, 128), mean) <= TOL


def test_one_query_a_million_keys():
    # hundreds of workgroups share the one problem, several key blocks per wavefront, ragged end
    Q, K, V = bb_inputs.make_attn(1, 1, 1_000_003, 128, 128, seed=12)
    assert run(Q, K, V) <= TOL


def test_one_query_replays_from_a_captured_graph():
    # the arrival counters are device memory that every launch leaves at zero, so a captured launch can be
    # replayed: several replays, with eager one-query calls (other batch sizes too) and new inputs in
    # between, each compared with the eager result on the same inputs
    B, N = 8, 3000
    Q, K, V = [t.cuda() for t in bb_inputs.make_attn(B, 1, N, 128, 128, seed=21)]
    other = [t.cuda() for t in bb_inputs.make_attn(20, 1, 777, 128, 128, seed=22)]
    out_g = torch.empty((B, 1, 128), dtype=torch.bfloat16, device="cuda")
    out_e = torch.empty_like(out_g)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        bb.bb_attention(*other)                        # warm-up: workspace and counters for the larger batch
        bb.bb_attention(Q, K, V, O=out_g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        bb.bb_attention(Q, K, V, O=out_g)
    for rep in range(4):
        Q.copy_(bb_inputs.make_attn(B, 1, N, 128, 128, seed=50 + rep)[0].cuda())
        graph.replay()
        torch.cuda.synchronize()
        bb.bb_attention(Q, K, V, O=out_e)              # eager, same inputs
        bb.bb_attention(*other)
        torch.cuda.synchronize()
        assert torch.equal(out_g.view(torch.uint16), out_e.view(torch.uint16)), rep
    ref = orc.attention(Q.cpu(), K.cpu(), V.cpu())
    assert rel_err(out_g.reshape(-1, 128), ref) <= TOL
