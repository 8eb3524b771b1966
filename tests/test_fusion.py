"""The host-side fusion tool (block programs, substitution rules, fuse()) against what the paper
states for its three worked examples: the rules applied step by step, the structure of every
snapshot (loop nest, intermediate lists, accumulations), and that every single substitution
preserves what the program computes."""
import os

import numpy as np
import pytest

from paper_2505_07829_amd import fusion
from paper_2505_07829_amd.fusion import algorithm, check, emit, lower, rules
from paper_2505_07829_amd.fusion.ir import (Graph, In, Map, MapIn, MapOut, Op, Out, Reduce, all_graphs,
                                            clone, dims_of)

GOLD = os.path.join(os.path.dirname(__file__), "golden")
NAMES = ["example1", "example2", "example3"]


def golden_traces():
    out = {}
    for line in open(os.path.join(GOLD, "fusion_traces.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, seq = line.split(":")
        out[name.strip()] = [tuple(int(x) for x in tok.split("|")) for tok in seq.split()]
    return out


def run(name):
    steps = []
    snaps = fusion.fuse(lower.EXAMPLES[name](), lambda r, w: steps.append((r, w)))
    return snaps, steps


@pytest.mark.parametrize("name", NAMES)
def test_initial_block_program_computes_the_array_program(name):
    g = lower.EXAMPLES[name]()
    g.check()
    assert check.max_error(g, name) < 1e-12
    # fully unfused: every operator of the top-level graph is a map over the row blocks
    assert all(isinstance(n, (In, Out)) or (isinstance(n, Map) and n.dim == "M") for n in g.nodes)


def test_initial_top_level_operator_counts():
    # Example 1: the two products, the division by sqrt(d) and softmax's four operators;
    # Example 2: LayerNorm's seven and the product; Example 3: RMSNorm's four, three products,
    # the Swish and the Hadamard product.  (The step headings fuse them 6, 7 and 8 times.)
    assert [len(lower.EXAMPLES[n]().maps()) for n in NAMES] == [7, 8, 9]


@pytest.mark.parametrize("name", NAMES)
def test_rule_sequence_matches_the_papers_steps(name):
    _, steps = run(name)
    want = golden_traces()[name]
    got = [r for r, _ in steps]
    assert len(got) == len(want) == {"example1": 17, "example2": 22, "example3": 26}[name]
    for i, (r, alts) in enumerate(zip(got, want)):
        assert r in alts, f"step {i + 1}: rule {r}, the paper applies {alts}"
    if name == "example2":
        assert sorted(got[11:17]) == [1, 1, 1, 1, 1, 2]


# What the paper says of the program after each round of fusion without map extension, as structure:
# the loop nest (emit.nest: X(...) a parallel loop over dimension X, x(...) a serial one), the number of
# intermediate lists left in global memory, of accumulating statements and of stores.
#   Example 1: first the softmax statistics and the unnormalised scores are produced per row block by a
#     serial loop over key blocks (one list of score blocks is left for the value product, which is a
#     parallel loop over value blocks); the extension moves that loop inside: one nest, nothing buffered.
#   Example 2: a statistics loop, then a parallel loop over column blocks with one contraction loop; the
#     extension fuses the statistics into that contraction loop.
#   Example 3: statistics loop, K-map (both products in one contraction loop), N-map over the hidden list;
#     the first extension pulls statistics and K-map under the N-map, the second fuses the statistics into
#     the products' contraction loop.
STRUCTURE = {
    "example1": [("M(n(d) L(n))", 1, 3, 2), ("M(L(n(d)))", 0, 3, 1)],
    "example2": [("M(k N(k))", 0, 4, 1), ("M(N(k))", 0, 4, 1)],
    "example3": [("M(d K(d) N(k))", 1, 4, 2), ("M(N(d k(d)))", 0, 4, 1), ("M(N(k(d)))", 0, 4, 1)],
}


@pytest.mark.parametrize("name", NAMES)
def test_snapshots_have_the_structure_the_paper_describes(name):
    snaps, _ = run(name)
    assert len(snaps) == len(STRUCTURE[name])
    for i, (s, (nest, lists, accumulations, stores)) in enumerate(zip(snaps, STRUCTURE[name])):
        s.check()
        lines = emit.skeleton(s).splitlines()
        got = (emit.nest(s), emit.intermediate_buffers(s), sum("+=" in l for l in lines),
               sum("store(" in l for l in lines))
        assert got == (nest, lists, accumulations, stores), f"{name} snapshot {i + 1}: {got}"
        # and it still is the array program, for block counts that differ per dimension
        assert check.max_error(s, name) < 1e-12


@pytest.mark.parametrize("name", NAMES)
@pytest.mark.parametrize("seed", [0, 1])
def test_every_substitution_preserves_the_result(name, seed):
    g = clone(lower.EXAMPLES[name]())
    errs = []

    def after(rule, what):
        g.check()
        errs.append((rule, check.max_error(g, name, seed)))

    algorithm.fuse_in_place(g, after)
    assert len(errs) >= 17
    assert max(e for _, e in errs) < 1e-12, errs


def test_fuse_leaves_its_argument_alone_and_snapshots_are_independent():
    g = lower.example3()
    before = emit.listing(g)
    snaps = fusion.fuse(g)
    assert emit.listing(g) == before
    texts = [emit.listing(s) for s in snaps]
    assert len(set(texts)) == 3
    rules.apply(rules.rule6_match(all_graphs(snaps[0])[1]))      # mutating one snapshot ...
    assert [emit.listing(s) for s in snaps[1:]] == texts[1:]     # ... leaves the others alone


def test_intermediate_lists_disappear():
    # buffered edges that are not program inputs / outputs, before and in each snapshot
    want = {"example1": (8, [1, 0]), "example2": (8, [0, 0]), "example3": (11, [1, 0, 0])}
    for name in NAMES:
        snaps, _ = run(name)
        assert emit.intermediate_buffers(lower.EXAMPLES[name]()) == want[name][0]
        assert [emit.intermediate_buffers(s) for s in snaps] == want[name][1]


def test_shared_parents_are_loaded_once():
    # Rule 2 merges the edges from the shared parent: one load where there were two or three
    def loads(g):
        return [l.split("load(")[1].split("[")[0] for l in emit.listing(g).splitlines() if "load(" in l]
    assert sorted(loads(run("example1")[0][-1])) == ["KT", "Q", "VT"]
    assert sorted(loads(run("example2")[0][-1])) == ["X", "YT"]
    assert sorted(loads(run("example3")[0][-1])) == ["UT", "VT", "WT", "X"]
    assert sorted(loads(run("example3")[0][0])) == ["I1", "UT", "VT", "WT", "X", "X"]


def test_first_snapshot_of_example3_is_the_program_the_tiled_kernels_run():
    # hidden activations written once per (row block, hidden block), nothing else materialised:
    # a statistics loop, a K-map with both products, scaling, Swish and Hadamard product in its
    # body, and an N-map contracting over K
    s = run("example3")[0][0]
    m_map = s.maps()[0]
    kinds = [(type(n).__name__, getattr(n, "dim", None)) for n in m_map.inner.nodes if not isinstance(n, In)]
    assert kinds == [("Map", "D"), ("Op", None), ("Map", "K"), ("Map", "N")]
    assert emit.intermediate_buffers(s) == 1
    assert "store(t13,I1[m,k])" in emit.listing(s)


# ---------------------------------------------------------------- single rules on small graphs
def _chain(with_detour):
    """top-level N-maps  A -> B  (elementwise each), optionally with A -> C(Reduce-like path) -> B"""
    p = lower.Program()
    x = p.input("X", ("N", "D"))
    a = p.elementwise(x, "{0}+1")
    if with_detour:
        s = p.row_sums(a)                       # A -> S
        r = p.reduce_then(s, "1/{0}")           # S -> R (per row vector)
        b = p.row_apply(a, r, "row_scale")      # A -> B and R -> B: indirect path A -> S -> R -> B
    else:
        b = p.elementwise(a, "{0}*2")
    p.output("Y", b)
    return p.g


def test_rule1_needs_no_indirect_path():
    g = _chain(False)
    m = rules.rule1_match(g)
    assert m and m.dim == "N"
    g2 = _chain(True)
    a, s, r, b = g2.maps()
    for _ in range(2):                          # A+S and then (A+S)+R fuse; B keeps waiting for R
        m = rules.rule1_match(g2)
        assert b not in m.nodes
        rules.apply(m)
    # now the only path is direct: the rest fuses
    m = rules.rule1_match(g2)
    assert m is not None and m.nodes[1] is b


def test_rule1_does_not_fuse_through_a_finished_reduction():
    # V takes U's reduced result whole: U must finish first
    g = lower.example1()
    snaps = fusion.fuse(g)
    inner = all_graphs(snaps[0])[1]             # [N-map (serial), 1/t, L-map]
    n_map, l_map = inner.maps()
    assert n_map.serial and rules.rule1_match(inner) is None and rules.rule2_match(inner) is None


def test_rule2_needs_mutually_unreachable_maps():
    p = lower.Program()
    x = p.input("X", ("M", "D"))
    a = p.elementwise(x, "{0}+1")
    b = p.binary(a, x, "add")                   # b depends on a and shares the parent X with it
    p.output("Y", b)
    assert rules.rule2_match(p.g) is None       # reachable: this case belongs to Rule 1
    assert rules.rule1_match(p.g) is not None
    p2 = lower.Program()
    x = p2.input("X", ("M", "D"))
    p2.output("A", p2.elementwise(x, "{0}+1"))
    p2.output("B", p2.elementwise(x, "{0}*2"))
    m = rules.rule2_match(p2.g)
    assert m is not None
    rules.apply(m)
    assert len(p2.g.maps()) == 1 and len(p2.g.maps()[0].ins) == 1     # one shared edge from X
    p2.g.check()


def test_rule3_keeps_a_list_somebody_else_reads():
    p = lower.Program()
    x = p.input("X", ("M", "D"))
    e = p.elementwise(x, "exp({0})")
    s = p.row_sums(e)
    r = p.reduce_then(s, "1/{0}")
    p.output("Y", p.row_apply(e, r, "row_scale"))
    p.output("S", s)                            # the list of partial sums is also an output
    g = p.g
    while rules.rule1_match(g):
        rules.apply(rules.rule1_match(g))
    inner = all_graphs(g)[1]
    m = rules.rule3_match(inner)
    assert m is not None
    u = m.nodes[0]
    n_outs = len(u.outs)
    rules.apply(m)
    assert len(u.outs) == n_outs + 1 and u.outs[-1].reduced and not u.outs[0].reduced
    g.check()


def test_rule4_needs_the_scaled_list_to_have_one_consumer():
    # Example 3 before Rule 8: the scaled X feeds two products, Rule 4 does not match, Rule 8 does
    g = lower.example3()
    algorithm.saturate(g)                       # top level: the M-maps
    inner = all_graphs(g)[1]
    assert rules.rule4_match(inner) is None
    m8 = rules.rule8_match(inner)
    assert m8 is not None and len(m8.nodes) == 3
    rules.apply(m8)
    assert rules.rule8_match(inner) is None and rules.rule4_match(inner) is not None


def test_rule4_only_for_the_left_operand():
    # scaling the rows of the RIGHT operand of a product is not a scaling of the result's rows
    p = lower.Program()
    a = p.input("A", ("M", "K"))
    b = p.input("B", ("N", "K"))
    c = p.input("C", ("N", "K"))
    s = p.row_sums(c)
    r = p.reduce_then(s, "1/{0}")
    bs = p.row_apply(b, r, "row_scale")          # rows of B scaled
    p.output("Y", p.matmul(a, bs))
    for gr in all_graphs(p.g):
        assert rules.rule4_match(gr) is None


def test_rule6_needs_the_map_at_the_end_of_its_graph():
    snaps, _ = run("example3")
    inner = all_graphs(snaps[0])[1]             # [D-map, 1/sqrt, K-map, N-map]
    m = rules.rule6_match(inner)
    assert m.dim == "N" and m.info == "a"       # not the K-map: the N-map consumes it
    final_graphs = all_graphs(snaps[-1])
    assert all(rules.rule6_match(gr) is None for gr in final_graphs)


def test_rule9_composes_expressions():
    p = lower.Program()
    x = p.input("X", ("M", "N"))
    p.output("Y", p.elementwise(p.elementwise(x, "{0}*(DD**-0.5)"), "exp({0})"))
    snaps = fusion.fuse(p.g)
    assert "exp(t1*(DD**-0.5))" in emit.listing(snaps[-1])
    p2 = lower.Program()
    x = p2.input("X", ("M", "N"))
    p2.output("Y", p2.elementwise(p2.elementwise(x, "{0}+1"), "{0}**2"))
    assert "(t1+1)**2" in emit.listing(fusion.fuse(p2.g)[-1])


def test_other_programs_fuse_and_stay_correct():
    # not one of the paper's examples: softmax of a product, both operands row-normalised
    p = lower.Program()
    a = p.input("Q", ("M", "D"))
    b = p.input("KT", ("N", "D"))
    p.output("O", p.softmax(p.matmul(p.rmsnorm(a), b)))
    rng = np.random.default_rng(3)
    A, B = rng.standard_normal((6, 8)), rng.standard_normal((4, 8))
    An = A / np.sqrt((A ** 2).sum(1, keepdims=True))
    P = np.exp(An @ B.T)
    want = P / P.sum(1, keepdims=True)
    from paper_2505_07829_amd.fusion.interp import assemble, evaluate, split
    for s in fusion.fuse(p.g):
        s.check()
        got = assemble(evaluate(s, {"Q": split(A, 2, 2), "KT": split(B, 2, 2)}, {})["O"])
        assert np.abs(got - want).max() < 1e-12


# ---------------------------------------------------------------- numerical safety (Appendix)
def _attention_blocks(scale, seed=0):
    from paper_2505_07829_amd.fusion.interp import split
    rng = np.random.default_rng(seed)
    c, e = check.COUNTS, check.EDGE
    Q = scale * rng.standard_normal((c["M"] * e["M"], c["D"] * e["D"]))
    K = rng.standard_normal((c["N"] * e["N"], c["D"] * e["D"]))
    V = rng.standard_normal((c["N"] * e["N"], c["L"] * e["L"]))
    dd = Q.shape[1]
    S = Q @ K.T / np.sqrt(dd)
    P = np.exp(S - S.max(axis=1, keepdims=True))                 # the textbook stable softmax
    want = (P / P.sum(axis=1, keepdims=True)) @ V
    ins = {"Q": split(Q, c["M"], c["D"]), "KT": split(K, c["N"], c["D"]), "VT": split(V.T.copy(), c["L"], c["N"])}
    return ins, {"DD": float(dd)}, want, S


def test_safety_pass_agrees_with_plain_arithmetic_on_moderate_scores():
    from paper_2505_07829_amd.fusion.interp import assemble, evaluate
    ins, consts, want, _ = _attention_blocks(1.0)
    for s in [lower.example1()] + fusion.fuse(lower.example1()):
        plain = assemble(evaluate(s, ins, consts)["O"])
        safe = assemble(evaluate(s, ins, consts, safe=True)["O"])
        assert np.abs(plain - want).max() < 1e-12 and np.abs(safe - want).max() < 1e-12


def test_safety_pass_survives_scores_that_overflow_the_plain_program():
    # scores of several thousand: exp overflows float64 (709), the unsafe programs return inf/nan,
    # the same programs evaluated with significand-exponent pairs match the stable softmax
    from paper_2505_07829_amd.fusion.interp import assemble, evaluate
    ins, consts, want, S = _attention_blocks(3000.0)
    assert S.max() > 1000
    for s in [lower.example1()] + fusion.fuse(lower.example1()):
        with np.errstate(over="ignore", invalid="ignore"):
            plain = assemble(evaluate(s, ins, consts)["O"])
        assert not np.all(np.isfinite(plain))
        safe = assemble(evaluate(s, ins, consts, safe=True)["O"])
        assert np.all(np.isfinite(safe)) and np.abs(safe - want).max() < 1e-9


def test_pair_addition_is_the_appendix_formula():
    from paper_2505_07829_amd.fusion.interp import Pair, pair_add
    a = Pair(np.array([[1.0, 2.0], [3.0, 4.0]]), np.array([5.0, -2.0]))
    b = Pair(np.array([[0.5, 0.25], [1.0, 1.0]]), np.array([3.0, 1.0]))
    c = pair_add(a, b)
    assert np.array_equal(c.t, [5.0, 1.0])                         # z = max(t1, t2) per row
    assert np.allclose(c.plain(), a.plain() + b.plain(), rtol=1e-15)
    assert np.allclose(c.s[0], a.s[0] + b.s[0] * np.exp(-2.0)) and np.allclose(c.s[1], a.s[1] * np.exp(-3.0) + b.s[1])
