"""Substitution rules 1-6, 8 and 9 (Section 4) on one graph of a block program.

Every ruleN_match(g) returns a Match (rule number, graph, what was matched)
or None; apply(match) performs the substitution in place and returns a short
description.  Rule 7 (peel off the first iteration) is not part of the
paper's algorithm and is not implemented.

Readings of points the text leaves open:
  * "if several subgraphs match, one is chosen arbitrarily": for the fusion
    rules 1 and 2 the pair of maps closest to each other in statement order,
    then the earliest; for the other rules the earliest.
  * a fused map takes the place of the first of the two maps; whatever the
    second one needs and stood between them moves in front of it.
  * Rule 4: the product moves to just behind the operator that produces its
    (now unscaled) left operand, or to the place of the removed scaling if
    that operand is an input of the graph; the new scaling takes the old
    place of the product.  Rule 5 puts its four new operators at the place of
    the removed shift.
  * Rule 2's "common parent": any value both maps take as an input.
  * Rule 9 composes unary elementwise operators.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Tuple

from .ir import Graph, In, Map, MapIn, MapOut, Node, Op, Out, Reduce, Value, dims_of


@dataclass
class Match:
    rule: int
    graph: Graph
    nodes: tuple
    dim: Optional[str] = None
    info: str = ""


# ------------------------------------------------------------------ helpers
def _body(g: Graph) -> List[Node]:
    return [n for n in g.nodes if not isinstance(n, In)]


def _new_map(dim: str, iterated: List[Value], broadcast: List[Value]) -> Tuple[Map, List[Value], List[Value]]:
    inner = Graph()
    m = Map(dim, inner)
    inner.parent = m
    ps, bs = [], []
    for v in iterated:
        p = In("", dims_of(v)[1:])
        inner.nodes.append(p)
        m.ins.append(MapIn(v, p, True))
        ps.append((p, 0))
    for v in broadcast:
        p = In("", dims_of(v))
        inner.nodes.append(p)
        m.ins.append(MapIn(v, p, False))
        bs.append((p, 0))
    return m, ps, bs


def _used_outside(g: Graph, v: Value, besides: Node) -> bool:
    return g.exported(v) or any(c is not besides for c in g.consumers(v))


def _merge_maps(g: Graph, u: Map, v: Map) -> None:
    """v's inner graph is appended to u's; edges u -> v become inner edges; inputs both take
    are shared; u stays where it is, v disappears"""
    g.hoist_dependencies(v, u)
    for vi in list(v.ins):
        if vi.outer[0] is u:                                  # produced by u: now an inner value
            v.inner.replace_uses((vi.param, 0), u.outs[vi.outer[1]].inner)
            v.inner.remove(vi.param)
            continue
        twin = next((ui for ui in u.ins if ui.outer == vi.outer and ui.iterated == vi.iterated), None)
        if twin is not None:                                  # the shared edge
            v.inner.replace_uses((vi.param, 0), (twin.param, 0))
            v.inner.remove(vi.param)
        else:
            u.ins.append(vi)
    # v's exported values may now be u's parameters or inner values: all live in u.inner
    params = [n for n in v.inner.nodes if isinstance(n, In)]
    rest = [n for n in v.inner.nodes if not isinstance(n, In)]
    n_params_u = sum(isinstance(n, In) for n in u.inner.nodes)
    u.inner.nodes[n_params_u:n_params_u] = params
    u.inner.nodes.extend(rest)
    for n in u.inner.nodes:
        if isinstance(n, Map):
            n.inner.parent = n
    # outputs: u's that are still wanted by someone else, then v's
    keep = [k for k in range(len(u.outs)) if _used_outside(g, (u, k), v)]
    new_outs = [u.outs[k] for k in keep] + list(v.outs)
    remap_u = {k: i for i, k in enumerate(keep)}
    base = len(keep)
    placeholder = Map(u.dim, Graph())                         # stands for the fused map while renumbering
    for k, i in remap_u.items():
        g.replace_uses((u, k), (placeholder, i))
    for j in range(len(v.outs)):
        g.replace_uses((v, j), (placeholder, base + j))
    u.outs = new_outs
    for i in range(len(new_outs)):
        g.replace_uses((placeholder, i), (u, i))
    g.remove(v)


def _closest(pairs):
    """of (u, v, gap, position) tuples the one with the smallest gap, then the earliest"""
    return min(pairs, key=lambda p: (p[2], p[3])) if pairs else None


# ------------------------------------------------------------------ rule 1
def rule1_match(g: Graph, dim: Optional[str] = None) -> Optional[Match]:
    cands = []
    maps = g.maps()
    for u in maps:
        for v in maps:
            if u is v or u.dim != v.dim or (dim and u.dim != dim):
                continue
            edges = [i for i in v.ins if i.outer[0] is u]
            if not edges or g.index(u) > g.index(v):
                continue
            # every edge must be a list u produces element by element and v consumes element by element
            if any(not i.iterated or u.outs[i.outer[1]].reduced for i in edges):
                continue
            if g.indirect_path(u, v):
                continue
            cands.append((u, v, g.index(v) - g.index(u), g.index(u)))
    best = _closest(cands)
    return Match(1, g, (best[0], best[1]), best[0].dim) if best else None


# ------------------------------------------------------------------ rule 2
def rule2_match(g: Graph, dim: Optional[str] = None) -> Optional[Match]:
    cands = []
    maps = g.maps()
    for a, u in enumerate(maps):
        for v in maps[a + 1:]:
            if u.dim != v.dim or (dim and u.dim != dim):
                continue
            if not any(x == y for x in u.args() for y in v.args()):
                continue
            if g.reachable(u, v) or g.reachable(v, u):
                continue
            cands.append((u, v, g.index(v) - g.index(u), g.index(u)))
    best = _closest(cands)
    return Match(2, g, (best[0], best[1]), best[0].dim) if best else None


# ------------------------------------------------------------------ rule 3
def rule3_match(g: Graph, dim: Optional[str] = None) -> Optional[Match]:
    for r in g.nodes:
        if isinstance(r, Reduce) and isinstance(r.arg[0], Map):
            u = r.arg[0]
            if u.dim == r.dim and not u.outs[r.arg[1]].reduced and (not dim or dim == u.dim):
                if dims_of(r.arg) == (u.dim,):
                    return Match(3, g, (u, r), u.dim)
    return None


def _apply3(m: Match) -> str:
    g, (u, r) = m.graph, m.nodes
    k = r.arg[1]
    if _used_outside(g, (u, k), r):
        u.outs.append(MapOut(u.outs[k].inner, True))
        new = (u, len(u.outs) - 1)
    else:
        u.outs[k].reduced = True
        new = (u, k)
    g.replace_uses((r, 0), new)
    g.remove(r)
    return f"fuse {u.dim}-map with reduction"


# ------------------------------------------------------------------ rule 9
def rule9_match(g: Graph) -> Optional[Match]:
    for v in g.nodes:
        if isinstance(v, Op) and v.fn == "ew" and len(v.operands) == 1:
            u = v.operands[0][0]
            if isinstance(u, Op) and u.fn == "ew" and len(u.operands) == 1:
                if g.consumers((u, 0)) == [v] and not g.exported((u, 0)):
                    return Match(9, g, (u, v))
    return None


def _apply9(m: Match) -> str:
    g, (u, v) = m.graph, m.nodes
    # f(g(x)): no extra parentheses where the placeholder already stands alone between parentheses
    bare = v.expr.count("{0}") == v.expr.count("({0})")
    v.expr = v.expr.replace("{0}", u.expr if bare else "(" + u.expr + ")")
    v.operands = list(u.operands)
    g.remove(u)
    return "fuse consecutive elementwise"


# ------------------------------------------------------------------ matmul / mapped scale recognition
def _mapped_row_op(u: Node, fns) -> Optional[Tuple[Value, Value]]:
    """u is a map whose inner graph is one row_scale / row_shift of the iterated element by a
    vector passed whole: returns (the list, the vector) as values of the enclosing graph"""
    if not isinstance(u, Map) or len(u.outs) != 1 or u.outs[0].reduced:
        return None
    body = _body(u.inner)
    if len(body) != 1 or not isinstance(body[0], Op) or body[0].fn not in fns:
        return None
    op = body[0]
    if u.outs[0].inner != (op, 0) or len(u.ins) != 2:
        return None
    a, c = op.operands
    ia = next((i for i in u.ins if (i.param, 0) == a), None)
    ic = next((i for i in u.ins if (i.param, 0) == c), None)
    if ia is None or ic is None or not ia.iterated or ic.iterated:
        return None
    return ia.outer, ic.outer


def _as_matmul(v: Node, left: Value, kdim: str):
    """v multiplies the list `left` (blocks along kdim, passed whole) with the rows of another
    list of lists: returns (MapIn of left, MapIn of the other operand, inner map over kdim) or None"""
    if not isinstance(v, Map) or len(v.ins) != 2 or len(v.outs) != 1 or v.outs[0].reduced:
        return None
    il = next((i for i in v.ins if i.outer == left), None)
    io = next((i for i in v.ins if i.outer != left), None)
    if il is None or io is None or il.iterated or not io.iterated:
        return None
    body = _body(v.inner)
    if len(body) == 2 and isinstance(body[0], Map) and isinstance(body[1], Reduce):
        km, red = body
        if red.arg != (km, 0) or red.dim != km.dim or v.outs[0].inner != (red, 0) or km.outs[0].reduced:
            return None
    elif len(body) == 1 and isinstance(body[0], Map):
        km = body[0]
        if v.outs[0].inner != (km, 0) or not km.outs[0].reduced:
            return None
    else:
        return None
    if km.dim != kdim or len(km.outs) != 1 or len(km.ins) != 2:
        return None
    kb = _body(km.inner)
    if len(kb) != 1 or not isinstance(kb[0], Op) or kb[0].fn != "dot" or km.outs[0].inner != (kb[0], 0):
        return None
    ka = next((i for i in km.ins if i.outer == (il.param, 0)), None)
    kbi = next((i for i in km.ins if i.outer == (io.param, 0)), None)
    if ka is None or kbi is None or not ka.iterated or not kbi.iterated:
        return None
    if kb[0].operands != [(ka.param, 0), (kbi.param, 0)]:       # the scaled / shifted list is the LEFT operand
        return None
    return il, io, km


def _scale_dot_match(g: Graph, fns, rule: int) -> Optional[Match]:
    for u in g.maps():
        got = _mapped_row_op(u, fns)
        if got is None or g.exported((u, 0)):
            continue
        cons = g.consumers((u, 0))
        if len(cons) != 1:                      # the mapped scale / shift may have no other outgoing edge
            continue
        mm = _as_matmul(cons[0], (u, 0), u.dim)
        if mm is None:
            continue
        return Match(rule, g, (u, cons[0]), cons[0].dim)
    return None


def rule4_match(g: Graph) -> Optional[Match]:
    return _scale_dot_match(g, ("row_scale",), 4)


def rule5_match(g: Graph) -> Optional[Match]:
    return _scale_dot_match(g, ("row_shift",), 5)


def _place_product(g: Graph, u: Map, v: Map, x: Value) -> None:
    """moves the product v to just behind the producer of its new left operand, or to u's place"""
    g.remove(v)
    if isinstance(x[0], In):
        g.insert_before(u, v)
    else:
        g.insert_after(x[0], v)


def _apply4(m: Match) -> str:
    g, (u, v) = m.graph, m.nodes
    x, c = _mapped_row_op(u, ("row_scale",))
    il, _, _ = _as_matmul(v, (u, 0), u.dim)
    s, ps, bs = _new_map(v.dim, [(v, 0)], [c])
    op = Op("row_scale", [ps[0], bs[0]])
    s.inner.nodes.append(op)
    s.outs.append(MapOut((op, 0), False))
    g.replace_uses((v, 0), (s, 0))
    s.ins[0].outer = (v, 0)
    g.insert_after(v, s)                       # the scaling takes the old place of the product
    il.outer = x
    _place_product(g, u, v, x)
    g.remove(u)
    return f"swap scale and dot: scaling moves behind the {v.dim}-map product"


def _apply5(m: Match) -> str:
    g, (u, v) = m.graph, m.nodes
    x, c = _mapped_row_op(u, ("row_shift",))
    il, io, km = _as_matmul(v, (u, 0), u.dim)
    # column sums of the right operand: per row of it, row_sum of every block, summed over the blocks
    cs, ps, _ = _new_map(v.dim, [io.outer], [])
    k2, p2, _ = _new_map(u.dim, [ps[0]], [])
    rs = Op("row_sum", [p2[0]])
    k2.inner.nodes.append(rs)
    k2.outs.append(MapOut((rs, 0), False))
    red = Reduce(u.dim, (k2, 0))
    cs.inner.nodes += [k2, red]
    cs.outs.append(MapOut((red, 0), False))
    # outer product of the shift vector with them
    om, po, bo = _new_map(v.dim, [(cs, 0)], [c])
    oo = Op("outer", [bo[0], po[0]])
    om.inner.nodes.append(oo)
    om.outs.append(MapOut((oo, 0), False))
    # sum of the two
    am, pa, _ = _new_map(v.dim, [(om, 0), (v, 0)], [])
    ao = Op("add", [pa[0], pa[1]])
    am.inner.nodes.append(ao)
    am.outs.append(MapOut((ao, 0), False))
    g.replace_uses((v, 0), (am, 0))
    am.ins[1].outer = (v, 0)
    il.outer = x
    g.remove(v)
    anchor = u if isinstance(x[0], In) else None
    new = [cs, om, v, am]
    if anchor is not None:
        for n in new:
            g.insert_before(u, n)
    else:
        at = x[0]
        for n in new:
            g.insert_after(at, n)
            at = n
    g.remove(u)
    return f"swap shift and dot: column sums, outer product and sum behind the {v.dim}-map product"


# ------------------------------------------------------------------ rule 8
def rule8_match(g: Graph) -> Optional[Match]:
    for u in g.maps():
        if _mapped_row_op(u, ("row_scale",)) is None or g.exported((u, 0)):
            continue
        cons = g.consumers((u, 0))
        if len(cons) >= 2 and all(_as_matmul(c, (u, 0), u.dim) is not None for c in cons):
            return Match(8, g, (u,) + tuple(cons), u.dim)
    return None


def _apply8(m: Match) -> str:
    g, u = m.graph, m.nodes[0]
    x, c = _mapped_row_op(u, ("row_scale",))
    for consumer in m.nodes[2:]:
        d, ps, bs = _new_map(u.dim, [x], [c])
        op = Op("row_scale", [ps[0], bs[0]])
        d.inner.nodes.append(op)
        d.outs.append(MapOut((op, 0), False))
        g.insert_before(consumer, d)
        consumer.replace_arg((u, 0), (d, 0))
    return "duplicate mapped scale"


# ------------------------------------------------------------------ rule 6
def rule6_match(g: Graph) -> Optional[Match]:
    """an X-map at the end of the graph (nothing in the graph consumes it) whose inner graph holds
    a Y-map, and a Y-map next to it in the graph, related as producer and consumer (a), through
    the same input of the graph (b) or through the same parent operator (c)"""
    body = [n for n in g.nodes if not isinstance(n, (In, Out))]
    for vx in g.maps():
        if g.node_consumers(vx) and any(not isinstance(c, Out) for c in g.node_consumers(vx)):
            continue
        others = [n for n in body if n is not vx]
        if not others:
            continue
        # everything the graph hands to its parent (or to the program's outputs) must come from vx
        if g.parent is not None and any(o.inner[0] is not vx for o in g.parent.outs):
            continue
        if g.parent is None and any(isinstance(n, Out) and n.arg[0] is not vx for n in g.nodes):
            continue
        for vy in vx.inner.maps():
            for u in others:
                if not isinstance(u, Map) or u.dim != vy.dim:
                    continue
                for yi in vy.ins:
                    if not yi.iterated or not isinstance(yi.outer[0], In):
                        continue
                    xi = next((i for i in vx.ins if i.param is yi.outer[0]), None)
                    if xi is None or xi.iterated:
                        continue
                    src = xi.outer                          # what vy walks, seen from the outer graph
                    if src[0] is u and not u.outs[src[1]].reduced:
                        return Match(6, g, (vx, u, vy), vx.dim, "a")
                    if any(ui.outer == src and ui.iterated for ui in u.ins):
                        return Match(6, g, (vx, u, vy), vx.dim, "b" if isinstance(src[0], In) else "c")
    return None


def _apply6(m: Match) -> str:
    g, vx = m.graph, m.nodes[0]
    moved = [n for n in g.nodes if not isinstance(n, (In, Out)) and n is not vx]
    for n in moved:
        g.remove(n)
    # values of the outer graph the moved operators use: graph inputs become parameters of vx
    def param_for(v: Value) -> Value:
        twin = next((i for i in vx.ins if i.outer == v and not i.iterated), None)
        if twin is None:
            p = In("", dims_of(v))
            n_params = sum(isinstance(n, In) for n in vx.inner.nodes)
            vx.inner.nodes.insert(n_params, p)
            twin = MapIn(v, p, False)
            vx.ins.append(twin)
        return (twin.param, 0)
    for n in moved:
        for a in n.args():
            if isinstance(a[0], In):
                n.replace_arg(a, param_for(a))
    # inputs of vx that the moved operators produce become inner edges
    for i in list(vx.ins):
        if any(i.outer[0] is n for n in moved):
            assert not i.iterated
            vx.inner.replace_uses((i.param, 0), i.outer)
            vx.inner.remove(i.param)
            vx.ins.remove(i)
    n_params = sum(isinstance(n, In) for n in vx.inner.nodes)
    vx.inner.nodes[n_params:n_params] = moved
    return f"extend {vx.dim}-map to the entire graph (variant {m.info})"


# ------------------------------------------------------------------ apply
def apply(m: Match) -> str:
    if m.rule == 1:
        u, v = m.nodes
        _merge_maps(m.graph, u, v)
        return f"fuse consecutive {u.dim}-maps"
    if m.rule == 2:
        u, v = m.nodes
        _merge_maps(m.graph, u, v)
        return f"fuse sibling {u.dim}-maps"
    return {3: _apply3, 4: _apply4, 5: _apply5, 6: _apply6, 8: _apply8, 9: _apply9}[m.rule](m)
