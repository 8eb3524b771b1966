"""Array program -> block program by lookup (Section 3.2, Table 2).

Every array operator becomes its predefined, fully unfused subgraph of block
operators: a map over the row-block dimension at the top level, everything
else nested inside.  The table's figures are not part of the text of the
paper; the subgraphs here are the ones its examples start from (the first
listing of each example is these subgraphs after the row maps were fused).

Matrices are lists of lists of blocks, (rows, columns) = two dimension names.
The second operand of a product is given transposed, as in the paper's block
programs (dot multiplies a block with the transpose of another).
"""
from __future__ import annotations

from typing import Dict, List, Tuple

from .ir import Graph, In, Map, MapIn, MapOut, Op, Out, Reduce, Value, dims_of


class Program:
    """Builder of a top-level block program."""

    def __init__(self):
        self.g = Graph()

    # ---- plumbing
    def input(self, name: str, dims: Tuple[str, str]) -> Value:
        n = In(name, tuple(dims))
        self.g.nodes.append(n)
        return (n, 0)

    def output(self, name: str, v: Value) -> None:
        self.g.nodes.append(Out(name, v))

    @staticmethod
    def _make_map(lists: List[Value], broadcast: List[Value], build) -> Map:
        """a map over the first dimension of `lists` (walked element by element) with `broadcast`
        passed whole; build(inner graph, parameters of lists, parameters of broadcast) returns
        the (inner value, reduced) pairs that become the map's outputs"""
        dim = dims_of(lists[0])[0]
        inner = Graph()
        m = Map(dim, inner)
        inner.parent = m
        ps, bs = [], []
        for v in lists:
            p = In("", dims_of(v)[1:])
            inner.nodes.append(p)
            m.ins.append(MapIn(v, p, True))
            ps.append((p, 0))
        for v in broadcast:
            p = In("", dims_of(v))
            inner.nodes.append(p)
            m.ins.append(MapIn(v, p, False))
            bs.append((p, 0))
        for v, red in build(inner, ps, bs):
            m.outs.append(MapOut(v, red))
        return m

    def _row_map(self, lists: List[Value], broadcast: List[Value], build) -> Map:
        """a top-level operator: the map over the row blocks (the caller appends it)"""
        return self._make_map(lists, broadcast, build)

    @classmethod
    def _sub_map(cls, g: Graph, lists: List[Value], broadcast: List[Value], build) -> Map:
        """a map appended to the inner graph g"""
        m = cls._make_map(lists, broadcast, build)
        g.nodes.append(m)
        return m

    @staticmethod
    def _op(g: Graph, fn: str, operands: List[Value], expr=None) -> Value:
        n = Op(fn, list(operands), expr)
        g.nodes.append(n)
        return (n, 0)

    # ---- Table 2
    def elementwise(self, a: Value, expr: str) -> Value:
        """f applied to every element: map over rows, map over columns, one elementwise operator"""
        def rows(g, ps, bs):
            m = self._sub_map(g, [ps[0]], [], lambda g2, p2, b2: [(self._op(g2, "ew", [p2[0]], expr), False)])
            return [((m, 0), False)]
        m = self._row_map([a], [], rows)
        self.g.nodes.append(m)
        return (m, 0)

    def binary(self, a: Value, b: Value, fn: str) -> Value:
        """blockwise add / mul of two equally blocked matrices"""
        def rows(g, ps, bs):
            m = self._sub_map(g, [ps[0], ps[1]], [], lambda g2, p2, b2: [(self._op(g2, fn, [p2[0], p2[1]]), False)])
            return [((m, 0), False)]
        m = self._row_map([a, b], [], rows)
        self.g.nodes.append(m)
        return (m, 0)

    def matmul(self, a: Value, bt: Value) -> Value:
        """a (rows x K blocks) times the transpose of bt (columns x K blocks): per row block and
        column block a map over K of dot, then the sum over K"""
        def rows(g, ps, bs):
            def cols(g2, p2, b2):
                def ks(g3, p3, b3):
                    return [(self._op(g3, "dot", [p3[0], p3[1]]), False)]
                km = self._sub_map(g2, [b2[0], p2[0]], [], ks)
                r = Reduce(km.dim, (km, 0))
                g2.nodes.append(r)
                return [((r, 0), False)]
            cm = self._sub_map(g, [bs[0]], [ps[0]], cols)
            return [((cm, 0), False)]
        m = self._row_map([a], [bt], rows)
        self.g.nodes.append(m)
        return (m, 0)

    def row_sums(self, a: Value) -> Value:
        """per row block: the list of row sums of its blocks (one map), as the softmax and the
        norms use it; the sum over the list is a separate operator (reduce_rows)"""
        def rows(g, ps, bs):
            m = self._sub_map(g, [ps[0]], [], lambda g2, p2, b2: [(self._op(g2, "row_sum", [p2[0]]), False)])
            return [((m, 0), False)]
        m = self._row_map([a], [], rows)
        self.g.nodes.append(m)
        return (m, 0)

    def reduce_then(self, partial: Value, expr: str, extra: List[Value] = ()) -> Value:
        """per row block: sum the list of partial results, then a scalar function of the sum
        (and of further per-row vectors): one map at the top level"""
        def rows(g, ps, bs):
            r = Reduce(dims_of(ps[0])[0], ps[0])
            g.nodes.append(r)
            return [(self._op(g, "ew", [(r, 0)] + ps[1:], expr), False)]
        m = self._row_map([partial] + list(extra), [], rows)
        self.g.nodes.append(m)
        return (m, 0)

    def row_apply(self, a: Value, c: Value, fn: str) -> Value:
        """row_scale / row_shift of every block of a row block by that row block's vector c"""
        def rows(g, ps, bs):
            m = self._sub_map(g, [ps[0]], [ps[1]], lambda g2, p2, b2: [(self._op(g2, fn, [p2[0], b2[0]]), False)])
            return [((m, 0), False)]
        m = self._row_map([a, c], [], rows)
        self.g.nodes.append(m)
        return (m, 0)

    # ---- array operators made of several block operators
    def softmax(self, a: Value) -> Value:
        e = self.elementwise(a, "exp({0})")
        s = self.row_sums(e)
        r = self.reduce_then(s, "1/{0}")
        return self.row_apply(e, r, "row_scale")

    def rmsnorm(self, a: Value) -> Value:
        """as Example 3 writes it: x / sqrt(sum of squares) per row"""
        sq = self.elementwise(a, "{0}**2")
        s = self.row_sums(sq)
        r = self.reduce_then(s, "1/sqrt({0})")
        return self.row_apply(a, r, "row_scale")

    def layernorm(self, a: Value, count: str) -> Value:
        """as Example 2 writes it: shift by minus the mean, scale by the inverse standard
        deviation sqrt(s2/k - (s1/k)^2); `count` names the constant k"""
        s1 = self.row_sums(a)
        neg_mean = self.reduce_then(s1, "-{0}/" + count)
        shifted = self.row_apply(a, neg_mean, "row_shift")
        sq = self.elementwise(a, "{0}**2")
        s2 = self.row_sums(sq)
        rstd = self.reduce_then(s2, "({0}/" + count + "-{1}**2)**(-0.5)", [neg_mean])
        return self.row_apply(shifted, rstd, "row_scale")


def example1() -> Graph:
    """Attention: softmax(Q K^T / sqrt(d)) V; K and V transposed as block-program inputs."""
    p = Program()
    q = p.input("Q", ("M", "D"))
    kt = p.input("KT", ("N", "D"))
    vt = p.input("VT", ("L", "N"))
    s = p.matmul(q, kt)
    s = p.elementwise(s, "{0}*(DD**-0.5)")
    pr = p.softmax(s)
    p.output("O", p.matmul(pr, vt))
    return p.g


def example2() -> Graph:
    """LayerNorm followed by a matrix product."""
    p = Program()
    x = p.input("X", ("M", "K"))
    yt = p.input("YT", ("N", "K"))
    p.output("Z", p.matmul(p.layernorm(x, "KK"), yt))
    return p.g


def example3() -> Graph:
    """RMSNorm followed by FFN-SwiGLU: (swish(X' W) * (X' V)) U."""
    p = Program()
    x = p.input("X", ("M", "D"))
    wt = p.input("WT", ("K", "D"))
    vt = p.input("VT", ("K", "D"))
    ut = p.input("UT", ("N", "K"))
    xn = p.rmsnorm(x)
    a = p.elementwise(p.matmul(xn, wt), "{0}/(1+exp(-{0}))")
    b = p.matmul(xn, vt)
    p.output("O", p.matmul(p.binary(a, b, "mul"), ut))
    return p.g


EXAMPLES = {"example1": example1, "example2": example2, "example3": example3}
