"""Block programs (Section 3): a hierarchical DAG of block operators.

A graph is an ORDERED list of nodes (always a valid topological order; the
order is the order statements are printed in).  Node kinds:

  In      an input of the graph: a program input (top level) or a parameter
          bound by the enclosing map
  Op      functional operator on items in local memory (Table 1 and
          elementwise expressions)
  Map     embarrassingly parallel loop over one dimension with an inner graph;
          an output flagged `reduced` is summed over the iterations instead of
          collected into a list (Rule 3 moved a reduction inside): the loop is
          then printed as a serial `for`
  Reduce  sum of a list over one dimension
  Out     a program output (top level only)

A value is a pair (node, k): output k of the node.  The type of a value is the
tuple of dimensions it is a list over, outermost first: () is a single block,
vector or scalar in local memory (an unbuffered edge), anything else lives in
global memory (a buffered edge).
"""
from __future__ import annotations

import copy
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

Value = Tuple["Node", int]

FUNCTIONAL = ("dot", "row_sum", "row_scale", "row_shift", "outer", "add", "mul", "ew")


class Node:
    def args(self) -> List[Value]:
        return []

    def replace_arg(self, old: Value, new: Value) -> None:
        pass

    @property
    def n_out(self) -> int:
        return 1


@dataclass(eq=False)
class In(Node):
    name: str
    dims: Tuple[str, ...]


@dataclass(eq=False)
class Op(Node):
    fn: str                      # one of FUNCTIONAL
    operands: List[Value]
    expr: Optional[str] = None   # fn == "ew": expression with placeholders {0}, {1}, ...

    def args(self):
        return list(self.operands)

    def replace_arg(self, old, new):
        self.operands = [new if a == old else a for a in self.operands]


@dataclass(eq=False)
class Reduce(Node):
    dim: str
    arg: Value

    def args(self):
        return [self.arg]

    def replace_arg(self, old, new):
        if self.arg == old:
            self.arg = new


@dataclass(eq=False)
class Out(Node):
    name: str
    arg: Value

    def args(self):
        return [self.arg]

    def replace_arg(self, old, new):
        if self.arg == old:
            self.arg = new

    @property
    def n_out(self):
        return 0


@dataclass(eq=False)
class MapIn:
    outer: Value          # value in the enclosing graph
    param: In             # the In node of the inner graph it is bound to
    iterated: bool        # True: the map walks this list; False: passed whole


@dataclass(eq=False)
class MapOut:
    inner: Value          # value of the inner graph
    reduced: bool         # True: summed over the iterations


@dataclass(eq=False)
class Map(Node):
    dim: str
    inner: "Graph"
    ins: List[MapIn] = field(default_factory=list)
    outs: List[MapOut] = field(default_factory=list)

    def args(self):
        return [i.outer for i in self.ins]

    def replace_arg(self, old, new):
        for i in self.ins:
            if i.outer == old:
                i.outer = new

    @property
    def n_out(self):
        return len(self.outs)

    @property
    def serial(self) -> bool:
        return any(o.reduced for o in self.outs)


@dataclass(eq=False)
class Graph:
    nodes: List[Node] = field(default_factory=list)
    parent: Optional[Map] = None      # the map this graph is the inner graph of

    # ---- queries
    def index(self, n: Node) -> int:
        for i, m in enumerate(self.nodes):
            if m is n:
                return i
        raise ValueError("node not in graph")

    def maps(self) -> List[Map]:
        return [n for n in self.nodes if isinstance(n, Map)]

    def consumers(self, v: Value) -> List[Node]:
        return [n for n in self.nodes if any(a == v for a in n.args())]

    def node_consumers(self, n: Node) -> List[Node]:
        return [m for m in self.nodes if any(a[0] is n for a in m.args())]

    def exported(self, v: Value) -> bool:
        """is v an output of the enclosing map?"""
        return self.parent is not None and any(o.inner == v for o in self.parent.outs)

    def reachable(self, a: Node, b: Node) -> bool:
        """is there a path a -> ... -> b (one or more edges)?"""
        seen, stack = set(), [a]
        while stack:
            x = stack.pop()
            for c in self.node_consumers(x):
                if c is b:
                    return True
                if id(c) not in seen:
                    seen.add(id(c))
                    stack.append(c)
        return False

    def indirect_path(self, a: Node, b: Node) -> bool:
        """a path from a to b through at least one other node"""
        return any(c is not b and self.reachable(c, b) for c in self.node_consumers(a))

    def ancestors(self, n: Node) -> List[Node]:
        seen, out, stack = set(), [], [n]
        while stack:
            x = stack.pop()
            for a in x.args():
                if id(a[0]) not in seen:
                    seen.add(id(a[0]))
                    out.append(a[0])
                    stack.append(a[0])
        return out

    # ---- edits
    def replace_uses(self, old: Value, new: Value) -> None:
        for n in self.nodes:
            n.replace_arg(old, new)
        if self.parent is not None:
            for o in self.parent.outs:
                if o.inner == old:
                    o.inner = new

    def remove(self, n: Node) -> None:
        self.nodes.pop(self.index(n))

    def insert_before(self, anchor: Node, new: Node) -> None:
        self.nodes.insert(self.index(anchor), new)

    def insert_after(self, anchor: Node, new: Node) -> None:
        self.nodes.insert(self.index(anchor) + 1, new)

    def hoist_dependencies(self, n: Node, floor: Node) -> None:
        """moves every ancestor of n that currently sits after `floor` to just
        before `floor`, keeping their order (used when two maps fuse at the
        position of the first one)"""
        fi = self.index(floor)
        anc = {id(a) for a in self.ancestors(n)}
        late = [m for m in self.nodes[fi + 1:] if id(m) in anc]
        for m in late:
            self.remove(m)
        fi = self.index(floor)
        for k, m in enumerate(late):
            self.nodes.insert(fi + k, m)

    def check(self) -> None:
        """order is topological, every argument is defined in this graph"""
        seen = set()
        for n in self.nodes:
            for a in n.args():
                assert id(a[0]) in seen, f"use before definition: {n}"
            seen.add(id(n))
            if isinstance(n, Map):
                assert n.inner.parent is n
                for i in n.ins:
                    assert any(p is i.param for p in n.inner.nodes)
                    want = dims_of(i.outer)
                    if i.iterated:
                        assert want and want[0] == n.dim, (want, n.dim)
                        want = want[1:]
                    assert tuple(i.param.dims) == tuple(want), (i.param.dims, want)
                for o in n.outs:
                    assert any(o.inner[0] is m for m in n.inner.nodes)
                    if o.reduced:
                        assert dims_of(o.inner) == ()
                n.inner.check()


def dims_of(v: Value) -> Tuple[str, ...]:
    n, k = v
    if isinstance(n, In):
        return tuple(n.dims)
    if isinstance(n, Op):
        return ()
    if isinstance(n, Reduce):
        d = dims_of(n.arg)
        assert d and d[0] == n.dim
        return d[1:]
    if isinstance(n, Map):
        o = n.outs[k]
        return dims_of(o.inner) if o.reduced else (n.dim,) + dims_of(o.inner)
    raise TypeError(n)


def all_graphs(g: Graph) -> List[Graph]:
    """g and every inner graph, breadth first"""
    out, queue = [], [g]
    while queue:
        x = queue.pop(0)
        out.append(x)
        queue.extend(m.inner for m in x.maps())
    return out


def clone(g: Graph) -> Graph:
    return copy.deepcopy(g)
