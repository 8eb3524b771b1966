"""Block program -> code, in the conventions of the paper's listings
(Section 3.1 and the examples): a map is a `forall` loop, a map that carries a
reduction and a reduction operator are serial `for` loops, list elements are
read with load(...) right before their first use in a loop body and written
with store(...) right after they are computed, local variables are t1, t2, ...
in order of appearance and accumulators start at zero, intermediate lists in
global memory are I1, I2, ... in order of their first store.

`listing(g)` returns the text; `skeleton(g)` the same program with the loads
folded into the expressions that use them and no variable numbers on plain
loads, one statement per line; `nest(g)` only the loop structure.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

from .ir import Graph, In, Map, Node, Op, Out, Reduce, Value, dims_of


class _Buffer:
    def __init__(self, name=None):
        self.name = name


class _Emitter:
    def __init__(self, fold_loads: bool):
        self.lines: List[str] = []
        self.nt = 0
        self.nbuf = 0
        self.fold = fold_loads

    def temp(self) -> str:
        self.nt += 1
        return f"t{self.nt}"

    def bufname(self, b: _Buffer) -> str:
        if b.name is None:
            self.nbuf += 1
            b.name = f"I{self.nbuf}"
        return b.name

    def put(self, depth: int, text: str) -> None:
        self.lines.append("\t" * depth + text)

    # env: id(node) -> list (one per output) of locations:
    #   ("temp", name) | ("list", buffer, [index vars]) | ("elem", buffer, [index vars]) (not loaded yet)
    def ref(self, env, v: Value, depth: int) -> str:
        loc = env[id(v[0])][v[1]]
        if loc[0] == "temp":
            return loc[1]
        if loc[0] == "elem":
            text = f"load({self.bufname(loc[1])}[{','.join(loc[2])}])"
            if self.fold:
                return text[5:-1]
            t = self.temp()
            self.put(depth, f"{t} = {text}")
            env[id(v[0])][v[1]] = ("temp", t)
            return t
        raise TypeError("a list has no local name")

    def expr(self, n: Op, names: List[str]) -> str:
        if n.fn == "ew":
            return n.expr.format(*names)
        return f"{n.fn}({','.join(names)})"

    def graph(self, g: Graph, env, depth: int, dest: Dict[Tuple[int, int], tuple]) -> None:
        """dest: (id(node), k) -> ("store", buffer, index vars) for values the enclosing map
        collects into a list, ("acc", temp name) for values it sums"""
        for n in g.nodes:
            if isinstance(n, (In, Out)):
                continue
            if isinstance(n, Op):
                names = [self.ref(env, a, depth) for a in n.operands]
                d = dest.get((id(n), 0))
                only_acc = d is not None and d[0] == "acc" and not g.consumers((n, 0))
                if only_acc:
                    self.put(depth, f"{d[1]} += {self.expr(n, names)}")
                    env[id(n)] = [("temp", d[1])]
                    continue
                t = self.temp()
                self.put(depth, f"{t} = {self.expr(n, names)}")
                env[id(n)] = [("temp", t)]
                self.finish(n, 0, t, d, depth)
            elif isinstance(n, Reduce):
                loc = env[id(n.arg[0])][n.arg[1]]
                assert loc[0] == "list"
                var = n.dim.lower()
                self.put(depth, f"for {var} in range({n.dim}):")
                src = f"{self.bufname(loc[1])}[{','.join(loc[2] + [var])}]"
                d = dest.get((id(n), 0))
                acc = d[1] if (d is not None and d[0] == "acc" and not g.consumers((n, 0))) else None
                if self.fold:
                    t = acc or self.temp()
                    self.put(depth + 1, f"{t} += {src}")
                else:
                    t1 = self.temp()
                    self.put(depth + 1, f"{t1} = load({src})")
                    t = acc or self.temp()
                    self.put(depth + 1, f"{t} += {t1}")
                env[id(n)] = [("temp", t)]
                if acc is None:
                    self.finish(n, 0, t, d, depth)
            elif isinstance(n, Map):
                self.map(g, n, env, depth, dest)

    def finish(self, n: Node, k: int, t: str, d, depth: int) -> None:
        if d is None:
            return
        if d[0] == "store":
            self.put(depth, f"store({t},{self.bufname(d[1])}[{','.join(d[2])}])")
        else:
            self.put(depth, f"{d[1]} += {t}")

    def map(self, g: Graph, m: Map, env, depth: int, dest) -> None:
        var = m.dim.lower()
        self.put(depth, f"{'for' if m.serial else 'forall'} {var} in range({m.dim}):")
        inner_env = dict()
        for i in m.ins:
            loc = env[id(i.outer[0])][i.outer[1]]
            if i.iterated:
                assert loc[0] == "list"
                idx = loc[2] + [var]
                inner_env[id(i.param)] = [("list", loc[1], idx) if i.param.dims else ("elem", loc[1], idx)]
            else:
                inner_env[id(i.param)] = [loc]
        inner_dest: Dict[Tuple[int, int], tuple] = {}
        outs_loc = []
        for k, o in enumerate(m.outs):
            key = (id(o.inner[0]), o.inner[1])
            if o.reduced:
                d = dest.get((id(m), k))
                reuse = d is not None and d[0] == "acc" and not g.consumers((m, k))
                t = d[1] if reuse else self.temp_later()
                inner_dest[key] = ("acc", t)
                outs_loc.append(("temp", t))
            else:
                d = dest.get((id(m), k))
                if d is not None and d[0] == "store":
                    buf, idx = d[1], d[2]          # the enclosing map collects this list: same buffer
                else:
                    buf, idx = self.buffer_for(g, m, k), self.scope_index(env)
                inner_dest[key] = ("store", buf, idx + [var])
                outs_loc.append(("list", buf, idx))
        env[id(m)] = outs_loc
        inner_env["__index__"] = self.scope_index(env) + [var]
        # a value that is both collected and summed, or exported twice, keeps the first destination only
        self.graph(m.inner, inner_env, depth + 1, inner_dest)
        # accumulators whose name was reserved lazily are named when first used inside
        for k, o in enumerate(m.outs):
            if o.reduced:
                loc = outs_loc[k]
                if isinstance(loc[1], _Lazy):
                    outs_loc[k] = ("temp", loc[1].name or self.temp())
        env[id(m)] = outs_loc
        for k, o in enumerate(m.outs):
            if o.reduced:
                d = dest.get((id(m), k))
                reuse = d is not None and d[0] == "acc" and not g.consumers((m, k))
                if d is not None and not reuse:
                    self.finish(m, k, outs_loc[k][1], d, depth)

    # -- helpers
    def temp_later(self):
        return _Lazy(self)

    def scope_index(self, env) -> List[str]:
        return list(env.get("__index__", []))

    def buffer_for(self, g: Graph, m: Map, k: int) -> _Buffer:
        for n in g.nodes:
            if isinstance(n, Out) and n.arg == (m, k):
                return _Buffer(n.name)
        return _Buffer()


class _Lazy:
    """an accumulator's name, numbered when it is first printed"""

    def __init__(self, em: _Emitter):
        self.em = em
        self.name: Optional[str] = None

    def __str__(self):
        if self.name is None:
            self.name = self.em.temp()
        return self.name

    def __format__(self, spec):
        return str(self)


def _emit(g: Graph, fold: bool) -> _Emitter:
    em = _Emitter(fold)
    env: Dict = {}
    for n in g.nodes:
        if isinstance(n, In):
            env[id(n)] = [("list", _Buffer(n.name), [])]
    em.graph(g, env, 0, {})
    return em


def listing(g: Graph) -> str:
    return "\n".join(str(l) for l in _emit(g, False).lines)


def skeleton(g: Graph) -> str:
    return "\n".join(str(l) for l in _emit(g, True).lines)


def nest(g: Graph) -> str:
    """The loop structure of the program without its statements: a parallel loop over dimension X
    is written X(...), a serial one x(...), siblings are separated by blanks, an innermost loop has no parentheses; e.g. "M(n(d) L(n))"
    is a parallel loop over M that holds a serial loop over N with a serial loop over D inside,
    followed by a parallel loop over L with a serial loop over N inside."""
    out: List[str] = []
    depth_open: List[int] = []

    def close_to(depth: int) -> None:
        while depth_open and depth_open[-1] >= depth:
            depth_open.pop()
            out.append(")")

    for line in _emit(g, True).lines:
        text = str(line)
        depth = len(text) - len(text.lstrip("\t"))
        body = text.strip()
        close_to(depth)
        for kw, par in (("forall ", True), ("for ", False)):
            if body.startswith(kw):
                var = body[len(kw):].split(" ")[0]
                if out and out[-1] != "(":
                    out.append(" ")
                out.append((var.upper() if par else var.lower()) + "(")
                depth_open.append(depth)
                break
    close_to(0)
    return "".join(out).replace("( ", "(").replace("()", "")


def intermediate_buffers(g: Graph) -> int:
    """number of intermediate lists the program materialises in global memory (the buffered
    edges that are not program inputs or outputs)"""
    return _emit(g, False).nbuf
