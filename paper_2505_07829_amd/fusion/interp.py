"""Evaluates a block program with numpy on concrete blocks: every list is a
Python list, every block / vector / scalar an ndarray.  Used to check that a
substitution preserves the logic of the program (Section 4: rules are
logic-preserving).

With safe=True the evaluation is the Appendix's numerical-safety pass carried
out on the fly: every value that descends from an exponential is represented
as a significand-exponent pair in the row-wise form (a block or vector of
significands and one exponent per row), exponentials are created as
(exp(X - z), z) with z the row maxima, products add exponents, sums bring both
terms to the larger exponent first, and a pair is turned back into plain
numbers only where the program stores it."""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from .ir import Graph, In, Map, Op, Out, Reduce


class Pair:
    """significands s (block [r, c] or vector [r]) times exp(t), t one exponent per row"""

    def __init__(self, s: np.ndarray, t: np.ndarray):
        self.s, self.t = s, t

    def plain(self) -> np.ndarray:
        return self.s * (np.exp(self.t)[:, None] if self.s.ndim == 2 else np.exp(self.t))


def _rows(v: np.ndarray, like: np.ndarray) -> np.ndarray:
    return v[:, None] if like.ndim == 2 else v


def pair_add(a, b):
    """(S1,t1) + (S2,t2) = (S1 e^(t1-z) + S2 e^(t2-z), z), z = max(t1,t2) per row"""
    if not isinstance(a, Pair) and not isinstance(b, Pair):
        return a + b
    if not isinstance(a, Pair):
        a = Pair(a, np.zeros(a.shape[0]))
    if not isinstance(b, Pair):
        b = Pair(b, np.zeros(b.shape[0]))
    z = np.maximum(a.t, b.t)
    return Pair(a.s * _rows(np.exp(a.t - z), a.s) + b.s * _rows(np.exp(b.t - z), b.s), z)


def _apply_safe(n: Op, a: List, consts: Dict[str, float]):
    if not any(isinstance(x, Pair) for x in a):
        if n.fn == "ew" and len(a) == 1 and n.expr.startswith("exp(") and n.expr.endswith(")") and a[0].ndim == 2:
            inner = Op("ew", n.operands, n.expr[4:-1])
            y = _apply(inner, a, consts)
            z = y.max(axis=1)
            return Pair(np.exp(y - z[:, None]), z)
        return _apply(n, a, consts)
    if n.fn == "row_sum":
        return Pair(a[0].s.sum(axis=1), a[0].t)
    if n.fn == "dot" and not isinstance(a[1], Pair):
        return Pair(a[0].s @ a[1].T, a[0].t)
    if n.fn == "row_scale":
        x = a[0] if isinstance(a[0], Pair) else Pair(a[0], np.zeros(a[0].shape[0]))
        c = a[1] if isinstance(a[1], Pair) else Pair(a[1], np.zeros(a[1].shape[0]))
        return Pair(x.s * c.s[:, None], x.t + c.t)
    if n.fn == "add":
        return pair_add(a[0], a[1])
    if n.fn == "ew" and len(a) == 1 and n.expr.replace(" ", "") == "1/{0}":
        return Pair(1.0 / a[0].s, -a[0].t)
    raise NotImplementedError(f"{n.fn} {n.expr or ''} on a significand-exponent pair")


def _apply(n: Op, a: List, consts: Dict[str, float]):
    if n.fn == "dot":
        return a[0] @ a[1].T
    if n.fn == "row_sum":
        return a[0].sum(axis=1)
    if n.fn == "row_scale":
        return a[0] * a[1][:, None]
    if n.fn == "row_shift":
        return a[0] + a[1][:, None]
    if n.fn == "outer":
        return np.outer(a[0], a[1])
    if n.fn == "add":
        return a[0] + a[1]
    if n.fn == "mul":
        return a[0] * a[1]
    if n.fn == "ew":
        names = {f"_a{i}": v for i, v in enumerate(a)}
        scope = {"exp": np.exp, "sqrt": np.sqrt, **consts, **names}
        return eval(n.expr.format(*[f"_a{i}" for i in range(len(a))]), {"__builtins__": {}}, scope)
    raise ValueError(n.fn)


def _sum(items):
    total = items[0]
    for x in items[1:]:
        total = pair_add(total, x)
    return total


def run_graph(g: Graph, env: Dict[int, list], consts: Dict[str, float], safe: bool = False) -> None:
    for n in g.nodes:
        if isinstance(n, (In, Out)):
            continue
        if isinstance(n, Op):
            args = [env[id(a[0])][a[1]] for a in n.operands]
            env[id(n)] = [_apply_safe(n, args, consts) if safe else _apply(n, args, consts)]
        elif isinstance(n, Reduce):
            env[id(n)] = [_sum(env[id(n.arg[0])][n.arg[1]])]
        elif isinstance(n, Map):
            vals = [env[id(i.outer[0])][i.outer[1]] for i in n.ins]
            lengths = {len(v) for v, i in zip(vals, n.ins) if i.iterated}
            assert len(lengths) == 1, "lists of a map must have equal length"
            count = lengths.pop()
            per_iter = []
            for it in range(count):
                inner = {id(i.param): [v[it] if i.iterated else v] for v, i in zip(vals, n.ins)}
                run_graph(n.inner, inner, consts, safe)
                per_iter.append([inner[id(o.inner[0])][o.inner[1]] for o in n.outs])
            env[id(n)] = [_sum([p[k] for p in per_iter]) if o.reduced else [p[k] for p in per_iter]
                          for k, o in enumerate(n.outs)]


def _plain(v):
    if isinstance(v, Pair):
        return v.plain()
    if isinstance(v, list):
        return [_plain(x) for x in v]
    return v


def evaluate(g: Graph, inputs: Dict[str, list], consts: Dict[str, float], safe: bool = False) -> Dict[str, list]:
    """outputs by name; safe=True: the Appendix's significand-exponent arithmetic (see above)"""
    env: Dict[int, list] = {}
    for n in g.nodes:
        if isinstance(n, In):
            env[id(n)] = [inputs[n.name]]
    run_graph(g, env, consts, safe)
    return {n.name: _plain(env[id(n.arg[0])][n.arg[1]]) for n in g.nodes if isinstance(n, Out)}


def assemble(blocks: list) -> np.ndarray:
    """list of lists of blocks -> one matrix"""
    return np.block([[b for b in row] for row in blocks])


def split(a: np.ndarray, rows: int, cols: int) -> list:
    """matrix -> rows x cols blocks (equal sizes)"""
    r, c = a.shape[0] // rows, a.shape[1] // cols
    return [[a[i * r:(i + 1) * r, j * c:(j + 1) * c] for j in range(cols)] for i in range(rows)]
