"""Evaluates a block program with numpy on concrete blocks: every list is a
Python list, every block / vector / scalar an ndarray.  Used to check that a
substitution preserves the logic of the program (Section 4: rules are
logic-preserving)."""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from .ir import Graph, In, Map, Op, Out, Reduce


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
        total = total + x
    return total


def run_graph(g: Graph, env: Dict[int, list], consts: Dict[str, float]) -> None:
    for n in g.nodes:
        if isinstance(n, (In, Out)):
            continue
        if isinstance(n, Op):
            env[id(n)] = [_apply(n, [env[id(a[0])][a[1]] for a in n.operands], consts)]
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
                run_graph(n.inner, inner, consts)
                per_iter.append([inner[id(o.inner[0])][o.inner[1]] for o in n.outs])
            env[id(n)] = [_sum([p[k] for p in per_iter]) if o.reduced else [p[k] for p in per_iter]
                          for k, o in enumerate(n.outs)]


def evaluate(g: Graph, inputs: Dict[str, list], consts: Dict[str, float]) -> Dict[str, list]:
    env: Dict[int, list] = {}
    for n in g.nodes:
        if isinstance(n, In):
            env[id(n)] = [inputs[n.name]]
    run_graph(g, env, consts)
    return {n.name: env[id(n.arg[0])][n.arg[1]] for n in g.nodes if isinstance(n, Out)}


def assemble(blocks: list) -> np.ndarray:
    """list of lists of blocks -> one matrix"""
    return np.block([[b for b in row] for row in blocks])


def split(a: np.ndarray, rows: int, cols: int) -> list:
    """matrix -> rows x cols blocks (equal sizes)"""
    r, c = a.shape[0] // rows, a.shape[1] // cols
    return [[a[i * r:(i + 1) * r, j * c:(j + 1) * c] for j in range(cols)] for i in range(rows)]
