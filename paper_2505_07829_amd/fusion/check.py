"""Numerical check of a block program against the array program it came from
(numpy, fp64, random inputs): the logic-preservation test for every rule."""
from __future__ import annotations

from typing import Dict

import numpy as np

from .interp import assemble, evaluate, split
from .ir import Graph

# blocks per dimension and block edge used by the checks (small, all different)
COUNTS = {"M": 2, "N": 3, "D": 2, "L": 2, "K": 3}
EDGE = {"M": 3, "N": 2, "D": 4, "L": 5, "K": 2}


def _matrix(rng, rows: str, cols: str) -> np.ndarray:
    return rng.standard_normal((COUNTS[rows] * EDGE[rows], COUNTS[cols] * EDGE[cols]))


def reference(name: str, seed: int = 0):
    """inputs (as blocks), constants and the expected output matrix of an example, computed
    from the array program's definition"""
    rng = np.random.default_rng(seed)
    if name == "example1":
        Q, K, V = _matrix(rng, "M", "D"), _matrix(rng, "N", "D"), _matrix(rng, "N", "L")
        dd = Q.shape[1]
        P = np.exp(Q @ K.T / np.sqrt(dd))
        want = (P / P.sum(axis=1, keepdims=True)) @ V
        ins = {"Q": split(Q, COUNTS["M"], COUNTS["D"]), "KT": split(K, COUNTS["N"], COUNTS["D"]),
               "VT": split(V.T.copy(), COUNTS["L"], COUNTS["N"])}
        return ins, {"DD": float(dd)}, {"O": want}
    if name == "example2":
        X, Y = _matrix(rng, "M", "K") + 0.7, _matrix(rng, "K", "N")
        kk = X.shape[1]
        mu = X.mean(axis=1, keepdims=True)
        sd = np.sqrt((X ** 2).mean(axis=1, keepdims=True) - mu ** 2)
        want = ((X - mu) / sd) @ Y
        ins = {"X": split(X, COUNTS["M"], COUNTS["K"]), "YT": split(Y.T.copy(), COUNTS["N"], COUNTS["K"])}
        return ins, {"KK": float(kk)}, {"Z": want}
    if name == "example3":
        X, W, V, U = _matrix(rng, "M", "D"), _matrix(rng, "D", "K"), _matrix(rng, "D", "K"), _matrix(rng, "K", "N")
        Xn = X / np.sqrt((X ** 2).sum(axis=1, keepdims=True))
        a = Xn @ W
        want = ((a / (1 + np.exp(-a))) * (Xn @ V)) @ U
        ins = {"X": split(X, COUNTS["M"], COUNTS["D"]), "WT": split(W.T.copy(), COUNTS["K"], COUNTS["D"]),
               "VT": split(V.T.copy(), COUNTS["K"], COUNTS["D"]), "UT": split(U.T.copy(), COUNTS["N"], COUNTS["K"])}
        return ins, {}, {"O": want}
    raise KeyError(name)


def max_error(g: Graph, name: str, seed: int = 0) -> float:
    ins, consts, want = reference(name, seed)
    got = evaluate(g, ins, consts)
    err = 0.0
    for k, w in want.items():
        err = max(err, float(np.abs(assemble(got[k]) - w).max() / np.abs(w).max()))
    return err
