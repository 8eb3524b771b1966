"""The fusion algorithm (Section 5): fuse_no_extend on one graph, breadth
first over the hierarchy, map extension, and fuse() that alternates the two
and returns the snapshots.

The pseudo-code's queue is read as first-in first-out (the text says breadth
first), and its append of a list as extending the queue."""
from __future__ import annotations

from typing import Callable, List, Optional, Tuple

from . import rules
from .ir import Graph, clone

Trace = List[Tuple[int, str]]          # (rule number, description) per applied substitution


def fuse_no_extend(g: Graph, on_step: Optional[Callable] = None) -> Graph:
    """all rules but 6 on ONE graph, priority 8, 4, 5, 9, 3, 1, 2, until none matches"""
    while True:
        m = (rules.rule8_match(g) or rules.rule4_match(g) or rules.rule5_match(g) or rules.rule9_match(g)
             or rules.rule3_match(g) or rules.rule1_match(g) or rules.rule2_match(g))
        if not m:
            return g
        what = rules.apply(m)
        if on_step:
            on_step(m.rule, what)


def get_inner_graphs(g: Graph) -> List[Graph]:
    return [n.inner for n in g.maps()]


def bfs_fuse_no_extend(g: Graph, on_step: Optional[Callable] = None) -> Graph:
    fuse_no_extend(g, on_step)
    queue = get_inner_graphs(g)
    while queue:
        c = queue.pop(0)
        fuse_no_extend(c, on_step)
        queue.extend(get_inner_graphs(c))
    return g


def bfs_extend(g: Graph, on_step: Optional[Callable] = None) -> Optional[Graph]:
    """the first opportunity for Rule 6, breadth first; None if there is none"""
    queue = [g]
    while queue:
        c = queue.pop(0)
        m = rules.rule6_match(c)
        if m:
            what = rules.apply(m)
            if on_step:
                on_step(6, what)
            return g
        queue.extend(get_inner_graphs(c))
    return None


def fuse(g: Graph, on_step: Optional[Callable] = None) -> List[Graph]:
    """returns the snapshots: the program after each round of fusion without extension
    (the last one is the most aggressively fused).  g is not modified."""
    g = clone(g)
    bfs_fuse_no_extend(g, on_step)
    snapshots = [clone(g)]
    while bfs_extend(g, on_step) is not None:
        bfs_fuse_no_extend(g, on_step)
        snapshots.append(clone(g))
    return snapshots
