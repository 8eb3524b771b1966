"""The fusion algorithm (Section 5) as a table of rules driven over the hierarchy of graphs.

A block program is a hierarchy: the top-level graph, the inner graph of every map in it, and so on.
The algorithm alternates two kinds of pass over that hierarchy, both breadth first:

  * a SATURATING pass: in every graph, apply the first matching rule of `PRIORITY` until none of them
    matches, then move on to the graphs of the level below (which the substitutions may just have
    created or merged, so they are looked up afterwards, not before);
  * an EXTENDING pass: the first graph, in the same order, that offers an opportunity for Rule 6 takes
    it - exactly one substitution per pass.

`fuse()` saturates, records a snapshot, and repeats both for as long as an extension is found.  The
snapshots are the candidates the paper leaves to a selection step; the last one is the most aggressively
fused.

Readings of the text: the pseudo-code's queue is first-in first-out (the text says breadth first), and
its append of a list extends the queue.
"""
from __future__ import annotations

from collections import deque
from typing import Callable, Iterator, List, Optional, Tuple

from . import rules
from .ir import Graph, clone

Trace = List[Tuple[int, str]]          # (rule number, description) per applied substitution
OnStep = Optional[Callable[[int, str], None]]

# Rules of the saturating pass, most urgent first: rewrites that create fusion opportunities (8: a row
# scaling that several products consume gets a copy per product; 4, 5: a scaling or a shift moves behind
# the product; 9: elementwise operators are composed), then the structural ones (3: a reduction is folded
# into the map that feeds it; 1: consecutive maps are fused; 2: maps with a common input are fused).
# Rule 6 (map extension) has a pass of its own; Rule 7 is not used by the algorithm.
PRIORITY: Tuple[int, ...] = (8, 4, 5, 9, 3, 1, 2)
EXTENSION_RULE = 6
MATCHERS = {n: getattr(rules, f"rule{n}_match") for n in PRIORITY + (EXTENSION_RULE,)}


def levels(root: Graph) -> Iterator[Graph]:
    """The graphs of the hierarchy, breadth first.  The inner graphs of a graph are read when the
    traversal leaves it, so a caller may rewrite the graph it has just been handed."""
    pending = deque([root])
    while pending:
        g = pending.popleft()
        yield g
        pending.extend(node.inner for node in g.maps())


def first_match(g: Graph, numbers: Tuple[int, ...]):
    """the match of the first rule in `numbers` that applies to g, or None"""
    for n in numbers:
        m = MATCHERS[n](g)
        if m:
            return m
    return None


def saturate(g: Graph, on_step: OnStep = None) -> int:
    """Rules of PRIORITY on ONE graph until none matches; returns the number of substitutions."""
    done = 0
    while (m := first_match(g, PRIORITY)) is not None:
        what = rules.apply(m)
        done += 1
        if on_step:
            on_step(m.rule, what)
    return done


def saturate_all(root: Graph, on_step: OnStep = None) -> int:
    """the saturating pass over the whole hierarchy"""
    return sum(saturate(g, on_step) for g in levels(root))


def extend_once(root: Graph, on_step: OnStep = None) -> bool:
    """the extending pass: one application of Rule 6 at the first graph that allows it"""
    for g in levels(root):
        m = first_match(g, (EXTENSION_RULE,))
        if m is not None:
            what = rules.apply(m)
            if on_step:
                on_step(EXTENSION_RULE, what)
            return True
    return False


def fuse_in_place(g: Graph, on_step: OnStep = None, on_snapshot: Optional[Callable[[Graph], None]] = None) -> None:
    """the whole algorithm on g itself; on_snapshot(g) is called where fuse() records a snapshot"""
    while True:
        saturate_all(g, on_step)
        if on_snapshot:
            on_snapshot(g)
        if not extend_once(g, on_step):
            return


def fuse(g: Graph, on_step: OnStep = None) -> List[Graph]:
    """returns the snapshots: the program after each saturating pass (the last one is the most
    aggressively fused).  g is not modified."""
    snapshots: List[Graph] = []
    fuse_in_place(clone(g), on_step, lambda cur: snapshots.append(clone(cur)))
    return snapshots
