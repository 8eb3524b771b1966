"""python -m paper_2505_07829_amd.fusion example1|example2|example3 [--steps] [--initial]

Runs fuse() on one of the paper's worked examples and prints the rules applied
and every snapshot as code; --steps prints the program after every single
substitution, --initial the unfused block program first."""
from __future__ import annotations

import argparse

from . import algorithm, check, emit, lower
from .ir import clone


def main() -> None:
    ap = argparse.ArgumentParser(prog="python -m paper_2505_07829_amd.fusion")
    ap.add_argument("example", choices=sorted(lower.EXAMPLES))
    ap.add_argument("--steps", action="store_true", help="print the program after every substitution")
    ap.add_argument("--initial", action="store_true", help="print the initial (unfused) block program")
    args = ap.parse_args()
    g = clone(lower.EXAMPLES[args.example]())
    if args.initial:
        print(f"# initial block program, {emit.intermediate_buffers(g)} intermediate lists in global memory")
        print(emit.listing(g), "\n")
    count = [0]

    def after(rule: int, what: str) -> None:
        count[0] += 1
        print(f"step {count[0]:2d}: rule {rule}: {what}")
        if args.steps:
            print(emit.listing(g), "\n")

    taken = [0]

    def snapshot(cur) -> None:
        taken[0] += 1
        err = check.max_error(cur, args.example)
        print(f"\n# snapshot {taken[0]}: {emit.intermediate_buffers(cur)} intermediate lists in global memory, "
              f"loop nest {emit.nest(cur)}, "
              f"max relative deviation from the array program on random blocks {err:.1e}")
        print(emit.listing(cur), "\n")

    algorithm.fuse_in_place(g, after, snapshot)


if __name__ == "__main__":
    main()
