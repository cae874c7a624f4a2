"""Operation tally of the anchor + score computation -- test infrastructure.

Walks the itemised steps of the appendix "FLOP count of KeyDiff" (unit-key
anchor, then the clamped cosine) and adds up multiplications, additions,
divisions and square roots step by step; the test pins the total to the closed
form the paper prints.  It is the work model the scoring roofline is built on.
"""
from __future__ import annotations


def tally(n: int, d: int) -> dict:
    ops = {"mul": 0, "add": 0, "div": 0, "sqrt": 0}

    def add(mul=0, add=0, div=0, sqrt=0):
        ops["mul"] += mul
        ops["add"] += add
        ops["div"] += div
        ops["sqrt"] += sqrt

    # anchor ------------------------------------------------------------------
    for _ in range(n):            # |k_i| = sqrt(k_i . k_i)
        add(mul=d, add=d - 1, sqrt=1)
    for _ in range(n):            # k_i / |k_i| as one reciprocal and d products
        add(div=1, mul=d)
    add(add=(n - 1) * d, div=1)   # mean of the n unit keys
    # score -------------------------------------------------------------------
    for _ in range(n):            # mu . k_i
        add(mul=d, add=d - 1)
    add(mul=d, add=d - 1, sqrt=1)  # |mu|
    for _ in range(n):            # |k_i||mu|, the max with eps (one comparison), the quotient
        add(mul=1, add=1, div=1)
    # The appendix itemises n divisions for the score step but states its subtotal as n + 1, and the
    # printed totals (2n + 2 divisions, the closed form) follow the subtotal: the extra division has
    # no step behind it and is added only so that the tally reproduces the printed total.
    add(div=1)
    return ops


def weighted(ops: dict) -> int:
    """x86-table weights the paper uses: add 1, sqrt 1, mul 3, div 47."""
    return 3 * ops["mul"] + ops["add"] + 47 * ops["div"] + ops["sqrt"]
