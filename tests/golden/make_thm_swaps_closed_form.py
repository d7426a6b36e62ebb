"""Writes thm_swaps_closed_form.txt from the closed form PRINTED in the paper
(App. A, proof of the first theorem): after n swaps of the list [1..5],
    s_0 = n * (sum_i i * pi(i) - 54.5),   head output = exp(s_0)/(exp(s_0)+n) * e_1.
Only list manipulation and that formula are used -- no oracle, no GPU code.
"""
import math
import os

CASES = [
    "1-2",
    "1-2 1-2",
    "1-2 2-3 1-2 2-3 1-2 2-3",
    "1-5 2-4 3-1 4-5",
    "3-4 4-5 3-4 1-2 4-5 1-2 3-5",
    "1-2 3-4 1-2 3-4",
    "2-5 2-5 1-3 1-3 4-1 4-1",
    "1-2 2-3 3-4 4-5 5-1 1-3 2-4",
]

here = os.path.dirname(os.path.abspath(__file__))
with open(os.path.join(here, "thm_swaps_closed_form.txt"), "w") as f:
    f.write("# swaps | s_0 = n(sum_i i*pi(i) - 54.5) | a_0 = exp(s_0)/(exp(s_0)+n)\n")
    f.write("# source: closed form in the paper's App. A (swap-tracking theorem); written by\n")
    f.write("# make_thm_swaps_closed_form.py\n")
    for case in CASES:
        swaps = [tuple(int(c) for c in p.split("-")) for p in case.split()]
        lst = [1, 2, 3, 4, 5]
        for x, y in swaps:
            lst[x - 1], lst[y - 1] = lst[y - 1], lst[x - 1]
        n = len(swaps)
        s0 = n * (sum((i + 1) * lst[i] for i in range(5)) - 54.5)
        a0 = 1.0 / (1.0 + n * math.exp(-s0))
        f.write(f"{case} | {s0!r} | {a0!r}\n")
