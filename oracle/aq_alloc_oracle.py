"""CPU oracle for the layer-balanced bit allocation (TEST INFRASTRUCTURE, not product code).

Plain Python, one candidate after the other; shares nothing with the library's host code.

What it follows (Section 4.1, paragraphs "Layer-balanced bit allocation" and "Solver"):
  - predicted error of tensor j of layer l at b bits: S[l][j] * eta(b), eta(b) = 2^(-2 b);
  - objective: sum over layers of E_l^2, E_l = sum_j S[l][j] eta(b[l][j])            (Eq. 6);
  - constraint: sum(b * size) / sum(size) <= budget                                   (Eq. 6);
  - greedy solver: every tensor starts at the cheapest type; at each step the upgrade with the
    largest gain per bit (E_l^2 - E~_l^2) / delta_bits is applied; the loop ends when the budget is met.
Readings where the paragraphs are silent (the library's too):
  - an upgrade moves one tensor to the next larger bit-width of the list (one step at a time);
  - an upgrade that would exceed the budget is not a candidate; the loop ends when no candidate is left
    or the best gain is not positive (S may be negative: Eq. 5 is a difference of two terms);
  - ties go to the first candidate in (layer, tensor) order; delta_bits = (b_next - b_cur) * size.
"""
from __future__ import annotations

import itertools
from typing import List, Sequence


def eta(b: int) -> float:
    return 2.0 ** (-2 * b)


def layer_error(S_row: Sequence[float], b_row: Sequence[int]) -> float:
    e = 0.0
    for s, b in zip(S_row, b_row):
        e += s * eta(b)
    return e


def objective(S, bits) -> float:
    return sum(layer_error(S[l], bits[l]) ** 2 for l in range(len(S)))


def average_bits(sizes, bits) -> float:
    num = sum(b * n for rb, rn in zip(bits, sizes) for b, n in zip(rb, rn))
    return num / sum(n for rn in sizes for n in rn)


def greedy(S, sizes, choices: Sequence[int], budget: float) -> List[List[int]]:
    L, J = len(S), len(S[0])
    level = [[0] * J for _ in range(L)]
    bits = [[choices[0]] * J for _ in range(L)]
    total = sum(n for rn in sizes for n in rn)
    used = sum(choices[0] * n for rn in sizes for n in rn)
    while True:
        best, best_ratio = None, 0.0
        for l in range(L):
            e_now = layer_error(S[l], bits[l])
            for j in range(J):
                if level[l][j] + 1 >= len(choices):
                    continue
                nb = choices[level[l][j] + 1]
                dbits = (nb - bits[l][j]) * sizes[l][j]
                if used + dbits > budget * total:
                    continue
                trial = list(bits[l])
                trial[j] = nb
                ratio = (e_now ** 2 - layer_error(S[l], trial) ** 2) / dbits
                if ratio > best_ratio:
                    best, best_ratio = (l, j, nb, dbits), ratio
        if best is None:
            return bits
        l, j, nb, dbits = best
        level[l][j] += 1
        bits[l][j] = nb
        used += dbits


def exhaustive(S, sizes, choices: Sequence[int], budget: float):
    """The true optimum of Eq. 6 by trying every assignment (tiny problems only)."""
    L, J = len(S), len(S[0])
    best, best_obj = None, float("inf")
    for flat in itertools.product(choices, repeat=L * J):
        bits = [list(flat[l * J:(l + 1) * J]) for l in range(L)]
        if average_bits(sizes, bits) <= budget + 1e-12:
            o = objective(S, bits)
            if o < best_obj:
                best, best_obj = bits, o
    return best, best_obj
