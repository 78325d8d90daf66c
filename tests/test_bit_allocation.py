"""Layer-balanced bit allocation (Section 4.1, Eq. 6 and "Solver"): the oracle against a hand-worked run and
exhaustive search, and the library's host-only solver against the oracle.  No GPU."""
import os

import numpy as np
import pytest

import paper_2605_24011_amd as aq
from oracle import aq_alloc_oracle as ao

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "bit_allocation_example.txt")


def _problem(rng, L, J, signed=False):
    S = rng.gamma(1.0, 1.0, size=(L, J)) * np.exp(rng.standard_normal((L, 1)))
    if signed:
        S = S - 0.3 * S.mean()
    sizes = rng.choice([256 * 2048, 2048 * 2048, 4096 * 4096, 4096 * 11008], size=(L, J))
    return S.tolist(), sizes.tolist()


def test_hand_worked_run():
    g = {}
    for line in open(GOLDEN):
        if not line.startswith("#") and line.strip():
            k, *v = line.split()
            g[k] = v
    S = [[float(x)] for x in g["S"]]
    sizes = [[int(x)] for x in g["sizes"]]
    choices = [int(x) for x in g["choices"]]
    bits = ao.greedy(S, sizes, choices, float(g["budget"][0]))
    assert [b[0] for b in bits] == [int(x) for x in g["bits"]]
    assert ao.objective(S, bits) == float(g["objective"][0])
    assert ao.exhaustive(S, sizes, choices, float(g["budget"][0]))[1] == float(g["objective"][0])
    assert aq.aq_allocate_bits(S, sizes, choices, float(g["budget"][0])) == bits


@pytest.mark.parametrize("seed", range(6))
def test_greedy_against_exhaustive_search(seed):
    """The greedy result is feasible, never better than the true optimum, and close to it; with one tensor per layer
    and equal sizes the objective is separable and convex in the bit-widths, where the greedy choice is optimal."""
    rng = np.random.default_rng(seed)
    S, sizes = _problem(rng, 3, 3)
    for budget in (2.4, 2.75, 3.3, 4.0):
        bits = ao.greedy(S, sizes, [2, 3, 4], budget)
        assert ao.average_bits(sizes, bits) <= budget + 1e-12
        best, best_obj = ao.exhaustive(S, sizes, [2, 3, 4], budget)
        obj = ao.objective(S, bits)
        assert obj >= best_obj * (1 - 1e-12)
        assert obj <= best_obj * 4.0
    S1 = [[s[0]] for s in S] + [[s[1]] for s in S]
    n1 = [[1000]] * 6
    for budget in (2.5, 3.0, 3.5):
        bits = ao.greedy(S1, n1, [2, 3, 4], budget)
        assert ao.objective(S1, bits) == pytest.approx(ao.exhaustive(S1, n1, [2, 3, 4], budget)[1], rel=1e-12)


def test_budget_extremes_and_negative_sensitivities():
    rng = np.random.default_rng(7)
    S, sizes = _problem(rng, 4, 7)
    assert all(b == 2 for row in ao.greedy(S, sizes, [2, 3, 4], 2.0) for b in row)
    assert all(b == 4 for row in ao.greedy(S, sizes, [2, 3, 4], 4.0) for b in row)
    # a negative sensitivity inside an otherwise positive layer (Eq. 5 is a difference): layer 0 has
    # E = eta(b0) - 0.2 eta(b1).  At [2,2] E = 0.05; [3,2] gives 1/64 - 0.0125 = 0.003125; going on to [4,2] gives
    # 1/256 - 0.0125 = -0.0086 and raising b1 gives 1/64 - 0.2/64 = 0.0125: both larger in magnitude, so the loop
    # leaves layer 0 at [3,2] with budget to spare, while the all-positive layer 1 goes to [4,4]
    S2 = [[1.0, -0.2], [2.0, 0.5]]
    bits = ao.greedy(S2, [[10, 10], [10, 10]], [2, 3, 4], 4.0)
    assert bits == [[3, 2], [4, 4]]
    assert aq.aq_allocate_bits(S2, [[10, 10], [10, 10]], (2, 3, 4), 4.0) == bits


@pytest.mark.parametrize("seed", range(8))
def test_library_solver_equals_the_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    L, J = int(rng.integers(1, 33)), int(rng.integers(1, 8))
    S, sizes = _problem(rng, L, J, signed=seed % 2 == 1)
    for budget, choices in ((2.5, (2, 3, 4)), (3.0, (2, 3, 4)), (3.5, (2, 4)), (5.0, (3, 4, 6, 8))):
        if choices[0] > budget:
            continue
        assert aq.aq_allocate_bits(S, sizes, choices, budget) == ao.greedy(S, sizes, list(choices), budget)


def test_library_solver_on_the_llama_shaped_backbone():
    """224 tensors (32 layers x 7) at a mean of 2.5 code bits: feasible, uses the budget, spends bits where S is large."""
    import aq_workloads as wl
    rng = np.random.default_rng(9)
    shapes = [(N, K) for _name, N, K in wl.LLAMA2_7B_LAYER]
    sizes = [[N * K for N, K in shapes] for _ in range(32)]
    S = (rng.gamma(0.7, 1.0, size=(32, 7)) * np.exp(0.5 * rng.standard_normal((32, 1)))).tolist()
    bits = aq.aq_allocate_bits(S, sizes, (2, 3, 4), 2.5)
    assert bits == ao.greedy(S, sizes, [2, 3, 4], 2.5)
    avg = ao.average_bits(sizes, bits)
    assert 2.45 < avg <= 2.5
    flatS = np.array(S).ravel()
    flatb = np.array(bits).ravel()
    assert flatS[flatb == 4].mean() > flatS[flatb == 2].mean()


def test_library_solver_validation():
    S, n = [[1.0, 2.0]], [[10, 10]]
    with pytest.raises(aq.AqError):
        aq.aq_allocate_bits(S, n, (3, 2), 3.0)              # not ascending
    with pytest.raises(aq.AqError):
        aq.aq_allocate_bits(S, n, (2, 3, 4), 1.5)           # cheapest type already over budget
    with pytest.raises(aq.AqError):
        aq.aq_allocate_bits(S, [[10, 0]], (2, 3, 4), 3.0)   # empty tensor
