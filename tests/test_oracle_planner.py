"""Pins of the allocation-optimizer oracle (Algorithms 1 and 2, BBS, Eq. 1 and 2)."""
import itertools
import json
import os

import pytest

from oracle import planner as P

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


def simple_memory(sizes, caps, kinds=None):
    """One pool per row; a worker of model m costs sizes[m] whatever its batch size."""
    kinds = kinds or ["GPU"] * len(caps)
    return P.Memory([0] * len(sizes), lambda m, b: sizes[m], list(range(len(caps))), kinds, caps)


# ------------------------------------------------------------------ equations
def test_total_matrices_example_and_brute_force():
    g = GOLD["total_matrices_example"]
    v = P.total_matrices(g["B"], g["gpus"] + g["cpus"], g["M"])
    assert v == 7775 ** 8
    assert abs(v / g["approx"] - 1) < 0.05
    for B, D, M in [(1, 2, 2), (2, 2, 2), (2, 3, 1), (1, 2, 3)]:
        vals = range(B + 1)
        count = 0
        for cells in itertools.product(vals, repeat=D * M):
            A = [list(cells[d * M:(d + 1) * M]) for d in range(D)]
            count += P.is_valid(A)
        assert count == P.total_matrices(B, D, M)


def test_total_neighs_example_and_definition():
    g = GOLD["total_neighs_example"]
    assert P.total_neighs_paper(g["B"], g["D"], g["M"], 0) == g["max"]
    assert P.total_neighs_paper(g["B"], g["D"], g["M"], g["M"]) == g["min"]
    # the definition (valid matrices at distance exactly one) counted by brute force
    domain = [8, 16]
    for A in ([[8, 0], [0, 16]], [[8, 8], [16, 0]], [[8, 16], [8, 16]], [[0, 8, 0], [16, 0, 8]]):
        D, M = len(A), len(A[0])
        brute = 0
        for cells in itertools.product([0] + domain, repeat=D * M):
            Bm = [list(cells[d * M:(d + 1) * M]) for d in range(D)]
            diff = sum(Bm[d][m] != A[d][m] for d in range(D) for m in range(M))
            brute += (diff == 1 and P.is_valid(Bm))
        neighs = P.neighborhood(A, domain)
        assert len(neighs) == brute == len(domain) * D * M - P.forbidden_moves(A)
        assert all(P.is_valid(n) for n in neighs)
        assert len({tuple(map(tuple, n)) for n in neighs}) == len(neighs)


def test_budget_and_bbs_counts():
    g = GOLD["greedy_budget"]
    assert g["max_neighs"] * g["max_iter"] == g["max_benches"]
    assert g["max_benches"] * g["seconds_per_bench"] / 3600.0 <= g["hours"]
    b = GOLD["bbs_benches"]
    for m, n in zip(b["models"], b["benches"]):
        _, count = P.best_batch_size(m, lambda mm, bb: float(bb), GOLD["batch_domain"]["values"])
        assert count == n == b["batch_values"] * m


def test_table_matrix_is_valid_and_reads_as_described():
    A = GOLD["imn4_matrix"]["A"]
    assert P.is_valid(A)
    assert A[0] == [0, 0, 0, 0]                                   # an unused device is legal
    assert sum(v != 0 for v in A[1]) == 2                         # co-localization on GPU1
    assert sorted(A[d][1] for d in range(5) if A[d][1]) == [8, 128]   # data-parallel ResNet101
    bad = [row[:] for row in A]
    bad[4][3] = 0
    assert not P.is_valid(bad)                                    # a zero column is illegal


# ------------------------------------------------------------------ Algorithm 1
def test_wfd_trace_on_toy_instance():
    sizes = [5, 9, 3, 7]                  # decreasing order: 1, 3, 0, 2
    mem = simple_memory(sizes, [12, 12, 12])
    A = P.worst_fit_decreasing(4, mem, 8)
    # 9 -> row0 (rem 3); 7 -> row1 (rem 5); 5 -> row2 (rem 7); 3 -> row2 (most remaining)
    assert A == [[0, 8, 0, 0], [0, 0, 0, 8], [8, 0, 8, 0]]
    assert P.fit_mem(A, mem) and P.is_valid(A)


def test_wfd_each_step_takes_most_remaining_memory():
    sizes = [4, 4, 3, 2, 2, 1]
    caps = [9, 8, 7]
    mem = simple_memory(sizes, caps)
    A = P.worst_fit_decreasing(len(sizes), mem, 8)
    rem = list(caps)
    for m in sorted(range(len(sizes)), key=lambda i: (-sizes[i], i)):
        d = max(range(3), key=lambda r: (rem[r], -r))
        assert A[d][m] == 8
        rem[d] -= sizes[m]
    assert min(rem) >= 0


def test_wfd_prefers_gpus_and_spills_to_cpu():
    mem = simple_memory([6, 5, 4], [7, 100], kinds=["GPU", "CPU"])
    A = P.worst_fit_decreasing(3, mem, 8)
    assert A == [[8, 0, 0], [0, 8, 8]]
    mem = simple_memory([6, 5, 4], [20, 100], kinds=["GPU", "CPU"])
    assert P.worst_fit_decreasing(3, mem, 8) == [[8, 8, 8], [0, 0, 0]]
    with pytest.raises(MemoryError):
        P.worst_fit_decreasing(2, simple_memory([6, 5], [5, 5]), 8)


def exhaustive_feasible(sizes, caps):
    for assign in itertools.product(range(len(caps)), repeat=len(sizes)):
        load = [0] * len(caps)
        for m, d in enumerate(assign):
            load[d] += sizes[m]
        if all(l <= c for l, c in zip(load, caps)):
            return True
    return False


def test_wfd_against_exhaustive_search():
    # success implies feasibility, always
    for sizes in itertools.product(range(1, 6), repeat=4):
        for caps in ([6, 6], [7, 5], [9], [4, 4, 4]):
            try:
                A = P.worst_fit_decreasing(4, simple_memory(sizes, caps), 8)
                ok = True
                assert P.fit_mem(A, simple_memory(sizes, caps))
            except MemoryError:
                ok = False
            feas = exhaustive_feasible(sizes, caps)
            assert (not ok) or feas
            if len(caps) == 1 or len(set(sizes)) == 1:   # complete on one bin / equal items
                assert ok == feas
    # M <= D with equal capacities: complete
    for sizes in itertools.product(range(1, 6), repeat=2):
        caps = [4, 4]
        try:
            P.worst_fit_decreasing(2, simple_memory(sizes, caps), 8)
            ok = True
        except MemoryError:
            ok = False
        assert ok == exhaustive_feasible(sizes, caps)
    # known negative fixtures of the heuristic: feasible, yet worst-fit-decreasing fails
    for sizes, caps in (([3, 3, 2, 2, 2], [6, 6]), ([5, 3, 3, 2, 2, 2], [6, 6, 6])):
        assert exhaustive_feasible(sizes, caps)
        with pytest.raises(MemoryError):
            P.worst_fit_decreasing(len(sizes), simple_memory(sizes, caps), 8)


def test_wfd_max_load_is_optimal_for_few_items_on_two_bins():
    for sizes in itertools.product(range(1, 8), repeat=4):
        A = P.worst_fit_decreasing(4, simple_memory(sizes, [100, 100]), 8)
        load = [sum(sizes[m] for m in range(4) if A[d][m]) for d in range(2)]
        best = min(max(sum(s for s, a in zip(sizes, asg) if a == 0), sum(s for s, a in zip(sizes, asg) if a == 1))
                   for asg in itertools.product(range(2), repeat=4))
        assert max(load) == best


def test_pooled_slots_share_weights_and_capacity():
    # three instance slots on one pool: weights once per member, arena per worker
    mem = P.Memory([100, 50], lambda m, b: 10 * b, [0, 0, 0], ["GPU"] * 3, [1000])
    A = P.worst_fit_decreasing(2, mem, 8)
    assert A == [[8, 8], [0, 0], [0, 0]]
    assert mem.pool_used(A, 0) == 100 + 50 + 80 + 80
    A2 = [[8, 8], [16, 0], [0, 0]]
    assert mem.pool_used(A2, 0) == 100 + 50 + 80 + 80 + 160
    assert P.fit_mem(A2, mem)
    assert not P.fit_mem([[8, 8], [128, 0], [0, 0]], mem)


# ------------------------------------------------------------------ Algorithm 2
DOMAIN = GOLD["batch_domain"]["values"]


def separable_cost(best):
    """Score that is a sum over cells; each cell has one best value."""
    def bench(A):
        s = 0.0
        for d, row in enumerate(A):
            for m, v in enumerate(row):
                s += 10.0 if v == best[d][m] else (1.0 if v != 0 else 0.0)
        return s
    return bench


def test_greedy_reaches_global_optimum_of_separable_cost():
    best = [[16, 0], [64, 8]]
    bench = separable_cost(best)
    start = [[8, 8], [0, 0]]
    A, s, _ = P.bounded_greedy(start, bench, [8, 16, 64], max_iter=20, max_neighs=10 ** 6)
    brute = max((bench([list(c[:2]), list(c[2:])]) for c in itertools.product([0, 8, 16, 64], repeat=4)
                 if P.is_valid([list(c[:2]), list(c[2:])])))
    assert A == [[16, 8], [64, 8]] or s == brute
    assert s == brute


def test_greedy_never_worse_and_respects_bounds():
    import random
    rnd = random.Random(5)
    table = {}

    def bench(A):
        key = tuple(map(tuple, A))
        if key not in table:
            table[key] = rnd.random()
        bench.calls += 1
        return table[key]

    for max_iter, max_neighs in [(1, 5), (3, 7), (10, 100)]:
        bench.calls = 0
        start = [[8, 8, 8], [0, 0, 0]]
        A, s, n_bench = P.bounded_greedy(start, bench, DOMAIN, max_iter, max_neighs, seed=3)
        assert s >= table[tuple(map(tuple, start))]
        assert n_bench == bench.calls <= 1 + max_neighs * (max_iter + 1)
        assert P.is_valid(A)


def test_greedy_stops_on_plateau_and_moves_only_if_strictly_better():
    calls = []

    def flat(A):
        calls.append(1)
        return 5.0

    start = [[8, 8]]
    A, s, n = P.bounded_greedy(start, flat, DOMAIN, max_iter=10, max_neighs=1000)
    assert A == start and s == 5.0
    assert n == 1 + len(P.neighborhood(start, DOMAIN))      # one iteration only


def test_greedy_takes_best_neighbour_each_iteration():
    def bench(A):                      # faster with a larger total batch, zero if "out of memory"
        tot = sum(v for row in A for v in row)
        return 0.0 if tot > 200 else float(tot)

    A, s, _ = P.bounded_greedy([[8, 8]], bench, DOMAIN, max_iter=10, max_neighs=1000)
    assert s == 192.0 and sorted(A[0]) == [64, 128]
    A1, s1, _ = P.bounded_greedy([[8, 8]], bench, DOMAIN, max_iter=1, max_neighs=1000)
    assert A1 == [[128, 8]] and s1 == 136.0                 # first-best in enumeration order


def test_greedy_iteration_floor_for_many_devices():
    moves = []

    def bench(A):
        s = float(sum(1 for row in A for v in row if v))
        moves.append(s)
        return s

    start = [[8]] + [[0]] * 14                               # D - M = 14 > max_iter = 2
    A, s, _ = P.bounded_greedy(start, bench, [8], max_iter=2, max_neighs=1000)
    assert s == 15.0                                          # all 14 extra moves were allowed


def test_draw_is_the_published_splitmix64_sequence():
    d = P.Draw(0)
    assert [d.next() for _ in range(3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    d = P.Draw(42)
    s = d.sample(range(50), 20)
    assert len(set(s)) == 20 and all(0 <= v < 50 for v in s)
    assert P.Draw(42).sample(range(50), 20) == s
    assert sorted(P.Draw(1).sample(range(9), 9)) == list(range(9))
