"""Oracle of the allocation-matrix optimizer (test infrastructure only).

Follows section "The allocation optimizer": Algorithm 1 (worst-fit-decreasing with
priority to GPUs) builds a feasible matrix at the default batch size, Algorithm 2
(bounded greedy) refines it with benchmarks.  A matrix has one row per device
and one column per DNN; 0 = no worker, otherwise the worker's batch size; a
column of zeros is illegal (section "The allocation matrix data structure").

Memory model (the paper leaves it to the framework's out-of-memory error; here
it is explicit so that it can be tested): a memory pool holds, for every member
with at least one worker in the pool, that member's weights once, plus one
activation arena per worker.  Rows map to pools; with one row per pool this is
the paper's per-device model, with several rows on one pool the rows are
instance slots of one device.
"""
import copy

GOLDEN = 0x9E3779B97F4A7C15
MASK = 0xFFFFFFFFFFFFFFFF


def _mix(z):
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK
    return z ^ (z >> 31)


class Draw:
    """SplitMix64 sequence: state += GOLDEN; output mix(state)."""

    def __init__(self, seed):
        self.state = seed & MASK

    def next(self):
        self.state = (self.state + GOLDEN) & MASK
        return _mix(self.state)

    def sample(self, items, k):
        """k items without replacement: partial Fisher-Yates, j = i + next() mod (n - i)."""
        items = list(items)
        n = len(items)
        for i in range(k):
            j = i + self.next() % (n - i)
            items[i], items[j] = items[j], items[i]
        return items[:k]


class Memory:
    def __init__(self, weights, arena, row_pool, row_kind, pool_cap):
        self.weights = list(weights)          # bytes per member
        self.arena = arena                    # arena(m, b) -> bytes of one worker
        self.row_pool = list(row_pool)        # pool index of each matrix row
        self.row_kind = list(row_kind)        # 'GPU' or 'CPU' per row
        self.pool_cap = list(pool_cap)        # bytes per pool

    def pool_used(self, A, pool):
        used = 0
        n_models = len(A[0])
        for m in range(n_models):
            cells = [A[d][m] for d in range(len(A)) if self.row_pool[d] == pool and A[d][m] != 0]
            if cells:
                used += self.weights[m] + sum(self.arena(m, b) for b in cells)
        return used

    def remaining(self, A, row):
        p = self.row_pool[row]
        return self.pool_cap[p] - self.pool_used(A, p)


def fit_mem(A, mem):
    return all(mem.pool_used(A, p) <= mem.pool_cap[p] for p in range(len(mem.pool_cap)))


def more_remaining_memory(A, mem, kind):
    """Row of the given device kind whose pool has the most remaining memory
    (lowest row index on ties); None when there is no device of that kind."""
    best = None
    for d in range(len(A)):
        if mem.row_kind[d] != kind:
            continue
        if best is None or mem.remaining(A, d) > mem.remaining(A, best):
            best = d
    return best


def worst_fit_decreasing(n_models, mem, default_batch):
    """Algorithm 1.  Raises MemoryError when a model fits on no device."""
    n_rows = len(mem.row_pool)
    A = [[0] * n_models for _ in range(n_rows)]
    order = sorted(range(n_models),
                   key=lambda m: (-(mem.weights[m] + mem.arena(m, default_batch)), m))
    for m in order:
        g = more_remaining_memory(A, mem, "GPU")
        c = more_remaining_memory(A, mem, "CPU")
        placed = False
        for row in (g, c):                       # priority to the GPU side
            if row is None:
                continue
            trial = copy.deepcopy(A)
            trial[row][m] = default_batch
            if fit_mem(trial, mem):
                A = trial
                placed = True
                break
        if not placed:
            raise MemoryError("no device has enough memory for model %d" % m)
    return A


def is_valid(A):
    return all(any(A[d][m] != 0 for d in range(len(A))) for m in range(len(A[0])))


def neighborhood(A, domain):
    """All valid matrices that differ from A in exactly one element, enumerated
    row by row, column by column, candidate values 0 then the domain ascending."""
    out = []
    for d in range(len(A)):
        for m in range(len(A[0])):
            for v in [0] + sorted(domain):
                if v == A[d][m]:
                    continue
                B = copy.deepcopy(A)
                B[d][m] = v
                if is_valid(B):
                    out.append(B)
    return out


def bounded_greedy(A, bench, domain, max_iter=10, max_neighs=100, seed=0):
    """Algorithm 2.  `bench(matrix)` returns the score to maximise (0 when the
    matrix does not fit in memory).  Returns (matrix, score, number of benches)."""
    n_rows, n_models = len(A), len(A[0])
    if n_rows - n_models > max_iter:             # section "Offline benchmark settings"
        max_iter = n_rows - n_models
    draw = Draw(seed)
    A = copy.deepcopy(A)
    a_speed = bench(A)
    n_bench = 1
    it = 0
    while it < max_iter:
        neighs = neighborhood(A, domain)
        if len(neighs) > max_neighs:
            neighs = draw.sample(neighs, max_neighs)
        best_a, best_speed = None, None
        for nb in neighs:
            s = bench(nb)
            n_bench += 1
            if best_speed is None or s > best_speed:
                best_a, best_speed = nb, s
        if best_speed is not None and best_speed > a_speed:
            A, a_speed = best_a, best_speed
            it += 1
        else:
            it = max_iter                         # local maximum or plateau
    return A, a_speed, n_bench


def best_batch_size(n_models, bench_single, domain):
    """The BBS baseline: every model alone on its own device, each batch size of
    the domain benchmarked once, the fastest kept.  Returns (batch sizes, #bench)."""
    chosen, n_bench = [], 0
    for m in range(n_models):
        best_b, best_s = None, None
        for b in sorted(domain):
            s = bench_single(m, b)
            n_bench += 1
            if best_s is None or s > best_s:
                best_b, best_s = b, s
        chosen.append(best_b)
    return chosen, n_bench


def total_matrices(B, D, M):
    """Equation (1) of section "Algorithm 2": ((B+1)^D - 1)^M."""
    return ((B + 1) ** D - 1) ** M


def total_neighs_paper(B, D, M, F):
    """Equation (2) of section "Algorithm 2" as printed: (B+1)*(D*M) - F."""
    return (B + 1) * (D * M) - F


def forbidden_moves(A):
    """Number of one-element changes that would empty a column."""
    return sum(1 for m in range(len(A[0])) if sum(1 for d in range(len(A)) if A[d][m] != 0) == 1)
