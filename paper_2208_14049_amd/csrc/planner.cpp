// Host-side allocation-matrix optimizer (section "The allocation optimizer"): Algorithm 1,
// worst-fit-decreasing with priority to GPUs; Algorithm 2, bounded greedy over one-cell
// neighbours; and the BBS baseline.  Pure host code over an explicit memory model and a
// benchmark callback; the GPU engine plugs its own timing in as the callback.
#include "planner.h"

#include <algorithm>
#include <numeric>

namespace ens {

static int domain_index(const ens_plan_problem& p, int batch) {
    for (int j = 0; j < p.n_domain; j++)
        if (p.domain[j] == batch) return j;
    return -1;
}

bool problem_ok(const ens_plan_problem* p) {
    if (!p || p->n_models <= 0 || p->n_rows <= 0 || p->n_pools <= 0 || p->n_domain <= 0) return false;
    if (!p->domain || !p->weight_bytes || !p->arena_bytes || !p->row_pool || !p->row_is_gpu || !p->pool_cap)
        return false;
    for (int j = 0; j < p->n_domain; j++)
        if (p->domain[j] <= 0) return false;
    for (int d = 0; d < p->n_rows; d++)
        if (p->row_pool[d] < 0 || p->row_pool[d] >= p->n_pools) return false;
    return domain_index(*p, p->default_batch) >= 0;
}

// Bytes in use in one pool: weights once per member present, one arena per worker.
// Returns -1 when a cell holds a batch size outside the domain.
int64_t pool_used(const ens_plan_problem& p, const int32_t* A, int pool) {
    int64_t used = 0;
    for (int m = 0; m < p.n_models; m++) {
        bool present = false;
        for (int d = 0; d < p.n_rows; d++) {
            const int b = A[d * p.n_models + m];
            if (p.row_pool[d] != pool || b == 0) continue;
            const int j = domain_index(p, b);
            if (j < 0) return -1;
            used += p.arena_bytes[(int64_t)m * p.n_domain + j];
            present = true;
        }
        if (present) used += p.weight_bytes[m];
    }
    return used;
}

bool fit_mem(const ens_plan_problem& p, const int32_t* A) {
    for (int pool = 0; pool < p.n_pools; pool++) {
        const int64_t u = pool_used(p, A, pool);
        if (u < 0 || u > p.pool_cap[pool]) return false;
    }
    return true;
}

bool matrix_valid(int n_rows, int n_models, const int32_t* A) {
    for (int m = 0; m < n_models; m++) {
        bool any = false;
        for (int d = 0; d < n_rows; d++) any = any || A[d * n_models + m] != 0;
        if (!any) return false;
    }
    return true;
}

// Row of the wanted kind whose pool has the most memory left; lowest index wins ties; -1 if none.
static int more_remaining_memory(const ens_plan_problem& p, const int32_t* A, bool gpu) {
    int best = -1;
    int64_t best_rem = 0;
    for (int d = 0; d < p.n_rows; d++) {
        if ((p.row_is_gpu[d] != 0) != gpu) continue;
        const int64_t rem = p.pool_cap[p.row_pool[d]] - pool_used(p, A, p.row_pool[d]);
        if (best < 0 || rem > best_rem) { best = d; best_rem = rem; }
    }
    return best;
}

int wfd(const ens_plan_problem& p, int32_t* A) {
    const int jd = domain_index(p, p.default_batch);
    std::fill(A, A + (size_t)p.n_rows * p.n_models, 0);
    std::vector<int> order(p.n_models);
    std::iota(order.begin(), order.end(), 0);
    auto size_of = [&](int m) { return p.weight_bytes[m] + p.arena_bytes[(int64_t)m * p.n_domain + jd]; };
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return size_of(a) > size_of(b); });
    for (int m : order) {
        const int cand[2] = {more_remaining_memory(p, A, true), more_remaining_memory(p, A, false)};
        bool placed = false;
        for (int c = 0; c < 2 && !placed; c++) {          // the GPU side is tried first
            if (cand[c] < 0) continue;
            A[cand[c] * p.n_models + m] = p.default_batch;
            if (fit_mem(p, A)) placed = true;
            else A[cand[c] * p.n_models + m] = 0;
        }
        if (!placed) return ENS_E_NOFIT;
    }
    return ENS_OK;
}

// Every valid matrix that differs from A in exactly one cell, as (cell, value) moves in the
// order row, column, value (0 first, then the domain ascending).
std::vector<Move> neighborhood(const ens_plan_problem& p, const int32_t* A) {
    std::vector<int> values(p.domain, p.domain + p.n_domain);
    std::sort(values.begin(), values.end());
    values.insert(values.begin(), 0);
    std::vector<int> per_col(p.n_models, 0);
    for (int d = 0; d < p.n_rows; d++)
        for (int m = 0; m < p.n_models; m++) per_col[m] += A[d * p.n_models + m] != 0;
    std::vector<Move> out;
    for (int d = 0; d < p.n_rows; d++)
        for (int m = 0; m < p.n_models; m++) {
            const int cur = A[d * p.n_models + m];
            for (int v : values) {
                if (v == cur) continue;
                if (v == 0 && per_col[m] == 1) continue;    // would leave the column empty
                out.push_back(Move{d * p.n_models + m, v});
            }
        }
    return out;
}

struct SplitMix {
    uint64_t state;
    uint64_t next() {
        state += 0x9E3779B97F4A7C15ull;
        uint64_t z = state;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
};

// The fastest of up to max_neighs one-cell neighbours of A (all of them, or a seeded draw without
// replacement by a partial Fisher-Yates shuffle); the first in enumeration order wins ties.
// Returns false when A has no neighbour.
static bool fastest_neighbour(const ens_plan_problem& p, const int32_t* A, SplitMix& rng,
                              const std::function<double(const int32_t*)>& bench, int* benches, Move* move, double* speed) {
    std::vector<Move> cand = neighborhood(p, A);
    if ((int)cand.size() > p.max_neighs) {
        const size_t n = cand.size();
        for (int i = 0; i < p.max_neighs; i++) {
            const size_t j = i + (size_t)(rng.next() % (uint64_t)(n - i));
            std::swap(cand[i], cand[j]);
        }
        cand.resize(p.max_neighs);
    }
    const size_t cells = (size_t)p.n_rows * p.n_models;
    std::vector<int32_t> trial(A, A + cells);
    bool found = false;
    for (const Move& mv : cand) {
        const int32_t keep = trial[mv.cell];
        trial[mv.cell] = mv.value;
        const double s = bench(trial.data());
        trial[mv.cell] = keep;
        ++*benches;
        if (!found || s > *speed) { found = true; *move = mv; *speed = s; }
    }
    return found;
}

// Algorithm 2: hill climbing from A, one cell per move, each move to the fastest benchmarked
// neighbour, only while that is strictly faster than the matrix held; at most `moves_allowed`
// moves.  Section "Offline benchmark settings" raises that bound to (rows - models) when there are
// more rows than the bound lets the search fill, and so does this function.
int greedy(const ens_plan_problem& p, int32_t* A, const std::function<double(const int32_t*)>& bench,
           double* score, int32_t* n_bench) {
    const int moves_allowed = std::max(p.max_iter, p.n_rows - p.n_models);
    SplitMix rng{p.seed};
    double held = bench(A);
    int benches = 1;
    for (int moves = 0; moves < moves_allowed; moves++) {
        Move mv{0, 0};
        double s = 0;
        if (!fastest_neighbour(p, A, rng, bench, &benches, &mv, &s) || !(s > held)) break;   // local maximum or plateau
        A[mv.cell] = mv.value;
        held = s;
    }
    if (score) *score = held;
    if (n_bench) *n_bench = benches;
    return ENS_OK;
}

int bbs(const ens_plan_problem& p, const std::function<double(int, int)>& bench_single, int32_t* batch_out,
        int32_t* n_bench) {
    std::vector<int> values(p.domain, p.domain + p.n_domain);
    std::sort(values.begin(), values.end());
    int benches = 0;
    for (int m = 0; m < p.n_models; m++) {
        bool have = false;
        double best = 0;
        for (int b : values) {
            const double s = bench_single(m, b);
            benches++;
            if (!have || s > best) { have = true; best = s; batch_out[m] = b; }
        }
    }
    if (n_bench) *n_bench = benches;
    return ENS_OK;
}

int partition(int64_t nb_images, int seg, int batch, std::vector<std::pair<int64_t, int64_t>>* out) {
    if (nb_images < 0 || seg <= 0 || batch <= 0) return ENS_E_INVALID;
    out->clear();
    for (int64_t s = 0; s * seg < nb_images; s++) {
        const int64_t start = s * seg, end = std::min<int64_t>((s + 1) * seg, nb_images);
        for (int64_t a = start; a < end; a += batch) out->push_back({a, std::min<int64_t>(a + batch, end)});
    }
    return ENS_OK;
}

// Which of a member's workers takes which segment.  In the paper the workers of one DNN take
// segment ids from the same FIFO queue (section "Data-parallelism"): whoever is free takes the next
// one, so a worker gets segments in proportion to its speed.  Here the hand-out is decided on the
// host before anything is launched, by running that queue in estimated time: a worker with batch
// size b needs ceil(L / b) * launch_cost + L * image_cost for a segment of L images (a batch costs a
// fixed amount for its kernel launches plus an amount per image), and every segment, in order, goes
// to the worker that becomes free first (lowest index on ties).  Deterministic; with equal batch
// sizes it is round-robin.
int hand_out(int64_t nb_images, int seg, const int32_t* batch, int n_workers, double launch_cost, double image_cost,
             std::vector<int32_t>* owner) {
    if (nb_images < 0 || seg <= 0 || n_workers <= 0 || !batch || launch_cost < 0 || image_cost < 0) return ENS_E_INVALID;
    for (int k = 0; k < n_workers; k++)
        if (batch[k] <= 0) return ENS_E_INVALID;
    owner->clear();
    std::vector<double> free_at(n_workers, 0.0);
    for (int64_t s = 0; s * seg < nb_images; s++) {
        const int64_t len = std::min<int64_t>((s + 1) * seg, nb_images) - s * seg;
        int pick = 0;
        for (int k = 1; k < n_workers; k++)
            if (free_at[k] < free_at[pick]) pick = k;
        free_at[pick] += (double)((len + batch[pick] - 1) / batch[pick]) * launch_cost + (double)len * image_cost;
        owner->push_back(pick);
    }
    return ENS_OK;
}

}  // namespace ens

// ---------------------------------------------------------------------------- C interface
using namespace ens;

extern "C" {

int ens_planner_fit_mem(const ens_plan_problem* p, const int32_t* matrix) {
    if (!problem_ok(p) || !matrix) return ENS_E_INVALID;
    return fit_mem(*p, matrix) ? 1 : 0;
}

int ens_planner_wfd(const ens_plan_problem* p, int32_t* matrix_out) {
    if (!problem_ok(p) || !matrix_out) return ENS_E_INVALID;
    return wfd(*p, matrix_out);
}

int ens_planner_neighbors(const ens_plan_problem* p, const int32_t* matrix, int32_t* out, int32_t max_out,
                          int32_t* n_out) {
    if (!problem_ok(p) || !matrix || !n_out) return ENS_E_INVALID;
    if (!matrix_valid(p->n_rows, p->n_models, matrix)) return ENS_E_INVALID;
    const std::vector<Move> mv = neighborhood(*p, matrix);
    *n_out = (int32_t)mv.size();
    const size_t cells = (size_t)p->n_rows * p->n_models;
    for (size_t i = 0; i < mv.size() && (int32_t)i < max_out && out; i++) {
        std::copy(matrix, matrix + cells, out + i * cells);
        out[i * cells + mv[i].cell] = mv[i].value;
    }
    return ENS_OK;
}

int ens_planner_greedy(const ens_plan_problem* p, int32_t* matrix_inout, ens_bench_fn bench, void* user,
                       double* score, int32_t* n_bench) {
    if (!problem_ok(p) || !matrix_inout || !bench) return ENS_E_INVALID;
    if (!matrix_valid(p->n_rows, p->n_models, matrix_inout)) return ENS_E_INVALID;
    return greedy(*p, matrix_inout, [&](const int32_t* A) { return bench(A, user); }, score, n_bench);
}

int ens_planner_bbs(const ens_plan_problem* p, ens_bench_single_fn bench, void* user, int32_t* batch_out,
                    int32_t* n_bench) {
    if (!problem_ok(p) || !bench || !batch_out) return ENS_E_INVALID;
    return bbs(*p, [&](int m, int b) { return bench(m, b, user); }, batch_out, n_bench);
}

int ens_partition(int64_t nb_images, int32_t segment_size, int32_t batch, int64_t* starts, int64_t* ends,
                  int32_t max_out, int32_t* n_out) {
    std::vector<std::pair<int64_t, int64_t>> v;
    const int rc = partition(nb_images, segment_size, batch, &v);
    if (rc != ENS_OK || !n_out) return ENS_E_INVALID;
    *n_out = (int32_t)v.size();
    for (size_t i = 0; i < v.size() && (int32_t)i < max_out && starts && ends; i++) {
        starts[i] = v[i].first;
        ends[i] = v[i].second;
    }
    return ENS_OK;
}

int ens_hand_out(int64_t nb_images, int32_t segment_size, const int32_t* batch, int32_t n_workers, double launch_cost,
                 double image_cost, int32_t* owner_out, int32_t max_out, int32_t* n_out) {
    std::vector<int32_t> v;
    const int rc = hand_out(nb_images, segment_size, batch, n_workers, launch_cost, image_cost, &v);
    if (rc != ENS_OK || !n_out) return ENS_E_INVALID;
    *n_out = (int32_t)v.size();
    for (size_t i = 0; i < v.size() && (int32_t)i < max_out && owner_out; i++) owner_out[i] = v[i];
    return ENS_OK;
}

}  // extern "C"
