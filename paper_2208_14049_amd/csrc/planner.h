// Host-side allocation-matrix optimizer; see planner.cpp.
#pragma once
#include <functional>
#include <utility>
#include <vector>

#include "../../include/ens.h"

namespace ens {

struct Move { int cell; int value; };

bool problem_ok(const ens_plan_problem* p);
int64_t pool_used(const ens_plan_problem& p, const int32_t* A, int pool);
bool fit_mem(const ens_plan_problem& p, const int32_t* A);
bool matrix_valid(int n_rows, int n_models, const int32_t* A);
int wfd(const ens_plan_problem& p, int32_t* A);
std::vector<Move> neighborhood(const ens_plan_problem& p, const int32_t* A);
int greedy(const ens_plan_problem& p, int32_t* A, const std::function<double(const int32_t*)>& bench,
           double* score, int32_t* n_bench);
int bbs(const ens_plan_problem& p, const std::function<double(int, int)>& bench_single, int32_t* batch_out,
        int32_t* n_bench);
int partition(int64_t nb_images, int seg, int batch, std::vector<std::pair<int64_t, int64_t>>* out);
int hand_out(int64_t nb_images, int seg, const int32_t* batch, int n_workers, double launch_cost, double image_cost,
             std::vector<int32_t>* owner);

}  // namespace ens
