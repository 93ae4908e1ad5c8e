#pragma once
#include "../../include/ens.h"

namespace ens {
// Fills `blob` (n_params floats) from the parameter specs; ENS_E_INVALID on a malformed spec.
int draw_params(const ens_param* specs, int n_specs, uint64_t seed, int member, float* blob, int64_t n_params);
}
