// Parameters drawn from a seed when a member description carries no parameter blob.
// Counter-based: every value is a function of (seed, member, parameter index, element index).
//   mix(z): SplitMix64 finaliser;  key = mix(mix(mix(mix(seed) + member) + index) + kind)
//   bits(i) = mix(key + (i + 1) * 0x9E3779B97F4A7C15);  uniform = ((bits >> 11) + 0.5) * 2^-53
//   normal(i) = sqrt(-2 ln uniform(2i)) * cos(2 pi uniform(2i + 1))
// Weights: normal * scale.  Biases: normal * 0.1.  Batch-norm: gamma = scale, beta = 0,
// mean = normal * 0.1, variance uniform in [0.5, 1.5).
#include "seedgen.h"

#include <cmath>

namespace ens {

static inline uint64_t mix(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static inline uint64_t stream_key(uint64_t seed, uint64_t a, uint64_t b, uint64_t c) {
    return mix(mix(mix(mix(seed) + a) + b) + c);
}
static inline double uniform(uint64_t key, uint64_t i) {
    const uint64_t b = mix(key + (i + 1) * 0x9E3779B97F4A7C15ull);
    return ((double)(b >> 11) + 0.5) * (1.0 / 9007199254740992.0);
}
static inline double normal(uint64_t key, uint64_t i) {
    const double u1 = uniform(key, 2 * i), u2 = uniform(key, 2 * i + 1);
    return std::sqrt(-2.0 * std::log(u1)) * std::cos(2.0 * M_PI * u2);
}

enum { KIND_WEIGHT = 2, KIND_BIAS = 3, KIND_BN_MEAN = 4, KIND_BN_VAR = 5 };

int draw_params(const ens_param* specs, int n_specs, uint64_t seed, int member, float* blob, int64_t n_params) {
    for (int t = 0; t < n_specs; t++) {
        const ens_param& p = specs[t];
        if (p.offset < 0 || p.size < 0 || p.offset + p.size > n_params) return ENS_E_INVALID;
        float* dst = blob + p.offset;
        if (p.role == ENS_PARAM_WEIGHT) {
            const uint64_t k = stream_key(seed, member, t, KIND_WEIGHT);
            for (int64_t i = 0; i < p.size; i++) dst[i] = (float)(normal(k, i) * p.scale);
        } else if (p.role == ENS_PARAM_BIAS) {
            const uint64_t k = stream_key(seed, member, t, KIND_BIAS);
            for (int64_t i = 0; i < p.size; i++) dst[i] = (float)(normal(k, i) * 0.1);
        } else if (p.role == ENS_PARAM_BN) {
            const int64_t c = p.channels;
            if (c <= 0 || p.size != 4 * c) return ENS_E_INVALID;
            const uint64_t km = stream_key(seed, member, t, KIND_BN_MEAN);
            const uint64_t kv = stream_key(seed, member, t, KIND_BN_VAR);
            for (int64_t i = 0; i < c; i++) {
                dst[i] = (float)p.scale;
                dst[c + i] = 0.f;
                dst[2 * c + i] = (float)(normal(km, i) * 0.1);
                dst[3 * c + i] = (float)(0.5 + uniform(kv, i));
            }
        } else {
            return ENS_E_INVALID;
        }
    }
    return ENS_OK;
}

}  // namespace ens
