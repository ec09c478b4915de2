// Role-conditioned advantage estimation: host-only, float64 (Alg. 1, policy-optimisation loop;
// RAE equation, Sec. 3).  One EMA baseline per (game, role); update first, then subtract.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <new>
#include <vector>

#include "spiral.h"

struct spiral_rae {
    int n_games;
    double alpha;
    std::vector<double> b;      // [n_games][2]
};

// defined in spiral_api.hip; sets the thread-local error text
extern "C" const char* spiral_last_error(void);
int spiral_set_error(int code, const char* text);

extern "C" int spiral_rae_create(int n_games, double alpha, spiral_rae** out) {
    if (!out) return spiral_set_error(SPIRAL_ERR_INVALID_ARG, "rae_create: null out");
    *out = nullptr;
    if (n_games < 1) return spiral_set_error(SPIRAL_ERR_INVALID_ARG, "rae_create: n_games must be positive");
    if (!(alpha >= 0.0 && alpha <= 1.0)) return spiral_set_error(SPIRAL_ERR_INVALID_ARG, "rae_create: alpha outside [0,1]");
    spiral_rae* r = new (std::nothrow) spiral_rae();
    if (!r) return spiral_set_error(SPIRAL_ERR_INVALID_ARG, "rae_create: out of host memory");
    r->n_games = n_games;
    r->alpha = alpha;
    r->b.assign((size_t)n_games * 2, 0.0);     // baselines start at zero
    *out = r;
    return SPIRAL_OK;
}

extern "C" int spiral_rae_update(spiral_rae* r, const int32_t* host_game_id, const double* host_r0, int n, double* host_adv) {
    if (!r) return spiral_set_error(SPIRAL_ERR_NOT_LOADED, "rae_update: null state");
    if (n < 0 || (n > 0 && (!host_game_id || !host_r0 || !host_adv)))
        return spiral_set_error(SPIRAL_ERR_INVALID_ARG, "rae_update: null array or negative n");
    for (int i = 0; i < n; ++i) {
        if (host_game_id[i] < 0 || host_game_id[i] >= r->n_games)
            return spiral_set_error(SPIRAL_ERR_INVALID_ARG, "rae_update: game id out of range");
        if (!std::isfinite(host_r0[i])) return spiral_set_error(SPIRAL_ERR_INVALID_ARG, "rae_update: non-finite reward");
    }
    const double a = r->alpha;
    for (int i = 0; i < n; ++i) {
        double* b = &r->b[(size_t)host_game_id[i] * 2];
        for (int p = 0; p < 2; ++p) {
            const double R = p == 0 ? host_r0[i] : -host_r0[i];     // zero-sum: R_1 = -R_0
            b[p] = a * b[p] + (1.0 - a) * R;
            host_adv[(size_t)i * 2 + p] = R - b[p];
        }
    }
    return SPIRAL_OK;
}

extern "C" int spiral_rae_get(const spiral_rae* r, double* host_b) {
    if (!r) return spiral_set_error(SPIRAL_ERR_NOT_LOADED, "rae_get: null state");
    if (!host_b) return spiral_set_error(SPIRAL_ERR_INVALID_ARG, "rae_get: null output");
    for (size_t i = 0; i < r->b.size(); ++i) host_b[i] = r->b[i];
    return SPIRAL_OK;
}

extern "C" int spiral_rae_set(spiral_rae* r, const double* host_b) {
    if (!r) return spiral_set_error(SPIRAL_ERR_NOT_LOADED, "rae_set: null state");
    if (!host_b) return spiral_set_error(SPIRAL_ERR_INVALID_ARG, "rae_set: null input");
    for (size_t i = 0; i < r->b.size(); ++i)
        if (!std::isfinite(host_b[i])) return spiral_set_error(SPIRAL_ERR_INVALID_ARG, "rae_set: non-finite baseline");
    for (size_t i = 0; i < r->b.size(); ++i) r->b[i] = host_b[i];
    return SPIRAL_OK;
}

extern "C" void spiral_rae_free(spiral_rae* r) { delete r; }
