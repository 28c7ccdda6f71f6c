// The host-only part of the library: error reporting, the control flow of Algorithm 1 (stage plan), the host decision
// of the adaptive velocity decay cache (Eq.7, Eq.8), the decision of the data-dependent reuse trigger, and the fit of
// Eq.7's timestep-aware factor.  Plain C++ without any GPU header, so that it also builds for the CPU alone (the tests
// compile it with the address and undefined-behaviour sanitizers and run the same cases through it).
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <algorithm>
#include <functional>
#include <vector>
#include "regione.h"

void regione_set_error(const char* fmt, ...);
#define RG_FAIL(code, ...) do { regione_set_error(__VA_ARGS__); return (code); } while (0)

static thread_local char g_last_error[512] = "";

void regione_set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof(g_last_error), fmt, ap);
    va_end(ap);
}

extern "C" const char* regione_last_error(void) { return g_last_error; }

extern "C" int regione_stage_plan_host(int32_t T, int32_t t_st, int32_t t_sm, const int32_t* forced_k, int32_t n_forced,
                                       regione_plan_step* steps_out, int32_t max_steps, int32_t* n_steps_out) {
    if (!steps_out || !n_steps_out || (n_forced > 0 && !forced_k)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "stage_plan: null argument");
    if (T < 1 || t_st < 1 || t_sm < 1 || n_forced < 0 || t_st + t_sm > T)
        RG_FAIL(REGIONE_ERR_INVALID_ARG, "stage_plan: T=%d t_st=%d t_sm=%d do not fit", T, t_st, t_sm);
    // boundaries of the segments, as timestep indices in descending order: the index after the stabilization stage,
    // one below every forced step, and t_sm - 1
    std::vector<int32_t> forced_i(forced_k, forced_k + n_forced);
    for (auto& k : forced_i) k = T - k;
    std::sort(forced_i.begin(), forced_i.end(), std::greater<int32_t>());
    std::vector<int32_t> bounds;
    bounds.push_back(T - t_st);
    for (int32_t i : forced_i) {
        // a forced step has to lie strictly inside the region-aware stage and below the step before it
        if (i - 1 >= bounds.back() - 0 || i - 1 <= t_sm - 1)
            RG_FAIL(REGIONE_ERR_INVALID_ARG, "stage_plan: forced step k=%d outside the region-aware stage or not descending", T - i);
        bounds.push_back(i - 1);
    }
    bounds.push_back(t_sm - 1);
    int32_t n = 0;
    auto put = [&](int32_t i, int32_t kind, int32_t first, int32_t next) {
        if (n < max_steps) steps_out[n] = regione_plan_step{i, kind, first, next};
        ++n;
    };
    for (int32_t i = T; i > T - t_st; --i) put(i, i == T - t_st + 1 ? REGIONE_STEP_FULL_STORE : REGIONE_STEP_FULL, 0, -1);
    for (size_t s = 0; s + 1 < bounds.size(); ++s) {
        const int32_t prev = bounds[s], next = bounds[s + 1];
        for (int32_t j = prev; j > next + 1; --j) put(j, REGIONE_STEP_REGION, j == prev, next);
        put(next + 1, REGIONE_STEP_FULL_STORE, 0, -1);
    }
    for (int32_t i = t_sm - 1; i >= 1; --i) put(i, REGIONE_STEP_FULL, 0, -1);
    *n_steps_out = n;
    if (n > max_steps) RG_FAIL(REGIONE_ERR_INVALID_ARG, "stage_plan: %d steps do not fit max_steps=%d", n, max_steps);
    return REGIONE_OK;
}

extern "C" int regione_velocity_decision_host(const float* t_host, const float* gamma_host, int32_t n_steps,
                                              float delta, int32_t j, regione_avd_state* st,
                                              int32_t* reuse, float* factor) {
    if (!t_host || !gamma_host || !st || !reuse || !factor) RG_FAIL(REGIONE_ERR_INVALID_ARG, "velocity_decision: null argument");
    if (n_steps < 1 || j < 1 || j >= n_steps) RG_FAIL(REGIONE_ERR_INVALID_ARG, "velocity_decision: step index %d outside [1, %d)", j, n_steps);
    // Eq.7: factor of the step at index j relative to the step before it (index j+1)
    const double d = (1.0 - (static_cast<double>(t_host[j + 1]) - static_cast<double>(t_host[j]))) * static_cast<double>(gamma_host[j]);
    const double prod = st->prod * d;
    const double criterion = 1.0 - prod;  // Eq.8, product over the steps after the cached one up to j
    if (!st->valid || criterion > static_cast<double>(delta)) {
        st->valid = 1;
        st->prod = 1.0;
        *reuse = 0;
        *factor = 1.0f;
    } else {
        st->prod = prod;
        *reuse = 1;
        *factor = static_cast<float>(prod);
    }
    return REGIONE_OK;
}

// The data-dependent reuse trigger beside Eq.8 (see regione_rel_change): decision before a region step, update after a
// fresh one.  The state starts as zeros at the first step of every segment.
extern "C" int regione_rel_decision_host(regione_rel_state* st, float decay, int32_t* reuse, float* factor) {
    if (!st || !reuse || !factor) RG_FAIL(REGIONE_ERR_INVALID_ARG, "rel_decision: null argument");
    const bool r = st->reuse_next && st->have_cache;     // never without a cached velocity, never two reuses in a row
    st->reuse_next = 0;
    *reuse = r ? 1 : 0;
    *factor = r ? decay : 1.0f;
    return REGIONE_OK;
}

extern "C" int regione_rel_update_host(regione_rel_state* st, const double* sums_host_opt, float threshold, double* rel_out_opt) {
    if (!st) RG_FAIL(REGIONE_ERR_INVALID_ARG, "rel_update: null state");
    if (sums_host_opt && st->have_cache) {
        const double s_diff = sums_host_opt[0], s_old = sums_host_opt[1];
        if (!(s_diff >= 0.0) || !(s_old >= 0.0)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "rel_update: a sum of squares is negative or NaN");
        const double rel = s_old > 0.0 ? sqrt(s_diff) / sqrt(s_old) : INFINITY;
        st->reuse_next = rel < static_cast<double>(threshold) ? 1 : 0;
        if (rel_out_opt) *rel_out_opt = rel;
    } else {
        st->reuse_next = 0;
        if (rel_out_opt) *rel_out_opt = INFINITY;
    }
    st->have_cache = 1;
    return REGIONE_OK;
}

extern "C" int regione_gamma_fit_host(const double* sq_norms_host, int32_t n_samples, const float* t_host, int32_t n_steps,
                                      float* gamma_out) {
    if (!sq_norms_host || !t_host || !gamma_out) RG_FAIL(REGIONE_ERR_INVALID_ARG, "gamma_fit: null argument");
    if (n_samples < 1 || n_steps < 1) RG_FAIL(REGIONE_ERR_INVALID_ARG, "gamma_fit: n_samples=%d n_steps=%d", n_samples, n_steps);
    const int64_t ld = static_cast<int64_t>(n_steps) + 1;
    for (int32_t j = 0; j <= n_steps; ++j) gamma_out[j] = 1.0f;
    for (int32_t j = 1; j < n_steps; ++j) {
        // least squares through the origin of |v_{t_j}| against |v_{t_{j+1}}| over the samples (Eq.7's left-hand side)
        double ab = 0.0, bb = 0.0;
        for (int32_t s = 0; s < n_samples; ++s) {
            const double a2 = sq_norms_host[s * ld + j], b2 = sq_norms_host[s * ld + j + 1];
            if (!(a2 >= 0.0) || !(b2 >= 0.0)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "gamma_fit: squared norm of sample %d is negative or NaN", s);
            ab += sqrt(a2) * sqrt(b2);
            bb += b2;
        }
        const double solver = 1.0 - (static_cast<double>(t_host[j + 1]) - static_cast<double>(t_host[j]));
        if (!(bb > 0.0) || !(solver > 0.0)) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "gamma_fit: step %d has zero velocities or a time step of one", j);
        gamma_out[j] = static_cast<float>(ab / bb / solver);
    }
    return REGIONE_OK;
}

