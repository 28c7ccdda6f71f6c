// Test driver for the library's host-only entry points (csrc/host_logic.cpp), built for the CPU with the address and
// undefined-behaviour sanitizers by tests/test_host_sanitizers.py.  Reads one case from stdin, calls the entry point
// through the public header, prints return code and results (floating point as hexadecimal literals, so the test can
// compare them bit for bit with what the shipped library returns).
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>
#include "regione.h"

static long rd_i() { long v; if (scanf("%ld", &v) != 1) { fprintf(stderr, "bad input\n"); exit(2); } return v; }
static double rd_f() { double v; if (scanf("%lf", &v) != 1) { fprintf(stderr, "bad input\n"); exit(2); } return v; }

int main() {
    char cmd[32];
    if (scanf("%31s", cmd) != 1) return 2;
    if (!strcmp(cmd, "plan")) {
        const int T = rd_i(), t_st = rd_i(), t_sm = rd_i(), n_forced = rd_i();
        std::vector<int32_t> forced(n_forced > 0 ? n_forced : 1);
        for (int i = 0; i < n_forced; ++i) forced[i] = rd_i();
        const int max_steps = rd_i();
        std::vector<regione_plan_step> steps(max_steps > 0 ? max_steps : 1);
        int32_t n = -1;
        const int rc = regione_stage_plan_host(T, t_st, t_sm, forced.data(), n_forced, steps.data(), max_steps, &n);
        printf("%d %d\n", rc, n);
        if (rc == REGIONE_OK) for (int i = 0; i < n; ++i) printf("%d %d %d %d\n", steps[i].i, steps[i].kind, steps[i].seg_first, steps[i].seg_next);
        else printf("%s\n", regione_last_error());
    } else if (!strcmp(cmd, "avd")) {
        const int n_steps = rd_i(); const float delta = rd_f(); const int n_j = rd_i();
        std::vector<int> js(n_j);
        for (auto& j : js) j = rd_i();
        std::vector<float> t(n_steps + 1), g(n_steps + 1);
        for (auto& v : t) v = rd_f();
        for (auto& v : g) v = rd_f();
        regione_avd_state st = {0, 1.0};
        for (int j : js) {
            int32_t reuse = -1; float factor = -1.f;
            const int rc = regione_velocity_decision_host(t.data(), g.data(), n_steps, delta, j, &st, &reuse, &factor);
            printf("%d %d %a %d %a\n", rc, reuse, (double)factor, st.valid, st.prod);
        }
    } else if (!strcmp(cmd, "gamma")) {
        const int n_samples = rd_i(), n_steps = rd_i();
        std::vector<double> sq((size_t)n_samples * (n_steps + 1));
        for (auto& v : sq) v = rd_f();
        std::vector<float> t(n_steps + 1), out(n_steps + 1, -1.f);
        for (auto& v : t) v = rd_f();
        const int rc = regione_gamma_fit_host(sq.data(), n_samples, t.data(), n_steps, out.data());
        printf("%d\n", rc);
        if (rc == REGIONE_OK) for (float v : out) printf("%a\n", (double)v); else printf("%s\n", regione_last_error());
    } else if (!strcmp(cmd, "rel")) {
        const float thr = rd_f(), decay = rd_f(); const int n = rd_i();
        regione_rel_state st = {0, 0};
        for (int i = 0; i < n; ++i) {
            const int op = rd_i();
            if (op == 0) { int32_t reuse = -1; float f = -1.f; const int rc = regione_rel_decision_host(&st, decay, &reuse, &f); printf("%d %d %a %d %d\n", rc, reuse, (double)f, st.have_cache, st.reuse_next); }
            else { double sums[2] = {0, 0}; if (op == 1) { sums[0] = rd_f(); sums[1] = rd_f(); } double rel = -1.0;
                   const int rc = regione_rel_update_host(&st, op == 1 ? sums : nullptr, thr, &rel); printf("%d %a %d %d\n", rc, rel, st.have_cache, st.reuse_next); }
        }
    } else if (!strcmp(cmd, "nulls")) {   // every entry point with null pointers: an error code, never a crash
        int32_t n = 0, reuse = 0; float f = 0.f; regione_avd_state st = {0, 1.0};
        printf("%d %d %d %d %d\n", regione_stage_plan_host(28, 6, 2, nullptr, 1, nullptr, 0, &n), regione_velocity_decision_host(nullptr, nullptr, 28, 0.1f, 3, &st, &reuse, &f),
               regione_gamma_fit_host(nullptr, 1, nullptr, 1, nullptr), regione_rel_decision_host(nullptr, 0.9f, &reuse, &f), regione_rel_update_host(nullptr, nullptr, 0.1f, nullptr));
    } else {
        return 2;
    }
    return 0;
}
