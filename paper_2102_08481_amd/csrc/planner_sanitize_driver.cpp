// Host-only driver for the planner's control logic (plan_core in planner.hip), built by tests/test_sanitizers.py under
// AddressSanitizer and UndefinedBehaviorSanitizer (host pass only) and run as a plain executable: random answer tables
// and random configurations, including videos shorter than a chunk, one-frame videos, batches of one, reuse distances
// beyond the video, and an evaluation callback that fails.  It touches no device.  Plans are checked for what must hold
// for any input (chunks tile the video in order, exits in range); equality with the paper's recursion is the business of
// tests/test_planner_host.py.  Not part of libthia.so.
#include <cstdio>
#include <cstdlib>
#include <random>

#include "thia_internal.h"

using namespace thia;

int main() {
    std::mt19937 rng(12345);
    int plans = 0;
    for (int it = 0; it < 400; ++it) {
        const int n = it < 8 ? it : 1 + (int)(rng() % 3000);
        const int E = 1 + (int)(rng() % 5);
        thia_planner_cfg cfg;
        thia_planner_defaults(&cfg);
        cfg.min_chunk = 1 + (int)(rng() % 200);
        cfg.final_span = 1 + (int)(rng() % 12);
        cfg.precision = (rng() % 11) / 10.0;
        cfg.recall = (rng() % 11) / 10.0;
        cfg.posi_enough = (rng() % 11) / 10.0;
        cfg.posi_skip = (rng() % 4) / 10.0;
        cfg.reuse_dist = (rng() % 3 == 0) ? (int)(rng() % 5000) : 0;
        cfg.eval_batch = (int)(rng() % 4) * (int)(rng() % 40);
        if (planner_cfg_error(cfg)) { std::fprintf(stderr, "valid configuration refused\n"); return 1; }
        std::vector<uint8_t> table((size_t)n * E);
        const unsigned dens = 1 + rng() % 9;
        for (auto& v : table) v = (rng() % 10) < dens;
        const bool failing = it % 50 == 49;
        int calls = 0;
        PlanEval eval = [&](const int* fr, int k, uint8_t* out, std::string& err) -> int {
            if (failing && ++calls == 2) { err = "forced failure"; return THIA_E_HIP; }
            for (int i = 0; i < k; ++i) {
                if (fr[i] < 0 || fr[i] >= n) { std::fprintf(stderr, "sample outside the video\n"); std::exit(1); }
                for (int e = 0; e < E; ++e) out[(size_t)i * E + e] = table[(size_t)fr[i] * E + e];
            }
            return THIA_OK;
        };
        std::vector<PlanChunk> plan;
        thia_plan_stats st;
        std::vector<uint8_t> mask(n ? n : 1);
        std::string err;
        const int rc = plan_core(n, E, cfg, eval, plan, st, mask.data(), err);
        if (rc != THIA_OK) {
            if (!failing || err.empty()) { std::fprintf(stderr, "unexpected failure %d\n", rc); return 1; }
            continue;
        }
        int pos = 0;
        for (const PlanChunk& c : plan) {
            if (c.start != pos || c.len <= 0 || c.ep < 0 || c.ep > E) { std::fprintf(stderr, "plan does not tile the video\n"); return 1; }
            pos += c.len;
        }
        if (pos != n || st.n_chunks != (int)plan.size()) { std::fprintf(stderr, "plan does not cover the video\n"); return 1; }
        ++plans;
    }
    thia_planner_cfg bad;
    thia_planner_defaults(&bad);
    bad.min_chunk = 0;
    if (!planner_cfg_error(bad)) return 1;
    double prf[3];
    const int32_t zero[3] = {0, 0, 0}, some[3] = {3, 1, 2};
    thia_metrics_from_counts(zero, prf);
    thia_metrics_from_counts(some, prf);
    thia_metrics_from_counts(nullptr, prf);
    std::printf("planner_sanitize_driver: ok (%d plans)\n", plans);
    return 0;
}
