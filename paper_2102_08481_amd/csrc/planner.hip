// Fine-grained query planning (Sec. 5.2, Algorithm 1) as host logic around one batched device step.
//
// The paper states the planner as a recursion that samples a chunk, evaluates every exit on the samples,
// and either settles the chunk (an exit, or skip) or halves it and doubles the sampling rate.  Here the
// recursion is walked level by level: all chunks of one depth are sampled first, the frames none of them
// finds memoised are evaluated together in as few device batches as possible (every exit in one backbone
// pass), and only then are the chunks decided.  Chunks of one level are disjoint and a chunk consults only
// memoised frames inside its own range, so the plan, the set of evaluated frames and the reuse count are
// those of the depth-first recursion.
#include "thia_internal.h"

#include <algorithm>
#include <set>

namespace thia {

namespace {

// Count(class) >= t on one frame's detection slots (Table 2).  One thread per frame.
__global__ void count_predicate_kernel(const int32_t* __restrict__ labels, const float* __restrict__ scores, long rows, int D,
                                       int label, int min_count, float min_score, uint8_t* __restrict__ flags) {
    const long r = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= rows) return;
    int c = 0;
    for (int d = 0; d < D; ++d) c += (labels[r * D + d] == label && scores[r * D + d] >= min_score) ? 1 : 0;
    flags[r] = c >= min_count ? 1 : 0;
}

struct Node {
    int a, b;
    long long span;
    int depth;
};

}  // namespace

hipError_t launch_count_predicate(const int32_t* labels, const float* scores, long rows, int D, int label, int min_count,
                                  float min_score, uint8_t* flags, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    const int threads = 256;
    const long blocks = (rows + threads - 1) / threads;
    hipLaunchKernelGGL(count_predicate_kernel, dim3((unsigned)blocks), dim3(threads), 0, s, labels, scores, rows, D, label, min_count,
                       min_score, flags);
    return hipGetLastError();
}

const char* planner_cfg_error(const thia_planner_cfg& c) {
    if (!(c.precision >= 0.0 && c.precision <= 1.0) || !(c.recall >= 0.0 && c.recall <= 1.0)) return "precision / recall outside 0..1";
    if (c.min_chunk < 1 || c.final_span < 1 || c.final_span > (1 << 20)) return "min_chunk and final_span must be at least 1";
    if (!(c.posi_enough >= 0.0 && c.posi_enough <= 1.0) || !(c.posi_skip >= 0.0 && c.posi_skip <= 1.0)) return "positive-ratio thresholds outside 0..1";
    if (c.reuse_dist < 0 || c.eval_batch < 0) return "negative reuse_dist / eval_batch";
    return nullptr;
}

int plan_core(int n, int E, const thia_planner_cfg& cfg, const PlanEval& eval, std::vector<PlanChunk>& plan, thia_plan_stats& st,
              uint8_t* evaluated_mask, std::string& err) {
    plan.clear();
    st = thia_plan_stats{};
    if (evaluated_mask) std::fill(evaluated_mask, evaluated_mask + n, (uint8_t)0);
    if (n == 0) return THIA_OK;

    // EstimateSamplingRate: the deepest level halves the video d times; its rate is 1/final_span, so the first
    // level samples every final_span * 2^d frames.
    int d = 0;
    while ((long long)cfg.min_chunk << d < n) ++d;
    const long long span0 = (long long)cfg.final_span << d;

    std::set<int> known;                        // frames with memoised answers
    std::vector<uint8_t> memo((size_t)n * E);   // answers of memoised frames, [frame][exit]
    std::vector<Node> level{{0, n, span0, 0}}, next;
    std::vector<int> need, src;                 // frames to evaluate; per sample, the frame whose answers it uses
    std::vector<size_t> first;                  // node i's samples are src[first[i] .. first[i + 1])
    std::vector<uint8_t> fresh;

    while (!level.empty()) {
        need.clear(); src.clear(); first.assign(1, 0);
        for (const Node& nd : level) {
            for (long long f = nd.a; f < nd.b; f += nd.span) {
                const int fi = (int)f;
                int use = -1;
                if (known.count(fi)) {
                    use = fi;
                } else if (cfg.reuse_dist > 0 && !known.empty()) {
                    // nearest memoised frame inside the chunk, the earlier one on a tie
                    auto hi = known.lower_bound(fi);
                    long long best = -1;
                    if (hi != known.begin()) {
                        const int g = *std::prev(hi);
                        if (g >= nd.a && fi - g <= cfg.reuse_dist) { use = g; best = fi - g; }
                    }
                    if (hi != known.end()) {
                        const int g = *hi;
                        if (g < nd.b && g - fi <= cfg.reuse_dist && (use < 0 || g - fi < best)) use = g;
                    }
                }
                if (use >= 0) ++st.samples_reused;
                else { need.push_back(fi); use = fi; }
                src.push_back(use);
            }
            first.push_back(src.size());
        }
        if (!need.empty()) {
            const size_t step = cfg.eval_batch > 0 ? (size_t)cfg.eval_batch : need.size();
            fresh.resize(step * E);
            for (size_t o = 0; o < need.size(); o += step) {
                const int k = (int)std::min(step, need.size() - o);
                const int rc = eval(need.data() + o, k, fresh.data(), err);
                if (rc != THIA_OK) return rc;
                ++st.eval_batches;
                for (int i = 0; i < k; ++i) {
                    const int f = need[o + i];
                    std::copy(fresh.begin() + (size_t)i * E, fresh.begin() + (size_t)(i + 1) * E, memo.begin() + (size_t)f * E);
                    known.insert(f);
                    if (evaluated_mask) evaluated_mask[f] = 1;
                }
            }
            st.frames_evaluated += (int)need.size();
        }
        next.clear();
        for (size_t i = 0; i < level.size(); ++i) {
            const Node& nd = level[i];
            st.depth = std::max(st.depth, nd.depth);
            const size_t k = first[i + 1] - first[i];
            // PickBestEP: the fastest exit whose frame answers reach the precision and recall asked for, measured
            // against the last exit on the samples; and the reference exit's ratio of positive frames.
            int npos = 0;
            for (size_t j = first[i]; j < first[i + 1]; ++j) npos += memo[(size_t)src[j] * E + (E - 1)] ? 1 : 0;
            int best_ep = E;
            for (int e = 0; e < E; ++e) {
                int tp = 0, fp = 0, fn = 0;
                for (size_t j = first[i]; j < first[i + 1]; ++j) {
                    const bool p = memo[(size_t)src[j] * E + e] != 0, r = memo[(size_t)src[j] * E + (E - 1)] != 0;
                    tp += (p && r) ? 1 : 0; fp += (p && !r) ? 1 : 0; fn += (!p && r) ? 1 : 0;
                }
                const double prec = tp + fp == 0 ? 1.0 : (double)tp / (double)(tp + fp);
                const double rec = tp + fn == 0 ? 1.0 : (double)tp / (double)(tp + fn);
                if (prec >= cfg.precision && rec >= cfg.recall) { best_ep = e + 1; break; }
            }
            const double posi_ratio = (double)npos / (double)k;
            const int len = nd.b - nd.a;
            const bool small = len < 2 * (long long)cfg.min_chunk;
            if ((posi_ratio >= cfg.posi_enough && best_ep == 1) || small) {
                plan.push_back({nd.a, len, best_ep});
            } else if (posi_ratio <= cfg.posi_skip) {
                plan.push_back({nd.a, len, 0});
            } else {
                const int mid = nd.a + len / 2;
                next.push_back({nd.a, mid, nd.span / 2, nd.depth + 1});
                next.push_back({mid, nd.b, nd.span / 2, nd.depth + 1});
            }
        }
        level.swap(next);
    }
    std::sort(plan.begin(), plan.end(), [](const PlanChunk& x, const PlanChunk& y) { return x.start < y.start; });
    st.n_chunks = (int)plan.size();
    return THIA_OK;
}

}  // namespace thia
