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

// TP, FP, FN of frame answers against the reference answers (Sec. 6.1).  One block; integer sums, so the order is immaterial.
__global__ void __launch_bounds__(1024) answer_counts_kernel(const uint8_t* __restrict__ ans, const uint8_t* __restrict__ ref, long n,
                                                             int32_t* __restrict__ counts) {
    __shared__ int s[3];
    if (threadIdx.x < 3) s[threadIdx.x] = 0;
    __syncthreads();
    int tp = 0, fp = 0, fn = 0;
    for (long i = threadIdx.x; i < n; i += 1024) {
        const bool a = ans[i] != 0, r = ref[i] != 0;
        tp += (a && r) ? 1 : 0; fp += (a && !r) ? 1 : 0; fn += (!a && r) ? 1 : 0;
    }
    atomicAdd(&s[0], tp); atomicAdd(&s[1], fp); atomicAdd(&s[2], fn);
    __syncthreads();
    if (threadIdx.x < 3) counts[threadIdx.x] = s[threadIdx.x];
}

// Mean over the positions of an NHWC map, one thread per channel: feat [n][HW][C] -> pooled [n][C].
template <typename T>
__global__ void spatial_mean_kernel(const T* __restrict__ feat, int HW, int C, float* __restrict__ pooled) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x, f = blockIdx.y;
    if (c >= C) return;
    const T* p = feat + (size_t)f * HW * C + c;
    float acc = 0.f;
    for (int i = 0; i < HW; ++i) {
        if constexpr (sizeof(T) == 2) acc += bf16_to_f32(p[(size_t)i * C]);
        else acc += p[(size_t)i * C];
    }
    pooled[(size_t)f * C + c] = acc / (float)HW;
}

// The exit estimator's two layers on one frame per block (Sec. 5.3): hidden = relu(W1 pooled + b1),
// logits = W2 hidden + b2, estimate = 1 + index of the largest logit (the first on a tie).
// w1t is W1 transposed, [C][hid], so that consecutive threads read consecutive addresses.
__global__ void __launch_bounds__(256) estimator_mlp_kernel(const float* __restrict__ pooled, int C, int hid, int E,
                                                            const float* __restrict__ w1t, const float* __restrict__ b1,
                                                            const float* __restrict__ w2, const float* __restrict__ b2,
                                                            int32_t* __restrict__ opt, float* __restrict__ logits_out) {
    extern __shared__ float sm[];
    float *sp = sm, *sh = sm + C, *sl = sh + hid;
    const int f = blockIdx.x, tid = threadIdx.x;
    for (int c = tid; c < C; c += 256) sp[c] = pooled[(size_t)f * C + c];
    __syncthreads();
    for (int j = tid; j < hid; j += 256) {
        float acc = b1[j];
        for (int c = 0; c < C; ++c) acc += w1t[(size_t)c * hid + j] * sp[c];
        sh[j] = acc > 0.f ? acc : 0.f;
    }
    __syncthreads();
    for (int e = tid; e < E; e += 256) {
        float acc = b2[e];
        for (int j = 0; j < hid; ++j) acc += w2[(size_t)e * hid + j] * sh[j];
        sl[e] = acc;
        if (logits_out) logits_out[(size_t)f * E + e] = acc;
    }
    __syncthreads();
    if (tid == 0) {
        int best = 0;
        for (int e = 1; e < E; ++e)
            if (sl[e] > sl[best]) best = e;
        opt[f] = best + 1;
    }
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

// answers[i] = over[i] where over[i] < 2 (frames whose answer is already known), else unchanged
__global__ void apply_known_answers_kernel(const uint8_t* __restrict__ over, long n, uint8_t* __restrict__ answers) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n && over[i] < 2) answers[i] = over[i];
}
hipError_t launch_apply_known_answers(const uint8_t* over, long n, uint8_t* answers, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(apply_known_answers_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, over, n, answers);
    return hipGetLastError();
}

hipError_t launch_answer_counts(const uint8_t* ans, const uint8_t* ref, long n, int32_t* counts, hipStream_t s) {
    hipLaunchKernelGGL(answer_counts_kernel, dim3(1), dim3(1024), 0, s, ans, ref, n, counts);
    return hipGetLastError();
}

hipError_t launch_estimator(const void* feat, int n, int HW, int C, int precision, float* pooled, int hid, int E, const float* w1t,
                            const float* b1, const float* w2, const float* b2, int32_t* opt, float* logits, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    const dim3 grid((C + 255) / 256, n);
    if (precision == 1) hipLaunchKernelGGL(spatial_mean_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t*>(feat), HW, C, pooled);
    else hipLaunchKernelGGL(spatial_mean_kernel<float>, grid, dim3(256), 0, s, static_cast<const float*>(feat), HW, C, pooled);
    const size_t lds = sizeof(float) * ((size_t)C + hid + E);
    hipLaunchKernelGGL(estimator_mlp_kernel, dim3(n), dim3(256), lds, s, pooled, C, hid, E, w1t, b1, w2, b2, opt, logits);
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
              uint8_t* evaluated_mask, std::string& err, std::vector<uint8_t>* memo_out) {
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
    if (memo_out) memo_out->swap(memo);   // rows of evaluated frames hold their answers, the rest is zero
    return THIA_OK;
}

}  // namespace thia
