// Internal declarations shared by the HIP translation units of libthia.
// gfx950 (CDNA4) only.  No part of this library depends on the CPU oracle.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <functional>
#include <mutex>
#include <set>
#include <string>
#include <utility>
#include <vector>

#include "../../include/thia.h"

namespace thia {

// Raises a kernel's dynamic LDS limit to `bytes` once per (kernel, device): the attribute belongs to the device's copy of
// the code object, so a flag per process is not enough when a second GPU or a second thread comes along.
inline hipError_t ensure_dynamic_lds(const void* kernel, size_t bytes) {
    static std::mutex mu;
    static std::set<std::pair<const void*, int>> done;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    if (done.count({kernel, dev})) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) done.insert({kernel, dev});
    return e;
}

// ---------------------------------------------------------------- element helpers
typedef uint16_t bf16_t;  // raw bfloat16 bits

__host__ __device__ inline bf16_t f32_to_bf16(float x) {
    union { float f; uint32_t u; } v;
    v.f = x;
    uint32_t u = v.u;
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);                                           // round to nearest even
    return (bf16_t)(u >> 16);
}
// Two floats -> packed bf16 pair (lo in bits 0..15) with the hardware conversion (round to nearest even).
__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_v;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_v;
    const f32x2_v v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_v));
}
__host__ __device__ inline float bf16_to_f32(bf16_t h) {
    union { float f; uint32_t u; } v;
    v.u = ((uint32_t)h) << 16;
    return v.f;
}

// ---------------------------------------------------------------- convolution (implicit GEMM)
// NHWC activations; weights [Cout][kh][kw][Cin] (K contiguous per output channel).
// out[m, n] = act(bias[n] + sum_k W[n, k] * im2col(in)[m, k] + res[m, n]),  m = (img, oy, ox).
// Output columns n < n_split go to out0 (row stride ld0), the others to out1 (row stride ld1).
struct ConvArgs {
    const void* in;
    const void* w;
    const float* bias;
    const void* res;  // may be null
    void* out0;
    void* out1;       // == nullptr unless the output is split
    int N, H, W, Cin, Ho, Wo, Cout, kh, kw, stride, pad;
    int relu, n_split, ld0, ld1;
    // Optional second source of a 1x1 convolution: out += W[:, Cin:Cin+Cin2] * in2[pixel (oy*stride2, ox*stride2)].
    // Used to sum a bottleneck's last 1x1 convolution and its projection shortcut in one accumulator.
    const void* in2;  // null = single source
    int Cin2, H2, W2, stride2;
    // Optional fused RPN predictors (bf16, Cout == 256, ReLU, large-tile kernel only; conv_heads_supported): instead of
    // storing the convolution's output t, the block rounds its 256-pixel x 256-channel tile to bf16 in LDS and
    // multiplies it by the 1x1 predictor weights: logits[m, a] = bl[a] + sum_c Wl[a, c] t[m, c] (a < head_a) and
    // deltas[m, j] = bd[j] + sum_c Wd[j, c] t[m, c] (j < 4 head_a), both fp32 and dense.  head_w: bf16 [96][256] rows
    // ordered (4 head_a delta rows, head_a logit rows, zero rows) in MFMA fragment order; head_b: fp32 [96] likewise.
    const void* head_w;  // null = plain convolution
    const float* head_b;
    float* head_logits;
    float* head_deltas;
    int head_a;
    // Optional expansion tail (bf16, Cout == 256, ReLU, large-tile kernel only; conv_tail_supported): the bottleneck's
    // last 1x1 is applied to the block's own 256-pixel x 256-channel output tile while it sits in LDS, so neither the
    // 256-channel tensor nor a second launch is needed: tail_out[m, n] = relu(tb[n] + sum_c Wt[n, c] t[m, c] + tail_res[m, n]),
    // n < tail_n (a multiple of 512).  tail_w: bf16 [tail_n][256] in MFMA fragment order; tail_res / tail_out: bf16 [M][tail_n].
    const void* tail_w = nullptr;  // null = no tail
    const float* tail_b = nullptr;
    const void* tail_res = nullptr;
    void* tail_out = nullptr;
    int tail_n = 0;
};
// precision 0: float tensors, fp32 MFMA; 1: bf16 tensors, bf16 MFMA with fp32 accumulation.
// out_f32: store float outputs even when tensors are bf16.  Returns hipSuccess or the launch error.
hipError_t launch_conv(const ConvArgs& a, int precision, bool out_f32, hipStream_t s);
// Shapes the kernel accepts.
bool conv_supported(const ConvArgs& a, int precision);
// True if launch_conv would run `a` (bf16, with head_* set) on the kernel variant that has the fused predictors.
bool conv_heads_supported(const ConvArgs& a, int precision);
// True if `a` (bf16, with tail_* set) fits the kernel variant with the expansion tail.
bool conv_tail_supported(const ConvArgs& a, int precision);

// ---------------------------------------------------------------- single-kernel bottleneck (bf16, stride 1)
// first == 0 (identity block): y = relu(W3 relu(W2 * relu(W1 x + b1) + b2) + b3 + x), x [N][H][W][4*width].
// first != 0 (projection block): y = relu(W3 relu(W2 * relu(W1 x + b1) + b2) + Ws x + b3), x [N][H][W][width]; w3f is
//   [W3 | Ws] concatenated along K ([4 width][2 width]) and b3 the sum of the two biases.
// y [N][H][W][4*width]; NHWC bf16, distinct buffers.  w1f / w2f / w3f: weight matrices ([width][Cin],
// [width][3][3][width], [4 width][K3], K contiguous) in MFMA fragment order (pack_mfma_fragments).
struct FusedBlockArgs {
    const bf16_t* x;
    bf16_t* y;
    const bf16_t *w1f, *w2f, *w3f;
    const float *b1, *b2, *b3;
    int N, H, W;
    int first;
    // optional tail layer (64-wide identity blocks): z = [relu](Wt y + bt), Wt [tail_n][4 * width] in fragment order,
    // z [N, H, W, tail_n]; tail_n = 0: none
    const bf16_t* wtf = nullptr;
    const float* bt = nullptr;
    bf16_t* z = nullptr;
    int tail_n = 0, tail_relu = 0;
};
bool fused_block_supported(const FusedBlockArgs& a, int width);
hipError_t launch_fused_block(const FusedBlockArgs& a, int width, hipStream_t s);
// w [Cout][K] (Cout % 32 == 0, K % 16 == 0) -> dst, Cout*K elements: fragment (ct, ks) = 64 lanes x 8 elements,
// lane l holds w[32 ct + l % 32][16 ks + 8 (l / 32) .. + 7].
void pack_mfma_fragments(const bf16_t* w, int Cout, int K, bf16_t* dst);

// ---------------------------------------------------------------- stem + pool
// frames u8 [n,3,H,W].  x = (u8 - mean) / stdv, zero padding after normalisation.
// fp32 models: launch_stem (out float [n,Hs,Ws,64] NHWC with ReLU applied; w: fp32 [(c*7+ky)*7+kx][64]) followed by
// launch_maxpool.
hipError_t launch_stem(const uint8_t* frames, int n, int H, int W, const float* w, const float* bias, float mean, float stdv, void* out,
                       hipStream_t s);
// wk: bf16 [64][22][8] with wk[ch][c*7+ky][j] = weight(ch, c, ky, kx = j-1) for j = 1..7, zero for j = 0 and row 21.
// bf16 models: stem and 3x3 / stride 2 / pad 1 max-pool in one kernel; out [n,Hp,Wp,64] NHWC bf16.
hipError_t launch_stem_pool(const uint8_t* frames, int n, int H, int W, const bf16_t* wk, const float* bias, float mean, float stdv,
                            void* out, hipStream_t s);
hipError_t launch_maxpool(const void* in, int n, int H, int W, int C, int precision, void* out, hipStream_t s);

// ---------------------------------------------------------------- RPN proposal path
struct AnchorSpec {
    int n_sizes, n_ratios;
    float sizes[8];
    float sqrt_ratios[4];
};
// Entries of a frame's candidate list in the top-k of `pre`: the radix select stops as soon as the keys at or above its
// current bound fit, the list is sorted and its first `pre` entries are the result.
inline int topk_cand_cap(int pre) {
    int p = 1;
    while (p < pre) p <<= 1;
    return p >= 4096 ? p : 2 * p;
}
struct TopkWork {          // device scratch for n frames
    uint32_t* hist;        // [n][2048]
    uint64_t* state;       // [n][4]: prefix key, k remaining, done flag, collected count
    uint64_t* cand;        // [n][topk_cand_cap(pre)]
};
// logits [n,nA]; deltas [n,nA,4]; out_idx [n,pre] (-1 pad); out_boxes [n,pre,4] (0 pad); out_n [n].
hipError_t launch_rpn_proposals(const float* logits, const float* deltas, int n, long nA, int pre, int Wk, int stride,
                                float imgW, float imgH, const AnchorSpec& anc, const TopkWork& work, int32_t* out_idx,
                                float* out_boxes, int32_t* out_n, hipStream_t s);
// boxes [n,cap,4], counts [n]; mask scratch [n][cap][ceil(cap/64)] u64; out_keep [n,max_keep] (-1 pad), out_n [n];
// rois_out (optional) [n,max_keep,4] gets the kept boxes, zero padded.
hipError_t launch_nms(const float* boxes, const int32_t* counts, int n, int cap, float thr, int max_keep, uint64_t* mask,
                      int32_t* out_keep, int32_t* out_n, float* rois_out, hipStream_t s);

// ---------------------------------------------------------------- ROI head
hipError_t launch_roialign(const void* feat, const float* rois, int n, int post, int Hk, int Wk, int Ch, int stride, int P,
                           int precision, void* out, hipStream_t s);
// cls [n*post,Kc] logits, deltas [n*post,4Kc], rois [n,post,4] -> scores [n,post,Kc], boxes [n,post,Kc,4]
hipError_t launch_scores_boxes(const float* cls, const float* deltas, const float* rois, int n, int post, int Kc, float imgW,
                               float imgH, float* scores, float* boxes, hipStream_t s);
// keys scratch [n][pow2 >= post*Kc] u64
hipError_t launch_select(const float* scores, const float* boxes, const int32_t* roi_n, int n, int post, int Kc,
                         float score_thr, float nms_thr, int D, uint64_t* keys, int key_cap, float* out_boxes,
                         float* out_scores, int32_t* out_labels, int32_t* out_n, hipStream_t s);
// fills the empty pattern for n frames
hipError_t launch_fill_empty(int n, int D, float* out_boxes, float* out_scores, int32_t* out_labels, hipStream_t s);

// ---------------------------------------------------------------- query planning (host logic + the predicate kernel)
// flags[r] = (number of slots d of row r with labels[r][d] == label and scores[r][d] >= min_score) >= min_count
hipError_t launch_count_predicate(const int32_t* labels, const float* scores, long rows, int D, int label, int min_count,
                                  float min_score, uint8_t* flags, hipStream_t s);
// counts[0..2] = TP, FP, FN of answers against reference answers (both uint8 [n], non-zero = positive)
hipError_t launch_answer_counts(const uint8_t* ans, const uint8_t* ref, long n, int32_t* counts, hipStream_t s);
// Exit estimator (Sec. 5.3) on NHWC last-stage features [n][HW][C]: pooled scratch [n][C]; w1t = W1 transposed [C][hid];
// C + hid + E floats of LDS (the caller keeps that within 64 KB); opt int32 [n] in 1..E, logits [n][E] or nullptr.
hipError_t launch_estimator(const void* feat, int n, int HW, int C, int precision, float* pooled, int hid, int E, const float* w1t,
                            const float* b1, const float* w2, const float* b2, int32_t* opt, float* logits, hipStream_t s);
struct PlanChunk { int start, len, ep; };
// Evaluates every exit on k frames (indices in `frames`) and writes their answers, flags[i * E + e]; blocks until done.
using PlanEval = std::function<int(const int* frames, int k, uint8_t* flags, std::string& err)>;
const char* planner_cfg_error(const thia_planner_cfg& c);  // nullptr if the configuration is usable
// memo_out (optional): receives the per-frame answers the planner memoised, [n][E]; rows of frames it did not evaluate are zero.
int plan_core(int n, int E, const thia_planner_cfg& cfg, const PlanEval& eval, std::vector<PlanChunk>& plan, thia_plan_stats& st,
              uint8_t* evaluated_mask, std::string& err, std::vector<uint8_t>* memo_out = nullptr);
// answers[i] = over[i] for the frames with over[i] < 2 (uint8, device)
hipError_t launch_apply_known_answers(const uint8_t* over, long n, uint8_t* answers, hipStream_t s);

}  // namespace thia
