// Proposal path of one exit: exact top-k of the RPN logits, anchor decoding, clipping
// and greedy NMS.
//
// Top-k: an element's rank key is 54 bits = (order-preserving map of the logit) << 22 |
// (2^22 - 1 - anchor index), so keys are unique and "largest key first" is exactly
// (logit descending, index ascending).  The k-th largest key is found by a most-significant
// -digit-first radix select (digits of 11,11,10,11,11 bits): each pass histograms, with
// many blocks per frame and integer atomics only, the digit of the elements that still match
// the prefix, then one block per frame picks the digit holding the k-th element.  A pass
// ends the search as soon as the keys at or above the digit bucket's lower bound fit the
// candidate list (twice the next power of two of k, at most 4096): with real-valued logits
// that is after the second digit, and the last three digits only ever run when logits tie
// at the cut.  All elements with key >= that bound are then gathered (any order) and
// sorted by key in LDS with a bitonic network, which makes the output order deterministic;
// the first k are the result.  The same block decodes the k anchors and compacts the
// non-empty boxes in order.
//
// NMS: a k x k upper-triangular overlap bit matrix (64-bit words) is computed by
// 64-thread blocks, then one wavefront per frame scans it 64 rows at a time from LDS,
// holding the "removed" bit vector one word per lane.
#include "device_util.h"

namespace thia {

constexpr int IDX_BITS = 22;
constexpr uint32_t IDX_MASK = (1u << IDX_BITS) - 1u;
constexpr int N_PASS = 5;
__host__ __device__ inline int pass_shift(int p) { return p == 0 ? 43 : p == 1 ? 32 : p == 2 ? 22 : p == 3 ? 11 : 0; }
__host__ __device__ inline int pass_bits(int p) { return p == 2 ? 10 : 11; }
constexpr int HIST_BINS = 2048;
constexpr int HIST_CHUNK = 8192;  // elements per histogram block
// Frames with at most this many anchors run the whole proposal step in one block per frame (one launch instead of twelve:
// 98 -> 74 / 51 us per 32 frames at 30 600 / 7 650 anchors).  Larger maps keep the multi-block histogram passes: a single
// block is bound by same-address LDS atomics (neighbouring logits share their leading digit), 161 against 99 us at 122 400
// anchors and 814 against 137 us at 486 000; counting a wavefront's shared digits once per ballot round was slower still.
constexpr long FUSED_MAX_ANCHORS = 50000;

__device__ inline uint64_t rank_key(float logit, uint32_t idx) {
    return ((uint64_t)score_key(logit) << IDX_BITS) | (uint64_t)(IDX_MASK - idx);
}

// state[f]: [0] prefix, [1] k remaining, [2] done, [3] gathered count
__global__ void topk_init_kernel(uint32_t* hist, uint64_t* state, int k) {
    const int f = blockIdx.x;
    for (int i = threadIdx.x; i < HIST_BINS; i += blockDim.x) hist[(size_t)f * HIST_BINS + i] = 0u;
    if (threadIdx.x == 0) {
        state[4 * f + 0] = 0ull;
        state[4 * f + 1] = (uint64_t)k;
        state[4 * f + 2] = 0ull;
        state[4 * f + 3] = 0ull;
    }
}

__global__ __launch_bounds__(256) void topk_hist_kernel(const float* __restrict__ logits, long nA, int pass,
                                                        uint32_t* __restrict__ hist, const uint64_t* __restrict__ state) {
    const int f = blockIdx.y;
    if (state[4 * f + 2]) return;
    __shared__ uint32_t lh[HIST_BINS];
    for (int i = threadIdx.x; i < HIST_BINS; i += 256) lh[i] = 0u;
    __syncthreads();
    const int shift = pass_shift(pass), bits = pass_bits(pass);
    const uint64_t prefix = state[4 * f + 0];
    const int hi_shift = shift + bits;  // bits above the current digit must equal the prefix
    const long i0 = (long)blockIdx.x * HIST_CHUNK;
    const long i1 = i0 + HIST_CHUNK < nA ? i0 + HIST_CHUNK : nA;
    const float* lg = logits + (size_t)f * nA;
    auto count = [&](float v, long i) {
        const uint64_t key = rank_key(v, (uint32_t)i);
        if (pass == 0 || (key >> hi_shift) == (prefix >> hi_shift)) atomicAdd(&lh[(key >> shift) & ((1u << bits) - 1u)], 1u);
    };
    if ((nA & 3) == 0) {   // every frame's logits start on a 16-byte boundary: four per load
        for (long i = i0 + 4 * threadIdx.x; i < i1; i += 4 * 256) {
            const float4 v = *reinterpret_cast<const float4*>(lg + i);
            count(v.x, i); count(v.y, i + 1); count(v.z, i + 2); count(v.w, i + 3);
        }
    } else {
        for (long i = i0 + threadIdx.x; i < i1; i += 256) count(lg[i], i);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < HIST_BINS; i += 256)
        if (lh[i]) atomicAdd(&hist[(size_t)f * HIST_BINS + i], lh[i]);
}

// One block per frame: find digit d with  #(digit > d) < k_rem <= #(digit >= d); clears the histogram.
__global__ __launch_bounds__(256) void topk_scan_kernel(uint32_t* __restrict__ hist, uint64_t* __restrict__ state, int pass, int k_want,
                                                        int cand_cap) {
    const int f = blockIdx.x;
    if (state[4 * f + 2]) return;  // uniform: written only by this block in earlier launches
    __shared__ uint32_t part[256];
    __shared__ uint32_t above[256];
    const int t = threadIdx.x;
    uint32_t h[8], sum = 0;
    uint32_t* hf = hist + (size_t)f * HIST_BINS;
    const uint32_t k_rem = (uint32_t)state[4 * f + 1];  // read before the barriers: written below by one thread
#pragma unroll
    for (int q = 0; q < 8; ++q) { h[q] = hf[8 * t + q]; sum += h[q]; hf[8 * t + q] = 0u; }
    part[t] = sum;
    __syncthreads();
    if (t == 0) {
        uint32_t run = 0;
        for (int i = 255; i >= 0; --i) { above[i] = run; run += part[i]; }
    }
    __syncthreads();
    uint32_t run = above[t];  // elements in bins above this thread's 8 bins
    for (int q = 7; q >= 0; --q) {
        if (run < k_rem && k_rem <= run + h[q]) {
            const uint64_t digit = (uint64_t)(8 * t + q);
            state[4 * f + 0] |= digit << pass_shift(pass);
            state[4 * f + 1] = (uint64_t)(k_rem - run);
            // keys at or above the bucket's lower bound: those above the prefix from earlier passes, above the digit, the bucket
            if ((uint32_t)k_want - k_rem + run + h[q] <= (uint32_t)cand_cap || pass == N_PASS - 1) state[4 * f + 2] = 1ull;
        }
        run += h[q];
    }
}

// Keys at or above the threshold, in any order.  A block collects its hits in LDS and reserves their places in the frame's
// list with one atomic (one per element made ~1500 same-address atomics per frame the whole cost of the kernel); hits
// beyond the block's LDS list, which only a frame of near-equal logits produces, take their places one by one.
constexpr int GATHER_LDS_KEYS = 1024;
__global__ __launch_bounds__(256) void topk_gather_kernel(const float* __restrict__ logits, long nA,
                                                          uint64_t* __restrict__ state, uint64_t* __restrict__ cand, int cap) {
    __shared__ uint64_t s_keys[GATHER_LDS_KEYS];
    __shared__ uint32_t s_n;
    __shared__ unsigned long long s_base;
    const int f = blockIdx.y;
    const uint64_t thr = state[4 * f + 0];
    const long i0 = (long)blockIdx.x * HIST_CHUNK;
    const long i1 = i0 + HIST_CHUNK < nA ? i0 + HIST_CHUNK : nA;
    const float* lg = logits + (size_t)f * nA;
    unsigned long long* total = reinterpret_cast<unsigned long long*>(&state[4 * f + 3]);
    if (threadIdx.x == 0) s_n = 0u;
    __syncthreads();
    auto take = [&](float v, long i) {
        const uint64_t key = rank_key(v, (uint32_t)i);
        if (key >= thr) {
            const uint32_t slot = atomicAdd(&s_n, 1u);
            if (slot < (uint32_t)GATHER_LDS_KEYS) {
                s_keys[slot] = key;
            } else {
                const unsigned long long g = atomicAdd(total, 1ull);
                if (g < (unsigned long long)cap) cand[(size_t)f * cap + g] = key;
            }
        }
    };
    if ((nA & 3) == 0) {
        for (long i = i0 + 4 * threadIdx.x; i < i1; i += 4 * 256) {
            const float4 v = *reinterpret_cast<const float4*>(lg + i);
            take(v.x, i); take(v.y, i + 1); take(v.z, i + 2); take(v.w, i + 3);
        }
    } else {
        for (long i = i0 + threadIdx.x; i < i1; i += 256) take(lg[i], i);
    }
    __syncthreads();
    const uint32_t mine = s_n < (uint32_t)GATHER_LDS_KEYS ? s_n : (uint32_t)GATHER_LDS_KEYS;
    if (mine == 0u) return;   // uniform
    if (threadIdx.x == 0) s_base = atomicAdd(total, (unsigned long long)mine);
    __syncthreads();
    const unsigned long long base = s_base;
    for (uint32_t j = threadIdx.x; j < mine; j += 256)
        if (base + j < (unsigned long long)cap) cand[(size_t)f * cap + base + j] = s_keys[j];
}

// Tail shared by the two top-k paths, run by a 1024-thread block for frame f: `keys` (LDS, cap entries, the gathered
// candidates first, the rest zero) is sorted, the first k emitted as indices, their anchors decoded and clipped, non-empty
// boxes compacted in order.
__device__ inline void sort_decode_emit(uint64_t* keys, int got, int k_want, int cap, int pre, long nA, const float* __restrict__ deltas,
                                        int Wk, int stride, float imgW, float imgH, const AnchorSpec& anc, int f,
                                        int32_t* __restrict__ out_idx, float* __restrict__ out_boxes, int32_t* __restrict__ out_n) {
    __shared__ int wave_tot[16];
    __shared__ int base_sh;
    const int t = threadIdx.x;
    if (t == 0) base_sh = 0;
    __syncthreads();
    const int k = got < k_want ? got : k_want;
    // the usual case gathers k or a few more keys: half the list then holds them all, and the network is a stage shorter
    bitonic_sort_desc_lds(keys, 2 * got <= cap ? cap / 2 : cap);

    const int A = anc.n_sizes * anc.n_ratios;
    const float* dl = deltas + (size_t)f * nA * 4;
    for (int j0 = 0; j0 < pre; j0 += 1024) {
        const int j = j0 + t;
        bool ok = false;
        Box b = {0.f, 0.f, 0.f, 0.f};
        if (j < pre) {
            int32_t idx = -1;
            if (j < k) {
                idx = (int32_t)(IDX_MASK - (uint32_t)(keys[j] & IDX_MASK));
                const int a = idx % A, loc = idx / A, x = loc % Wk, y = loc / Wk;
                const float size = anc.sizes[a / anc.n_ratios], sr = anc.sqrt_ratios[a % anc.n_ratios];
                const float cx = ((float)x + 0.5f) * (float)stride, cy = ((float)y + 0.5f) * (float)stride;
                const float w = size / sr, h = size * sr;
                const float4 d = *reinterpret_cast<const float4*>(dl + 4 * (size_t)idx);
                ok = decode_box(cx, cy, w, h, d.x, d.y, d.z, d.w, imgW, imgH, b);
            }
            out_idx[(size_t)f * pre + j] = idx;
        }
        // ordered compaction: position = valid boxes before j
        const unsigned long long bal = __ballot(ok);
        const int lane = t & 63, wv = t >> 6;
        const int before = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) wave_tot[wv] = __popcll(bal);
        __syncthreads();
        int off = base_sh;
        for (int q = 0; q < wv; ++q) off += wave_tot[q];
        if (ok) *reinterpret_cast<float4*>(out_boxes + ((size_t)f * pre + off + before) * 4) = make_float4(b.x1, b.y1, b.x2, b.y2);
        __syncthreads();
        if (t == 0) {
            int tot = 0;
            for (int q = 0; q < 16; ++q) tot += wave_tot[q];
            base_sh += tot;
        }
        __syncthreads();
    }
    const int total = base_sh;
    for (int j = total + t; j < pre; j += 1024)
        *reinterpret_cast<float4*>(out_boxes + ((size_t)f * pre + j) * 4) = make_float4(0.f, 0.f, 0.f, 0.f);
    if (t == 0) out_n[f] = total;
}

// One block per frame: sort the gathered keys, emit indices, decode, clip, compact non-empty boxes.
__global__ __launch_bounds__(1024) void topk_sort_decode_kernel(const uint64_t* __restrict__ cand, const uint64_t* __restrict__ state,
                                                                int cap, int k_want, int pre, long nA, const float* __restrict__ deltas,
                                                                int Wk, int stride, float imgW, float imgH, AnchorSpec anc,
                                                                int32_t* __restrict__ out_idx, float* __restrict__ out_boxes,
                                                                int32_t* __restrict__ out_n) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint64_t* keys = reinterpret_cast<uint64_t*>(smem_raw);  // [cap]
    const int f = blockIdx.x, t = threadIdx.x;
    int got = (int)state[4 * f + 3];
    if (got > cap) got = cap;
    for (int i = t; i < cap; i += 1024) keys[i] = i < got ? cand[(size_t)f * cap + i] : 0ull;
    sort_decode_emit(keys, got, k_want, cap, pre, nA, deltas, Wk, stride, imgW, imgH, anc, f, out_idx, out_boxes, out_n);
}

// Radix-select passes first .. N_PASS - 1 of one frame by one 1024-thread block: LDS histogram of the digit of the elements
// that match the prefix, then the digit holding the k-th element.  prefix / k_rem / done are the block's shared search
// state (k_rem and prefix as left by the passes before `first`); hist [HIST_BINS], part and above [256] are LDS scratch.
__device__ inline void block_select_passes(const float* __restrict__ lg, long nA, int first, int k_want, int cand_cap, uint32_t* hist,
                                           uint32_t* part, uint32_t* above, uint64_t* s_prefix, uint32_t* s_krem, uint32_t* s_done) {
    const int t = threadIdx.x;
    for (int pass = first; pass < N_PASS; ++pass) {
        if (*s_done) break;                                                  // uniform: written before the last barrier
        for (int i = t; i < HIST_BINS; i += 1024) hist[i] = 0u;
        __syncthreads();
        const int shift = pass_shift(pass), bits = pass_bits(pass), hi_shift = shift + bits;
        const uint64_t prefix = *s_prefix;
        // (eight loads in flight per thread: with one the block reads at a few GB/s)
        for (long b = 0; b < nA; b += 8 * 1024) {
            float v[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) { const long i = b + q * 1024 + t; v[q] = i < nA ? lg[i] : 0.f; }
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const long i = b + q * 1024 + t;
                const uint64_t key = rank_key(v[q], (uint32_t)i);
                if (i < nA && (pass == 0 || (key >> hi_shift) == (prefix >> hi_shift))) atomicAdd(&hist[(key >> shift) & ((1u << bits) - 1u)], 1u);
            }
        }
        __syncthreads();
        // digit d with  #(digit > d) < k_rem <= #(digit >= d)
        uint32_t h[8], sum = 0;
        const uint32_t k_rem = *s_krem;
        if (t < 256) {
#pragma unroll
            for (int q = 0; q < 8; ++q) { h[q] = hist[8 * t + q]; sum += h[q]; }
            part[t] = sum;
        }
        __syncthreads();
        if (t == 0) {
            uint32_t run = 0;
            for (int i = 255; i >= 0; --i) { above[i] = run; run += part[i]; }
        }
        __syncthreads();
        if (t < 256) {
            uint32_t run = above[t];
            for (int q = 7; q >= 0; --q) {
                if (run < k_rem && k_rem <= run + h[q]) {                    // exactly one (thread, q) satisfies this
                    *s_prefix = prefix | ((uint64_t)(8 * t + q) << shift);
                    *s_krem = k_rem - run;
                    if ((uint32_t)k_want - k_rem + run + h[q] <= (uint32_t)cand_cap || pass == N_PASS - 1) *s_done = 1u;
                }
                run += h[q];
            }
        }
        __syncthreads();
    }
}

// Multi-kernel path, after the first two digits: one 1024-thread block per frame runs whatever passes the frame still
// needs (none unless more keys than the candidate list holds share the cut's first two digits, i.e. logits all but tie
// there; only the elements matching the prefix touch the histogram, so the block is not bound by LDS atomics).
__global__ __launch_bounds__(1024) void topk_finish_kernel(const float* __restrict__ logits, long nA, uint64_t* __restrict__ state,
                                                           int k_want, int cand_cap) {
    const int f = blockIdx.x, t = threadIdx.x;
    if (state[4 * f + 2]) return;   // uniform
    __shared__ uint32_t hist[HIST_BINS];
    __shared__ uint32_t part[256];
    __shared__ uint32_t above[256];
    __shared__ uint64_t s_prefix;
    __shared__ uint32_t s_krem, s_done;
    if (t == 0) { s_prefix = state[4 * f + 0]; s_krem = (uint32_t)state[4 * f + 1]; s_done = 0u; }
    __syncthreads();
    block_select_passes(logits + (size_t)f * nA, nA, 2, k_want, cand_cap, hist, part, above, &s_prefix, &s_krem, &s_done);
    if (t == 0) { state[4 * f + 0] = s_prefix; state[4 * f + 1] = (uint64_t)s_krem; state[4 * f + 2] = 1ull; }
}

// The whole proposal step of one frame in one 1024-thread block (frames with up to a few ten thousand anchors): the
// radix select runs its passes back to back with block-level barriers and an LDS histogram, the elements at or above the
// threshold key are gathered into LDS (keys are unique, so their order there does not matter), then sorted, decoded and
// emitted as above.  Same keys, same digits, same result as the multi-kernel path; its launches become one.
__global__ __launch_bounds__(1024) void topk_fused_kernel(const float* __restrict__ logits, long nA, int k_want, int cap, int pre,
                                                          const float* __restrict__ deltas, int Wk, int stride, float imgW, float imgH,
                                                          AnchorSpec anc, int32_t* __restrict__ out_idx, float* __restrict__ out_boxes,
                                                          int32_t* __restrict__ out_n) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint64_t* keys = reinterpret_cast<uint64_t*>(smem_raw);                  // [cap]
    uint32_t* hist = reinterpret_cast<uint32_t*>(keys + cap);                // [HIST_BINS]
    __shared__ uint32_t part[256];
    __shared__ uint32_t above[256];
    __shared__ uint64_t s_prefix;
    __shared__ uint32_t s_krem, s_done, s_count;
    const int f = blockIdx.x, t = threadIdx.x;
    const float* lg = logits + (size_t)f * nA;
    if (t == 0) { s_prefix = 0ull; s_krem = (uint32_t)k_want; s_done = 0u; s_count = 0u; }
    __syncthreads();
    block_select_passes(lg, nA, 0, k_want, cap, hist, part, above, &s_prefix, &s_krem, &s_done);
    const uint64_t thr = s_prefix;
    for (int i = t; i < cap; i += 1024) keys[i] = 0ull;
    __syncthreads();
    for (long b = 0; b < nA; b += 8 * 1024) {
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) { const long i = b + q * 1024 + t; v[q] = i < nA ? lg[i] : 0.f; }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const long i = b + q * 1024 + t;
            const uint64_t key = rank_key(v[q], (uint32_t)i);
            if (i < nA && key >= thr) {
                const uint32_t slot = atomicAdd(&s_count, 1u);
                if (slot < (uint32_t)cap) keys[slot] = key;
            }
        }
    }
    __syncthreads();
    int got = (int)s_count;
    if (got > cap) got = cap;
    sort_decode_emit(keys, got, k_want, cap, pre, nA, deltas, Wk, stride, imgW, imgH, anc, f, out_idx, out_boxes, out_n);
}

hipError_t launch_rpn_proposals(const float* logits, const float* deltas, int n, long nA, int pre, int Wk, int stride,
                                float imgW, float imgH, const AnchorSpec& anc, const TopkWork& work, int32_t* out_idx,
                                float* out_boxes, int32_t* out_n, hipStream_t s) {
    if (n <= 0 || nA <= 0 || nA > (long)IDX_MASK || pre <= 0 || pre > 4096) return hipErrorInvalidValue;
    const int k = (long)pre < nA ? pre : (int)nA;
    const int cap = topk_cand_cap(pre);
    const unsigned bpf = (unsigned)((nA + HIST_CHUNK - 1) / HIST_CHUNK);
    if (n > 65535) return hipErrorInvalidValue;
    if (nA <= FUSED_MAX_ANCHORS) {
        hipLaunchKernelGGL(topk_fused_kernel, dim3(n), dim3(1024), (size_t)cap * 8 + HIST_BINS * 4, s, logits, nA, k, cap, pre, deltas, Wk,
                           stride, imgW, imgH, anc, out_idx, out_boxes, out_n);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(topk_init_kernel, dim3(n), dim3(256), 0, s, work.hist, work.state, k);
    for (int pass = 0; pass < 2; ++pass) {   // the two leading digits with many blocks per frame (every element takes part in the first)
        hipLaunchKernelGGL(topk_hist_kernel, dim3(bpf, n), dim3(256), 0, s, logits, nA, pass, work.hist, work.state);
        hipLaunchKernelGGL(topk_scan_kernel, dim3(n), dim3(256), 0, s, work.hist, work.state, pass, k, cap);
    }
    hipLaunchKernelGGL(topk_finish_kernel, dim3(n), dim3(1024), 0, s, logits, nA, work.state, k, cap);
    hipLaunchKernelGGL(topk_gather_kernel, dim3(bpf, n), dim3(256), 0, s, logits, nA, work.state, work.cand, cap);
    hipLaunchKernelGGL(topk_sort_decode_kernel, dim3(n), dim3(1024), (size_t)cap * 8, s, work.cand, work.state, cap, k, pre, nA,
                       deltas, Wk, stride, imgW, imgH, anc, out_idx, out_boxes, out_n);
    return hipGetLastError();
}

// ------------------------------------------------------------------------- NMS
__global__ __launch_bounds__(64) void nms_mask_kernel(const float* __restrict__ boxes, const int32_t* __restrict__ counts,
                                                      int cap, int words, float thr, uint64_t* __restrict__ mask) {
    const int bx = blockIdx.x, by = blockIdx.y, f = blockIdx.z;
    if (bx < by) return;
    const int cnt = counts[f] < cap ? counts[f] : cap;
    if (64 * by >= cnt || 64 * bx >= cnt) return;
    __shared__ Box cb[64];
    const int t = threadIdx.x;
    const float* bf = boxes + (size_t)f * cap * 4;
    const int cj = 64 * bx + t;
    if (cj < cnt) {
        const float4 v = *reinterpret_cast<const float4*>(bf + 4 * (size_t)cj);
        cb[t] = {v.x, v.y, v.z, v.w};
    }
    __syncthreads();
    const int i = 64 * by + t;
    if (i >= cnt) return;
    const float4 v = *reinterpret_cast<const float4*>(bf + 4 * (size_t)i);
    const Box me = {v.x, v.y, v.z, v.w};
    uint64_t bits = 0ull;
    const int jn = (cnt - 64 * bx) < 64 ? (cnt - 64 * bx) : 64;
    for (int b = 0; b < jn; ++b) {
        const int j = 64 * bx + b;
        if (j > i && iou_over(me, cb[b], thr)) bits |= 1ull << b;
    }
    mask[((size_t)f * cap + i) * words + bx] = bits;
}

// One 256-thread block per frame.  The bit matrix is consumed 64 rows at a time: all threads
// fetch the next 64 x words tile into registers while wavefront 0 resolves the current one from
// LDS.  Within a tile the greedy decisions only need the diagonal word of each row, which is
// held one row per lane and broadcast with readlane, so the serial chain is register-only; the
// rows that were kept are then OR-ed into the "removed" vector (one 64-bit word per lane).
__global__ __launch_bounds__(256) void nms_reduce_kernel(const uint64_t* __restrict__ mask, const float* __restrict__ boxes,
                                                         const int32_t* __restrict__ counts, int cap, int words, int max_keep,
                                                         int32_t* __restrict__ out_keep, int32_t* __restrict__ out_n,
                                                         float* __restrict__ rois_out) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint64_t* tile = reinterpret_cast<uint64_t*>(smem_raw);                 // [64][words]
    int32_t* keep = reinterpret_cast<int32_t*>(tile + (size_t)64 * words);  // [max_keep]
    __shared__ int s_nk;
    const int f = blockIdx.x, t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int cnt = counts[f] < cap ? counts[f] : cap;
    const int wc = (cnt + 63) / 64;
    const uint64_t* mf = mask + (size_t)f * cap * words;
    const int per_thread = (64 * words + 255) / 256;   // <= 16 for words <= 64
    // two tiles ahead: a tile's words are requested while the tile before the previous one is resolved
    uint64_t stage_a[16], stage_b[16];
    auto fetch = [&](int c, uint64_t (&stage)[16]) {
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            if (q >= per_thread) break;
            const int e = q * 256 + t, r = e / words, w = e - r * words;
            uint64_t v = 0ull;
            if (e < 64 * words && 64 * c + r < cnt && w >= c && w < wc) v = mf[(size_t)(64 * c + r) * words + w];
            stage[q] = v;
        }
    };
    auto stash = [&](const uint64_t (&stage)[16]) {
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            if (q >= per_thread) break;
            const int e = q * 256 + t;
            if (e < 64 * words) tile[e] = stage[q];
        }
    };
    if (t == 0) s_nk = -1;    // becomes the final count as soon as max_keep boxes are kept (early exit for all wavefronts)
    uint64_t removed = 0ull;  // wavefront 0: lane w holds word w
    int nk = 0;
    if (wc > 0) fetch(0, stage_a);
    if (wc > 1) fetch(1, stage_b);
    __syncthreads();
    // one tile: returns true once max_keep boxes are kept
    auto step = [&](int c, uint64_t (&stage)[16]) {
        stash(stage);
        __syncthreads();
        if (c + 2 < wc) fetch(c + 2, stage);
        if (wv == 0) {
            const int rows = (cnt - 64 * c) < 64 ? (cnt - 64 * c) : 64;
            const uint64_t diag = lane < rows ? tile[(size_t)lane * words + c] : 0ull;
            const uint32_t dlo = (uint32_t)diag, dhi = (uint32_t)(diag >> 32);
            const uint32_t rlo = (uint32_t)removed, rhi = (uint32_t)(removed >> 32);
            uint64_t cur = (uint64_t)(uint32_t)__builtin_amdgcn_readlane(rlo, c) | ((uint64_t)(uint32_t)__builtin_amdgcn_readlane(rhi, c) << 32);
            // serial greedy chain over the tile's rows, registers and scalars only.  It steps from one kept row to the next
            // (lowest row not yet suppressed): with one wavefront on the SIMD every dependent instruction pays its full
            // latency, ~120 cycles per step, so stepping over suppressed rows one by one was most of the kernel.
            uint64_t kept = 0ull;
            int room = max_keep - nk;
            uint64_t avail = ~cur & (rows < 64 ? (1ull << rows) - 1ull : ~0ull);
            while (avail != 0ull && room > 0) {
                const int b = __builtin_ctzll(avail);
                kept |= 1ull << b;
                --room;
                const uint64_t d = (uint64_t)(uint32_t)__builtin_amdgcn_readlane(dlo, b) | ((uint64_t)(uint32_t)__builtin_amdgcn_readlane(dhi, b) << 32);
                avail &= ~d & ~((2ull << b) - 1ull);   // rows b suppresses, and rows up to b, are decided
            }
            // kept rows -> keep list (lane b writes its own slot) and OR of their mask rows into the removed set
            if ((kept >> lane) & 1ull) keep[nk + __popcll(kept & ((1ull << lane) - 1ull))] = 64 * c + lane;
            nk += __popcll(kept);
            if (nk < max_keep && lane < words) {
                uint64_t acc = 0ull;
                for (uint64_t k = kept; k != 0ull; k &= k - 1ull) acc |= tile[(size_t)__builtin_ctzll(k) * words + lane];   // kept rows only
                removed |= acc;
            }
            if (nk == max_keep && lane == 0) s_nk = nk;
        }
        __syncthreads();
        return s_nk >= 0;   // uniform: written before the barrier
    };
    for (int c = 0; c < wc; c += 2) {
        if (step(c, stage_a)) break;
        if (c + 1 < wc && step(c + 1, stage_b)) break;
    }
    if (t == 0 && s_nk < 0) s_nk = nk;
    __syncthreads();
    nk = s_nk;
    const float* bf = boxes + (size_t)f * cap * 4;
    for (int j = t; j < max_keep; j += 256) {
        const int src = j < nk ? keep[j] : -1;
        out_keep[(size_t)f * max_keep + j] = src;
        if (rois_out) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (src >= 0) v = *reinterpret_cast<const float4*>(bf + 4 * (size_t)src);
            *reinterpret_cast<float4*>(rois_out + ((size_t)f * max_keep + j) * 4) = v;
        }
    }
    if (t == 0) out_n[f] = nk;
}

hipError_t launch_nms(const float* boxes, const int32_t* counts, int n, int cap, float thr, int max_keep, uint64_t* mask,
                      int32_t* out_keep, int32_t* out_n, float* rois_out, hipStream_t s) {
    if (n <= 0 || cap <= 0 || cap > 4096 || max_keep <= 0 || max_keep > 4096 || n > 65535) return hipErrorInvalidValue;
    const int words = (cap + 63) / 64;
    hipLaunchKernelGGL(nms_mask_kernel, dim3(words, words, n), dim3(64), 0, s, boxes, counts, cap, words, thr, mask);
    const size_t lds = (size_t)64 * words * 8 + (size_t)max_keep * 4;
    hipLaunchKernelGGL(nms_reduce_kernel, dim3(n), dim3(256), lds, s, mask, boxes, counts, cap, words, max_keep, out_keep, out_n,
                       rois_out);
    return hipGetLastError();
}

}  // namespace thia
