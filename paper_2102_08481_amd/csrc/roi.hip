// ROI head kernels: ROIAlign gather on the NHWC head feature map, class scores and
// per-class box decoding, and the final detection selection (threshold, ordering,
// same-class greedy NMS, top-D).
#include "device_util.h"

#include <type_traits>

namespace thia {

// ------------------------------------------------------------------ ROIAlign
// One block per ROI; threads run over channels, so every tap is one contiguous run of Ch
// elements of the NHWC map.  Convention: texel j has centre j + 0.5; a sample more than one
// texel outside the map contributes zero; otherwise its coordinates are clamped to the
// texel-centre range.  Output layout [(ph*P + pw)][c].
//
// A bin averages 2 x 2 samples of 2 x 2 texels each, and both the sample grid and the bilinear
// weights are products of a row factor and a column factor.  So a bin is sum_y sum_x Wy[y] Wx[x] F[y][x]
// over the DISTINCT rows and columns its samples touch (2 to 4 of each), with the weights of coinciding
// texels added up: a bin narrower than two texels gathers 4, 6 or 9 texels instead of 16.  The per-axis
// lists are built once per ROI (2 P threads), expanded to one tap table per bin in LDS (texel offset and
// weight, the 1/4 of the average folded in, entries past the bin's count zero), and every work item runs
// the smallest unrolled gather that covers its bin's count.
constexpr int ROI_TAPS = 16;   // most taps per bin (4 rows x 4 columns)

__host__ __device__ inline size_t roialign_lds_bytes(int P) {
    return (size_t)P * P * (ROI_TAPS * 8 + 4) + (size_t)2 * P * (4 * 8 + 4);
}

template <typename T>
__global__ __launch_bounds__(256) void roialign_kernel(const T* __restrict__ feat, const float* __restrict__ rois, int post,
                                                       int Hk, int Wk, int Ch, float scale, int P, T* __restrict__ out) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int nb = P * P;
    int* s_off = reinterpret_cast<int*>(smem_raw);             // [nb][16] texel offsets (in pixels of the map)
    float* s_w = reinterpret_cast<float*>(s_off + ROI_TAPS * nb);   // [nb][16]
    int* s_nt = reinterpret_cast<int*>(s_w + ROI_TAPS * nb);   // [nb] taps of the bin
    int* ax_i = s_nt + nb;                                     // [2 P][4] distinct texel rows (first P lists) / columns
    float* ax_w = reinterpret_cast<float*>(ax_i + 8 * P);      // [2 P][4] their summed weights
    int* ax_n = reinterpret_cast<int*>(ax_w + 8 * P);          // [2 P] entries per list
    const int roi = blockIdx.x, f = roi / post;
    const float4 r = *reinterpret_cast<const float4*>(rois + 4 * (size_t)roi);
    const float x1 = r.x * scale, y1 = r.y * scale;
    const float bw = (r.z * scale - x1) / (float)P, bh = (r.w * scale - y1) / (float)P;
    if ((int)threadIdx.x < 2 * P) {
        const int lst = threadIdx.x, isx = lst >= P, p = isx ? lst - P : lst;
        const float start = isx ? x1 : y1, b = isx ? bw : bh;
        const int L = isx ? Wk : Hk;
        int n = 0;
        auto add = [&](int j, float w) {
            for (int k = 0; k < n; ++k)
                if (ax_i[4 * lst + k] == j) { ax_w[4 * lst + k] += w; return; }
            ax_i[4 * lst + n] = j; ax_w[4 * lst + n] = w; ++n;
        };
        for (int i = 0; i < 2; ++i) {
            float tc = start + (float)p * b + ((float)i + 0.5f) * b * 0.5f - 0.5f;
            if (tc < -1.f || tc > (float)L) continue;
            tc = fminf(fmaxf(tc, 0.f), (float)(L - 1));
            const int i0 = (int)floorf(tc), i1 = i0 + 1 < L ? i0 + 1 : L - 1;
            const float l = tc - (float)i0;
            add(i0, 1.f - l);
            add(i1, l);
        }
        ax_n[lst] = n;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < ROI_TAPS * nb; e += blockDim.x) {
        const int bin = e / ROI_TAPS, k = e - bin * ROI_TAPS, ph = bin / P, pw = bin - ph * P;
        const int ny = ax_n[ph], nx = ax_n[P + pw], nt = ny * nx;
        int off = 0;
        float w = 0.f;
        if (k < nt) {
            const int ia = k / nx, ib = k - ia * nx;
            off = ax_i[4 * ph + ia] * Wk + ax_i[4 * (P + pw) + ib];
            w = ax_w[4 * ph + ia] * ax_w[4 * (P + pw) + ib] * 0.25f;
        }
        s_off[e] = off;
        s_w[e] = w;
        if (k == 0) s_nt[bin] = nt;
    }
    __syncthreads();
    const T* fm = feat + (size_t)f * Hk * Wk * Ch;
    T* o = out + (size_t)roi * nb * Ch;
    // one work item = one bin x one 16-byte run of channels; consecutive threads take consecutive runs
    constexpr int VEC = 16 / (int)sizeof(T);
    const int runs = Ch / VEC;
    for (int i = threadIdx.x; i < nb * runs; i += blockDim.x) {
        const int bin = i / runs, c = (i - bin * runs) * VEC;
        const int nt = s_nt[bin];
        const int* toff = s_off + ROI_TAPS * bin;
        const float* tw = s_w + ROI_TAPS * bin;
        float sum[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) sum[e] = 0.f;
        auto gather = [&](auto nc) {
            constexpr int N = decltype(nc)::value;
            uint4 raw[N];
#pragma unroll
            for (int k = 0; k < N; ++k) raw[k] = *reinterpret_cast<const uint4*>(fm + (size_t)toff[k] * Ch + c);
#pragma unroll
            for (int k = 0; k < N; ++k) {
                const float w = tw[k];
                if constexpr (sizeof(T) == 2) {
                    const uint32_t wd[4] = {raw[k].x, raw[k].y, raw[k].z, raw[k].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        sum[2 * e] += w * __uint_as_float(wd[e] << 16);
                        sum[2 * e + 1] += w * __uint_as_float(wd[e] & 0xffff0000u);
                    }
                } else {
                    sum[0] += w * __uint_as_float(raw[k].x); sum[1] += w * __uint_as_float(raw[k].y);
                    sum[2] += w * __uint_as_float(raw[k].z); sum[3] += w * __uint_as_float(raw[k].w);
                }
            }
        };
        if (nt <= 4) gather(std::integral_constant<int, 4>{});
        else if (nt <= 6) gather(std::integral_constant<int, 6>{});
        else if (nt <= 9) gather(std::integral_constant<int, 9>{});
        else if (nt <= 12) gather(std::integral_constant<int, 12>{});
        else gather(std::integral_constant<int, 16>{});
        uint4 pk;
        if constexpr (sizeof(T) == 2) {
            pk = make_uint4(pack_bf16x2(sum[0], sum[1]), pack_bf16x2(sum[2], sum[3]), pack_bf16x2(sum[4], sum[5]),
                            pack_bf16x2(sum[6], sum[7]));
        } else {
            pk = make_uint4(__float_as_uint(sum[0]), __float_as_uint(sum[1]), __float_as_uint(sum[2]), __float_as_uint(sum[3]));
        }
        *reinterpret_cast<uint4*>(o + (size_t)bin * Ch + c) = pk;
    }
}

hipError_t launch_roialign(const void* feat, const float* rois, int n, int post, int Hk, int Wk, int Ch, int stride, int P,
                           int precision, void* out, hipStream_t s) {
    if (n <= 0 || post <= 0 || P <= 0 || P > 16 || Ch % 8) return hipErrorInvalidValue;
    const size_t lds = roialign_lds_bytes(P);
    const float scale = 1.0f / (float)stride;
    const unsigned blocks = (unsigned)n * (unsigned)post;
    if (precision)
        hipLaunchKernelGGL(roialign_kernel<bf16_t>, dim3(blocks), dim3(256), lds, s, static_cast<const bf16_t*>(feat), rois, post,
                           Hk, Wk, Ch, scale, P, static_cast<bf16_t*>(out));
    else
        hipLaunchKernelGGL(roialign_kernel<float>, dim3(blocks), dim3(256), lds, s, static_cast<const float*>(feat), rois, post, Hk,
                           Wk, Ch, scale, P, static_cast<float*>(out));
    return hipGetLastError();
}

// ------------------------------------------------------------------ scores + per-class boxes
// One thread per ROI: softmax over Kc logits (max subtracted) and, for every foreground
// class, the ROI decoded with that class's deltas and clipped.
__global__ void scores_boxes_kernel(const float* __restrict__ cls, const float* __restrict__ deltas,
                                    const float* __restrict__ rois, int total, int Kc, float imgW, float imgH,
                                    float* __restrict__ scores, float* __restrict__ boxes) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= total) return;
    const float* x = cls + (size_t)r * Kc;
    float mx = x[0];
    for (int c = 1; c < Kc; ++c) mx = fmaxf(mx, x[c]);
    float sum = 0.f;
    for (int c = 0; c < Kc; ++c) sum += expf(x[c] - mx);
    const float4 q = *reinterpret_cast<const float4*>(rois + 4 * (size_t)r);
    const float rw = q.z - q.x, rh = q.w - q.y;
    const float cx = q.x + 0.5f * rw, cy = q.y + 0.5f * rh;
    for (int c = 0; c < Kc; ++c) {
        scores[(size_t)r * Kc + c] = expf(x[c] - mx) / sum;
        Box b = {0.f, 0.f, 0.f, 0.f};
        if (c > 0) {
            const float4 d = *reinterpret_cast<const float4*>(deltas + ((size_t)r * Kc + c) * 4);
            decode_box(cx, cy, rw, rh, d.x, d.y, d.z, d.w, imgW, imgH, b);
        }
        *reinterpret_cast<float4*>(boxes + ((size_t)r * Kc + c) * 4) = make_float4(b.x1, b.y1, b.x2, b.y2);
    }
}

hipError_t launch_scores_boxes(const float* cls, const float* deltas, const float* rois, int n, int post, int Kc, float imgW,
                               float imgH, float* scores, float* boxes, hipStream_t s) {
    const int total = n * post;
    if (total <= 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(scores_boxes_kernel, dim3((total + 127) / 128), dim3(128), 0, s, cls, deltas, rois, total, Kc, imgW, imgH,
                       scores, boxes);
    return hipGetLastError();
}

// ------------------------------------------------------------------ detection selection
// One block per frame.  Candidates (roi < roi_n, class >= 1, score > thr, non-empty box)
// get the key (order-preserving score) << 32 | (2^32 - 1 - (roi*Kc + class)); the keys are
// sorted descending (LDS when they fit, else in the global scratch), then wavefront 0
// runs greedy same-class NMS 64 candidates at a time against the list of kept boxes.
constexpr int SEL_LDS_KEYS = 4096;
constexpr int SEL_MAX_D = 512;

__global__ __launch_bounds__(1024) void select_kernel(const float* __restrict__ scores, const float* __restrict__ boxes,
                                                      const int32_t* __restrict__ roi_n, int post, int Kc, float score_thr,
                                                      float nms_thr, int D, uint64_t* __restrict__ gkeys, int key_cap,
                                                      float* __restrict__ out_boxes, float* __restrict__ out_scores,
                                                      int32_t* __restrict__ out_labels, int32_t* __restrict__ out_n) {
    __shared__ uint64_t lkeys[SEL_LDS_KEYS];
    __shared__ Box kbox[SEL_MAX_D];
    __shared__ int klab[SEL_MAX_D];
    __shared__ float kscore[SEL_MAX_D];
    __shared__ int s_count, s_nk;
    const int f = blockIdx.x, t = threadIdx.x;
    int nr = roi_n[f];
    nr = nr < post ? nr : post;
    const float* sc = scores + (size_t)f * post * Kc;
    const float* bx = boxes + (size_t)f * post * Kc * 4;
    uint64_t* gk = gkeys + (size_t)f * key_cap;
    if (t == 0) { s_count = 0; s_nk = 0; }
    __syncthreads();
    const int total = nr * Kc;
    for (int j = t; j < total; j += 1024) {
        const int c = j % Kc;
        if (c == 0) continue;
        const float s = sc[j];
        if (!(s > score_thr)) continue;
        const float4 b = *reinterpret_cast<const float4*>(bx + 4 * (size_t)j);
        if (!((b.z - b.x >= 1e-3f) && (b.w - b.y >= 1e-3f))) continue;
        const int slot = atomicAdd(&s_count, 1);
        gk[slot] = ((uint64_t)score_key(s) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)j);
    }
    __syncthreads();
    const int nc = s_count;
    int n2 = 1;
    while (n2 < nc) n2 <<= 1;
    uint64_t* keys;
    if (n2 <= SEL_LDS_KEYS) {
        for (int i = t; i < n2; i += 1024) lkeys[i] = i < nc ? gk[i] : 0ull;
        keys = lkeys;
    } else {
        for (int i = nc + t; i < n2; i += 1024) gk[i] = 0ull;
        keys = gk;
    }
    __syncthreads();
    bitonic_sort_desc(keys, n2);

    if (t < 64) {
        const int lane = t;
        int nk = 0;
        for (int s0 = 0; s0 < nc && nk < D; s0 += 64) {
            const int i = s0 + lane;
            bool alive = i < nc;
            Box me = {0.f, 0.f, 0.f, 0.f};
            int lab = -1;
            float myscore = 0.f;
            if (alive) {
                const uint64_t key = keys[i];
                const uint32_t j = 0xFFFFFFFFu - (uint32_t)(key & 0xFFFFFFFFull);
                const float4 b = *reinterpret_cast<const float4*>(bx + 4 * (size_t)j);
                me = {b.x, b.y, b.z, b.w};
                lab = (int)(j % (uint32_t)Kc);
                myscore = key_score((uint32_t)(key >> 32));
                for (int q = 0; q < nk; ++q)
                    if (klab[q] == lab && iou_over(kbox[q], me, nms_thr)) { alive = false; break; }
            }
            for (int b = 0; b < 64 && nk < D; ++b) {
                const int ab = __shfl((int)alive, b);
                if (!ab) continue;
                const Box kb = {__shfl(me.x1, b), __shfl(me.y1, b), __shfl(me.x2, b), __shfl(me.y2, b)};
                const int kl = __shfl(lab, b);
                const float ks = __shfl(myscore, b);
                if (lane == 0) { kbox[nk] = kb; klab[nk] = kl; kscore[nk] = ks; }
                ++nk;
                if (lane > b && alive && lab == kl && iou_over(kb, me, nms_thr)) alive = false;
            }
            __builtin_amdgcn_wave_barrier();
            __threadfence_block();
        }
        if (lane == 0) s_nk = nk;
    }
    __syncthreads();
    const int nk = s_nk;
    for (int d = t; d < D; d += 1024) {
        float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
        float s = 0.f;
        int l = -1;
        if (d < nk) { b = make_float4(kbox[d].x1, kbox[d].y1, kbox[d].x2, kbox[d].y2); s = kscore[d]; l = klab[d]; }
        *reinterpret_cast<float4*>(out_boxes + ((size_t)f * D + d) * 4) = b;
        out_scores[(size_t)f * D + d] = s;
        out_labels[(size_t)f * D + d] = l;
    }
    if (t == 0 && out_n) out_n[f] = nk;
}

// Same selection with one wavefront per foreground class (post <= 512, Kc - 1 <= 16, D <= 128).  Same-class NMS
// never looks across classes and the global walk stops after D kept boxes, so the result equals: per class, greedy
// NMS over that class's candidates in key order, cut after its first D kept; then the D largest keys among all
// kept.  Every wavefront gathers and sorts its class's candidates in LDS (wave-level barriers only), resolves 64
// candidates at a time (overlap bits against the earlier candidates of the group, then a register-only greedy
// chain), and the block finally ranks the <= (Kc - 1) * D kept keys by counting.
constexpr int SELC_MAX_POST = 512, SELC_MAX_CLASSES = 16, SELC_MAX_D = 128;

__global__ __launch_bounds__(1024) void select_classes_kernel(const float* __restrict__ scores, const float* __restrict__ boxes,
                                                              const int32_t* __restrict__ roi_n, int post, int Kc,
                                                              float score_thr, float nms_thr, int D,
                                                              float* __restrict__ out_boxes, float* __restrict__ out_scores,
                                                              int32_t* __restrict__ out_labels, int32_t* __restrict__ out_n) {
    extern __shared__ __align__(16) unsigned char sel_smem[];
    const int NC = Kc - 1;
    Box* gbox = reinterpret_cast<Box*>(sel_smem);                        // [NC][64] boxes of the group being resolved
    Box* kbox = gbox + (size_t)NC * 64;                                  // [NC][D] kept boxes (16-byte aligned: read as float4)
    uint64_t* keys = reinterpret_cast<uint64_t*>(kbox + (size_t)NC * D); // [NC][SELC_MAX_POST]
    uint64_t* kkey = keys + (size_t)NC * SELC_MAX_POST;                  // [NC][D]
    int* kcount = reinterpret_cast<int*>(kkey + (size_t)NC * D);         // [NC]
    const int f = blockIdx.x, t = threadIdx.x, lane = t & 63, wv = t >> 6;
    int nr = roi_n[f];
    nr = nr < post ? nr : post;
    const float* sc = scores + (size_t)f * post * Kc;
    const float* bx = boxes + (size_t)f * post * Kc * 4;

    if (wv < NC) {
        const int c = wv;                       // label c + 1
        uint64_t* ck = keys + (size_t)c * SELC_MAX_POST;
        // candidates of the class, packed to the front of the list in ROI order
        int nc = 0;
        for (int r0 = 0; r0 < nr; r0 += 64) {
            const int roi = r0 + lane;
            uint64_t key = 0ull;
            if (roi < nr) {
                const int j = roi * Kc + c + 1;
                const float s = sc[j];
                if (s > score_thr) {
                    const float4 b = *reinterpret_cast<const float4*>(bx + 4 * (size_t)j);
                    if ((b.z - b.x >= 1e-3f) && (b.w - b.y >= 1e-3f)) key = ((uint64_t)score_key(s) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)j);
                }
            }
            const uint64_t has = __ballot(key != 0ull);
            if (key != 0ull) ck[nc + __popcll(has & ((1ull << lane) - 1ull))] = key;
            nc += __popcll(has);
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_wave_barrier();
        // Sorted descending by counting: keys are unique, so a key's place is the number of larger keys.  Every lane holds up
        // to SELC_MAX_POST / 64 keys in registers and walks the list once (all lanes read the same entry: a broadcast);
        // ~15 000 cycles for 300 candidates against ~57 000 for a 512-key bitonic network run by one wavefront.
        {
            constexpr int QMAX = SELC_MAX_POST / 64;
            uint64_t mine[QMAX];
            int rank[QMAX];
#pragma unroll
            for (int q = 0; q < QMAX; ++q) {
                mine[q] = (lane + 64 * q < nc) ? ck[lane + 64 * q] : ~0ull;   // (absent slots compare as "nothing is larger")
                rank[q] = 0;
            }
            auto count = [&](auto qc) {
                constexpr int QN = decltype(qc)::value;
#pragma unroll 4
                for (int k = 0; k < nc; ++k) {
                    const uint64_t o = ck[k];
#pragma unroll
                    for (int q = 0; q < QN; ++q) rank[q] += (o > mine[q]) ? 1 : 0;
                }
            };
            if (nc <= 128) count(std::integral_constant<int, 2>{});
            else if (nc <= 256) count(std::integral_constant<int, 4>{});
            else count(std::integral_constant<int, QMAX>{});
            __builtin_amdgcn_s_waitcnt(0xc07f);   // every lane has read the whole list
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int q = 0; q < QMAX; ++q)
                if (lane + 64 * q < nc) ck[rank[q]] = mine[q];
            __builtin_amdgcn_s_waitcnt(0xc07f);
            __builtin_amdgcn_wave_barrier();
        }
        int nk = 0;
        for (int s0 = 0; s0 < nc && nk < D; s0 += 64) {
            const int i = s0 + lane;
            bool alive = i < nc;
            Box me = {0.f, 0.f, 0.f, 0.f};
            uint64_t key = 0ull;
            if (alive) {
                key = ck[i];
                const uint32_t j = 0xFFFFFFFFu - (uint32_t)(key & 0xFFFFFFFFull);
                const float4 b = *reinterpret_cast<const float4*>(bx + 4 * (size_t)j);
                me = {b.x, b.y, b.z, b.w};
            }
            {   // against the boxes this class has kept so far: four at a time, no early exit (the loads pipeline)
                bool hit = false;
                const Box* kb = kbox + (size_t)c * D;
                int q = 0;
                auto ld = [&](int k) { const float4 v = *reinterpret_cast<const float4*>(kb + k); return Box{v.x, v.y, v.z, v.w}; };
                for (; q + 4 <= nk; q += 4) {
                    const Box b0 = ld(q), b1 = ld(q + 1), b2 = ld(q + 2), b3 = ld(q + 3);
                    const int h = (int)iou_over(b0, me, nms_thr) | (int)iou_over(b1, me, nms_thr) | (int)iou_over(b2, me, nms_thr) | (int)iou_over(b3, me, nms_thr);
                    hit = hit || h != 0;
                }
                for (; q < nk; ++q) hit = hit || iou_over(ld(q), me, nms_thr);
                alive = alive && !hit;
            }
            // column b of the group's overlap matrix (which later candidates candidate b suppresses), held by lane b.
            // Every lane walks the group's boxes in LDS (all lanes read the same address: a broadcast) and tests its own
            // box against them; broadcasting box b through scalar registers and collecting a ballot per b instead made
            // each of the 64 steps a chain of dependent scalar and vector instructions.
            uint64_t col = 0ull;
            const int live = (nc - s0) < 64 ? (nc - s0) : 64;   // candidates in this group
            Box* gb = gbox + (size_t)c * 64;
            gb[lane] = me;
            __builtin_amdgcn_s_waitcnt(0xc07f);
            __builtin_amdgcn_wave_barrier();
            if (i < nc) {
                // four boxes per step, loaded together and tested independently (slots past `live` hold zero boxes: no overlap)
                uint32_t word[2] = {0u, 0u};
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    if (32 * h >= live) break;   // uniform
                    uint32_t w = 0u;
#pragma unroll 2
                    for (int j0 = 0; j0 < 32; j0 += 4) {
                        float4 q[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) q[u] = *reinterpret_cast<const float4*>(gb + 32 * h + j0 + u);
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const int j = 32 * h + j0 + u;
                            const Box o = {q[u].x, q[u].y, q[u].z, q[u].w};
                            w |= (j > lane && iou_over(me, o, nms_thr)) ? (1u << (j0 + u)) : 0u;
                        }
                    }
                    word[h] = w;
                }
                col = (uint64_t)word[0] | ((uint64_t)word[1] << 32);
            }
            uint64_t dead = ~__ballot(alive);
            uint64_t kept = 0ull;
            const uint32_t clo = (uint32_t)col, chi = (uint32_t)(col >> 32);
            for (uint64_t avail = ~dead; avail != 0ull;) {   // from one kept candidate to the next: suppressed ones are not visited
                const int b = __builtin_ctzll(avail);
                kept |= 1ull << b;
                const uint64_t d = (uint64_t)(uint32_t)__builtin_amdgcn_readlane(clo, b) | ((uint64_t)(uint32_t)__builtin_amdgcn_readlane(chi, b) << 32);
                avail &= ~d & ~((2ull << b) - 1ull);
            }
            if ((kept >> lane) & 1ull) {
                const int pos = nk + __popcll(kept & ((1ull << lane) - 1ull));
                if (pos < D) { kbox[(size_t)c * D + pos] = me; kkey[(size_t)c * D + pos] = key; }
            }
            nk += __popcll(kept);
            nk = nk < D ? nk : D;
            __builtin_amdgcn_s_waitcnt(0xc07f);
            __builtin_amdgcn_wave_barrier();
        }
        if (lane == 0) kcount[c] = nk;
    }
    __syncthreads();
    // rank of every kept key among all kept keys (each class list is sorted descending: binary search per class)
    int total = 0;
    for (int c = 0; c < NC; ++c) total += kcount[c];
    const int nk_out = total < D ? total : D;
    for (int e = t; e < NC * D; e += 1024) {
        const int c = e / D, q = e - c * D;
        if (q >= kcount[c]) continue;
        const uint64_t key = kkey[(size_t)c * D + q];
        int rank = 0;
        for (int c2 = 0; c2 < NC; ++c2) {
            const uint64_t* l = kkey + (size_t)c2 * D;
            int lo = 0, hi = kcount[c2];          // first position whose key is <= key
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (l[mid] > key) lo = mid + 1; else hi = mid;
            }
            rank += lo;
        }
        if (rank < D) {
            const Box b = kbox[(size_t)c * D + q];
            *reinterpret_cast<float4*>(out_boxes + ((size_t)f * D + rank) * 4) = make_float4(b.x1, b.y1, b.x2, b.y2);
            out_scores[(size_t)f * D + rank] = key_score((uint32_t)(key >> 32));
            out_labels[(size_t)f * D + rank] = c + 1;
        }
    }
    for (int d = nk_out + t; d < D; d += 1024) {
        *reinterpret_cast<float4*>(out_boxes + ((size_t)f * D + d) * 4) = make_float4(0.f, 0.f, 0.f, 0.f);
        out_scores[(size_t)f * D + d] = 0.f;
        out_labels[(size_t)f * D + d] = -1;
    }
    if (t == 0 && out_n) out_n[f] = nk_out;
}

hipError_t launch_select(const float* scores, const float* boxes, const int32_t* roi_n, int n, int post, int Kc,
                         float score_thr, float nms_thr, int D, uint64_t* keys, int key_cap, float* out_boxes,
                         float* out_scores, int32_t* out_labels, int32_t* out_n, hipStream_t s) {
    if (n <= 0 || D <= 0 || D > SEL_MAX_D || key_cap < post * Kc) return hipErrorInvalidValue;
    if (post <= SELC_MAX_POST && Kc >= 2 && Kc - 1 <= SELC_MAX_CLASSES && D <= SELC_MAX_D) {
        const int NC = Kc - 1;
        const size_t lds = (size_t)NC * 64 * sizeof(Box) + (size_t)NC * SELC_MAX_POST * 8 + (size_t)NC * D * (8 + sizeof(Box)) + (size_t)NC * 4;
        {
            const size_t lds_max = (size_t)SELC_MAX_CLASSES * 64 * sizeof(Box) + (size_t)SELC_MAX_CLASSES * SELC_MAX_POST * 8 +
                                   (size_t)SELC_MAX_CLASSES * SELC_MAX_D * (8 + sizeof(Box)) + (size_t)SELC_MAX_CLASSES * 4;
            hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(select_classes_kernel), lds_max);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(select_classes_kernel, dim3(n), dim3(1024), lds, s, scores, boxes, roi_n, post, Kc, score_thr, nms_thr, D,
                           out_boxes, out_scores, out_labels, out_n);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(select_kernel, dim3(n), dim3(1024), 0, s, scores, boxes, roi_n, post, Kc, score_thr, nms_thr, D, keys,
                       key_cap, out_boxes, out_scores, out_labels, out_n);
    return hipGetLastError();
}

__global__ void fill_empty_kernel(int total, float* __restrict__ out_boxes, float* __restrict__ out_scores,
                                  int32_t* __restrict__ out_labels) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    *reinterpret_cast<float4*>(out_boxes + 4 * (size_t)i) = make_float4(0.f, 0.f, 0.f, 0.f);
    out_scores[i] = 0.f;
    out_labels[i] = -1;
}

hipError_t launch_fill_empty(int n, int D, float* out_boxes, float* out_scores, int32_t* out_labels, hipStream_t s) {
    const int total = n * D;
    if (total <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_empty_kernel, dim3((total + 255) / 256), dim3(256), 0, s, total, out_boxes, out_scores, out_labels);
    return hipGetLastError();
}

}  // namespace thia
