// Device helpers shared by the proposal and ROI kernels: order-preserving score keys,
// a block-wide bitonic sort, box decoding and the NMS overlap test.  All geometry is
// plain fp32 with singly rounded operations (the library is built with
// -ffp-contract=off), so that orderings and keep decisions are reproducible.
#pragma once
#include "thia_internal.h"

namespace thia {

// Monotone map float -> uint32 (larger float = larger key); -0 and +0 map to the same key.
__device__ inline uint32_t score_key(float s) {
    const uint32_t b = __float_as_uint(s + 0.0f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ inline float key_score(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// n2 (a power of two) keys in LDS, sorted descending by the whole block (a multiple of 64 threads).  A thread owns
// compare-exchange pair q of a stage: lower element ((q & ~(j-1)) << 1) | (q & (j-1)), partner = lower | j.  The 64 pairs
// of one wavefront iteration lie within one aligned block of 128 elements for every distance j <= 64, so between two such
// stages only the wavefront's own LDS traffic has to be ordered; the block barrier is kept around the stages with j >= 128
// (10 of the 66 stages at 2048 keys) and after the last one.
__device__ inline void bitonic_sort_desc_lds(uint64_t* keys, int n2) {
    const int pairs = n2 >> 1, nt = blockDim.x;
    for (int k = 2; k <= n2; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int q = threadIdx.x; q < pairs; q += nt) {
                const int i = ((q & ~(j - 1)) << 1) | (q & (j - 1)), p = i | j;
                const uint64_t a = keys[i], b = keys[p];
                const bool desc = (i & k) == 0;
                if (desc ? (a < b) : (a > b)) { keys[i] = b; keys[p] = a; }
            }
            const int jn = j > 1 ? (j >> 1) : k;   // distance of the stage that follows (k: first stage of the next merge)
            if (j >= 128 || jn >= 128 || (j == 1 && k == n2)) {
                __syncthreads();
            } else {
                __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
                __builtin_amdgcn_wave_barrier();
                asm volatile("" ::: "memory");
            }
        }
}

// The same network with a block barrier after every stage: keys may live in LDS or in global memory.
__device__ inline void bitonic_sort_desc(uint64_t* keys, int n2) {
    for (int k = 2; k <= n2; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = threadIdx.x; i < n2; i += blockDim.x) {
                const int p = i ^ j;
                if (p > i) {
                    const uint64_t a = keys[i], b = keys[p];
                    const bool desc = (i & k) == 0;
                    if (desc ? (a < b) : (a > b)) { keys[i] = b; keys[p] = a; }
                }
            }
            __syncthreads();
        }
}

struct Box { float x1, y1, x2, y2; };

// Decoding of (dx,dy,dw,dh) against a reference box given as centre/size, unit weights,
// dw/dh clamped at ln(1000/16), corners clipped to the frame.  Returns false for boxes
// narrower or lower than 1e-3 px after clipping.
__device__ inline bool decode_box(float cx, float cy, float w, float h, float dx, float dy, float dw, float dh, float imgW,
                                  float imgH, Box& o) {
    const float clampv = 4.135166556742356f;
    dw = dw < clampv ? dw : clampv;
    dh = dh < clampv ? dh : clampv;
    const float ncx = cx + dx * w, ncy = cy + dy * h;
    const float nw = w * expf(dw), nh = h * expf(dh);
    const float hw = 0.5f * nw, hh = 0.5f * nh;
    o.x1 = fminf(fmaxf(ncx - hw, 0.f), imgW);
    o.y1 = fminf(fmaxf(ncy - hh, 0.f), imgH);
    o.x2 = fminf(fmaxf(ncx + hw, 0.f), imgW);
    o.y2 = fminf(fmaxf(ncy + hh, 0.f), imgH);
    return (o.x2 - o.x1 >= 1e-3f) && (o.y2 - o.y1 >= 1e-3f);
}

// Division-free overlap test: IoU(a, b) > thr  <=>  union > 0 and inter > thr * union.
__device__ inline bool iou_over(const Box& a, const Box& b, float thr) {
    float iw = fminf(a.x2, b.x2) - fmaxf(a.x1, b.x1);
    float ih = fminf(a.y2, b.y2) - fmaxf(a.y1, b.y1);
    iw = fmaxf(iw, 0.f);
    ih = fmaxf(ih, 0.f);
    const float inter = iw * ih;
    const float aa = (a.x2 - a.x1) * (a.y2 - a.y1);
    const float ab = (b.x2 - b.x1) * (b.y2 - b.y1);
    const float uni = (aa + ab) - inter;
    const float t = thr * uni;
    return uni > 0.f && inter > t;
}

}  // namespace thia
