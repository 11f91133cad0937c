// Image classifier with exits: the paper's generalisation of early inference to a VGG-16-style network (Sec. 4.2,
// "Generalization").  A stack of 3x3 convolutions (+ ReLU) with 2x2 max-pools in between; exit k taps the output of one
// convolution layer and owns a classifier unit: global average pooling, one fully connected layer, soft-max, arg-max.
// Inference stops at the chosen exit: layers behind the tapped one are never launched.
//
// The convolutions run on the library's implicit-GEMM matrix-core kernel (launch_conv); the first layer's three input
// channels are zero-padded to one K tile by the kernel that normalises the frames and lays them out as NHWC.  The pooled
// means are formed as per-slab partial sums that the unit's kernel adds in a fixed order (no floating-point atomics: the
// result does not depend on scheduling).
#include <algorithm>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "thia_internal.h"

using namespace thia;

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int32_t kClsMagic = 0x43494854;
constexpr int kMaxLayers = 16, kMaxExits = 8, kSlabs = 64;

// frames u8 [n,3,H,W] -> x [n,H,W,CP] with x[.., c] = (u8 - mean) / std for c < 3 and 0 above; one thread per 16-byte chunk.
template <bool BF16>
__global__ void pack_frames_kernel(const uint8_t* __restrict__ frames, size_t pixels, int HW, int CP, float mean, float stdv,
                                   void* __restrict__ out_) {
    constexpr int EPC = BF16 ? 8 : 4;
    const int chunks = CP / EPC;
    const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= pixels * chunks) return;
    const int ck = (int)(gid % chunks);
    const size_t px = gid / chunks;
    float v[3] = {0.f, 0.f, 0.f};
    if (ck == 0) {
        const size_t img = px / HW, p = px - img * HW;
        for (int c = 0; c < 3; ++c) v[c] = ((float)frames[(img * 3 + c) * HW + p] - mean) / stdv;
    }
    if (BF16) {
        const u32x4_t o = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], 0.f), 0u, 0u};
        *reinterpret_cast<u32x4_t*>(static_cast<bf16_t*>(out_) + px * CP + (size_t)ck * EPC) = o;
    } else {
        const f32x4_t o = {v[0], v[1], v[2], 0.f};
        *reinterpret_cast<f32x4_t*>(static_cast<float*>(out_) + px * CP + (size_t)ck * EPC) = o;
    }
}

// 2x2 / stride 2 max-pool without padding (a trailing odd row / column is dropped), NHWC; one thread per 16-byte chunk.
template <bool BF16>
__global__ void maxpool2x2_kernel(const void* __restrict__ in_, int n, int H, int W, int C, void* __restrict__ out_) {
    constexpr int EPC = BF16 ? 8 : 4;
    const int Ho = H / 2, Wo = W / 2, chunks = C / EPC;
    const size_t total = (size_t)n * Ho * Wo * chunks;
    const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const int ck = (int)(gid % chunks);
    size_t r = gid / chunks;
    const int ox = (int)(r % Wo); r /= Wo;
    const int oy = (int)(r % Ho);
    const int img = (int)(r / Ho);
    float best[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) best[q] = -INFINITY;
    for (int ky = 0; ky < 2; ++ky)
        for (int kx = 0; kx < 2; ++kx) {
            const size_t off = (((size_t)img * H + 2 * oy + ky) * W + 2 * ox + kx) * C + (size_t)ck * EPC;
            if (BF16) {
                const u32x4_t v = *reinterpret_cast<const u32x4_t*>(static_cast<const bf16_t*>(in_) + off);
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    best[2 * q] = fmaxf(best[2 * q], __uint_as_float(w[q] << 16));
                    best[2 * q + 1] = fmaxf(best[2 * q + 1], __uint_as_float(w[q] & 0xffff0000u));
                }
            } else {
                const f32x4_t v = *reinterpret_cast<const f32x4_t*>(static_cast<const float*>(in_) + off);
                best[0] = fmaxf(best[0], v.x); best[1] = fmaxf(best[1], v.y); best[2] = fmaxf(best[2], v.z); best[3] = fmaxf(best[3], v.w);
            }
        }
    const size_t o = (((size_t)img * Ho + oy) * Wo + ox) * C + (size_t)ck * EPC;
    if (BF16) {
        // the maximum of bf16 values is one of them: the conversion back is exact
        const u32x4_t ov = {pack_bf16x2(best[0], best[1]), pack_bf16x2(best[2], best[3]), pack_bf16x2(best[4], best[5]), pack_bf16x2(best[6], best[7])};
        *reinterpret_cast<u32x4_t*>(static_cast<bf16_t*>(out_) + o) = ov;
    } else {
        const f32x4_t ov = {best[0], best[1], best[2], best[3]};
        *reinterpret_cast<f32x4_t*>(static_cast<float*>(out_) + o) = ov;
    }
}

// Partial sums over the positions of an NHWC map: slab s of frame f covers positions [s * per, (s + 1) * per); the block's
// 256 threads are laid out as (position group, channel) and the groups are added in order through LDS.
// feat [n][HW][C] -> partial [n][kSlabs][C] (fp32).  C <= 1024.
template <typename T>
__global__ __launch_bounds__(256) void mean_partial_kernel(const T* __restrict__ feat, int HW, int C, float* __restrict__ partial) {
    __shared__ float red[256];
    const int s = blockIdx.x, f = blockIdx.y, t = threadIdx.x;
    const int lanes = C < 256 ? C : 256;          // channels handled side by side (C is a multiple of 32)
    const int groups = 256 / lanes;               // position groups
    const int g = t / lanes, l = t - g * lanes;
    const int per = (HW + kSlabs - 1) / kSlabs;
    const int p0 = s * per, p1 = (p0 + per < HW) ? p0 + per : HW;
    for (int c0 = 0; c0 < C; c0 += lanes) {
        float acc = 0.f;
        if (g < groups && c0 + l < C) {
            const T* p = feat + (size_t)f * HW * C + c0 + l;
            for (int i = p0 + g; i < p1; i += groups) {
                if constexpr (sizeof(T) == 2) acc += bf16_to_f32(p[(size_t)i * C]);
                else acc += p[(size_t)i * C];
            }
        }
        red[t] = acc;
        __syncthreads();
        if (g == 0 && c0 + l < C) {
            float sum = 0.f;
            for (int q = 0; q < groups; ++q) sum += red[q * lanes + l];
            partial[((size_t)f * kSlabs + s) * C + c0 + l] = sum;
        }
        __syncthreads();
    }
}

// The classifier unit on one frame per block: g = (sum of the slab sums) / HW, logits = V g + c, soft-max, arg-max (the
// lowest class on a tie).  V [classes][C] fp32.  LDS: C + classes floats.
__global__ __launch_bounds__(256) void classifier_head_kernel(const float* __restrict__ partial, int HW, int C, int classes,
                                                              const float* __restrict__ V, const float* __restrict__ cb,
                                                              int32_t* __restrict__ labels, float* __restrict__ conf,
                                                              float* __restrict__ logits_out) {
    extern __shared__ float sm[];
    float *sg = sm, *sl = sm + C;
    const int f = blockIdx.x, t = threadIdx.x;
    for (int c = t; c < C; c += 256) {
        float sum = 0.f;
        for (int s = 0; s < kSlabs; ++s) sum += partial[((size_t)f * kSlabs + s) * C + c];
        sg[c] = sum / (float)HW;
    }
    __syncthreads();
    for (int k = t; k < classes; k += 256) {
        float acc = cb[k];
        const float* v = V + (size_t)k * C;
        for (int c = 0; c < C; ++c) acc += v[c] * sg[c];
        sl[k] = acc;
        if (logits_out) logits_out[(size_t)f * classes + k] = acc;
    }
    __syncthreads();
    if (t == 0) {
        int best = 0;
        for (int k = 1; k < classes; ++k)
            if (sl[k] > sl[best]) best = k;
        float den = 0.f;
        for (int k = 0; k < classes; ++k) den += expf(sl[k] - sl[best]);
        labels[f] = best;
        conf[f] = 1.f / den;
    }
}

__global__ void fill_skipped_kernel(int n, int32_t* __restrict__ labels, float* __restrict__ conf) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { labels[i] = -1; conf[i] = 0.f; }
}

struct ConvLayer {
    void* w = nullptr;
    float* b = nullptr;
    int co = 0, ci = 0;   // ci: input channels as the kernel sees them (padded for the first layer)
};

}  // namespace

struct thia_classifier {
    int precision = 0, n_exits = 0, n_layers = 0, in_ch = 3, n_classes = 0, cin_pad = 64;
    float mean = 0.f, stdv = 1.f;
    int channels[kMaxLayers] = {}, pool[kMaxLayers] = {}, taps[kMaxExits] = {};
    size_t esz = 4;
    ConvLayer conv[kMaxLayers];
    float* fcw[kMaxExits] = {};
    float* fcb[kMaxExits] = {};
    hipStream_t stream = nullptr;
    void* act[2] = {nullptr, nullptr};
    size_t act_cap = 0;
    float* partial = nullptr;
    size_t partial_cap = 0;
    std::string err;
};

namespace {

int cfail(thia_classifier* c, int code, const std::string& msg) {
    if (c) c->err = msg;
    return code;
}

int ensure_buffers(thia_classifier* c, size_t act_bytes, size_t partial_floats) {
    if (act_bytes > c->act_cap) {
        if (hipStreamSynchronize(c->stream) != hipSuccess) return cfail(c, THIA_E_HIP, "stream synchronisation failed");
        for (void*& p : c->act) { (void)hipFree(p); p = nullptr; }
        c->act_cap = 0;
        for (void*& p : c->act)
            if (hipMalloc(&p, act_bytes) != hipSuccess) return cfail(c, THIA_E_NOMEM, "activation buffers: allocation failed");
        c->act_cap = act_bytes;
    }
    if (partial_floats > c->partial_cap) {
        if (hipStreamSynchronize(c->stream) != hipSuccess) return cfail(c, THIA_E_HIP, "stream synchronisation failed");
        (void)hipFree(c->partial);
        c->partial = nullptr; c->partial_cap = 0;
        if (hipMalloc(reinterpret_cast<void**>(&c->partial), partial_floats * 4) != hipSuccess) return cfail(c, THIA_E_NOMEM, "pooling buffer: allocation failed");
        c->partial_cap = partial_floats;
    }
    return THIA_OK;
}

hipError_t launch_pool2x2(const void* in, int n, int H, int W, int C, int precision, void* out, hipStream_t s) {
    const int epc = precision ? 8 : 4;
    const size_t total = (size_t)n * (H / 2) * (W / 2) * (C / epc);
    if (total == 0) return hipSuccess;
    const size_t blocks = (total + 255) / 256;
    if (blocks >= (1ull << 31)) return hipErrorInvalidValue;
    if (precision) hipLaunchKernelGGL(maxpool2x2_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, in, n, H, W, C, out);
    else hipLaunchKernelGGL(maxpool2x2_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, in, n, H, W, C, out);
    return hipGetLastError();
}

hipError_t launch_head(const thia_classifier* c, const void* feat, int n, int HW, int ep, float* partial, int32_t* labels, float* conf,
                       float* logits, hipStream_t s) {
    const int C = c->channels[c->taps[ep - 1] - 1];
    if (c->precision) hipLaunchKernelGGL(mean_partial_kernel<bf16_t>, dim3(kSlabs, n), dim3(256), 0, s, static_cast<const bf16_t*>(feat), HW, C, partial);
    else hipLaunchKernelGGL(mean_partial_kernel<float>, dim3(kSlabs, n), dim3(256), 0, s, static_cast<const float*>(feat), HW, C, partial);
    const size_t lds = sizeof(float) * ((size_t)C + c->n_classes);
    hipLaunchKernelGGL(classifier_head_kernel, dim3(n), dim3(256), lds, s, partial, HW, C, c->n_classes, c->fcw[ep - 1], c->fcb[ep - 1], labels,
                       conf, logits);
    return hipGetLastError();
}

// nb frames up to the layer exit ep taps; *feat points at the tapped tensor [nb,h,w,C] (NHWC), *hw = h * w.
int run_to_tap(thia_classifier* c, const uint8_t* frames, int nb, int H, int W, int ep, const void** feat, int* hw) {
    const int tap = c->taps[ep - 1];
    {
        const int epc = c->precision ? 8 : 4;
        const size_t total = (size_t)nb * H * W * (c->cin_pad / epc), blocks = (total + 255) / 256;
        if (blocks >= (1ull << 31)) return cfail(c, THIA_E_SHAPE, "chunk too large");
        if (c->precision) hipLaunchKernelGGL(pack_frames_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, c->stream, frames, (size_t)nb * H * W, H * W, c->cin_pad, c->mean, c->stdv, c->act[1]);
        else hipLaunchKernelGGL(pack_frames_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, c->stream, frames, (size_t)nb * H * W, H * W, c->cin_pad, c->mean, c->stdv, c->act[1]);
        if (hipGetLastError() != hipSuccess) return cfail(c, THIA_E_HIP, "frame packing launch failed");
    }
    void *x = c->act[1], *y = c->act[0];
    int h = H, w = W;
    for (int i = 0; i < tap; ++i) {
        const ConvLayer& L = c->conv[i];
        ConvArgs a{};
        a.in = x; a.w = L.w; a.bias = L.b; a.res = nullptr; a.out0 = y; a.out1 = nullptr;
        a.N = nb; a.H = h; a.W = w; a.Cin = L.ci; a.Cout = L.co; a.kh = 3; a.kw = 3; a.stride = 1; a.pad = 1; a.Ho = h; a.Wo = w;
        a.relu = 1; a.n_split = L.co; a.ld0 = L.co; a.ld1 = 0;
        if (!conv_supported(a, c->precision)) return cfail(c, THIA_E_SHAPE, "convolution shape not supported");
        if (launch_conv(a, c->precision, false, c->stream) != hipSuccess) return cfail(c, THIA_E_HIP, "convolution launch failed");
        std::swap(x, y);
        if (c->pool[i] && i + 1 < tap) {
            if (launch_pool2x2(x, nb, h, w, L.co, c->precision, y, c->stream) != hipSuccess) return cfail(c, THIA_E_HIP, "pooling launch failed");
            std::swap(x, y);
            h /= 2; w /= 2;
        }
    }
    *feat = x;
    *hw = h * w;
    return THIA_OK;
}

// Largest tensor of the stack (elements per frame), the packed input included.
size_t max_act_elems(const thia_classifier* c, int H, int W) {
    size_t mx = (size_t)H * W * c->cin_pad;
    int h = H, w = W;
    for (int i = 0; i < c->n_layers; ++i) {
        mx = std::max(mx, (size_t)h * w * c->channels[i]);
        if (c->pool[i]) { h /= 2; w /= 2; }
    }
    return mx;
}

}  // namespace

extern "C" {

int thia_classifier_load(const void* weights, size_t nbytes, int n_exits, thia_classifier** out) {
    if (!weights || !out) return THIA_E_BADARG;
    *out = nullptr;
    if (nbytes < 256 || (nbytes - 256) % 4) return THIA_E_BLOB;
    int32_t h[64];
    float hf[64];
    std::memcpy(h, weights, 256);
    std::memcpy(hf, weights, 256);
    if (h[0] != kClsMagic || h[1] != 1) return THIA_E_BLOB;
    if (h[3] != n_exits || n_exits < 1 || n_exits > kMaxExits || h[4] < 1 || h[4] > kMaxLayers) return THIA_E_BLOB;
    thia_classifier* c = new (std::nothrow) thia_classifier();
    if (!c) return THIA_E_NOMEM;
    auto bad = [&](int code) { thia_classifier_free(c); return code; };
    c->precision = h[2]; c->n_exits = n_exits; c->n_layers = h[4]; c->in_ch = h[5]; c->n_classes = h[6];
    c->mean = hf[7]; c->stdv = hf[8];
    if ((c->precision != 0 && c->precision != 1) || c->in_ch != 3 || c->n_classes < 2 || c->n_classes > 4096 || !(c->stdv > 0.f)) return bad(THIA_E_BLOB);
    c->esz = c->precision ? 2 : 4;
    c->cin_pad = c->precision ? 64 : 32;   // one K tile of the convolution kernel
    const int kt = c->cin_pad;
    for (int i = 0; i < c->n_layers; ++i) {
        c->channels[i] = h[9 + i]; c->pool[i] = h[25 + i] ? 1 : 0;
        // kernel limits: channel counts are whole K tiles of the next layer and at most 1024 (pooling kernel's LDS row)
        if (c->channels[i] < kt || c->channels[i] % kt || c->channels[i] > 1024) return bad(THIA_E_SHAPE);
    }
    for (int k = 0; k < n_exits; ++k) {
        c->taps[k] = h[41 + k];
        if (c->taps[k] < 1 || c->taps[k] > c->n_layers || (k > 0 && c->taps[k] <= c->taps[k - 1])) return bad(THIA_E_BLOB);
    }
    const float* p = reinterpret_cast<const float*>(static_cast<const char*>(weights) + 256);
    const float* end = reinterpret_cast<const float*>(static_cast<const char*>(weights) + nbytes);
    auto take = [&](size_t n, const float** q) { if ((size_t)(end - p) < n) return false; *q = p; p += n; return true; };
    int cin = c->in_ch;
    for (int i = 0; i < c->n_layers; ++i) {
        const int co = c->channels[i], ci_k = i == 0 ? c->cin_pad : cin;
        const float *w = nullptr, *b = nullptr;
        if (!take((size_t)co * cin * 9, &w) || !take((size_t)co, &b)) return bad(THIA_E_BLOB);
        // [O][I][3][3] fp32 -> [O][3][3][I (zero-padded for the first layer)] in the model's element type
        std::vector<unsigned char> host((size_t)co * 9 * ci_k * c->esz, 0);
        for (int o = 0; o < co; ++o)
            for (int t = 0; t < 9; ++t)
                for (int ic = 0; ic < cin; ++ic) {
                    const float v = w[((size_t)o * cin + ic) * 9 + t];
                    const size_t d = ((size_t)o * 9 + t) * ci_k + ic;
                    if (c->precision) reinterpret_cast<bf16_t*>(host.data())[d] = f32_to_bf16(v);
                    else reinterpret_cast<float*>(host.data())[d] = v;
                }
        ConvLayer& L = c->conv[i];
        L.co = co; L.ci = ci_k;
        if (hipMalloc(&L.w, host.size()) != hipSuccess || hipMalloc(reinterpret_cast<void**>(&L.b), (size_t)co * 4) != hipSuccess) return bad(THIA_E_NOMEM);
        if (hipMemcpy(L.w, host.data(), host.size(), hipMemcpyHostToDevice) != hipSuccess || hipMemcpy(L.b, b, (size_t)co * 4, hipMemcpyHostToDevice) != hipSuccess)
            return bad(THIA_E_HIP);
        cin = co;
    }
    for (int k = 0; k < n_exits; ++k) {
        const int C = c->channels[c->taps[k] - 1];
        const float *w = nullptr, *b = nullptr;
        if (!take((size_t)c->n_classes * C, &w) || !take((size_t)c->n_classes, &b)) return bad(THIA_E_BLOB);
        if (hipMalloc(reinterpret_cast<void**>(&c->fcw[k]), (size_t)c->n_classes * C * 4) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&c->fcb[k]), (size_t)c->n_classes * 4) != hipSuccess)
            return bad(THIA_E_NOMEM);
        if (hipMemcpy(c->fcw[k], w, (size_t)c->n_classes * C * 4, hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(c->fcb[k], b, (size_t)c->n_classes * 4, hipMemcpyHostToDevice) != hipSuccess)
            return bad(THIA_E_HIP);
    }
    if (p != end) return bad(THIA_E_BLOB);
    *out = c;
    return THIA_OK;
}

void thia_classifier_free(thia_classifier* c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->stream);
    for (ConvLayer& L : c->conv) { (void)hipFree(L.w); (void)hipFree(L.b); }
    for (int k = 0; k < kMaxExits; ++k) { (void)hipFree(c->fcw[k]); (void)hipFree(c->fcb[k]); }
    (void)hipFree(c->act[0]); (void)hipFree(c->act[1]); (void)hipFree(c->partial);
    delete c;
}

int thia_classifier_set_stream(thia_classifier* c, void* hip_stream) {
    if (!c) return THIA_E_BADARG;
    if (hipStreamSynchronize(c->stream) != hipSuccess) return cfail(c, THIA_E_HIP, "stream synchronisation failed");
    c->stream = static_cast<hipStream_t>(hip_stream);
    return THIA_OK;
}

const char* thia_classifier_last_error(const thia_classifier* c) { return c ? c->err.c_str() : "null classifier"; }

int thia_classify_chunk(thia_classifier* c, const uint8_t* frames, int n, int H, int W, int ep, int32_t* out_labels, float* out_conf,
                        float* out_logits) {
    if (!c) return THIA_E_BADARG;
    if (n < 0) return cfail(c, THIA_E_BADARG, "negative frame count");
    if (n > 0 && (!frames || !out_labels || !out_conf)) return cfail(c, THIA_E_BADARG, "null pointer");
    if (ep < 0 || ep > c->n_exits) return cfail(c, THIA_E_BADEP, "exit outside 0..n_exits");
    if (H < 1 || W < 1 || H > 16384 || W > 16384) return cfail(c, THIA_E_SHAPE, "frame size must be within 1..16384");
    if (n == 0) return THIA_OK;
    if (ep == 0) {
        hipLaunchKernelGGL(fill_skipped_kernel, dim3((n + 255) / 256), dim3(256), 0, c->stream, n, out_labels, out_conf);
        return hipGetLastError() == hipSuccess ? THIA_OK : cfail(c, THIA_E_HIP, "fill launch failed");
    }
    {   // every pool in front of the tapped layer must leave at least one position
        int h = H, w = W;
        for (int i = 0; i + 1 < c->taps[ep - 1]; ++i)
            if (c->pool[i]) { h /= 2; w /= 2; }
        if (h < 1 || w < 1) return cfail(c, THIA_E_SHAPE, "frame too small for the pools in front of this exit");
    }
    // micro-batches of at most ~512 MB per activation tensor
    const size_t per_frame = max_act_elems(c, H, W) * c->esz;
    const int mb = (int)std::max<size_t>(1, std::min<size_t>((size_t)n, ((size_t)512 << 20) / per_frame));
    int rc = ensure_buffers(c, (size_t)mb * per_frame, (size_t)mb * kSlabs * 1024);
    if (rc != THIA_OK) return rc;
    for (int f0 = 0; f0 < n; f0 += mb) {
        const int nb = std::min(mb, n - f0);
        const void* feat = nullptr;
        int hw = 0;
        rc = run_to_tap(c, frames + (size_t)f0 * 3 * H * W, nb, H, W, ep, &feat, &hw);
        if (rc != THIA_OK) return rc;
        if (launch_head(c, feat, nb, hw, ep, c->partial, out_labels + f0, out_conf + f0, out_logits ? out_logits + (size_t)f0 * c->n_classes : nullptr,
                        c->stream) != hipSuccess)
            return cfail(c, THIA_E_HIP, "classifier unit launch failed");
    }
    return THIA_OK;
}

int thia_classifier_op_pool(thia_classifier* c, const void* in, int n, int H, int W, int C, void* out) {
    if (!c || !in || !out || n <= 0 || H < 2 || W < 2) return cfail(c, THIA_E_BADARG, "bad arguments");
    if (C <= 0 || C % (c->precision ? 8 : 4)) return cfail(c, THIA_E_SHAPE, "channels must fill whole 16-byte chunks");
    if (launch_pool2x2(in, n, H, W, C, c->precision, out, c->stream) != hipSuccess) return cfail(c, THIA_E_HIP, "pooling launch failed");
    return THIA_OK;
}

int thia_classifier_op_unit(thia_classifier* c, const void* feat, int n, int HW, int ep, int32_t* out_labels, float* out_conf, float* out_logits) {
    if (!c || !feat || !out_labels || !out_conf || n <= 0 || HW <= 0) return cfail(c, THIA_E_BADARG, "bad arguments");
    if (ep < 1 || ep > c->n_exits) return cfail(c, THIA_E_BADEP, "exit outside 1..n_exits");
    const int rc = ensure_buffers(c, 0, (size_t)n * kSlabs * 1024);
    if (rc != THIA_OK) return rc;
    if (launch_head(c, feat, n, HW, ep, c->partial, out_labels, out_conf, out_logits, c->stream) != hipSuccess) return cfail(c, THIA_E_HIP, "classifier unit launch failed");
    return THIA_OK;
}

}  // extern "C"
