// Backbone entry: pixel normalisation fused into the 7x7 stride-2 stem convolution
// (+ bias, ReLU), and the 3x3 stride-2 max-pool.  Input frames are planar uint8
// [n,3,H,W]; outputs are NHWC.
//
// bf16 models: one persistent matrix-core kernel does normalisation, stem, ReLU and pool
// (stem_pool_mfma_kernel).  fp32 models: the stem contracts only K = 3*7*7 = 147 values per
// output and runs on the vector ALUs (stem_kernel: a 256-thread block owns a 16x16 tile of
// output pixels, stages the normalised 37x37x3 patch in LDS once, and every thread
// accumulates all 64 output channels of its pixel; weights are wavefront-uniform), followed
// by maxpool_kernel.
#include <algorithm>
#include <type_traits>

#include "thia_internal.h"

namespace thia {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int ST = 16;               // output tile side
constexpr int SP = 2 * ST + 5;       // input patch side (stride 2, 7 taps)
constexpr int SC = 64;               // stem output channels

template <bool BF16>
__global__ __launch_bounds__(256) void stem_kernel(const uint8_t* __restrict__ frames, int H, int W, int Hs, int Ws,
                                                   const float* __restrict__ w, const float* __restrict__ bias,
                                                   float mean, float stdv, void* __restrict__ out_) {
    __shared__ float patch[3][SP][SP + 1];
    const int t = threadIdx.x, tx = t & (ST - 1), ty = t / ST;
    const int ox0 = blockIdx.x * ST, oy0 = blockIdx.y * ST, img = blockIdx.z;
    const int ix0 = 2 * ox0 - 3, iy0 = 2 * oy0 - 3;
    const uint8_t* f = frames + (size_t)img * 3 * H * W;
    for (int i = t; i < 3 * SP * SP; i += 256) {
        const int c = i / (SP * SP), r = i - c * SP * SP, py = r / SP, px = r - py * SP;
        const int iy = iy0 + py, ix = ix0 + px;
        float v = 0.f;  // zero padding applies to the normalised tensor
        if ((unsigned)iy < (unsigned)H && (unsigned)ix < (unsigned)W) {
            v = ((float)f[((size_t)c * H + iy) * W + ix] - mean) / stdv;
            if (BF16) v = bf16_to_f32(f32_to_bf16(v));
        }
        patch[c][py][px] = v;
    }
    __syncthreads();

    float acc[SC];
#pragma unroll
    for (int ch = 0; ch < SC; ++ch) acc[ch] = 0.f;
    for (int c = 0; c < 3; ++c)
        for (int ky = 0; ky < 7; ++ky)
#pragma unroll
            for (int kx = 0; kx < 7; ++kx) {
                const float x = patch[c][2 * ty + ky][2 * tx + kx];
                const float* wt = w + ((c * 7 + ky) * 7 + kx) * SC;
#pragma unroll
                for (int ch = 0; ch < SC; ++ch) acc[ch] = fmaf(x, wt[ch], acc[ch]);
            }

    const int oy = oy0 + ty, ox = ox0 + tx;
    if (oy >= Hs || ox >= Ws) return;
    const size_t o = (((size_t)img * Hs + oy) * Ws + ox) * SC;
    if (BF16) {
        bf16_t* out = static_cast<bf16_t*>(out_) + o;
#pragma unroll
        for (int ch = 0; ch < SC; ch += 8) {
            u32x4_t v;
            float h[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) h[q] = fmaxf(acc[ch + q] + bias[ch + q], 0.f);
            v.x = pack_bf16x2(h[0], h[1]); v.y = pack_bf16x2(h[2], h[3]); v.z = pack_bf16x2(h[4], h[5]); v.w = pack_bf16x2(h[6], h[7]);
            *reinterpret_cast<u32x4_t*>(out + ch) = v;
        }
    } else {
        float* out = static_cast<float*>(out_) + o;
#pragma unroll
        for (int ch = 0; ch < SC; ch += 4) {
            f32x4_t v = {fmaxf(acc[ch] + bias[ch], 0.f), fmaxf(acc[ch + 1] + bias[ch + 1], 0.f),
                         fmaxf(acc[ch + 2] + bias[ch + 2], 0.f), fmaxf(acc[ch + 3] + bias[ch + 3], 0.f)};
            *reinterpret_cast<f32x4_t*>(out + ch) = v;
        }
    }
}

// ---------------------------------------------------------------------------------
// bf16 stem on the matrix cores.  The 7x7x3 window is laid out as K = 22 rows x 8 taps:
// row r = c*7 + ky (row 21 is padding), tap j = kx + 1 (j = 0 has a zero weight).  With
// that layout the 8 consecutive K values a lane feeds to one 32x32x16 MFMA are 8
// consecutive pixels of one input row of the normalised bf16 patch held in LDS (four
// dwords): no im2col copy is ever built.
typedef __attribute__((ext_vector_type(8))) __bf16 sbf16x8_t;
typedef __attribute__((ext_vector_type(16))) float sf32x16_t;

constexpr int MP_W = 72;                       // patch columns (2 * 32 stem columns + taps)
constexpr int MK_ROWS = 22;                    // 21 (c,ky) rows + 1 zero row
constexpr int MW_PITCH = MK_ROWS * 16 + 16;    // bytes per channel row of the weight tile (padded)
constexpr int ME_PITCH = 128 + 16;             // epilogue row pitch (64 bf16 + pad)

// Stem and max-pool in one kernel (bf16 models): the stem tensor is four times the size of the pooled one
// and is otherwise written and read back once.  A block owns 8 x 15 pooled pixels = stem rows 2 py0 - 1 ..
// 2 py0 + 15 and stem columns 2 px0 - 1 .. 2 px0 + 30 (32 columns = one MFMA pixel tile).  Each wavefront
// computes five stem rows (the fifth is shared with the next wavefront and recomputed) so that both of
// its pooled rows are maxima over its own accumulators; the column maximum is taken on the bf16 tile that
// goes through LDS for the store anyway.  Stem pixels outside the stem tensor count as 0, which equals the
// pool's "ignore" padding because every window holds its in-range centre and all values are >= 0 after the
// ReLU; rounding and ReLU are monotonic, so max-then-round equals round-then-max bit for bit.
constexpr int QP_ROWS = 8, QP_COLS = 15;            // pooled tile
constexpr int QS_ROWS = 2 * QP_ROWS + 1;            // 17 stem rows
constexpr int QPR = 2 * QS_ROWS + 5;                // 39 patch rows
typedef __attribute__((ext_vector_type(8))) unsigned short u16x8_t;

__global__ __launch_bounds__(256, 2) void stem_pool_mfma_kernel(const uint8_t* __restrict__ frames, int n, int H, int W, int Hs, int Ws,
                                                             int Hp, int Wp, const bf16_t* __restrict__ wk /*[64][22*8]*/,
                                                             const float* __restrict__ bias, float mean, float stdv,
                                                             bf16_t* __restrict__ out) {
    __shared__ __align__(16) bf16_t patch[3 * QPR * MP_W];
    __shared__ __align__(16) unsigned char wt[64 * MW_PITCH];
    __shared__ __align__(16) unsigned char etile[4 * 32 * ME_PITCH];
    __shared__ bf16_t lut[256];
    __shared__ __align__(16) float sbias[64];
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    if (t < 64) sbias[t] = bias[t];
    // Persistent blocks: weights and the normalisation table are staged once, and the raw pixels of the next
    // tile are requested (9 dwords per thread, held in registers) before the current tile is multiplied.
    lut[t] = f32_to_bf16(((float)t - mean) / stdv);
    for (int i = t; i < 64 * MK_ROWS; i += 256) {
        const int ch = i / MK_ROWS, r = i - ch * MK_ROWS;
        *reinterpret_cast<u32x4_t*>(wt + ch * MW_PITCH + r * 16) = *reinterpret_cast<const u32x4_t*>(wk + (size_t)ch * MK_ROWS * 8 + r * 8);
    }
    const int tiles_x = (Wp + QP_COLS - 1) / QP_COLS, tiles_y = (Hp + QP_ROWS - 1) / QP_ROWS;
    const int total = n * tiles_y * tiles_x;
    constexpr int DW_ROW = MP_W / 4;
    constexpr int N_DW = 3 * QPR * DW_ROW;
    constexpr int PER_T = (N_DW + 255) / 256;
    const bool dwords = (W & 3) == 0;   // every patch row then starts on a 4-byte boundary of the frame
    // patch coordinates (channel, row, dword) of dword q of this thread
    auto dword_pos = [&](int q, int& c, int& py, int& pd) {
        const int i = min(q * 256 + t, N_DW - 1);
        c = i / (QPR * DW_ROW);
        const int r = i - c * (QPR * DW_ROW);
        py = r / DW_ROW;
        pd = r - py * DW_ROW;
    };
    struct TileOrg { int img, px0, py0, ix0, iy0; };
    auto tile_org = [&](int tile) {
        TileOrg o;
        o.img = tile / (tiles_y * tiles_x);
        const int rem = tile - o.img * (tiles_y * tiles_x);
        o.py0 = (rem / tiles_x) * QP_ROWS;
        o.px0 = (rem % tiles_x) * QP_COLS;
        // stem origin (2 px0 - 1, 2 py0 - 1); patch column 0 is image column 2 sx0 - 6 (a multiple of 4): tap
        // j = kx + 1 of stem column sx0 + p sits at patch column 2 p + 2 + j
        o.ix0 = 2 * (2 * o.px0 - 1) - 6;
        o.iy0 = 2 * (2 * o.py0 - 1) - 3;
        return o;
    };
    uint32_t raw[PER_T];
    auto load_raw = [&](const TileOrg& o) {
        const uint8_t* f = frames + (size_t)o.img * 3 * H * W;
#pragma unroll
        for (int q = 0; q < PER_T; ++q) {
            int c, py, pd;
            dword_pos(q, c, py, pd);
            const int iy = o.iy0 + py, ix = o.ix0 + 4 * pd;
            raw[q] = 0u;
            if ((unsigned)iy < (unsigned)H && ix >= 0 && ix + 3 < W) raw[q] = *reinterpret_cast<const uint32_t*>(f + ((size_t)c * H + iy) * W + ix);
        }
    };
    int tile = blockIdx.x;
    if (tile >= total) return;
    TileOrg cur = tile_org(tile);
    if (dwords) load_raw(cur);
    __syncthreads();   // lut and weights visible
    const int g = lane >> 5, pxl = lane & 31;
    for (; tile < total; tile += gridDim.x) {
        // ---- patch fill: out-of-image pixels become the bf16 zero of the normalised tensor
        if (dwords) {
#pragma unroll
            for (int q = 0; q < PER_T; ++q) {
                if (q * 256 + t < N_DW) {
                    int c, py, pd;
                    dword_pos(q, c, py, pd);
                    const int iy = cur.iy0 + py, ix = cur.ix0 + 4 * pd;
                    const bool in = (unsigned)iy < (unsigned)H && ix >= 0 && ix + 3 < W;
                    uint32_t lo = 0u, hi = 0u;
                    if (in) {
                        lo = (uint32_t)lut[raw[q] & 0xffu] | ((uint32_t)lut[(raw[q] >> 8) & 0xffu] << 16);
                        hi = (uint32_t)lut[(raw[q] >> 16) & 0xffu] | ((uint32_t)lut[raw[q] >> 24] << 16);
                    }
                    uint32_t* d = reinterpret_cast<uint32_t*>(patch + (c * QPR + py) * MP_W + 4 * pd);
                    d[0] = lo;
                    d[1] = hi;
                }
            }
        } else {
            const uint8_t* f = frames + (size_t)cur.img * 3 * H * W;
            for (int i = t; i < 3 * QPR * MP_W; i += 256) {
                const int c = i / (QPR * MP_W), r = i - c * (QPR * MP_W), py = r / MP_W, px = r - py * MP_W;
                const int iy = cur.iy0 + py, ix = cur.ix0 + px;
                bf16_t v = 0;
                if ((unsigned)iy < (unsigned)H && (unsigned)ix < (unsigned)W) v = lut[f[((size_t)c * H + iy) * W + ix]];
                patch[i] = v;
            }
        }
        __syncthreads();
        const TileOrg nxt = tile_org(min(tile + (int)gridDim.x, total - 1));
        if (dwords && tile + (int)gridDim.x < total) load_raw(nxt);

        // Stem rows 0..2 of this wavefront give its first pooled row, rows 2..4 the second: rows 0..2 are
        // multiplied first, rows 3..4 after the first pooled row has left the registers (96 live accumulator
        // registers instead of 160).
        sf32x16_t bias_t[2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const f32x4_t q = *reinterpret_cast<const f32x4_t*>(sbias + i * 32 + 8 * v + 4 * g);   // LDS copy: no per-tile global wait
                bias_t[i][4 * v] = q.x; bias_t[i][4 * v + 1] = q.y; bias_t[i][4 * v + 2] = q.z; bias_t[i][4 * v + 3] = q.w;
            }
        const int sx0 = 2 * cur.px0 - 1, sy0 = 2 * cur.py0 - 1;
        unsigned char* ep = etile + wv * 32 * ME_PITCH;
        const bool colok = (unsigned)(sx0 + pxl) < (unsigned)Ws;
        sf32x16_t acc[3][2];   // rows (0, 1, 2), then (3, 4, 2)
        auto mma_rows = [&](auto r0c, auto nrc) {
            constexpr int r0 = decltype(r0c)::value, nr = decltype(nrc)::value;
#pragma unroll
            for (int r = 0; r < nr; ++r)
#pragma unroll
                for (int i = 0; i < 2; ++i) acc[r][i] = bias_t[i];   // accumulators start from the bias
#pragma unroll 2
            for (int s = 0; s < MK_ROWS / 2; ++s) {   // (a full unroll hoists every operand load and spills)
                const int rr = 2 * s + g;
                const int rq = rr < 21 ? rr : 0;
                const int c = rq / 7, ky = rq - 7 * c;
                u32x4_t fa[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) fa[i] = *reinterpret_cast<const u32x4_t*>(wt + (i * 32 + pxl) * MW_PITCH + rr * 16);
#pragma unroll
                for (int r = 0; r < nr; ++r) {
                    const int row = 2 * (4 * wv + r0 + r) + ky;
                    const uint32_t* src = reinterpret_cast<const uint32_t*>(patch + (c * QPR + row) * MP_W + 2 * pxl + 2);
                    u32x4_t fb = {src[0], src[1], src[2], src[3]};
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        acc[r][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(sbf16x8_t, fa[i]),
                                                                            __builtin_bit_cast(sbf16x8_t, fb), acc[r][i], 0, 0, 0);
                }
            }
        };
        auto pooled_row = [&](int half, const bool rowok[3]) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float m[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float best = 0.f;   // ReLU and the zero that stands for out-of-range stem pixels
#pragma unroll
                        for (int r = 0; r < 3; ++r) best = fmaxf(best, rowok[r] ? acc[r][i][4 * v + e] : 0.f);
                        m[e] = colok ? best : 0.f;
                    }
                    uint32_t* d = reinterpret_cast<uint32_t*>(ep + pxl * ME_PITCH + (i * 32 + 8 * v + 4 * g) * 2);
                    d[0] = pack_bf16x2(m[0], m[1]);
                    d[1] = pack_bf16x2(m[2], m[3]);
                }
            __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the tile is private to this wavefront
            __builtin_amdgcn_wave_barrier();
            const int py = cur.py0 + 2 * wv + half;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int item = it * 64 + lane;
                const int j = item >> 3, chunk = item & 7;
                if (j < QP_COLS) {
                    // non-negative bf16 values order like their bit patterns: packed 16-bit integer maximum
                    const u16x8_t a0 = *reinterpret_cast<const u16x8_t*>(ep + (2 * j) * ME_PITCH + chunk * 16);
                    const u16x8_t a1 = *reinterpret_cast<const u16x8_t*>(ep + (2 * j + 1) * ME_PITCH + chunk * 16);
                    const u16x8_t a2 = *reinterpret_cast<const u16x8_t*>(ep + (2 * j + 2) * ME_PITCH + chunk * 16);
                    const u16x8_t mx = __builtin_elementwise_max(__builtin_elementwise_max(a0, a1), a2);
                    const int px = cur.px0 + j;
                    if (py < Hp && px < Wp) *reinterpret_cast<u16x8_t*>(out + (((size_t)cur.img * Hp + py) * Wp + px) * SC + chunk * 8) = mx;
                }
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);
            __builtin_amdgcn_wave_barrier();
        };
        const int srow = sy0 + 4 * wv;
        mma_rows(std::integral_constant<int, 0>{}, std::integral_constant<int, 3>{});
        {
            const bool ok[3] = {(unsigned)srow < (unsigned)Hs, (unsigned)(srow + 1) < (unsigned)Hs, (unsigned)(srow + 2) < (unsigned)Hs};
            pooled_row(0, ok);
        }
        mma_rows(std::integral_constant<int, 3>{}, std::integral_constant<int, 2>{});   // rows 3, 4 replace rows 0, 1; row 2 stays
        __syncthreads();   // every wavefront is done with the patch: the next iteration may overwrite it
        {
            const bool ok[3] = {(unsigned)(srow + 3) < (unsigned)Hs, (unsigned)(srow + 4) < (unsigned)Hs, (unsigned)(srow + 2) < (unsigned)Hs};
            pooled_row(1, ok);
        }
        cur = nxt;
    }
}

hipError_t launch_stem_pool(const uint8_t* frames, int n, int H, int W, const bf16_t* wk, const float* bias, float mean, float stdv,
                            void* out, hipStream_t s) {
    const int Hs = (H + 6 - 7) / 2 + 1, Ws = (W + 6 - 7) / 2 + 1;
    const int Hp = (Hs + 2 - 3) / 2 + 1, Wp = (Ws + 2 - 3) / 2 + 1;
    const long long tiles = (long long)n * ((Wp + QP_COLS - 1) / QP_COLS) * ((Hp + QP_ROWS - 1) / QP_ROWS);
    if (n <= 0 || tiles <= 0 || tiles >= (1ll << 30)) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)std::min<long long>(tiles, 512);   // two resident blocks on each of the 256 CUs
    hipLaunchKernelGGL(stem_pool_mfma_kernel, dim3(grid), dim3(256), 0, s, frames, n, H, W, Hs, Ws, Hp, Wp, wk, bias, mean, stdv,
                       static_cast<bf16_t*>(out));
    return hipGetLastError();
}

hipError_t launch_stem(const uint8_t* frames, int n, int H, int W, const float* w, const float* bias, float mean, float stdv, void* out,
                       hipStream_t s) {
    const int Hs = (H + 6 - 7) / 2 + 1, Ws = (W + 6 - 7) / 2 + 1;
    dim3 grid((Ws + ST - 1) / ST, (Hs + ST - 1) / ST, n);
    if (grid.y > 65535u || grid.z > 65535u) return hipErrorInvalidValue;
    hipLaunchKernelGGL(stem_kernel<false>, grid, dim3(256), 0, s, frames, H, W, Hs, Ws, w, bias, mean, stdv, out);
    return hipGetLastError();
}

// 3x3 / stride 2 / pad 1 max-pool, NHWC; one thread per 16-byte channel chunk of an output pixel.
template <bool BF16>
__global__ void maxpool_kernel(const void* __restrict__ in_, int n, int H, int W, int C, int Ho, int Wo,
                               void* __restrict__ out_) {
    constexpr int EPC = BF16 ? 8 : 4;
    const int chunks = C / EPC;
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
    for (int ky = 0; ky < 3; ++ky) {
        const int iy = 2 * oy - 1 + ky;
        if ((unsigned)iy >= (unsigned)H) continue;
        for (int kx = 0; kx < 3; ++kx) {
            const int ix = 2 * ox - 1 + kx;
            if ((unsigned)ix >= (unsigned)W) continue;
            const size_t off = (((size_t)img * H + iy) * W + ix) * C + (size_t)ck * EPC;
            if (BF16) {
                const u32x4_t v = *reinterpret_cast<const u32x4_t*>(static_cast<const bf16_t*>(in_) + off);
                const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    best[2 * q] = fmaxf(best[2 * q], __uint_as_float(wv[q] << 16));
                    best[2 * q + 1] = fmaxf(best[2 * q + 1], __uint_as_float(wv[q] & 0xffff0000u));
                }
            } else {
                const f32x4_t v = *reinterpret_cast<const f32x4_t*>(static_cast<const float*>(in_) + off);
                best[0] = fmaxf(best[0], v.x); best[1] = fmaxf(best[1], v.y);
                best[2] = fmaxf(best[2], v.z); best[3] = fmaxf(best[3], v.w);
            }
        }
    }
    const size_t o = (((size_t)img * Ho + oy) * Wo + ox) * C + (size_t)ck * EPC;
    if (BF16) {
        u32x4_t v;
        uint32_t h[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) h[q] = __float_as_uint(best[q]) >> 16;  // values are bf16 already
        v.x = h[0] | (h[1] << 16); v.y = h[2] | (h[3] << 16); v.z = h[4] | (h[5] << 16); v.w = h[6] | (h[7] << 16);
        *reinterpret_cast<u32x4_t*>(static_cast<bf16_t*>(out_) + o) = v;
    } else {
        f32x4_t v = {best[0], best[1], best[2], best[3]};
        *reinterpret_cast<f32x4_t*>(static_cast<float*>(out_) + o) = v;
    }
}

hipError_t launch_maxpool(const void* in, int n, int H, int W, int C, int precision, void* out, hipStream_t s) {
    const int Ho = (H + 2 - 3) / 2 + 1, Wo = (W + 2 - 3) / 2 + 1;
    const int epc = precision ? 8 : 4;
    if (C % epc) return hipErrorInvalidValue;
    const size_t total = (size_t)n * Ho * Wo * (C / epc);
    const size_t blocks = (total + 255) / 256;
    if (blocks == 0 || blocks >= (1ull << 31)) return hipErrorInvalidValue;
    if (precision)
        hipLaunchKernelGGL(maxpool_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, in, n, H, W, C, Ho, Wo, out);
    else
        hipLaunchKernelGGL(maxpool_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, in, n, H, W, C, Ho, Wo, out);
    return hipGetLastError();
}

}  // namespace thia
