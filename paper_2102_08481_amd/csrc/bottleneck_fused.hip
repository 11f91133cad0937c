// One identity bottleneck block (1x1 -> 3x3 -> 1x1 + input, stride 1) of the backbone in a single
// kernel on the CDNA4 matrix cores (gfx950), bf16 tensors with fp32 accumulation.
//
// Layer by layer the narrow stages are pure HBM streaming: every 1x1 re-reads or re-writes the
// 4*WD-channel tensor.  Here a 256-thread block (4 wavefronts) owns an 8 x 16 pixel tile of one frame and
// keeps the two WD-channel intermediates in LDS, so the wide tensor is read once (plus halo) and written
// once per block:
//   phase 1  t1 = relu(W1 x + b1) on the 10 x 18 halo tile (192 rows with padding), K = 4*WD walked in
//            64-channel steps through an LDS staging tile (coalesced 16-byte loads); halo pixels outside
//            the frame are set to zero, which is the zero padding of the 3x3 that follows;
//   phase 2  t2 = relu(W2 * t1 + b2): the MFMA pixel operand is read straight from the t1 tile at the
//            tap's row offset, no im2col copy;
//   phase 3  y = relu(W3 t2 + b3 + x): per 32-pixel sub-tile the fp32 result goes through a
//            wavefront-private LDS transpose so that residual loads and stores are 16 bytes per lane
//            and cover whole lines of the NHWC tensors.
// Both intermediates are rounded to bf16 exactly where the layer-by-layer path stores them.
// Optionally (TAILN > 0) a fourth phase applies the 1x1 layer that reads this block's output - the exit's lateral or
// the next stage's first 1x1 - to the output tile while it is still on the CU, so that layer's own launch, and its
// read of the wide tensor, disappear.
// Weights never pass through LDS: they are pre-packed in MFMA fragment order (one coalesced 1 KiB
// load per 32-channel x 16-k fragment) and stay in L2.
#include <type_traits>

#include "thia_internal.h"

namespace thia {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

namespace {

__device__ inline void mma(f32x16_t& acc, const u32x4_t& a, const u32x4_t& b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), acc, 0, 0, 0);
}
__device__ inline uint32_t pack2(float lo, float hi) { return pack_bf16x2(lo, hi); }

// Scheduling fence for global memory instructions only: the compiler otherwise sinks prefetch loads
// down to their first use to save registers, which exposes the L2 latency once per fragment.
__device__ inline void pin_vmem() { __builtin_amdgcn_sched_barrier(0x78f); }

template <int I, int N, typename F>
__device__ inline void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

constexpr int TH = 8, TW = 16;          // output tile (pixels)
constexpr int HALO_W = TW + 2;          // halo tile width
constexpr int NH = (TH + 2) * HALO_W;   // halo pixels (180)
constexpr int NHP = 192;                // ... padded to whole 32-row MFMA tiles
constexpr int NPX = TH * TW;            // 128

}  // namespace

// FIRST = false: identity block, x has 4 WD channels and is the residual.
// FIRST = true:  a stage's first block at stride 1: x has WD channels and enters the output through the
//                projection shortcut; w3f holds [W3 | Ws] along K (2 WD) and b3 the summed biases, so phase 3 is one
//                contraction over (t2 channels, x channels) with the x operand read from the staging tile.
// TAILN = 128 or 256 (identity blocks only): z = [relu](Wt y + bt) with TAILN output channels is written to a.z as well.
template <int WD, bool FIRST, int TAILN = 0>
__global__ __launch_bounds__(256, 2) void bottleneck_fused_kernel(const FusedBlockArgs a) {
    static_assert(WD == 64, "work split below is written for 64-channel intermediates");
    static_assert(TAILN == 0 || (!FIRST && (TAILN == 128 || TAILN == 256)), "tail layer: identity blocks, 128 or 256 outputs");
    constexpr int C4 = 4 * WD;
    constexpr int CIN = FIRST ? WD : C4;
    constexpr int BK = 64;                 // phase-1 K step (channels)
    constexpr int XP = BK * 2 + 16;        // LDS row pitch of the x staging tile (bytes)
    constexpr int TP = WD * 2 + 16;        // LDS row pitch of t1 / t2 (bytes)
    constexpr int KT1 = CIN / BK;          // phase-1 K steps
    constexpr int KS1 = CIN / 16, KS2 = 9 * WD / 16, KS3 = (FIRST ? 2 * WD : WD) / 16;  // 16-wide MFMA k-steps per phase
    constexpr int EPITCH = 64 * 2 + 16;    // bf16 epilogue row: 64 channels + pad (bytes)
    constexpr int RING = 16;               // weight fragments in flight in phase 2
    static_assert(FIRST ? (KT1 == 1 && BK == WD) : KT1 == 4, "identity: one phase-1 K step per wavefront (residual hand-over)");

    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* T1 = smem;                        // [NHP][TP]
    unsigned char* XS = smem + NHP * TP;             // [NHP][XP]
    unsigned char* T2 = smem + NHP * (TP + XP);      // [NPX][TP]
    static_assert(4 * 32 * EPITCH <= NHP * TP, "epilogue tiles reuse the t1 area (the staging tile stays live for FIRST)");

    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int l32 = lane & 31, lh = lane >> 5;

    const int tiles_x = (a.W + TW - 1) / TW, tiles_y = (a.H + TH - 1) / TH;
    const int total = a.N * tiles_y * tiles_x;
    const int per_xcd = (total + 7) >> 3;   // contiguous tile range per XCD (block id & 7 selects the XCD)
    const int tile = (int)(blockIdx.x & 7u) * per_xcd + (int)(blockIdx.x >> 3);
    if (tile >= total) return;
    const int img = tile / (tiles_y * tiles_x);
    const int trem = tile - img * (tiles_y * tiles_x);
    const int y0 = (trem / tiles_x) * TH, x0 = (trem % tiles_x) * TW;
    const bf16_t* __restrict__ xin = a.x + (size_t)img * a.H * a.W * CIN;
    bf16_t* __restrict__ yout = a.y + (size_t)img * a.H * a.W * C4;

    // ------------------------------------------------------------------ phase 1: t1 on the halo tile
    // staging coordinates: 16-byte chunk lc of halo rows lr + 32 p; out-of-frame rows read a clamped
    // pixel (their t1 is forced to zero below)
    const int lc = t & 7, lr = t >> 3;
    uint32_t xoff[6];
#pragma unroll
    for (int p = 0; p < 6; ++p) {
        const int r = lr + 32 * p;
        const int hy = r / HALO_W, hx = r - hy * HALO_W;
        const int iy = min(max(y0 - 1 + hy, 0), a.H - 1), ix = min(max(x0 - 1 + hx, 0), a.W - 1);
        xoff[p] = (uint32_t)((iy * a.W + ix) * CIN + lc * 8);
    }
    const int cw = wv & 1;        // 32-channel half of the WD intermediates owned in phases 1 and 2
    const int pw = wv >> 1;       // pixel sub-tiles pw, pw + 2, ...
    const u32x4_t* __restrict__ w1f = reinterpret_cast<const u32x4_t*>(a.w1f) + (size_t)cw * KS1 * 64 + lane;
    const u32x4_t* __restrict__ w2f = reinterpret_cast<const u32x4_t*>(a.w2f) + (size_t)cw * KS2 * 64 + lane;
    const u32x4_t* __restrict__ w3f = reinterpret_cast<const u32x4_t*>(a.w3f) + (size_t)(2 * wv) * KS3 * 64 + lane;

    // the whole halo tile of x (4 K steps x 6 chunks per thread) is requested up front: one exposed
    // memory latency per tile instead of one per K step
    u32x4_t xs[KT1][6];
    u32x4_t wa[2][BK / 16];   // W1 fragments of the current and the next K step
#pragma unroll
    for (int p = 0; p < 6; ++p) xs[0][p] = *reinterpret_cast<const u32x4_t*>(xin + xoff[p]);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) wa[0][kk] = w1f[kk * 64];
#pragma unroll
    for (int kt = 1; kt < KT1; ++kt)
#pragma unroll
        for (int p = 0; p < 6; ++p) xs[kt][p] = *reinterpret_cast<const u32x4_t*>(xin + xoff[p] + kt * BK);

    // Accumulators start from the bias (element e of a lane is channel 8 (e / 4) + 4 (lane / 32) + e % 4 of the
    // 32-channel tile), so no epilogue waits for a bias load.
    auto bias_tile = [&](const float* b) {
        f32x16_t r;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const f32x4_t q = *reinterpret_cast<const f32x4_t*>(b + 8 * v + 4 * lh);
            r[4 * v] = q.x; r[4 * v + 1] = q.y; r[4 * v + 2] = q.z; r[4 * v + 3] = q.w;
        }
        return r;
    };
    f32x16_t acc1[3];
    acc1[0] = bias_tile(a.b1 + cw * 32);
    acc1[1] = acc1[0];
    acc1[2] = acc1[0];

    // Residual of phase 3: this wavefront's 64 output channels are K step wv of phase 1, so its share of
    // the centre pixels is copied out of the staging tile while that step is resident (no second read of x).
    u32x2_t rres[4][2][4];   // [pixel sub-tile][channel tile][accumulator quad], in accumulator layout

    static_for<0, KT1>([&](auto ktc) {
        constexpr int kt = decltype(ktc)::value;
        if (kt > 0) __syncthreads();   // every wavefront is done with the previous staging tile
#pragma unroll
        for (int p = 0; p < 6; ++p) *reinterpret_cast<u32x4_t*>(XS + (lr + 32 * p) * XP + lc * 16) = xs[kt][p];
        if (kt + 1 < KT1) {
#pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk) wa[(kt + 1) & 1][kk] = w1f[((kt + 1) * (BK / 16) + kk) * 64];
            pin_vmem();
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const u32x4_t b = *reinterpret_cast<const u32x4_t*>(XS + ((pw + 2 * j) * 32 + l32) * XP + kk * 32 + lh * 16);
                mma(acc1[j], wa[kt & 1][kk], b);
            }
        }
        if (!FIRST && wv == kt) {
#pragma unroll
            for (int pt = 0; pt < 4; ++pt)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int p = pt * 32 + l32;
                        const int hrow = (p / TW + 1) * HALO_W + (p % TW) + 1;
                        rres[pt][i][v] = *reinterpret_cast<const u32x2_t*>(XS + hrow * XP + (i * 32 + 8 * v + 4 * lh) * 2);
                    }
        }
    });

    // first weight fragments of phase 2 are requested before the t1 epilogue
    u32x4_t ring[RING];
#pragma unroll
    for (int s = 0; s < RING; ++s) ring[s] = w2f[s * 64];
    f32x16_t acc2[2];
    acc2[0] = bias_tile(a.b2 + cw * 32);
    acc2[1] = acc2[0];
    pin_vmem();

#pragma unroll
    for (int j = 0; j < 3; ++j) {
        const int r = (pw + 2 * j) * 32 + l32;
        const int hy = r / HALO_W, hx = r - hy * HALO_W;
        const int iy = y0 - 1 + hy, ix = x0 - 1 + hx;
        const bool ok = r < NH && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int ch = cw * 32 + 8 * v + 4 * lh;
            const float r0 = ok ? fmaxf(acc1[j][4 * v], 0.f) : 0.f, r1 = ok ? fmaxf(acc1[j][4 * v + 1], 0.f) : 0.f;
            const float r2 = ok ? fmaxf(acc1[j][4 * v + 2], 0.f) : 0.f, r3 = ok ? fmaxf(acc1[j][4 * v + 3], 0.f) : 0.f;
            u32x2_t o = {pack2(r0, r1), pack2(r2, r3)};
            *reinterpret_cast<u32x2_t*>(T1 + r * TP + ch * 2) = o;
        }
    }
    __syncthreads();

    // ------------------------------------------------------------------ phase 2: t2 = relu(W2 * t1 + b2)
    int hb[2];   // halo row of the tap (0, 0) input of this lane's pixel
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int p = (pw + 2 * j) * 32 + l32;
        hb[j] = (p / TW) * HALO_W + (p % TW);
    }
    // Software pipeline, pinned step by step (the scheduler would otherwise run the first RING steps before
    // issuing any refill): step s issues the weight fragment of step s + RING and the t1 operands of step
    // s + 1, then multiplies the operands fetched one step earlier.
    auto t1_frag = [&](int s, int j) {
        const int tap = s / (WD / 16), kk = s % (WD / 16);
        return *reinterpret_cast<const u32x4_t*>(T1 + (hb[j] + (tap / 3) * HALO_W + (tap % 3)) * TP + kk * 32 + lh * 16);
    };
    u32x4_t bq[2][2];
#pragma unroll
    for (int j = 0; j < 2; ++j) bq[0][j] = t1_frag(0, j);
    static_for<0, KS2>([&](auto sc) {
        constexpr int s = decltype(sc)::value;
        const u32x4_t wfrag = ring[s % RING];
        if (s + RING < KS2) ring[s % RING] = w2f[(s + RING) * 64];
        if (s + 1 < KS2) {
#pragma unroll
            for (int j = 0; j < 2; ++j) bq[(s + 1) & 1][j] = t1_frag(s + 1, j);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) mma(acc2[j], wfrag, bq[s & 1][j]);
        __builtin_amdgcn_sched_barrier(0);
    });

    // last-layer weights: requested now, used after the barrier
    u32x4_t w3[2][KS3];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int kk = 0; kk < KS3; ++kk) w3[i][kk] = w3f[(i * KS3 + kk) * 64];
    f32x16_t b3t[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) b3t[i] = bias_tile(a.b3 + wv * 64 + i * 32);
    pin_vmem();
    uint32_t ooff[4][4];   // element offset of the lane's 8 output channels; ~0u = outside the frame
#pragma unroll
    for (int pt = 0; pt < 4; ++pt)
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int item = lane + 64 * it;
            const int p = pt * 32 + (item >> 3), chunk = item & 7;
            const int oy = y0 + p / TW, ox = x0 + p % TW;
            ooff[pt][it] = (oy < a.H && ox < a.W) ? (uint32_t)((oy * a.W + ox) * C4 + wv * 64 + chunk * 8) : ~0u;
        }

#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int p = (pw + 2 * j) * 32 + l32;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int ch = cw * 32 + 8 * v + 4 * lh;
            u32x2_t o = {pack2(fmaxf(acc2[j][4 * v], 0.f), fmaxf(acc2[j][4 * v + 1], 0.f)),
                         pack2(fmaxf(acc2[j][4 * v + 2], 0.f), fmaxf(acc2[j][4 * v + 3], 0.f))};
            *reinterpret_cast<u32x2_t*>(T2 + p * TP + ch * 2) = o;
        }
    }
    __syncthreads();   // t2 complete; t1 and the staging tile are dead from here on

    // ------------------------------------------------------------------ phase 3: y = relu(W3 t2 + b3 + x)
    // this wavefront: output channels 64 wv .. 64 wv + 63 of all 128 pixels, one 32-pixel sub-tile at a time
    // The residual is added in accumulator layout (fp32), the sum is rounded once, and only the bf16 tile goes
    // through the wavefront's LDS region to be re-read as 16-byte runs of 8 channels per lane.
    unsigned char* ep = smem + wv * (32 * EPITCH);
    u32x2_t ypk[TAILN ? 4 : 1][2][4];   // tail layer: the block's rounded output in accumulator layout
    static_for<0, 4>([&](auto ptc) {
        constexpr int pt = decltype(ptc)::value;
        f32x16_t acc3[2] = {b3t[0], b3t[1]};
#pragma unroll
        for (int kk = 0; kk < KS3; ++kk) {
            u32x4_t b;
            if (kk < WD / 16) {
                b = *reinterpret_cast<const u32x4_t*>(T2 + (pt * 32 + l32) * TP + kk * 32 + lh * 16);
            } else {   // FIRST: the centre pixels of x, still resident in the staging tile
                const int p = pt * 32 + l32;
                const int hrow = (p / TW + 1) * HALO_W + (p % TW) + 1;
                b = *reinterpret_cast<const u32x4_t*>(XS + hrow * XP + (kk - WD / 16) * 32 + lh * 16);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) mma(acc3[i], w3[i][kk], b);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                u32x2_t q = {0u, 0u};
                if (!FIRST) q = rres[pt][i][v];
                const float r0 = fmaxf(acc3[i][4 * v] + __uint_as_float(q.x << 16), 0.f);
                const float r1 = fmaxf(acc3[i][4 * v + 1] + __uint_as_float(q.x & 0xffff0000u), 0.f);
                const float r2 = fmaxf(acc3[i][4 * v + 2] + __uint_as_float(q.y << 16), 0.f);
                const float r3 = fmaxf(acc3[i][4 * v + 3] + __uint_as_float(q.y & 0xffff0000u), 0.f);
                u32x2_t o = {pack2(r0, r1), pack2(r2, r3)};
                *reinterpret_cast<u32x2_t*>(ep + l32 * EPITCH + (i * 32 + 8 * v + 4 * lh) * 2) = o;
                if constexpr (TAILN > 0) ypk[pt][i][v] = o;
            }
        __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): the region is private to this wavefront
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int item = lane + 64 * it;
            const u32x4_t o = *reinterpret_cast<const u32x4_t*>(ep + (item >> 3) * EPITCH + (item & 7) * 16);
            if (ooff[pt][it] != ~0u) *reinterpret_cast<u32x4_t*>(yout + ooff[pt][it]) = o;
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_wave_barrier();
    });

    // ------------------------------------------------------------------ phase 4 (optional): z = [relu](Wt y + bt)
    // The output tile is laid out once more in LDS, now as one row of all 4 WD channels per pixel (the MFMA pixel
    // operand of a contraction over those channels); wavefront wv computes output channels TAILN / 4 * wv .. of all
    // 128 pixels with its weight fragments streamed from L2.
    if constexpr (TAILN > 0) {
        constexpr int YP = C4 * 2 + 16;            // row pitch of the output tile (bytes)
        constexpr int NTW = TAILN / 128;           // 32-channel tiles per wavefront
        constexpr int KS4 = C4 / 16;               // k-steps (16)
        constexpr int TRING = 8;                   // k-steps of weight fragments in flight
        constexpr int ZPITCH = NTW * 64 + 16;      // staging row: the wavefront's channels of one pixel + pad (bytes)
        static_assert(NPX * YP <= NHP * (TP + XP) + NPX * TP, "output tile fits in the block's LDS");
        static_assert(4 * 32 * ZPITCH <= NPX * YP, "staging fits");
        unsigned char* Y = smem;
        const u32x4_t* __restrict__ wtf = reinterpret_cast<const u32x4_t*>(a.wtf) + (size_t)(wv * NTW) * KS4 * 64 + lane;
        u32x4_t tring[NTW][TRING];
#pragma unroll
        for (int i = 0; i < NTW; ++i)
#pragma unroll
            for (int k = 0; k < TRING; ++k) tring[i][k] = wtf[(i * KS4 + k) * 64];
        f32x16_t acc4[NTW][4];
#pragma unroll
        for (int i = 0; i < NTW; ++i) {
            acc4[i][0] = bias_tile(a.bt + (wv * NTW + i) * 32);
#pragma unroll
            for (int j = 1; j < 4; ++j) acc4[i][j] = acc4[i][0];
        }
        pin_vmem();
        __syncthreads();   // every wavefront is done with t2 and with its staging region
#pragma unroll
        for (int pt = 0; pt < 4; ++pt)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    *reinterpret_cast<u32x2_t*>(Y + (pt * 32 + l32) * YP + (wv * 64 + i * 32 + 8 * v + 4 * lh) * 2) = ypk[pt][i][v];
        __syncthreads();
        static_for<0, KS4>([&](auto kc) {
            constexpr int kk = decltype(kc)::value;
            u32x4_t wf[NTW];
#pragma unroll
            for (int i = 0; i < NTW; ++i) {
                wf[i] = tring[i][kk % TRING];
                if (kk + TRING < KS4) tring[i][kk % TRING] = wtf[(i * KS4 + kk + TRING) * 64];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const u32x4_t b = *reinterpret_cast<const u32x4_t*>(Y + (j * 32 + l32) * YP + kk * 32 + lh * 16);
#pragma unroll
                for (int i = 0; i < NTW; ++i) mma(acc4[i][j], wf[i], b);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        __syncthreads();   // the output tile is dead: its space becomes the wavefronts' staging regions
        unsigned char* zp = smem + wv * (32 * ZPITCH);
        bf16_t* __restrict__ zout = a.z + (size_t)img * a.H * a.W * TAILN;
        const bool zrelu = a.tail_relu != 0;
        static_for<0, 4>([&](auto ptc) {
            constexpr int pt = decltype(ptc)::value;
#pragma unroll
            for (int i = 0; i < NTW; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float r0 = acc4[i][pt][4 * v], r1 = acc4[i][pt][4 * v + 1], r2 = acc4[i][pt][4 * v + 2], r3 = acc4[i][pt][4 * v + 3];
                    if (zrelu) { r0 = fmaxf(r0, 0.f); r1 = fmaxf(r1, 0.f); r2 = fmaxf(r2, 0.f); r3 = fmaxf(r3, 0.f); }
                    u32x2_t o = {pack2(r0, r1), pack2(r2, r3)};
                    *reinterpret_cast<u32x2_t*>(zp + l32 * ZPITCH + (i * 32 + 8 * v + 4 * lh) * 2) = o;
                }
            __builtin_amdgcn_s_waitcnt(0xc07f);
            __builtin_amdgcn_wave_barrier();
            constexpr int CPP = NTW * 4;           // 16-byte chunks per pixel of this wavefront's channels
#pragma unroll
            for (int it = 0; it < 32 * CPP / 64; ++it) {
                const int item = lane + 64 * it;
                const int pr = item / CPP, chunk = item % CPP;
                const int p = pt * 32 + pr;
                const int oy = y0 + p / TW, ox = x0 + p % TW;
                const u32x4_t o = *reinterpret_cast<const u32x4_t*>(zp + pr * ZPITCH + chunk * 16);
                if (oy < a.H && ox < a.W)
                    *reinterpret_cast<u32x4_t*>(zout + (size_t)(oy * a.W + ox) * TAILN + wv * (32 * NTW) + chunk * 8) = o;
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);
            __builtin_amdgcn_wave_barrier();
        });
    }
}

// ---------------------------------------------------------------------------------------------------
// 128-channel intermediates (identity blocks of the second stage): same tile and phases, other budgets.
// t1 / t2 rows are 256 bytes and are stored unpadded with the 16-byte chunk index XOR-ed with the row
// (t1 46 KB + t2 32 KB, the staging tile shares t2's space: two blocks per CU still fit).  Work split:
//   phase 1  wavefront = 2 channel tiles x 3 pixel tiles (each staged operand feeds two MFMAs),
//   phase 2  wavefront = 1 channel tile x 4 pixel tiles (each weight fragment is fetched by one wavefront only),
//   phase 3  wavefront = 128 output channels as two 64-channel halves x 4 pixel tiles; the residual is
//            re-read from global memory (L2) in 16-byte runs and added after an fp32 transpose through LDS.
__device__ inline int swz256(int row, int byteoff) {   // physical offset in a 256-byte-row swizzled tile
    return row * 256 + ((((byteoff >> 4) ^ row) & 15) << 4) + (byteoff & 15);
}

__global__ __launch_bounds__(256, 2) void bottleneck_fused128_kernel(const FusedBlockArgs a) {
    constexpr int WD = 128, C4 = 512, BK = 64;
    constexpr int XP = BK * 2 + 16;                  // staging tile row pitch (bytes)
    constexpr int KT1 = C4 / BK;                     // 8 phase-1 K steps
    constexpr int KS1 = C4 / 16, KS2 = 9 * WD / 16, KS3 = WD / 16;   // 32, 72, 8
    constexpr int XRING = 2;                         // staged K steps in flight (a third spills registers)
    constexpr int RING = 16;                         // phase-2 weight fragments in flight
    constexpr int EPITCH = 64 * 4 + 16;              // fp32 epilogue row: 64 channels + pad
    constexpr int T1_BYTES = NH * 256;               // 46080
    constexpr int T2_BYTES = NPX * 256;              // 32768 (>= the staging tile)
    static_assert(NHP * XP <= T2_BYTES, "the staging tile shares t2's space");
    static_assert(4 * 32 * EPITCH <= T1_BYTES, "epilogue tiles reuse the t1 area");

    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* T1 = smem;
    unsigned char* XS = smem + T1_BYTES;
    unsigned char* T2 = smem + T1_BYTES;

    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int tiles_x = (a.W + TW - 1) / TW, tiles_y = (a.H + TH - 1) / TH;
    const int total = a.N * tiles_y * tiles_x;
    const int per_xcd = (total + 7) >> 3;
    const int tile = (int)(blockIdx.x & 7u) * per_xcd + (int)(blockIdx.x >> 3);
    if (tile >= total) return;
    const int img = tile / (tiles_y * tiles_x);
    const int trem = tile - img * (tiles_y * tiles_x);
    const int y0 = (trem / tiles_x) * TH, x0 = (trem % tiles_x) * TW;
    const bf16_t* __restrict__ xin = a.x + (size_t)img * a.H * a.W * C4;
    bf16_t* __restrict__ yout = a.y + (size_t)img * a.H * a.W * C4;

    auto bias_tile = [&](const float* b) {
        f32x16_t r;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const f32x4_t q = *reinterpret_cast<const f32x4_t*>(b + 8 * v + 4 * lh);
            r[4 * v] = q.x; r[4 * v + 1] = q.y; r[4 * v + 2] = q.z; r[4 * v + 3] = q.w;
        }
        return r;
    };

    // ------------------------------------------------------------------ phase 1
    const int lc = t & 7, lr = t >> 3;
    uint32_t xoff[6];
#pragma unroll
    for (int p = 0; p < 6; ++p) {
        const int r = lr + 32 * p;
        const int hy = r / HALO_W, hx = r - hy * HALO_W;
        const int iy = min(max(y0 - 1 + hy, 0), a.H - 1), ix = min(max(x0 - 1 + hx, 0), a.W - 1);
        xoff[p] = (uint32_t)((iy * a.W + ix) * C4 + lc * 8);
    }
    const int cp = wv & 1;        // phase 1: channel tiles 2 cp, 2 cp + 1
    const int pw = wv >> 1;       // phase 1: pixel tiles pw, pw + 2, pw + 4
    const u32x4_t* __restrict__ w1f = reinterpret_cast<const u32x4_t*>(a.w1f) + (size_t)(2 * cp) * KS1 * 64 + lane;
    const u32x4_t* __restrict__ w2f = reinterpret_cast<const u32x4_t*>(a.w2f) + (size_t)wv * KS2 * 64 + lane;
    const u32x4_t* __restrict__ w3f = reinterpret_cast<const u32x4_t*>(a.w3f) + (size_t)(4 * wv) * KS3 * 64 + lane;

    u32x4_t xs[XRING][6];
    u32x4_t wa[2][2][BK / 16];   // [buffer][channel tile][k-step of the K step]
    auto load_x = [&](int kt, int slot) {
#pragma unroll
        for (int p = 0; p < 6; ++p) xs[slot][p] = *reinterpret_cast<const u32x4_t*>(xin + xoff[p] + kt * BK);
    };
    auto load_wa = [&](int kt, int buf) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk) wa[buf][i][kk] = w1f[(i * KS1 + kt * (BK / 16) + kk) * 64];
    };
    load_x(0, 0);
    load_wa(0, 0);
    load_x(1, 1);
    static_assert(XRING == 2, "prologue issues two K steps");
    f32x16_t acc1[2][3];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        acc1[i][0] = bias_tile(a.b1 + (2 * cp + i) * 32);
        acc1[i][1] = acc1[i][0];
        acc1[i][2] = acc1[i][0];
    }
    static_for<0, KT1>([&](auto ktc) {
        constexpr int kt = decltype(ktc)::value;
        if (kt > 0) __syncthreads();   // every wavefront is done with the previous staging tile
#pragma unroll
        for (int p = 0; p < 6; ++p) *reinterpret_cast<u32x4_t*>(XS + (lr + 32 * p) * XP + lc * 16) = xs[kt % XRING][p];
        if (kt + XRING < KT1) load_x(kt + XRING, kt % XRING);
        if (kt + 1 < KT1) load_wa(kt + 1, (kt + 1) & 1);
        pin_vmem();
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const u32x4_t b = *reinterpret_cast<const u32x4_t*>(XS + ((pw + 2 * j) * 32 + l32) * XP + kk * 32 + lh * 16);
#pragma unroll
                for (int i = 0; i < 2; ++i) mma(acc1[i][j], wa[kt & 1][i][kk], b);
            }
        }
    });

    // phase-2 prologue: first weight fragments and the bias tile
    u32x4_t ring[RING];
#pragma unroll
    for (int s = 0; s < RING; ++s) ring[s] = w2f[s * 64];
    f32x16_t acc2[4];
    acc2[0] = bias_tile(a.b2 + wv * 32);
    acc2[1] = acc2[0]; acc2[2] = acc2[0]; acc2[3] = acc2[0];
    pin_vmem();

#pragma unroll
    for (int j = 0; j < 3; ++j) {
        const int r = (pw + 2 * j) * 32 + l32;
        const int hy = r / HALO_W, hx = r - hy * HALO_W;
        const int iy = y0 - 1 + hy, ix = x0 - 1 + hx;
        const bool ok = (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
        if (r < NH) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int ch = (2 * cp + i) * 32 + 8 * v + 4 * lh;
                    const float r0 = ok ? fmaxf(acc1[i][j][4 * v], 0.f) : 0.f, r1 = ok ? fmaxf(acc1[i][j][4 * v + 1], 0.f) : 0.f;
                    const float r2 = ok ? fmaxf(acc1[i][j][4 * v + 2], 0.f) : 0.f, r3 = ok ? fmaxf(acc1[i][j][4 * v + 3], 0.f) : 0.f;
                    u32x2_t o = {pack2(r0, r1), pack2(r2, r3)};
                    *reinterpret_cast<u32x2_t*>(T1 + swz256(r, ch * 2)) = o;
                }
        }
    }
    __syncthreads();   // t1 complete; the staging tile is dead (t2 will take its place)

    // ------------------------------------------------------------------ phase 2: channel tile wv, pixel tiles 0..3
    int hb[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int p = j * 32 + l32;
        hb[j] = (p / TW) * HALO_W + (p % TW);
    }
    auto t1_frag = [&](int s, int j) {
        const int tap = s / (WD / 16), kk = s % (WD / 16);
        return *reinterpret_cast<const u32x4_t*>(T1 + swz256(hb[j] + (tap / 3) * HALO_W + (tap % 3), kk * 32 + lh * 16));
    };
    u32x4_t bq[2][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) bq[0][j] = t1_frag(0, j);
    static_for<0, KS2>([&](auto sc) {
        constexpr int s = decltype(sc)::value;
        const u32x4_t wfrag = ring[s % RING];
        if (s + RING < KS2) ring[s % RING] = w2f[(s + RING) * 64];
        if (s + 1 < KS2) {
#pragma unroll
            for (int j = 0; j < 4; ++j) bq[(s + 1) & 1][j] = t1_frag(s + 1, j);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) mma(acc2[j], wfrag, bq[s & 1][j]);
        __builtin_amdgcn_sched_barrier(0);
    });
    // (t2 takes the staging tile's place, which nobody has read since the barrier above; t1 is not touched)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int p = j * 32 + l32;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int ch = wv * 32 + 8 * v + 4 * lh;
            u32x2_t o = {pack2(fmaxf(acc2[j][4 * v], 0.f), fmaxf(acc2[j][4 * v + 1], 0.f)),
                         pack2(fmaxf(acc2[j][4 * v + 2], 0.f), fmaxf(acc2[j][4 * v + 3], 0.f))};
            *reinterpret_cast<u32x2_t*>(T2 + swz256(p, ch * 2)) = o;
        }
    }
    __syncthreads();   // t2 complete; t1 is dead from here on

    // ------------------------------------------------------------------ phase 3: output channels 128 wv .. 128 wv + 127
    unsigned char* ep = smem + wv * (32 * EPITCH);
    uint32_t ooff[4][4];   // element offset of the lane's 8 channels in the first 64-channel half; ~0u = outside the frame
#pragma unroll
    for (int pt = 0; pt < 4; ++pt)
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int item = lane + 64 * it;
            const int p = pt * 32 + (item >> 3), chunk = item & 7;
            const int oy = y0 + p / TW, ox = x0 + p % TW;
            ooff[pt][it] = (oy < a.H && ox < a.W) ? (uint32_t)((oy * a.W + ox) * C4 + wv * 128 + chunk * 8) : ~0u;
        }
    u32x4_t rq[2][4];   // residual of the current and the next (half, pixel tile) step
    auto fetch_res = [&](int step, int slot) {
        const int half = step >> 2, pt = step & 3;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const uint32_t off = ooff[pt][it];
            rq[slot][it] = *reinterpret_cast<const u32x4_t*>(xin + (off == ~0u ? 0u : off + half * 64));
        }
    };
    fetch_res(0, 0);
    static_for<0, 2>([&](auto hc) {
        constexpr int half = decltype(hc)::value;
        u32x4_t w3[2][KS3];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int kk = 0; kk < KS3; ++kk) w3[i][kk] = w3f[((2 * half + i) * KS3 + kk) * 64];
        f32x16_t b3t[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) b3t[i] = bias_tile(a.b3 + wv * 128 + half * 64 + i * 32);
        pin_vmem();
        // the products of pixel tile pt + 1 are issued before the epilogue of pixel tile pt, so that the matrix
        // pipe works while the vector ALUs and LDS transpose, add the residual and store
        f32x16_t acc3[2][2];
        auto products = [&](int pt, int slot) {
            acc3[slot][0] = b3t[0];
            acc3[slot][1] = b3t[1];
#pragma unroll
            for (int kk = 0; kk < KS3; ++kk) {
                const u32x4_t b = *reinterpret_cast<const u32x4_t*>(T2 + swz256(pt * 32 + l32, kk * 32 + lh * 16));
#pragma unroll
                for (int i = 0; i < 2; ++i) mma(acc3[slot][i], w3[i][kk], b);
            }
        };
        products(0, 0);
        static_for<0, 4>([&](auto ptc) {
            constexpr int pt = decltype(ptc)::value;
            constexpr int step = half * 4 + pt;
            if (step + 1 < 8) fetch_res(step + 1, (step + 1) & 1);
            if (pt + 1 < 4) products(pt + 1, (pt + 1) & 1);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    f32x4_t r = {acc3[pt & 1][i][4 * v], acc3[pt & 1][i][4 * v + 1], acc3[pt & 1][i][4 * v + 2], acc3[pt & 1][i][4 * v + 3]};
                    *reinterpret_cast<f32x4_t*>(ep + l32 * EPITCH + (i * 32 + 8 * v + 4 * lh) * 4) = r;
                }
            __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): the region is private to this wavefront
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int item = lane + 64 * it;
                const f32x4_t lo = *reinterpret_cast<const f32x4_t*>(ep + (item >> 3) * EPITCH + (item & 7) * 32);
                const f32x4_t hi = *reinterpret_cast<const f32x4_t*>(ep + (item >> 3) * EPITCH + (item & 7) * 32 + 16);
                const u32x4_t q = rq[step & 1][it];
                u32x4_t o;
                o.x = pack2(fmaxf(lo.x + __uint_as_float(q.x << 16), 0.f), fmaxf(lo.y + __uint_as_float(q.x & 0xffff0000u), 0.f));
                o.y = pack2(fmaxf(lo.z + __uint_as_float(q.y << 16), 0.f), fmaxf(lo.w + __uint_as_float(q.y & 0xffff0000u), 0.f));
                o.z = pack2(fmaxf(hi.x + __uint_as_float(q.z << 16), 0.f), fmaxf(hi.y + __uint_as_float(q.z & 0xffff0000u), 0.f));
                o.w = pack2(fmaxf(hi.z + __uint_as_float(q.w << 16), 0.f), fmaxf(hi.w + __uint_as_float(q.w & 0xffff0000u), 0.f));
                const uint32_t off = ooff[pt][it];
                if (off != ~0u) *reinterpret_cast<u32x4_t*>(yout + off + half * 64) = o;
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);
            __builtin_amdgcn_wave_barrier();
        });
    });
}

bool fused_block_supported(const FusedBlockArgs& a, int width) {
    if (width != 64 && !(width == 128 && !a.first)) return false;   // 128-wide: identity blocks only
    if (!a.x || !a.y || a.x == a.y || !a.w1f || !a.w2f || !a.w3f || !a.b1 || !a.b2 || !a.b3) return false;
    if (a.tail_n != 0) {   // tail layer: 64-wide identity blocks, 128 or 256 outputs
        if (width != 64 || a.first || (a.tail_n != 128 && a.tail_n != 256) || !a.wtf || !a.bt || !a.z || a.z == a.y || a.z == a.x) return false;
    }
    if (a.N <= 0 || a.H <= 0 || a.W <= 0) return false;
    if ((long long)a.H * a.W * 4 * width >= (1ll << 31)) return false;   // 32-bit element offsets within a frame
    const long long tiles = (long long)a.N * ((a.H + TH - 1) / TH) * ((a.W + TW - 1) / TW);
    return tiles < (1ll << 30);
}

template <typename Kern>
static hipError_t launch_fused_kernel(Kern kern, size_t lds, const FusedBlockArgs& a, hipStream_t s) {
    {
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
        if (e != hipSuccess) return e;
    }
    const long long tiles = (long long)a.N * ((a.H + TH - 1) / TH) * ((a.W + TW - 1) / TW);
    const long long grid = ((tiles + 7) / 8) * 8;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, s, a);
    return hipGetLastError();
}

hipError_t launch_fused_block(const FusedBlockArgs& a, int width, hipStream_t s) {
    if (!fused_block_supported(a, width)) return hipErrorInvalidValue;
    constexpr size_t lds64 = (size_t)NHP * ((64 * 2 + 16) + (64 * 2 + 16)) + (size_t)NPX * (64 * 2 + 16);
    constexpr size_t lds128 = (size_t)NH * 256 + (size_t)NPX * 256;
    if (width == 128) return launch_fused_kernel(bottleneck_fused128_kernel, lds128, a, s);
    if (a.tail_n == 128) return launch_fused_kernel(bottleneck_fused_kernel<64, false, 128>, lds64, a, s);
    if (a.tail_n == 256) return launch_fused_kernel(bottleneck_fused_kernel<64, false, 256>, lds64, a, s);
    if (a.first) return launch_fused_kernel(bottleneck_fused_kernel<64, true>, lds64, a, s);
    return launch_fused_kernel(bottleneck_fused_kernel<64, false>, lds64, a, s);
}

// Host-side packing of a [Cout][K] bf16 weight matrix (K contiguous) into MFMA fragment order:
// fragment (ct, ks) is 64 lanes x 8 elements, lane l holding W[32 ct + l % 32][16 ks + 8 (l / 32) .. + 7].
void pack_mfma_fragments(const bf16_t* w, int Cout, int K, bf16_t* dst) {
    const int KS = K / 16;
    for (int ct = 0; ct < Cout / 32; ++ct)
        for (int ks = 0; ks < KS; ++ks)
            for (int l = 0; l < 64; ++l)
                for (int e = 0; e < 8; ++e)
                    dst[(((size_t)ct * KS + ks) * 64 + l) * 8 + e] = w[(size_t)(ct * 32 + l % 32) * K + ks * 16 + 8 * (l / 32) + e];
}

}  // namespace thia
