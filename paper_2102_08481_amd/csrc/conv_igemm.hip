// Implicit-GEMM convolution on the CDNA4 matrix cores (gfx950).
//
// Every convolution and fully connected layer of the detector (bottleneck 1x1/3x3,
// shortcut, exit lateral, RPN 3x3 and heads, FC layers and predictors) is the
// contraction  out[m, n] = sum_k W[n, k] * X[m, k]  with m = (image, oy, ox),
// n = output channel and k = (ky, kx, ci); activations are NHWC so a K tile of one
// filter tap is a contiguous run of input channels of one input pixel.
//
// Tiling: a 256-thread block (4 wavefronts of 64) owns 128 pixels x BN channels and
// walks K in 128-byte steps (64 bf16 / 32 fp32 per row).  Global loads are 16 bytes
// per lane, staged in registers and written to a double-buffered LDS tile whose rows
// are padded to 144 bytes so that the 16-byte fragment reads of 32 consecutive rows
// fall in distinct banks.  Each wavefront owns 64 pixels x BN/2 channels as 32x32 MFMA
// tiles.  The weights are the MFMA "A" operand (rows = channels) and the activations the
// "B" operand (columns = pixels): each lane then holds 4 consecutive channels of one
// pixel per accumulator quad, which is the contiguous direction of the NHWC output.
// Epilogue: + bias (fp32) [+ residual] [ReLU], then one rounding to the output type.
#include <type_traits>

#include "thia_internal.h"

namespace thia {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;


template <typename T>
__device__ inline void mma_step(f32x16_t& acc, const u32x4_t& a, const u32x4_t& b);

template <>
__device__ inline void mma_step<bf16_t>(f32x16_t& acc, const u32x4_t& a, const u32x4_t& b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), acc, 0, 0, 0);
}
template <>
__device__ inline void mma_step<float>(f32x16_t& acc, const u32x4_t& a, const u32x4_t& b) {
    // 16 bytes = 4 consecutive k per lane half; MFMA step j contracts k = {j, 4 + j} of the 8-wide group
    const f32x4_t fa = __builtin_bit_cast(f32x4_t, a), fb = __builtin_bit_cast(f32x4_t, b);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.x, fb.x, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.y, fb.y, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.z, fb.z, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.w, fb.w, acc, 0, 0, 0);
}

__device__ inline float load_elem(const float* p) { return *p; }
__device__ inline float load_elem(const bf16_t* p) { return bf16_to_f32(*p); }
__device__ inline void store_elem(float* p, float v) { *p = v; }
__device__ inline void store_elem(bf16_t* p, float v) { *p = (bf16_t)pack_bf16x2(v, 0.f); }

__device__ inline void load4(const float* p, float r[4]) {
    const f32x4_t v = *reinterpret_cast<const f32x4_t*>(p);
    r[0] = v.x; r[1] = v.y; r[2] = v.z; r[3] = v.w;
}
__device__ inline void load4(const bf16_t* p, float r[4]) {
    const u32x2_t v = *reinterpret_cast<const u32x2_t*>(p);
    r[0] = __uint_as_float(v.x << 16); r[1] = __uint_as_float(v.x & 0xffff0000u);
    r[2] = __uint_as_float(v.y << 16); r[3] = __uint_as_float(v.y & 0xffff0000u);
}
__device__ inline void store4(float* p, const float r[4]) {
    f32x4_t v = {r[0], r[1], r[2], r[3]};
    *reinterpret_cast<f32x4_t*>(p) = v;
}
__device__ inline void store4(bf16_t* p, const float r[4]) {
    u32x2_t v;
    v.x = pack_bf16x2(r[0], r[1]);
    v.y = pack_bf16x2(r[2], r[3]);
    *reinterpret_cast<u32x2_t*>(p) = v;
}

// 8 consecutive elements of T as one register bundle
template <typename T> struct Vec8;
template <> struct __attribute__((aligned(16))) Vec8<bf16_t> { u32x4_t v; };
template <> struct __attribute__((aligned(16))) Vec8<float> { f32x4_t lo, hi; };
__device__ inline void unpack8(const Vec8<bf16_t>& x, float r[8]) {
    const uint32_t w[4] = {x.v.x, x.v.y, x.v.z, x.v.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) { r[2 * q] = __uint_as_float(w[q] << 16); r[2 * q + 1] = __uint_as_float(w[q] & 0xffff0000u); }
}
__device__ inline void unpack8(const Vec8<float>& x, float r[8]) {
    r[0] = x.lo.x; r[1] = x.lo.y; r[2] = x.lo.z; r[3] = x.lo.w; r[4] = x.hi.x; r[5] = x.hi.y; r[6] = x.hi.z; r[7] = x.hi.w;
}
__device__ inline void store8(bf16_t* p, const float r[8]) {
    u32x4_t v;
    v.x = pack_bf16x2(r[0], r[1]);
    v.y = pack_bf16x2(r[2], r[3]);
    v.z = pack_bf16x2(r[4], r[5]);
    v.w = pack_bf16x2(r[6], r[7]);
    *reinterpret_cast<u32x4_t*>(p) = v;
}
__device__ inline void store8(float* p, const float r[8]) {
    f32x4_t lo = {r[0], r[1], r[2], r[3]}, hi = {r[4], r[5], r[6], r[7]};
    *reinterpret_cast<f32x4_t*>(p) = lo;
    *reinterpret_cast<f32x4_t*>(p + 4) = hi;
}

// 16 bytes per lane from global memory straight into LDS: lane l's bytes land at lds + 16 l (lds is uniform over the
// wavefront).  Counted by vmcnt like any vector memory load.  (The builtin exists in the device pass only.)
__device__ inline void load_to_lds16(const void* g, void* lds) {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_global_load_lds(g, lds, 16, 0, 0);
#endif
}

// 16 zero bytes (and some more) in global memory: what a padded filter tap fetches on the direct-to-LDS path
__device__ __align__(256) unsigned char g_zero_page[256];

// compile-time loop: the body sees the index as a constant (keeps accumulator indices static)
template <int I, int N, typename F>
__device__ inline void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// MODE 0: any filter size; 1: 1x1 unpadded (no tap bookkeeping); 2: 1x1 with a second source tensor;
// 4: any filter size, followed by the expansion tail (ConvArgs::tail_*) on the block's output tile.
template <typename T, int BM, int BN, int BKB, int WAVES_M, int WAVES_N, int MODE, typename OutT>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void conv_igemm_kernel(const ConvArgs a) {
    constexpr bool ONE = MODE == 1 || MODE == 2, DUAL = MODE == 2;
    constexpr int NT = 64 * WAVES_M * WAVES_N;  // threads per block
    constexpr int BK = BKB / (int)sizeof(T);   // K elements per tile row
    constexpr int EPC = 16 / (int)sizeof(T);   // elements per 16-byte chunk
    constexpr int CPR = BKB / 16;              // 16-byte chunks per tile row
    constexpr int RPP = NT / CPR;              // tile rows covered by one pass of the block's threads
    constexpr int PB = BM / RPP, PA = BN / RPP;  // chunks staged per thread (activations, weights)
    // DIRECT (128-byte K rows): operand tiles go from global memory straight into LDS (global_load_lds_dwordx4: lane l of
    // a wavefront instruction lands at the instruction's LDS base + 16 l, i.e. one instruction fills 8 whole tile rows),
    // without staging registers or LDS-write instructions.  Rows are unpadded; instead a lane fetches the 16-byte chunk
    // (slot ^ swz(row)) of its row, swz(row) = (row & 7) ^ ((row >> 3) & 1), so that the fragment reads of 16 consecutive
    // rows at one logical chunk fall on 16 different 16-byte slots modulo 256 bytes (and any 8 aligned rows on 8 modulo 128).
    constexpr bool DIRECT = BKB == 128;
    constexpr int LDS_ROW = DIRECT ? BKB : BKB + 16;   // staged path: padded row pitch (an odd multiple of 16 bytes)
    constexpr int KK = BKB / 32;               // MFMA k-steps per tile row (32 bytes = 2 lane halves x 16 bytes)
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wavefront tile (pixels x channels)
    constexpr int TM = WM / 32, TN = WN / 32;  // 32x32 MFMA tiles per wavefront
    constexpr int LPP = WN / 8;                // epilogue: lanes per pixel (8 channels each)
    constexpr int PPI = 64 / LPP;              // epilogue: pixels per wavefront instruction
    constexpr int NIT = 32 / PPI;              // epilogue: instructions per 32-pixel sub-tile
    constexpr int EPITCH = WN * 4 + 16;        // epilogue: padded fp32 row pitch in LDS (bytes)
    constexpr bool PREFETCH_RES = TM * NIT <= 8;  // residual tile small enough to hold across the K loop
    static_assert(WAVES_M * WAVES_N * 32 * EPITCH <= 2 * (BN + BM) * LDS_ROW, "epilogue tile must fit in the pipeline buffers");
    static_assert(!DIRECT || (CPR == 8 && (NT / 64) % 2 == 0), "direct loads: 8 chunks per row, an even number of wavefronts");
    static_assert(BM % RPP == 0 && BN % RPP == 0, "tile rows must be a multiple of the rows staged per pass");

    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* sA = smem;                     // [2][BN][LDS_ROW]
    unsigned char* sB = smem + 2 * BN * LDS_ROW;  // [2][BM][LDS_ROW]

    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int wm = wv % WAVES_M, wn = wv / WAVES_M;
    const int HoWo = a.Ho * a.Wo;
    const int M = a.N * HoWo;
    const int K = a.kh * a.kw * a.Cin + (DUAL ? a.Cin2 : 0);
    const int tiles_n = (a.Cout + BN - 1) / BN;
    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): give every XCD a
    // contiguous range of tiles so that tiles sharing an activation tile hit the same L2.
    const int total_tiles = ((M + BM - 1) / BM) * tiles_n;
    const int per_xcd = (total_tiles + 7) >> 3;
    const int tile = (int)(blockIdx.x & 7u) * per_xcd + (int)(blockIdx.x >> 3);
    if (tile >= total_tiles) return;
    const int tile_n = tile % tiles_n, tile_m = tile / tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const T* __restrict__ in = static_cast<const T*>(a.in);
    const T* __restrict__ wgt = static_cast<const T*>(a.w);

    // ---- per-thread load coordinates: tile row lrow + RPP*p, 16-byte chunk lchunk of the row
    const int lrow = t / CPR;
    // staged path: the thread's chunk of the row; direct path: the chunk whose LDS slot is t % CPR (see DIRECT above;
    // row & 7 = lane / 8 and (row >> 3) & 1 = wavefront & 1 for every row lrow + RPP * p of this thread)
    const int lchunk = DIRECT ? ((t % CPR) ^ ((lane >> 3) ^ (wv & 1))) & 7 : t % CPR;
    // weight rows first: they need no pixel arithmetic, and on the direct path the first K tile's weight requests go out
    // before the (division-heavy) pixel coordinates are worked out
    size_t a_base[PA];
    bool a_ok[PA];
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        const int n = n0 + lrow + RPP * p;
        a_ok[p] = n < a.Cout;
        a_base[p] = (size_t)(a_ok[p] ? n : 0) * K + (size_t)lchunk * EPC;
    }
    if constexpr (DIRECT) {
        unsigned char* dA0 = sA + (size_t)((wv * 64) / CPR) * LDS_ROW;
#pragma unroll
        for (int p = 0; p < PA; ++p) load_to_lds16(wgt + a_base[p], dA0 + (size_t)(RPP * p) * LDS_ROW);
    }
    size_t b_base[PB];
    size_t b_base2[DUAL ? PB : 1];
    const T* __restrict__ in2 = static_cast<const T*>(a.in2);
    // general filters: signed element offset of the (tap 0, channel 0) input of the row's pixel and, per filter tap, one
    // bit "tap lies inside the image" (kh * kw <= 32)
    long long b_off0[ONE ? 1 : PB];
    uint32_t b_taps[ONE ? 1 : PB];
    bool b_ok[PB];
    // (image, row, column) of the thread's first tile row by division; its other rows are RPP pixels further on each and
    // are reached by stepping (a few carries) unless the output rows are very short
    int s_img, s_oy, s_ox;
    {
        const int m = m0 + lrow;
        const int mm = m < M ? m : 0;
        s_img = mm / HoWo;
        const int rem = mm - s_img * HoWo;
        s_oy = rem / a.Wo;
        s_ox = rem - s_oy * a.Wo;
    }
    const bool step_rows = a.Wo >= 16;
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        const int m = m0 + lrow + RPP * p;
        b_ok[p] = m < M;
        int img, oy, ox;
        if (p == 0 || !b_ok[p]) {   // (rows beyond M are clamped to row 0: they only feed outputs that are never stored)
            img = b_ok[p] ? s_img : 0; oy = b_ok[p] ? s_oy : 0; ox = b_ok[p] ? s_ox : 0;
        } else if (step_rows) {
            s_ox += RPP;
            while (s_ox >= a.Wo) { s_ox -= a.Wo; ++s_oy; }
            while (s_oy >= a.Ho) { s_oy -= a.Ho; ++s_img; }
            img = s_img; oy = s_oy; ox = s_ox;
        } else {
            img = m / HoWo;
            const int rem = m - img * HoWo;
            oy = rem / a.Wo;
            ox = rem - oy * a.Wo;
        }
        const int iy0 = oy * a.stride - a.pad, ix0 = ox * a.stride - a.pad;
        b_base[p] = (size_t)img * a.H * a.W * a.Cin + (size_t)lchunk * EPC;
        // 1x1, unpadded: the row's input pixel is fixed for the whole K loop
        if constexpr (ONE) {
            b_base[p] += ((size_t)iy0 * a.W + ix0) * a.Cin;
        } else {
            b_off0[p] = (long long)b_base[p] + ((long long)iy0 * a.W + ix0) * a.Cin;
            // tap (ky, kx) lies inside the image iff row iy0 + ky and column ix0 + kx do
            uint32_t cols = 0;
            for (int kx = 0; kx < a.kw; ++kx) cols |= ((unsigned)(ix0 + kx) < (unsigned)a.W) ? (1u << kx) : 0u;
            uint32_t bits = 0;
            for (int ky = 0; ky < a.kh; ++ky) bits |= ((unsigned)(iy0 + ky) < (unsigned)a.H) ? (cols << (ky * a.kw)) : 0u;
            b_taps[p] = bits;
        }
        if constexpr (DUAL)
            b_base2[p] = (((size_t)img * a.H2 + (size_t)oy * a.stride2) * a.W2 + (size_t)ox * a.stride2) * a.Cin2 + (size_t)lchunk * EPC;
    }
    const int cin_tiles = a.Cin / BK;
    const int KT = K / BK;

    // zmask: bit p set = activation chunk p is a padded tap and is written to LDS as zeros.  (The select is applied at
    // the LDS write, one step after the load: applied right after the load it would make every step wait for its data.)
    struct Stage { u32x4_t a[PA]; u32x4_t b[PB]; uint32_t zmask; };
    Stage st0;
    auto load_tiles = [&](int kt, Stage& st) {
        // All loads are unconditional: rows beyond M / Cout are clamped to row 0 (they only feed outputs that are
        // never stored), padded filter taps are fetched from a valid in-image address and zeroed at the LDS write.
        st.zmask = 0;
        if constexpr (ONE) {
            const int kt1 = a.Cin / BK;  // K tiles of the first source
            if (!DUAL || kt < kt1) {
#pragma unroll
                for (int p = 0; p < PB; ++p) st.b[p] = *reinterpret_cast<const u32x4_t*>(in + b_base[p] + (size_t)kt * BK);
            } else {
#pragma unroll
                for (int p = 0; p < PB; ++p)
                    st.b[p] = *reinterpret_cast<const u32x4_t*>(in2 + b_base2[DUAL ? p : 0] + (size_t)(kt - kt1) * BK);
            }
#pragma unroll
            for (int p = 0; p < PA; ++p) st.a[p] = *reinterpret_cast<const u32x4_t*>(wgt + a_base[p] + (size_t)kt * BK);
            return;
        }
        const int tap = kt / cin_tiles;
        const int c0 = (kt - tap * cin_tiles) * BK;
        const int ky = tap / a.kw, kx = tap - ky * a.kw;
        const long long tap_off = ((long long)ky * a.W + kx) * a.Cin + c0;   // uniform over the block
        uint32_t zm = 0;
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            const bool ok = (b_taps[ONE ? 0 : p] >> tap) & 1u;
            // a padded tap reads the row's (always valid) image base instead and is replaced by zeros at the LDS write
            const long long off = ok ? b_off0[ONE ? 0 : p] + tap_off : (long long)b_base[p];
            st.b[p] = *reinterpret_cast<const u32x4_t*>(in + off);
            zm |= ok ? 0u : (1u << p);
        }
        st.zmask = zm;
#pragma unroll
        for (int p = 0; p < PA; ++p) st.a[p] = *reinterpret_cast<const u32x4_t*>(wgt + a_base[p] + (size_t)kt * BK);
    };
    auto store_tiles = [&](int buf, const Stage& st) {
#pragma unroll
        for (int p = 0; p < PA; ++p)
            *reinterpret_cast<u32x4_t*>(sA + (size_t)(buf * BN + lrow + RPP * p) * LDS_ROW + lchunk * 16) = st.a[p];
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            const u32x4_t z = {0u, 0u, 0u, 0u};
            const u32x4_t v = (!ONE && ((st.zmask >> p) & 1u)) ? z : st.b[p];
            *reinterpret_cast<u32x4_t*>(sB + (size_t)(buf * BM + lrow + RPP * p) * LDS_ROW + lchunk * 16) = v;
        }
    };

    // direct path: request K tile kt into LDS buffer buf (PA + PB wavefront instructions, each filling 8 rows)
    auto issue_tiles = [&](int kt, int buf) {
        unsigned char* dA = sA + (size_t)(buf * BN + (wv * 64) / CPR) * LDS_ROW;
        unsigned char* dB = sB + (size_t)(buf * BM + (wv * 64) / CPR) * LDS_ROW;
        if constexpr (ONE) {
            const int kt1 = a.Cin / BK;  // K tiles of the first source
            if (!DUAL || kt < kt1) {
#pragma unroll
                for (int p = 0; p < PB; ++p)
                    load_to_lds16(in + b_base[p] + (size_t)kt * BK, dB + (size_t)(RPP * p) * LDS_ROW);
            } else {
#pragma unroll
                for (int p = 0; p < PB; ++p)
                    load_to_lds16(in2 + b_base2[DUAL ? p : 0] + (size_t)(kt - kt1) * BK, dB + (size_t)(RPP * p) * LDS_ROW);
            }
        } else {
            const int tap = kt / cin_tiles;
            const int c0 = (kt - tap * cin_tiles) * BK;
            const int ky = tap / a.kw, kx = tap - ky * a.kw;
            const long long tap_off = ((long long)ky * a.W + kx) * a.Cin + c0;   // uniform over the block
#pragma unroll
            for (int p = 0; p < PB; ++p) {
                // a padded tap reads 16 zero bytes instead
                const bool ok = (b_taps[ONE ? 0 : p] >> tap) & 1u;
                const T* src = ok ? in + (b_off0[ONE ? 0 : p] + tap_off) : reinterpret_cast<const T*>(g_zero_page);
                load_to_lds16(src, dB + (size_t)(RPP * p) * LDS_ROW);
            }
        }
        if (kt == 0) return;   // the first tile's weight rows were requested at the top of the kernel
#pragma unroll
        for (int p = 0; p < PA; ++p)
            load_to_lds16(wgt + a_base[p] + (size_t)kt * BK, dA + (size_t)(RPP * p) * LDS_ROW);
    };

    f32x16_t acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // 8-channel-per-lane epilogue needs Cout, ld0 multiples of 8 and one dense output
    const bool vec = (a.out1 == nullptr) && ((a.Cout & 7) == 0) && ((a.ld0 & 7) == 0);
    const T* __restrict__ res = static_cast<const T*>(a.res);
    Vec8<T> rres[PREFETCH_RES ? TM * NIT : 1];
    if (PREFETCH_RES && vec && res != nullptr) {  // residual tile: issued now, consumed after the K loop
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int pix = m0 + wm * WM + j * 32 + it * PPI + lane / LPP, ch = n0 + wn * WN + (lane % LPP) * 8;
                if (pix < M && ch < a.Cout) rres[PREFETCH_RES ? j * NIT + it : 0] = *reinterpret_cast<const Vec8<T>*>(res + (size_t)pix * a.Cout + ch);
            }
    }

    const int frag_row = lane & 31, frag_off = (lane >> 5) * 16;
    // direct path: slot of logical chunk c in this lane's fragment row is c ^ frag_swz (tile row offsets are multiples of 16)
    const int frag_swz = (frag_row & 7) ^ ((frag_row >> 3) & 1);
    struct Frags { u32x4_t a[TN], b[TM]; };
    auto read_frags = [&](int buf, int kk, Frags& f) {
        const int koff = DIRECT ? ((2 * kk + (lane >> 5)) ^ frag_swz) * 16 : kk * 32 + frag_off;
#pragma unroll
        for (int i = 0; i < TN; ++i)
            f.a[i] = *reinterpret_cast<const u32x4_t*>(sA + (size_t)(buf * BN + wn * WN + i * 32 + frag_row) * LDS_ROW + koff);
#pragma unroll
        for (int j = 0; j < TM; ++j)
            f.b[j] = *reinterpret_cast<const u32x4_t*>(sB + (size_t)(buf * BM + wm * WM + j * 32 + frag_row) * LDS_ROW + koff);
    };
    auto mma_frags = [&](const Frags& f) {
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j) mma_step<T>(acc[i][j], f.a[i], f.b[j]);
    };
    auto compute = [&](int buf) {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            Frags f;
            read_frags(buf, kk, f);
            mma_frags(f);
        }
    };

    // Software pipeline: while tile kt is multiplied out of LDS buffer kt&1, the loads of tile kt+1 are
    // in flight into registers; they are written to the other buffer at the end of the step.  (A second
    // register stage was measured: it costs the second resident block per CU and is slower.  Cycle stamps on
    // the 256 x 256 tile: of ~4700 cycles per step ~1800 go to issuing the 8 loads per thread - the CU's one
    // address unit takes ~20 cycles per 1 KiB instruction and a wavefront issues in order - but spreading the
    // loads between the MFMAs of the step, pinned with scheduling barriers, was measured 3-8 % slower, also
    // with the two wavefronts of a SIMD taking turns.)
    if constexpr (DIRECT) {
        // Two LDS buffers: tile kt + 1 is requested as soon as every wavefront has finished reading its buffer (the
        // barrier that ends step kt - 1) and has the whole of step kt to arrive.
        // The fragments of k-step kk + 1 are read while k-step kk is multiplied, and the barrier sits in front of a
        // tile's LAST k-step: by then every wavefront has read the whole tile (so its buffer can be refilled) and still
        // has a k-step of matrix work queued, which covers the first fragment reads of the next tile.
        static_assert(KK % 2 == 0, "the fragment double buffer alternates per k-step");
        issue_tiles(0, 0);
        __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0)
        __syncthreads();
        if (KT > 1) issue_tiles(1, 1);
        Frags f0, f1;
        read_frags(0, 0, f0);
        for (int kt = 0; kt < KT; ++kt) {
            const int buf = kt & 1;
            static_for<0, KK - 1>([&](auto kc) {
                constexpr int kk = decltype(kc)::value;
                read_frags(buf, kk + 1, (kk & 1) ? f0 : f1);
                mma_frags((kk & 1) ? f1 : f0);
            });
            __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): this thread's part of tile kt + 1 is in LDS
            __syncthreads();
            if (kt + 2 < KT) issue_tiles(kt + 2, buf);
            if (kt + 1 < KT) read_frags(buf ^ 1, 0, f0);
            mma_frags(f1);
        }
    } else {
    load_tiles(0, st0);
    store_tiles(0, st0);
    if (KT > 1) load_tiles(1, st0);
    __syncthreads();
    // The requests for tile kt + 2 go out right after the LDS write of tile kt + 1 has freed the staging
    // registers, so the data has a whole step to arrive.  With 8 wavefronts the two that share a SIMD (w and
    // w + 4) do this staging at opposite ends of the step - one before its MFMAs, one after - so that one of them
    // multiplies while the other writes LDS and queues at the CU's address unit (issued by all wavefronts at
    // once right after the barrier, the loads cost ~1300 of ~4100 cycles per step with the matrix pipe idle).
    const bool stage_first = NT == 512 && (wv >> 2) == 1;
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (stage_first) {
            if (kt + 1 < KT) store_tiles(buf ^ 1, st0);
            if (kt + 2 < KT) load_tiles(kt + 2, st0);
        }
        // the wavefront that multiplies wins issue arbitration over the SIMD's other wavefront, which is staging
        // (LDS writes, global loads) at that moment: measured 0.5-1 % on the whole sweep
        __builtin_amdgcn_s_setprio(3);
        compute(buf);
        __builtin_amdgcn_s_setprio(0);
        if (!stage_first) {
            if (kt + 1 < KT) store_tiles(buf ^ 1, st0);
            if (kt + 2 < KT) load_tiles(kt + 2, st0);
        }
        __syncthreads();
    }
    }

    // ---- fused RPN predictors (large bf16 tile only): the block's ReLU'd 256 x 256 tile, rounded to bf16 as the
    // stored tensor would be, stays in LDS and is contracted with the 1x1 predictor weights right away.
    if constexpr (std::is_same<T, bf16_t>::value && std::is_same<OutT, bf16_t>::value && BM == 256 && BN == 256 && WAVES_M == 2 &&
                  WAVES_N == 4 && MODE == 0) {
        if (a.head_w != nullptr) {
            constexpr int YP = BN * 2 + 16;            // LDS row pitch of the bf16 tile
            constexpr int HKS = BN / 16;               // k-steps of the predictor contraction (16)
            constexpr int HP = 96 * 4 + 16;            // fp32 row pitch of the per-wavefront output tile
            static_assert(BM * YP <= 160 * 1024 && 32 * HP <= 32 * YP, "tile and output staging fit (launch_cfg requests BM * YP bytes)");
            const u32x4_t* __restrict__ hwf = reinterpret_cast<const u32x4_t*>(a.head_w) + lane;
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int i = 0; i < TN; ++i)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int ch = wn * WN + i * 32 + 8 * v + 4 * (lane >> 5);
                        const f32x4_t bv = *reinterpret_cast<const f32x4_t*>(a.bias + n0 + ch);
                        u32x2_t o = {pack_bf16x2(fmaxf(acc[i][j][4 * v] + bv.x, 0.f), fmaxf(acc[i][j][4 * v + 1] + bv.y, 0.f)),
                                     pack_bf16x2(fmaxf(acc[i][j][4 * v + 2] + bv.z, 0.f), fmaxf(acc[i][j][4 * v + 3] + bv.w, 0.f))};
                        *reinterpret_cast<u32x2_t*>(smem + (size_t)(wm * WM + j * 32 + frag_row) * YP + ch * 2) = o;
                    }
            // predictor weight fragments (3 channel tiles per k-step) run HRING k-steps ahead of their use; the first
            // ones and the bias tile are requested once the accumulators are parked, in flight across the barrier
            constexpr int HRING = 4;   // (8 spills and is slower)
            __builtin_amdgcn_sched_barrier(0);   // (hoisted above the parking loop they would spill)
            u32x4_t hw[HRING * 3];
#pragma unroll
            for (int ks = 0; ks < HRING; ++ks)
#pragma unroll
                for (int i = 0; i < 3; ++i) hw[ks * 3 + i] = hwf[(i * HKS + ks) * 64];
            f32x16_t hacc[3];
#pragma unroll
            for (int i = 0; i < 3; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const f32x4_t q = *reinterpret_cast<const f32x4_t*>(a.head_b + i * 32 + 8 * v + 4 * (lane >> 5));
                    hacc[i][4 * v] = q.x; hacc[i][4 * v + 1] = q.y; hacc[i][4 * v + 2] = q.z; hacc[i][4 * v + 3] = q.w;
                }
            __syncthreads();
            // wavefront wv: pixels 32 wv .. 32 wv + 31 of the tile against all 96 (padded) predictor rows
            const unsigned char* yrow = smem + (size_t)(wv * 32 + frag_row) * YP + frag_off;
            static_for<0, HKS>([&](auto kc) {
                constexpr int ks = decltype(kc)::value;
                const u32x4_t b = *reinterpret_cast<const u32x4_t*>(yrow + ks * 32);
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    mma_step<T>(hacc[i], hw[(ks % HRING) * 3 + i], b);
                    if (ks + HRING < HKS) hw[(ks % HRING) * 3 + i] = hwf[(i * HKS + ks + HRING) * 64];
                }
                __builtin_amdgcn_sched_barrier(0);
            });
            // the wavefront's own 32 rows of the tile are dead now: fp32 results go there, then out in dense rows
            unsigned char* hp = smem + (size_t)(wv * 32) * YP;
            __builtin_amdgcn_s_waitcnt(0xc07f);
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int i = 0; i < 3; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    f32x4_t r = {hacc[i][4 * v], hacc[i][4 * v + 1], hacc[i][4 * v + 2], hacc[i][4 * v + 3]};
                    *reinterpret_cast<f32x4_t*>(hp + (size_t)frag_row * HP + (i * 32 + 8 * v + 4 * (lane >> 5)) * 4) = r;
                }
            __builtin_amdgcn_s_waitcnt(0xc07f);
            __builtin_amdgcn_wave_barrier();
            const int A = a.head_a;
            const int mbase = m0 + wv * 32;
            for (int e = lane; e < 32 * A; e += 64) {
                const int px = e / A, q = e - px * A;
                if (mbase + px >= M) continue;
                const f32x4_t d = *reinterpret_cast<const f32x4_t*>(hp + (size_t)px * HP + q * 16);
                *reinterpret_cast<f32x4_t*>(a.head_deltas + ((size_t)(mbase + px) * A + q) * 4) = d;
                a.head_logits[(size_t)(mbase + px) * A + q] = *reinterpret_cast<const float*>(hp + (size_t)px * HP + (4 * A + q) * 4);
            }
            return;
        }
    }

    // ---- expansion tail (large bf16 tile only): the block's ReLU'd 256 x 256 tile, rounded to bf16 as the stored tensor
    // would be, is parked in LDS (unpadded 512-byte rows, 16-byte chunk index XOR-ed with the row) and contracted with the
    // next 1x1 layer's weights (fragment order, streamed from L2).  Wavefront wv owns output channels tail_n / 8 * wv ..
    // and walks them 64 at a time over the two 128-pixel halves of the tile.  Residual and result pass through a 4 KB
    // wavefront-private LDS region as bf16 (32 pixels x 64 channels), so that global loads and stores are 16 bytes per
    // lane and cover whole 128-byte lines; the sum is formed in accumulator layout in fp32 and rounded once.
    if constexpr (std::is_same<T, bf16_t>::value && std::is_same<OutT, bf16_t>::value && BM == 256 && BN == 256 && WAVES_M == 2 &&
                  WAVES_N == 4 && MODE == 4) {
        constexpr int TKS = BN / 16;               // k-steps of the tail contraction (16)
        constexpr int TR = 4;                      // k-steps of weight fragments in flight
        const int lh = lane >> 5;
        auto yoff = [](int row, int byteoff) { return row * 512 + ((((byteoff >> 4) ^ row) & 31) << 4) + (byteoff & 15); };
        auto roff = [](int row, int byteoff) { return row * 128 + ((((byteoff >> 4) ^ row) & 7) << 4) + (byteoff & 15); };
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int ch = wn * WN + i * 32 + 8 * v + 4 * lh;
                    const f32x4_t bv = *reinterpret_cast<const f32x4_t*>(a.bias + n0 + ch);
                    u32x2_t o = {pack_bf16x2(fmaxf(acc[i][j][4 * v] + bv.x, 0.f), fmaxf(acc[i][j][4 * v + 1] + bv.y, 0.f)),
                                 pack_bf16x2(fmaxf(acc[i][j][4 * v + 2] + bv.z, 0.f), fmaxf(acc[i][j][4 * v + 3] + bv.w, 0.f))};
                    *reinterpret_cast<u32x2_t*>(smem + yoff(wm * WM + j * 32 + frag_row, ch * 2)) = o;
                }
        __syncthreads();
        const int N3 = a.tail_n, ctw = N3 / 256;   // 32-channel tiles per wavefront
        const u32x4_t* __restrict__ twf = reinterpret_cast<const u32x4_t*>(a.tail_w) + lane;
        const T* __restrict__ tres = static_cast<const T*>(a.tail_res);
        T* __restrict__ tout = static_cast<T*>(a.tail_out);
        unsigned char* R = smem + 256 * 512 + wv * 4096;
        // pixel operand of the tail's MFMAs: row q * 128 + j * 32 + frag_row, logical chunk 2 ks + lane / 32; the rows of one
        // fragment differ in their low five bits only (= frag_row), so the swizzled chunk is (x0 ^ 2 ks) for every j and q
        const int x0 = ((lane >> 5) ^ frag_row) & 31;
        const unsigned char* ylane = smem + frag_row * 512;
        const int pr0 = lane >> 3, chunk = lane & 7;   // this lane's 16-byte pieces: pixels pr0 + 8 it, channels 8 chunk .. + 7
        for (int cp = 0; cp < ctw; cp += 2) {
            const int ct0 = wv * ctw + cp;
            for (int q = 0; q < 2; ++q) {
                u32x4_t rq[2][4];
                auto fetch_res = [&](int j, u32x4_t* dst) {
#pragma unroll
                    for (int it = 0; it < 4; ++it) {
                        const int pix = m0 + q * 128 + j * 32 + pr0 + 8 * it;
                        dst[it] = *reinterpret_cast<const u32x4_t*>(tres + (size_t)(pix < M ? pix : 0) * N3 + ct0 * 32 + chunk * 8);
                    }
                };
                fetch_res(0, rq[0]);
                u32x4_t tw[2][TR];
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int k = 0; k < TR; ++k) tw[i][k] = twf[((size_t)(ct0 + i) * TKS + k) * 64];
                f32x16_t t4[2][4];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const f32x4_t bq = *reinterpret_cast<const f32x4_t*>(a.tail_b + (ct0 + i) * 32 + 8 * v + 4 * lh);
                        t4[i][0][4 * v] = bq.x; t4[i][0][4 * v + 1] = bq.y; t4[i][0][4 * v + 2] = bq.z; t4[i][0][4 * v + 3] = bq.w;
                    }
#pragma unroll
                    for (int j = 1; j < 4; ++j) t4[i][j] = t4[i][0];
                }
                __builtin_amdgcn_sched_barrier(0);
                static_for<0, TKS>([&](auto kc) {
                    constexpr int ks = decltype(kc)::value;
                    u32x4_t wf[2];
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        wf[i] = tw[i][ks % TR];
                        if (ks + TR < TKS) tw[i][ks % TR] = twf[((size_t)(ct0 + i) * TKS + ks + TR) * 64];
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const u32x4_t b = *reinterpret_cast<const u32x4_t*>(ylane + (q * 128 + j * 32) * 512 + ((x0 ^ (2 * ks)) << 4));
#pragma unroll
                        for (int i = 0; i < 2; ++i) mma_step<T>(t4[i][j], wf[i], b);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
                static_for<0, 4>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
                    if (j + 1 < 4) fetch_res(j + 1, rq[(j + 1) & 1]);
#pragma unroll
                    for (int it = 0; it < 4; ++it) *reinterpret_cast<u32x4_t*>(R + roff(pr0 + 8 * it, chunk * 16)) = rq[j & 1][it];
                    __builtin_amdgcn_s_waitcnt(0xc07f);
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            unsigned char* pp = R + roff(frag_row, (i * 32 + 8 * v + 4 * lh) * 2);
                            const u32x2_t r = *reinterpret_cast<const u32x2_t*>(pp);
                            const float r0 = fmaxf(t4[i][j][4 * v] + __uint_as_float(r.x << 16), 0.f);
                            const float r1 = fmaxf(t4[i][j][4 * v + 1] + __uint_as_float(r.x & 0xffff0000u), 0.f);
                            const float r2 = fmaxf(t4[i][j][4 * v + 2] + __uint_as_float(r.y << 16), 0.f);
                            const float r3 = fmaxf(t4[i][j][4 * v + 3] + __uint_as_float(r.y & 0xffff0000u), 0.f);
                            const u32x2_t o = {pack_bf16x2(r0, r1), pack_bf16x2(r2, r3)};
                            *reinterpret_cast<u32x2_t*>(pp) = o;   // the lane rewrites exactly the bytes it has read
                        }
                    __builtin_amdgcn_s_waitcnt(0xc07f);
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int it = 0; it < 4; ++it) {
                        const int pix = m0 + q * 128 + j * 32 + pr0 + 8 * it;
                        const u32x4_t o = *reinterpret_cast<const u32x4_t*>(R + roff(pr0 + 8 * it, chunk * 16));
                        if (pix < M) *reinterpret_cast<u32x4_t*>(tout + (size_t)pix * N3 + ct0 * 32 + chunk * 8) = o;
                    }
                    __builtin_amdgcn_s_waitcnt(0xc07f);
                    __builtin_amdgcn_wave_barrier();
                });
            }
        }
        return;
    }

    // ---- epilogue.  Accumulator element e of lane l: channel 8*(e/4) + 4*(l/32) + e%4, pixel l%32.
    OutT* __restrict__ out0 = static_cast<OutT*>(a.out0);
    OutT* __restrict__ out1 = static_cast<OutT*>(a.out1);
    if (vec) {
        // Coalesced path, one 32-pixel sub-tile at a time: the wavefront parks its 32 pixel x WN channel
        // fp32 tile (+ bias) in its own LDS region (the pipeline buffers are free now) and re-reads it so
        // that each lane owns 8 consecutive channels of one pixel: residual loads and output stores are
        // 16-byte and the lanes of one instruction cover whole lines of the NHWC tensors.
        unsigned char* ep = smem + (size_t)wv * (32 * EPITCH);
        if constexpr (std::is_same<OutT, bf16_t>::value && std::is_same<T, bf16_t>::value) {
            // No residual: bias, ReLU and the rounding to bf16 are applied in accumulator layout, and the tile goes through
            // LDS already rounded - half the LDS traffic, one 16-byte read per store (same values as the fp32 round trip).
            if (res == nullptr) {
                constexpr int EPB = WN * 2 + 16;   // bf16 row pitch
                f32x4_t bv[TN][4];
#pragma unroll
                for (int i = 0; i < TN; ++i)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int ch = n0 + wn * WN + i * 32 + 8 * v + 4 * (lane >> 5);
                        bv[i][v] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                        if (ch < a.Cout) bv[i][v] = *reinterpret_cast<const f32x4_t*>(a.bias + ch);
                    }
                const bool relu = a.relu != 0;
                static_for<0, TM>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
#pragma unroll
                    for (int i = 0; i < TN; ++i)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            float r0 = acc[i][j][4 * v] + bv[i][v].x, r1 = acc[i][j][4 * v + 1] + bv[i][v].y;
                            float r2 = acc[i][j][4 * v + 2] + bv[i][v].z, r3 = acc[i][j][4 * v + 3] + bv[i][v].w;
                            if (relu) { r0 = fmaxf(r0, 0.f); r1 = fmaxf(r1, 0.f); r2 = fmaxf(r2, 0.f); r3 = fmaxf(r3, 0.f); }
                            const u32x2_t o = {pack_bf16x2(r0, r1), pack_bf16x2(r2, r3)};
                            *reinterpret_cast<u32x2_t*>(ep + (size_t)frag_row * EPB + (i * 32 + 8 * v + 4 * (lane >> 5)) * 2) = o;
                        }
                    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the region is private to this wavefront
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int it = 0; it < NIT; ++it) {
                        const int pxl = it * PPI + lane / LPP, chunk = lane % LPP;
                        const int pix = m0 + wm * WM + j * 32 + pxl, ch = n0 + wn * WN + chunk * 8;
                        const u32x4_t q = *reinterpret_cast<const u32x4_t*>(ep + (size_t)pxl * EPB + chunk * 16);
                        if (pix < M && ch < a.Cout) *reinterpret_cast<u32x4_t*>(out0 + (size_t)pix * a.ld0 + ch) = q;
                    }
                    __builtin_amdgcn_s_waitcnt(0xc07f);
                    __builtin_amdgcn_wave_barrier();
                });
                return;
            }
        }
        // residual tiles that were not held across the K loop are fetched one sub-tile ahead of their use
        Vec8<T> rq0[NIT], rq1[NIT];
        auto fetch_res = [&](int j, Vec8<T>* dst) {
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int pix = m0 + wm * WM + j * 32 + it * PPI + lane / LPP, ch = n0 + wn * WN + (lane % LPP) * 8;
                if (pix < M && ch < a.Cout) dst[it] = *reinterpret_cast<const Vec8<T>*>(res + (size_t)pix * a.Cout + ch);
            }
        };
        if (!PREFETCH_RES && res != nullptr) fetch_res(0, rq0);
        static_for<0, TM>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            Vec8<T>* rnow = (j & 1) ? rq1 : rq0;
            if (!PREFETCH_RES && res != nullptr && j + 1 < TM) fetch_res(j + 1, (j & 1) ? rq0 : rq1);
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int chl = i * 32 + 8 * v + 4 * (lane >> 5);
                    const int ch = n0 + wn * WN + chl;
                    f32x4_t bv = {0.f, 0.f, 0.f, 0.f};
                    if (ch < a.Cout) bv = *reinterpret_cast<const f32x4_t*>(a.bias + ch);
                    f32x4_t r = {acc[i][j][4 * v] + bv.x, acc[i][j][4 * v + 1] + bv.y, acc[i][j][4 * v + 2] + bv.z,
                                 acc[i][j][4 * v + 3] + bv.w};
                    *reinterpret_cast<f32x4_t*>(ep + (size_t)frag_row * EPITCH + chl * 4) = r;
                }
            __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the region is private to this wavefront
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int pxl = it * PPI + lane / LPP, chunk = lane % LPP;
                const int pix = m0 + wm * WM + j * 32 + pxl, ch = n0 + wn * WN + chunk * 8;
                if (pix >= M || ch >= a.Cout) continue;
                const f32x4_t lo = *reinterpret_cast<const f32x4_t*>(ep + (size_t)pxl * EPITCH + chunk * 32);
                const f32x4_t hi = *reinterpret_cast<const f32x4_t*>(ep + (size_t)pxl * EPITCH + chunk * 32 + 16);
                float r[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                if (res) {
                    float q[8];
                    if (PREFETCH_RES) unpack8(rres[PREFETCH_RES ? j * NIT + it : 0], q);
                    else unpack8(rnow[it], q);
#pragma unroll
                    for (int e = 0; e < 8; ++e) r[e] += q[e];
                }
                if (a.relu) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) r[e] = fmaxf(r[e], 0.f);
                }
                store8(out0 + (size_t)pix * a.ld0 + ch, r);
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);
            __builtin_amdgcn_wave_barrier();
        });
        return;
    }
    // General path (split outputs, channel counts that are not multiples of 8): the same LDS round trip,
    // then one element per lane with consecutive lanes on consecutive channels of a pixel, so that stores
    // stay contiguous within each output row.
    {
        unsigned char* ep = smem + (size_t)wv * (32 * EPITCH);
        static_for<0, TM>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int chl = i * 32 + 8 * v + 4 * (lane >> 5);
                    f32x4_t r = {acc[i][j][4 * v], acc[i][j][4 * v + 1], acc[i][j][4 * v + 2], acc[i][j][4 * v + 3]};
                    *reinterpret_cast<f32x4_t*>(ep + (size_t)frag_row * EPITCH + chl * 4) = r;
                }
            __builtin_amdgcn_s_waitcnt(0xc07f);
            __builtin_amdgcn_wave_barrier();
            for (int e = lane; e < 32 * WN; e += 64) {
                const int pxl = e / WN, cl = e - pxl * WN;
                const int pix = m0 + wm * WM + j * 32 + pxl, c = n0 + wn * WN + cl;
                if (pix >= M || c >= a.Cout) continue;
                float val = *reinterpret_cast<const float*>(ep + (size_t)pxl * EPITCH + cl * 4) + a.bias[c];
                if (res) val += load_elem(res + (size_t)pix * a.Cout + c);
                if (a.relu) val = fmaxf(val, 0.f);
                if (c < a.n_split) store_elem(out0 + (size_t)pix * a.ld0 + c, val);
                else store_elem(out1 + (size_t)pix * a.ld1 + (c - a.n_split), val);
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);
            __builtin_amdgcn_wave_barrier();
        });
    }
}

// Whether launch_conv picks the 256 x 256 bf16 tile for this layer (the only variant with the fused predictors).
static bool takes_large_tile(const ConvArgs& a) {
    const long long M = (long long)a.N * a.Ho * a.Wo;
    const long long K = (long long)a.kh * a.kw * a.Cin + (a.in2 ? a.Cin2 : 0);
    const long long tiles_l = ((M + 255) / 256) * ((a.Cout + 255) / 256);
    return a.Cout % 256 == 0 && K >= 512 && (tiles_l >= 200 || (tiles_l >= 150 && K >= 8192)) && a.out1 == nullptr;
}

bool conv_heads_supported(const ConvArgs& a, int precision) {
    if (precision != 1 || a.head_w == nullptr || a.head_b == nullptr || a.head_logits == nullptr || a.head_deltas == nullptr) return false;
    if (a.Cout != 256 || a.in2 != nullptr || a.res != nullptr || !a.relu || a.head_a < 1 || 5 * a.head_a > 96) return false;
    if (a.kh == 1 && a.kw == 1 && a.pad == 0) return false;   // only the general-filter instantiation carries the predictor path
    return conv_supported(a, precision) && takes_large_tile(a);
}

bool conv_supported(const ConvArgs& a, int precision) {
    const int bk = precision ? 64 : 32;
    if (a.Cin <= 0 || a.Cin % bk) return false;
    if (a.kh < 1 || a.kw < 1 || a.kh * a.kw > 32) return false;   // one validity bit per filter tap
    if (a.N <= 0 || a.Cout <= 0 || a.Ho <= 0 || a.Wo <= 0) return false;
    if (a.in2 != nullptr) {
        if (a.kh != 1 || a.kw != 1 || a.pad != 0 || a.Cin2 <= 0 || a.Cin2 % bk || a.stride2 < 1) return false;
        if ((a.Ho - 1) * a.stride2 >= a.H2 || (a.Wo - 1) * a.stride2 >= a.W2) return false;
    }
    if ((long long)a.N * a.Ho * a.Wo >= (1ll << 31)) return false;
    if ((long long)a.N * a.H * a.W * a.Cin >= (1ll << 40)) return false;
    return true;
}

template <typename T, int BM, int BN, int BKB, int WAVES_M, int WAVES_N, int MODE, typename OutT>
static hipError_t launch_cfg(const ConvArgs& a, hipStream_t s) {
    // (the expansion tail parks an unpadded 256 x 512-byte tile and gives each of the 8 wavefronts 4 KB beside it: the CU's whole LDS)
    const size_t pipe = (size_t)2 * (BN + BM) * (BKB == 128 ? BKB : BKB + 16);
    // (the fused-predictor path of the large bf16 tile parks a padded 256 x 528-byte tile, more than the two pipeline buffers)
    const size_t heads = (std::is_same<T, bf16_t>::value && BM == 256 && BN == 256 && MODE == 0) ? (size_t)BM * (BN * 2 + 16) : 0;
    const size_t lds = MODE == 4 ? (size_t)160 * 1024 : (pipe > heads ? pipe : heads);
    auto kern = conv_igemm_kernel<T, BM, BN, BKB, WAVES_M, WAVES_N, MODE, OutT>;
    {
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
        if (e != hipSuccess) return e;
    }
    const long long M = (long long)a.N * a.Ho * a.Wo;
    const long long tiles = ((M + BM - 1) / BM) * ((a.Cout + BN - 1) / BN);
    if (tiles <= 0 || tiles >= (1ll << 30)) return hipErrorInvalidValue;
    const long long grid = ((tiles + 7) / 8) * 8;  // 8 XCDs x equal ranges; surplus workgroups exit at once
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * WAVES_M * WAVES_N), lds, s, a);
    return hipGetLastError();
}

// 1x1 unpadded convolutions (and the FC layers) get the variant without filter-tap bookkeeping.
template <typename T, int BM, int BN, int BKB, int WAVES_M, int WAVES_N, typename OutT, bool ALLOW_DUAL = false>
static hipError_t launch_one(const ConvArgs& a, hipStream_t s) {
    if (a.in2 != nullptr) {
        if constexpr (ALLOW_DUAL) return launch_cfg<T, BM, BN, BKB, WAVES_M, WAVES_N, 2, OutT>(a, s);
        else return hipErrorInvalidValue;
    }
    if (a.kh == 1 && a.kw == 1 && a.pad == 0) return launch_cfg<T, BM, BN, BKB, WAVES_M, WAVES_N, 1, OutT>(a, s);
    return launch_cfg<T, BM, BN, BKB, WAVES_M, WAVES_N, 0, OutT>(a, s);
}

bool conv_tail_supported(const ConvArgs& a, int precision) {
    if (precision != 1 || !conv_supported(a, precision)) return false;
    if (!a.tail_w || !a.tail_b || !a.tail_res || !a.tail_out || a.tail_res == a.tail_out) return false;
    if (a.tail_n < 512 || a.tail_n % 512 || a.tail_n > 4096) return false;
    if (a.Cout != 256 || !a.relu || a.res != nullptr || a.out1 != nullptr || a.in2 != nullptr || a.head_w != nullptr) return false;
    const long long M = (long long)a.N * a.Ho * a.Wo;
    return M * a.tail_n < (1ll << 31);
}

hipError_t launch_conv(const ConvArgs& a, int precision, bool out_f32, hipStream_t s) {
    if (!conv_supported(a, precision)) return hipErrorInvalidValue;
    if (a.tail_w != nullptr) {   // expansion tail: one kernel variant only
        if (out_f32 || !conv_tail_supported(a, precision)) return hipErrorInvalidValue;
        return launch_cfg<bf16_t, 256, 256, 128, 2, 4, 4, bf16_t>(a, s);
    }
    if (a.head_w != nullptr) {   // fused predictors exist in one kernel variant only
        if (out_f32 || !conv_heads_supported(a, precision)) return hipErrorInvalidValue;
        return launch_one<bf16_t, 256, 256, 128, 2, 4, bf16_t, true>(a, s);
    }
    const bool narrow = a.Cout <= 64;
    if (precision == 0) {
        return narrow ? launch_one<float, 128, 64, 128, 2, 2, float>(a, s) : launch_one<float, 128, 128, 128, 2, 2, float, true>(a, s);
    }
    if (out_f32) return narrow ? launch_one<bf16_t, 128, 64, 128, 2, 2, float>(a, s) : launch_one<bf16_t, 128, 128, 128, 2, 2, float>(a, s);
    // Long-K layers are bound by L2 -> CU bandwidth with a 128 x 128 tile (64 flop per byte staged); a
    // 256 x 256 tile halves that traffic.  It runs with 8 wavefronts (128 x 64 each), so that one block per
    // CU still keeps two wavefronts per SIMD, and with 128-byte K rows, which doubles the bytes in flight
    // per CU against the 64-byte variant (measured 15 % faster).  (4 wavefronts of 128 x 128 - also with the
    // K step software-pipelined by hand and pinned with scheduling-group barriers, 30 % slower - and
    // 256 x 128 with 64-byte K rows were measured and are slower; with fewer than ~200 tiles the 256 CUs
    // are better filled by the 128 x 128 tile, except for very long K; with K < 512 the kernel is mostly epilogue
    // (streaming the wide output), which two resident 128 x 128 blocks overlap with each other's K loop - except with a second source
    // (projection shortcut folded in), where K >= 384 already pays for the large tile: measured 30 us faster per launch; 16 wavefronts of 64 x 64 on the
    // 256 x 256 tile spill; 256 x 128 with 8 wavefronts and 64-byte rows is 1.5x slower.)
    {
        const long long M = (long long)a.N * a.Ho * a.Wo;
        const long long K = (long long)a.kh * a.kw * a.Cin + (a.in2 ? a.Cin2 : 0);
        // Short-K layers are pure streaming: what matters is how many independent tiles a CU has in
        // flight, so they take the small-footprint 128 x 64 tile (4 blocks of 4 wavefronts per CU).
        if (K <= 128 && a.out1 == nullptr && a.in2 == nullptr) return launch_one<bf16_t, 128, 64, 64, 2, 2, bf16_t>(a, s);
        const long long tiles_l = ((M + 255) / 256) * ((a.Cout + 255) / 256);
        // Very long K with a tile count that leaves CUs idle in a single round (the first FC layer: 152 tiles of
        // 256 x 256 on 256 CUs): 192-pixel tiles give 200 tiles of 3/4 the work each.
        const long long tiles_192 = ((M + 191) / 192) * ((a.Cout + 255) / 256);
        if (a.Cout % 256 == 0 && K >= 8192 && tiles_l < 200 && tiles_192 <= 256 && tiles_192 > tiles_l && a.out1 == nullptr && a.in2 == nullptr)
            return launch_one<bf16_t, 192, 256, 128, 2, 4, bf16_t>(a, s);
        if (a.Cout % 256 == 0 && (K >= 512 || (a.in2 != nullptr && K >= 384)) && (tiles_l >= 200 || (tiles_l >= 150 && K >= 8192)) && a.out1 == nullptr)
            return launch_one<bf16_t, 256, 256, 128, 2, 4, bf16_t, true>(a, s);
    }
    return narrow ? launch_one<bf16_t, 128, 64, 64, 2, 2, bf16_t>(a, s) : launch_one<bf16_t, 128, 128, 128, 2, 4, bf16_t, true>(a, s);
}

}  // namespace thia
