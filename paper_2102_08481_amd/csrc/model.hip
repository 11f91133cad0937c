// Host side of libthia: weights-blob parsing and repacking, workspace planning, the
// per-exit forward pass (micro-batched, one stream), plan execution and the C ABI.
// Every arithmetic step runs in the HIP kernels of this library; there is no CPU path.
#include <algorithm>
#include <cmath>
#include <new>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/thia.h"
#include "thia_internal.h"

using namespace thia;

namespace {

constexpr int32_t kMagic = 0x41494854;
constexpr size_t kHeaderBytes = 256;

struct Layer {
    void* w = nullptr;     // device, element type per precision, [Cout][k][k][Cin]
    float* b = nullptr;    // device fp32 [Cout]
    int co = 0, ci = 0, k = 1;
};
struct Block {
    Layer c1, c2, c3;  // for a stage's first block c3 holds [conv3 | projection shortcut] concatenated along K
    bool has_sc = false;
    int sc_ci = 0;     // input channels of the shortcut part
    int stride = 1;
    // identity blocks the single-kernel bottleneck covers: the three weight matrices in MFMA fragment order
    bf16_t *f1 = nullptr, *f2 = nullptr, *f3 = nullptr;
    // first block of the 128-wide stage: its 1x1 (256 -> 128) in fragment order, for use as the tail layer of the
    // 64-wide stage's last single-kernel block
    bf16_t* tf = nullptr;
    // identity blocks with 256-channel intermediates: the last 1x1 (256 -> 1024) in fragment order, applied by the 3x3's
    // kernel to its own output tile (ConvArgs::tail_*)
    bf16_t* t3f = nullptr;
};
struct ExitUnit {
    Layer lateral, rpn_conv, rpn_head /* obj (A) ++ delta (4A) */, fc1, fc2, pred /* cls (Kc) ++ box (4Kc) */;
    // RPN predictors for the convolution kernel's fused path: 96 rows (4A delta rows, A logit rows, zero rows) x 256
    // in MFMA fragment order, and the matching fp32 bias; null when the exit has no fused variant
    bf16_t* head_f = nullptr;
    float* head_fb = nullptr;
    bf16_t* lat_f = nullptr;   // lateral 256 -> 256 in fragment order (tail layer of the 64-wide stage's last block); else null
};

struct Tap {
    void* buf = nullptr;
    size_t cap = 0, bytes = 0, per_frame = 0;
};

struct Workspace {
    int H = 0, W = 0, mb = 0;
    char* arena = nullptr;
    size_t bytes = 0;
    void *act[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
    void *hf = nullptr, *rpn_t = nullptr;
    float *logits = nullptr, *deltas = nullptr;
    TopkWork topk{};
    int32_t *idx = nullptr, *prop_n = nullptr, *keep = nullptr, *roi_n = nullptr, *det_n = nullptr;
    float *prop_boxes = nullptr, *rois = nullptr;
    uint64_t *mask = nullptr, *sel_keys = nullptr;
    void *roi_feat = nullptr, *h1 = nullptr, *h2 = nullptr;
    float *cls = nullptr, *box = nullptr, *cand_scores = nullptr, *cand_boxes = nullptr;
    int key_cap = 0;
};

}  // namespace

struct thia_model {
    int precision = 0, n_exits = 0, blocks_n[4] = {0, 0, 0, 0}, stem_ch = 64, has_lateral = 0, head_ch = 256;
    // 1: exit 1 reads the pooled stem output and exit k >= 2 reads conv(k)_x (five exits, Sec. 4.2 / Table 4); 0: exit k reads conv(k+1)_x
    int stem_exit = 0;
    AnchorSpec anc{};
    int pre = 0, post = 0, pool = 7, sampling = 2, fc_dim = 0, Kc = 0, D = 0, base_width = 64;
    float rpn_thr = 0.7f, score_thr = 0.05f, det_thr = 0.5f, mean = 0.f, stdv = 1.f;
    size_t esz = 4;
    float* stem_w = nullptr;  // device fp32 [147][64] (fp32 path)
    bf16_t* stem_wk = nullptr;  // device bf16 [64][22][8] (matrix-core path)
    float* stem_b = nullptr;
    std::vector<Block> stage[4];
    ExitUnit ex[5];
    char* warena = nullptr;
    hipStream_t stream = nullptr;
    int user_mb = 0;
    bool fuse_blocks = true;  // identity bottlenecks as one kernel where a variant exists
    bool fuse_always = false; // take fused variants also below the sizes where they pay (tests)
    // exit estimator (two layers on the pooled last-stage features); est_hidden == 0: none set
    int est_hidden = 0;
    float *est_w1t = nullptr, *est_b1 = nullptr, *est_w2 = nullptr, *est_b2 = nullptr, *est_pooled = nullptr;
    size_t est_pooled_cap = 0;
    Workspace ws;
    // grow-only staging owned by the model (never allocated per call once large enough): gathered frames and their outputs
    // for micro-batches that mix chunks (plan execution) or sampled frames (planner); per-frame answers; query outputs
    struct Staging {
        uint8_t* frames = nullptr; size_t frames_cap = 0;
        float *ob = nullptr, *os = nullptr; int32_t* ol = nullptr; size_t out_rows = 0;   // rows of D detection slots
        uint8_t* flags = nullptr; size_t flags_cap = 0;
        int32_t* opt = nullptr; size_t opt_cap = 0;
    } stg, qry, qout;
    // Second lane.  The micro-batches of one call are independent, so they alternate between the caller's stream (workspace
    // ws, staging stg) and a stream of the model's own (ws_alt, stg_alt): the latency-bound proposal and selection kernels
    // of one micro-batch then run beside the convolutions of the next, and the last partial round of tiles of a launch
    // is filled by the other lane's blocks.  The model's stream starts after everything the caller had queued when the
    // call began (ev_fork) and the caller's stream waits for it before the call returns (ev_join), so callers see the
    // usual single-stream ordering.  Created on first use.
    Workspace ws_alt;
    Staging stg_alt;
    hipStream_t lane_stream = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    int lanes = 2;              // 1: everything on the caller's stream
    int lane_depth = 0;         // nesting of LaneScope
    int lane_next = 0;          // lane of the next micro-batch
    bool lane_ready = false;    // this call may use the second lane (set by LaneScope::begin)
    bool lane_forked = false;   // the model's stream holds work of the current call
    bool lane_active = false;   // the current code runs on the second lane (ws/stg/stream are swapped)
    bool debug = false;
    Tap taps[THIA_TAP_COUNT];
    bool profiling = false;
    std::vector<hipEvent_t> ev_pool;
    std::vector<int> ev_class;  // class of pair i (events 2i, 2i+1)
    size_t ev_used = 0;
    std::string err;
};

namespace {

// Overlap bit matrix of thia_op_nms_noalloc: fixed device storage, one copy per GPU, held until the process ends.
// Host code never uses this name as an address: it resolves the current device's copy once (nms_scratch_ptr).
constexpr size_t kNmsScratchWords = (size_t)1 << 20;   // 8 MiB
static __device__ __align__(256) unsigned long long nms_scratch[kNmsScratchWords];
constexpr int kMaxDevices = 64;
uint64_t* g_nms_scratch_ptr[kMaxDevices] = {};

int fail(thia_model* m, int code, const std::string& msg) {
    if (m) m->err = msg;
    return code;
}
int fail_hip(thia_model* m, hipError_t e, const char* what) {
    return fail(m, THIA_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
}
#define HIP_TRY(m, expr)                                          \
    do {                                                          \
        hipError_t e__ = (expr);                                  \
        if (e__ != hipSuccess) return fail_hip((m), e__, #expr);  \
    } while (0)

// Device address of the current GPU's copy of nms_scratch (each GPU holds its own copy at its own address).
int nms_scratch_ptr(thia_model* m, uint64_t** out) {
    int dev = -1;
    HIP_TRY(m, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(m, THIA_E_HIP, "device ordinal beyond the table of fixed buffers");
    if (!g_nms_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(m, hipGetSymbolAddress(&p, HIP_SYMBOL(nms_scratch)));
        if (!p) return fail(m, THIA_E_HIP, "hipGetSymbolAddress returned a null address");
        g_nms_scratch_ptr[dev] = static_cast<uint64_t*>(p);
    }
    *out = g_nms_scratch_ptr[dev];
    return THIA_OK;
}

inline int conv_out(int n, int k, int s, int p) { return (n + 2 * p - k) / s + 1; }
inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// ---------------------------------------------------------------- weights
struct BlobReader {
    const float* p;
    const float* end;
    bool take(size_t n, const float** out) {
        if ((size_t)(end - p) < n) return false;
        *out = p;
        p += n;
        return true;
    }
};

struct HostLayer {
    const float *w = nullptr, *b = nullptr;
    int co = 0, ci = 0, k = 1;
};
bool take_layer(BlobReader& r, HostLayer& L, int co, int ci, int k) {
    L.co = co; L.ci = ci; L.k = k;
    return r.take((size_t)co * ci * k * k, &L.w) && r.take((size_t)co, &L.b);
}

struct ArenaPlan {
    size_t off = 0;
    size_t add(size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes);
        return o;
    }
};

// Convert OIHW fp32 -> [O][kh][kw][I] in the model's element type, appended to `dst`.
void repack(const HostLayer& L, int precision, std::vector<unsigned char>& dst) {
    const size_t n = (size_t)L.co * L.ci * L.k * L.k, esz = precision ? 2 : 4;
    const size_t base = dst.size();
    dst.resize(base + n * esz);
    const int kk = L.k * L.k;
    for (int o = 0; o < L.co; ++o)
        for (int t = 0; t < kk; ++t)
            for (int i = 0; i < L.ci; ++i) {
                const float v = L.w[((size_t)o * L.ci + i) * kk + t];
                const size_t d = ((size_t)o * kk + t) * L.ci + i;
                if (precision) reinterpret_cast<bf16_t*>(dst.data() + base)[d] = f32_to_bf16(v);
                else reinterpret_cast<float*>(dst.data() + base)[d] = v;
            }
}

// Upload one layer (optionally the row-wise concatenation of two layers with equal ci, k).
int upload_layer(thia_model* m, const HostLayer& a, const HostLayer* b2, Layer& out) {
    std::vector<unsigned char> host;
    repack(a, m->precision, host);
    std::vector<float> bias(a.b, a.b + a.co);
    int co = a.co;
    if (b2) {
        repack(*b2, m->precision, host);
        bias.insert(bias.end(), b2->b, b2->b + b2->co);
        co += b2->co;
    }
    out.co = co; out.ci = a.ci; out.k = a.k;
    HIP_TRY(m, hipMalloc(&out.w, host.size()));
    HIP_TRY(m, hipMemcpy(out.w, host.data(), host.size(), hipMemcpyHostToDevice));
    HIP_TRY(m, hipMalloc(reinterpret_cast<void**>(&out.b), bias.size() * 4));
    HIP_TRY(m, hipMemcpy(out.b, bias.data(), bias.size() * 4, hipMemcpyHostToDevice));
    return THIA_OK;
}
// Upload one layer's weights in MFMA fragment order (bf16 models only).
int upload_fragments(thia_model* m, const HostLayer& a, bf16_t** out) {
    std::vector<unsigned char> host;
    repack(a, 1, host);
    const int K = a.ci * a.k * a.k;
    std::vector<bf16_t> frag((size_t)a.co * K);
    pack_mfma_fragments(reinterpret_cast<const bf16_t*>(host.data()), a.co, K, frag.data());
    HIP_TRY(m, hipMalloc(reinterpret_cast<void**>(out), frag.size() * 2));
    HIP_TRY(m, hipMemcpy(*out, frag.data(), frag.size() * 2, hipMemcpyHostToDevice));
    return THIA_OK;
}
void free_layer(Layer& L) {
    if (L.w) (void)hipFree(L.w);
    if (L.b) (void)hipFree(L.b);
    L.w = nullptr; L.b = nullptr;
}

// ---------------------------------------------------------------- geometry
struct ExitGeom { int C, Hk, Wk, stride; };
// Bottleneck stages in front of exit ep (0 = the exit reads the pooled stem output).
int exit_stages(const thia_model* m, int ep) { return ep - m->stem_exit; }
int exit_channels(const thia_model* m, int ep) {
    const int st = exit_stages(m, ep);
    return st == 0 ? m->stem_ch : 4 * (m->base_width << (st - 1));
}
ExitGeom exit_geom(const thia_model* m, int ep, int H, int W) {
    int h = conv_out(conv_out(H, 7, 2, 3), 3, 2, 1), w = conv_out(conv_out(W, 7, 2, 3), 3, 2, 1);
    const int st = exit_stages(m, ep);
    for (int s = 1; s < st; ++s) { h = conv_out(h, 3, 2, 1); w = conv_out(w, 3, 2, 1); }
    return {exit_channels(m, ep), h, w, st == 0 ? 4 : 4 << (st - 1)};
}
int head_channels(const thia_model* m, int ep) { return m->has_lateral ? m->head_ch : exit_channels(m, ep); }

int next_pow2(int v) {
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

// Largest activation tensor (elements per frame) among all layers of the backbone.
size_t max_act_elems(const thia_model* m, int H, int W) {
    int h = conv_out(H, 7, 2, 3), w = conv_out(W, 7, 2, 3);
    size_t mx = (size_t)h * w * m->stem_ch;
    h = conv_out(h, 3, 2, 1); w = conv_out(w, 3, 2, 1);
    for (int s = 0; s < exit_stages(m, m->n_exits); ++s) {
        const int width = m->base_width << s;
        if (s > 0) {
            mx = std::max(mx, (size_t)h * w * width);  // conv1 output before the strided 3x3
            h = conv_out(h, 3, 2, 1); w = conv_out(w, 3, 2, 1);
        }
        mx = std::max(mx, (size_t)h * w * 4 * width);
    }
    return mx;
}

int default_microbatch(const thia_model* m, int H, int W) {
    const double per_frame = (double)max_act_elems(m, H, W) * m->esz;
    int mb = (int)std::floor(600.0e6 / per_frame + 0.5);
    return std::min(32, std::max(1, mb));
}

int microbatch_frames(const thia_model* m, int H, int W) { return m->user_mb > 0 ? m->user_mb : default_microbatch(m, H, W); }

void free_workspace(thia_model* m) {   // the current lane's
    if (m->ws.arena) (void)hipFree(m->ws.arena);
    m->ws = Workspace{};
}

int ensure_workspace(thia_model* m, int H, int W) {
    const int mb = microbatch_frames(m, H, W);
    Workspace& ws = m->ws;
    if (ws.arena && ws.H == H && ws.W == W && ws.mb == mb) return THIA_OK;
    if (ws.arena) {
        HIP_TRY(m, hipStreamSynchronize(m->stream));
        free_workspace(m);
    }
    const size_t esz = m->esz;
    ArenaPlan ap;
    const size_t act_bytes = (size_t)mb * max_act_elems(m, H, W) * esz;
    size_t o_act[5];
    for (int i = 0; i < 5; ++i) o_act[i] = ap.add(act_bytes);
    // head buffers sized for the largest exit (exit 1 has the largest map)
    size_t hw_max = 0, na_max = 0, hf_max = 0;
    const int A = m->anc.n_sizes * m->anc.n_ratios;
    for (int ep = 1; ep <= m->n_exits; ++ep) {
        const ExitGeom g = exit_geom(m, ep, H, W);
        const size_t hw = (size_t)g.Hk * g.Wk;
        hw_max = std::max(hw_max, hw);
        na_max = std::max(na_max, hw * A);
        hf_max = std::max(hf_max, hw * head_channels(m, ep));
    }
    if (na_max >= (1u << 22)) return fail(m, THIA_E_SHAPE, "frame too large: more than 2^22 anchors per frame");
    int ch_max = 0;
    for (int ep = 1; ep <= m->n_exits; ++ep) ch_max = std::max(ch_max, head_channels(m, ep));
    const size_t o_hf = ap.add((size_t)mb * hf_max * esz), o_rt = ap.add((size_t)mb * hf_max * esz);
    const size_t o_lg = ap.add((size_t)mb * na_max * 4), o_dl = ap.add((size_t)mb * na_max * 16);
    const int cap = topk_cand_cap(m->pre);
    const size_t o_hist = ap.add((size_t)mb * 2048 * 4), o_state = ap.add((size_t)mb * 4 * 8), o_cand = ap.add((size_t)mb * cap * 8);
    const size_t o_idx = ap.add((size_t)mb * m->pre * 4), o_pb = ap.add((size_t)mb * m->pre * 16), o_pn = ap.add((size_t)mb * 4);
    const int words = (m->pre + 63) / 64;
    const size_t o_mask = ap.add((size_t)mb * m->pre * words * 8);
    const size_t o_keep = ap.add((size_t)mb * m->post * 4), o_rois = ap.add((size_t)mb * m->post * 16), o_rn = ap.add((size_t)mb * 4);
    const size_t o_dn = ap.add((size_t)mb * 4);
    const size_t rows = (size_t)mb * m->post;
    const size_t o_rf = ap.add(rows * m->pool * m->pool * ch_max * esz);
    const size_t o_h1 = ap.add(rows * m->fc_dim * esz), o_h2 = ap.add(rows * m->fc_dim * esz);
    const size_t o_cls = ap.add(rows * m->Kc * 4), o_box = ap.add(rows * m->Kc * 16);
    const size_t o_cs = ap.add(rows * m->Kc * 4), o_cb = ap.add(rows * m->Kc * 16);
    const int key_cap = next_pow2(m->post * m->Kc);
    const size_t o_keys = ap.add((size_t)mb * key_cap * 8);

    void* base = nullptr;
    hipError_t e = hipMalloc(&base, ap.off);
    if (e != hipSuccess) return fail(m, THIA_E_NOMEM, std::string("workspace hipMalloc: ") + hipGetErrorString(e));
    char* a = static_cast<char*>(base);
    ws.arena = a; ws.bytes = ap.off; ws.H = H; ws.W = W; ws.mb = mb;
    for (int i = 0; i < 5; ++i) ws.act[i] = a + o_act[i];
    ws.hf = a + o_hf; ws.rpn_t = a + o_rt;
    ws.logits = reinterpret_cast<float*>(a + o_lg); ws.deltas = reinterpret_cast<float*>(a + o_dl);
    ws.topk.hist = reinterpret_cast<uint32_t*>(a + o_hist);
    ws.topk.state = reinterpret_cast<uint64_t*>(a + o_state);
    ws.topk.cand = reinterpret_cast<uint64_t*>(a + o_cand);
    ws.idx = reinterpret_cast<int32_t*>(a + o_idx); ws.prop_boxes = reinterpret_cast<float*>(a + o_pb);
    ws.prop_n = reinterpret_cast<int32_t*>(a + o_pn); ws.mask = reinterpret_cast<uint64_t*>(a + o_mask);
    ws.keep = reinterpret_cast<int32_t*>(a + o_keep); ws.rois = reinterpret_cast<float*>(a + o_rois);
    ws.roi_n = reinterpret_cast<int32_t*>(a + o_rn); ws.det_n = reinterpret_cast<int32_t*>(a + o_dn);
    ws.roi_feat = a + o_rf; ws.h1 = a + o_h1; ws.h2 = a + o_h2;
    ws.cls = reinterpret_cast<float*>(a + o_cls); ws.box = reinterpret_cast<float*>(a + o_box);
    ws.cand_scores = reinterpret_cast<float*>(a + o_cs); ws.cand_boxes = reinterpret_cast<float*>(a + o_cb);
    ws.sel_keys = reinterpret_cast<uint64_t*>(a + o_keys); ws.key_cap = key_cap;
    return THIA_OK;
}

// ---------------------------------------------------------------- lanes
// Bracket of one call.  The outermost scope notes where the caller's stream stood when the call began (begin); join makes
// the caller's stream wait for what the call put on the model's stream.  On an error path the destructor waits for that
// work on the host instead, so no call returns with work of its own still running beside the caller's stream.
struct LaneScope {
    thia_model* m;
    explicit LaneScope(thia_model* m_) : m(m_) {
        if (m->lane_depth++ == 0) { m->lane_next = 0; m->lane_forked = false; m->lane_ready = false; }
    }
    int begin() {
        if (m->lane_depth != 1 || m->lanes < 2 || m->profiling || m->debug) return THIA_OK;
        if (!m->lane_stream) {
            HIP_TRY(m, hipStreamCreateWithFlags(&m->lane_stream, hipStreamNonBlocking));
            HIP_TRY(m, hipEventCreateWithFlags(&m->ev_fork, hipEventDisableTiming));
            HIP_TRY(m, hipEventCreateWithFlags(&m->ev_join, hipEventDisableTiming));
        }
        if (!m->ev_fork || !m->ev_join) return THIA_OK;   // an earlier creation failed half-way: stay on one lane
        HIP_TRY(m, hipEventRecord(m->ev_fork, m->stream));
        m->lane_ready = true;
        return THIA_OK;
    }
    int join() {
        if (m->lane_depth != 1 || !m->lane_forked) return THIA_OK;
        HIP_TRY(m, hipEventRecord(m->ev_join, m->lane_stream));
        HIP_TRY(m, hipStreamWaitEvent(m->stream, m->ev_join, 0));
        m->lane_forked = false;
        return THIA_OK;
    }
    ~LaneScope() {
        if (--m->lane_depth > 0) return;
        if (m->lane_forked) (void)hipStreamSynchronize(m->lane_stream);
        m->lane_forked = false;
        m->lane_ready = false;
    }
};

// Lane of the next micro-batch (0: the caller's stream).  The model's stream is held back to the call's start the first
// time a call uses it.  Call outside any LaneGuard.
int pick_lane(thia_model* m, int* lane) {
    *lane = 0;
    if (!m->lane_ready) return THIA_OK;
    *lane = m->lane_next;
    m->lane_next ^= 1;
    if (*lane == 1 && !m->lane_forked) {
        HIP_TRY(m, hipStreamWaitEvent(m->lane_stream, m->ev_fork, 0));
        m->lane_forked = true;
    }
    return THIA_OK;
}

// While it lives, the model's stream, workspace and staging are those of `lane`: everything below addresses them as
// m->stream, m->ws and m->stg.
struct LaneGuard {
    thia_model* m;
    bool on;
    LaneGuard(thia_model* m_, int lane) : m(m_), on(lane == 1) { if (on) flip(); }
    ~LaneGuard() { if (on) flip(); }
    LaneGuard(const LaneGuard&) = delete;
    LaneGuard& operator=(const LaneGuard&) = delete;
    void flip() {
        std::swap(m->ws, m->ws_alt);
        std::swap(m->stg, m->stg_alt);
        std::swap(m->stream, m->lane_stream);
        m->lane_active = !m->lane_active;
    }
};

// ---------------------------------------------------------------- launch bookkeeping
struct Scope {  // brackets one launch (group) with events when profiling is on
    thia_model* m;
    bool on;
    Scope(thia_model* m_, int cls) : m(m_), on(m_->profiling) {
        if (!on) return;
        if (m->ev_used + 2 > m->ev_pool.size()) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { on = false; return; }
            m->ev_pool.push_back(a);
            m->ev_pool.push_back(b);
        }
        m->ev_class.resize(m->ev_used / 2 + 1);
        m->ev_class[m->ev_used / 2] = cls;
        (void)hipEventRecord(m->ev_pool[m->ev_used], m->stream);
    }
    ~Scope() {
        if (!on) return;
        (void)hipEventRecord(m->ev_pool[m->ev_used + 1], m->stream);
        m->ev_used += 2;
    }
};

struct Second {  // second source of a dual 1x1 convolution
    const void* in = nullptr;
    int Cin = 0, H = 0, W = 0, stride = 1;
};
struct Heads {  // RPN predictors fused into the convolution (ConvArgs::head_*)
    const bf16_t* w = nullptr;
    const float* b = nullptr;
    float *logits = nullptr, *deltas = nullptr;
    int A = 0;
};

void fill_conv_args(const thia_model* m, ConvArgs& a, const Layer& L, const void* in, int n, int H, int W, int stride, int pad,
                    const void* res, bool relu, void* out0, void* out1, int n_split, const Second* second) {
    a = ConvArgs{};
    a.in = in; a.w = L.w; a.bias = L.b; a.res = res; a.out0 = out0; a.out1 = out1;
    a.N = n; a.H = H; a.W = W; a.Cin = L.ci; a.Cout = L.co;
    if (second) {
        a.in2 = second->in; a.Cin2 = second->Cin; a.H2 = second->H; a.W2 = second->W; a.stride2 = second->stride;
        a.Cin = L.ci - second->Cin;
    }
    a.kh = L.k; a.kw = L.k; a.stride = stride; a.pad = pad;
    a.Ho = conv_out(H, L.k, stride, pad); a.Wo = conv_out(W, L.k, stride, pad);
    a.relu = relu ? 1 : 0;
    if (out1) { a.n_split = n_split; a.ld0 = n_split; a.ld1 = L.co - n_split; }
    else { a.n_split = L.co; a.ld0 = L.co; a.ld1 = 0; }
}

int run_conv(thia_model* m, int cls, const Layer& L, const void* in, int n, int H, int W, int stride, int pad, const void* res,
             bool relu, bool out_f32, void* out0, void* out1 = nullptr, int n_split = -1, const Second* second = nullptr) {
    ConvArgs a;
    fill_conv_args(m, a, L, in, n, H, W, stride, pad, res, relu, out0, out1, n_split, second);
    Scope sc(m, cls);
    HIP_TRY(m, launch_conv(a, m->precision, out_f32, m->stream));
    return THIA_OK;
}

int tap_prepare(thia_model* m, int which, int n, size_t per_frame) {
    Tap& t = m->taps[which];
    const size_t need = (size_t)n * per_frame;
    if (need > t.cap) {
        if (t.buf) { HIP_TRY(m, hipStreamSynchronize(m->stream)); (void)hipFree(t.buf); t.buf = nullptr; t.cap = 0; }
        HIP_TRY(m, hipMalloc(&t.buf, need));
        t.cap = need;
    }
    t.bytes = need; t.per_frame = per_frame;
    return THIA_OK;
}
int tap_copy(thia_model* m, int which, int f0, int nb, const void* src) {
    Tap& t = m->taps[which];
    HIP_TRY(m, hipMemcpyAsync(static_cast<char*>(t.buf) + (size_t)f0 * t.per_frame, src, (size_t)nb * t.per_frame,
                              hipMemcpyDeviceToDevice, m->stream));
    return THIA_OK;
}

#define TRY(expr)                     \
    do {                              \
        int rc__ = (expr);            \
        if (rc__ != THIA_OK) return rc__; \
    } while (0)

// State of one backbone pass over nb frames: x holds the newest stage tensor (NHWC, h x w), y is the spare buffer.
struct Trunk {
    void *x = nullptr, *y = nullptr;
    int h = 0, w = 0;
    bool c1_done = false;   // the next stage's first 1x1 was applied by the previous stage's last block (result in ws.act[2])
    bool hf_done = false;   // the exit's lateral was applied by the stage's last block (result in ws.hf)
};

// A 1x1 layer applied by the stage's last single-kernel block to its own output tile (FusedBlockArgs::wtf ...).
struct Tail {
    const bf16_t* wtf = nullptr;
    const float* bt = nullptr;
    void* z = nullptr;
    int n = 0, relu = 0;
};

// Normalisation, stem and max-pool.
int run_stem(thia_model* m, const uint8_t* frames, int nb, int H, int W, Trunk& t) {
    Workspace& ws = m->ws;
    const int Hs = conv_out(H, 7, 2, 3), Ws = conv_out(W, 7, 2, 3);
    t.h = conv_out(Hs, 3, 2, 1); t.w = conv_out(Ws, 3, 2, 1);
    if (m->precision == 1) {
        Scope sc(m, THIA_K_STEM);
        HIP_TRY(m, launch_stem_pool(frames, nb, H, W, m->stem_wk, m->stem_b, m->mean, m->stdv, ws.act[0], m->stream));
    } else {
        {
            Scope sc(m, THIA_K_STEM);
            HIP_TRY(m, launch_stem(frames, nb, H, W, m->stem_w, m->stem_b, m->mean, m->stdv, ws.act[2], m->stream));
        }
        Scope sc(m, THIA_K_POOL);
        HIP_TRY(m, launch_maxpool(ws.act[2], nb, Hs, Ws, m->stem_ch, m->precision, ws.act[0], m->stream));
    }
    t.x = ws.act[0]; t.y = ws.act[1];
    return THIA_OK;
}

// The 1x1 layer that reads stage s's output next: exit `ep_here`'s lateral if the backbone stops after this stage
// (ep_here > 0), else the first 1x1 of stage s + 1.  Empty when no fragment-ordered copy of that layer exists.
Tail stage_tail(const thia_model* m, int s, int ep_here) {
    Tail tl;
    if (!m->fuse_blocks || m->precision != 1) return tl;
    if (ep_here > 0) {
        const ExitUnit& E = m->ex[ep_here - 1];
        if (m->has_lateral && E.lat_f) { tl.wtf = E.lat_f; tl.bt = E.lateral.b; tl.z = m->ws.hf; tl.n = E.lateral.co; tl.relu = 0; }
    } else if (s + 1 < 4 && !m->stage[s + 1].empty()) {
        const Block& N = m->stage[s + 1][0];
        if (N.tf) { tl.wtf = N.tf; tl.bt = N.c1.b; tl.z = m->ws.act[2]; tl.n = N.c1.co; tl.relu = 1; }
    }
    return tl;
}

// Bottleneck stage s (0-based) applied to t.x; the stage's output becomes t.x.  `tail` (optional) is handed to the
// stage's last block if that block runs as a single kernel of the 64-wide variant; *tail_applied tells whether it was.
int run_stage(thia_model* m, int s, int nb, Trunk& t, const Tail* tail = nullptr, bool* tail_applied = nullptr) {
    Workspace& ws = m->ws;
    void *&x = t.x, *&y = t.y;
    int &h = t.h, &w = t.w;
    const bool skip_c1 = t.c1_done;   // first block only: its 1x1 already sits in ws.act[2]
    t.c1_done = false;
    if (tail_applied) *tail_applied = false;
    const size_t nblocks = m->stage[s].size();
    for (size_t bi = 0; bi < nblocks; ++bi) {
        const Block& B = m->stage[s][bi];
        const int ho = conv_out(h, 3, B.stride, 1), wo = conv_out(w, 3, B.stride, 1);
        if (B.f1 && m->fuse_blocks) {
            FusedBlockArgs fa{};
            fa.x = static_cast<const bf16_t*>(x); fa.y = static_cast<bf16_t*>(y);
            fa.w1f = B.f1; fa.w2f = B.f2; fa.w3f = B.f3; fa.b1 = B.c1.b; fa.b2 = B.c2.b; fa.b3 = B.c3.b;
            fa.N = nb; fa.H = h; fa.W = w; fa.first = B.has_sc ? 1 : 0;
            if (B.stride == 1 && fused_block_supported(fa, B.c1.co)) {
                bool with_tail = false;
                if (tail && tail->wtf && bi + 1 == nblocks && !B.has_sc && B.c1.co == 64) {
                    FusedBlockArgs ft = fa;
                    ft.wtf = tail->wtf; ft.bt = tail->bt; ft.z = static_cast<bf16_t*>(tail->z); ft.tail_n = tail->n; ft.tail_relu = tail->relu;
                    if (fused_block_supported(ft, B.c1.co)) { fa = ft; with_tail = true; }
                }
                Scope sc(m, THIA_K_CONV);
                HIP_TRY(m, launch_fused_block(fa, B.c1.co, m->stream));
                if (with_tail && tail_applied) *tail_applied = true;
                std::swap(x, y);
                continue;
            }
        }
        if (!(bi == 0 && skip_c1)) TRY(run_conv(m, THIA_K_CONV, B.c1, x, nb, h, w, 1, 0, nullptr, true, false, ws.act[2]));
        if (B.t3f && m->fuse_blocks && !B.has_sc && B.stride == 1) {
            // 3x3 and the last 1x1 (+ residual) in one launch: the 256-channel tensor between them stays in LDS.  Worth it
            // only where the 3x3 runs on the large tile anyway (enough 256-pixel tiles to fill the chip).
            ConvArgs a;
            fill_conv_args(m, a, B.c2, ws.act[2], nb, h, w, 1, 1, nullptr, true, ws.act[3], nullptr, -1, nullptr);
            a.tail_w = B.t3f; a.tail_b = B.c3.b; a.tail_res = x; a.tail_out = y; a.tail_n = B.c3.co;
            const long long tiles_l = ((long long)nb * h * w + 255) / 256;
            if ((tiles_l >= 200 || m->fuse_always) && conv_tail_supported(a, m->precision)) {
                Scope sc(m, THIA_K_CONV);
                HIP_TRY(m, launch_conv(a, m->precision, false, m->stream));
                std::swap(x, y);
                continue;
            }
        }
        TRY(run_conv(m, THIA_K_CONV, B.c2, ws.act[2], nb, h, w, B.stride, 1, nullptr, true, false, ws.act[3]));
        if (B.has_sc) {
            // last 1x1 and projection shortcut share one accumulator: y = relu(W3 t2 + Ws x(strided) + b3 + bs)
            Second sec;
            sec.in = x; sec.Cin = B.sc_ci; sec.H = h; sec.W = w; sec.stride = B.stride;
            TRY(run_conv(m, THIA_K_CONV, B.c3, ws.act[3], nb, ho, wo, 1, 0, nullptr, true, false, y, nullptr, -1, &sec));
        } else {
            TRY(run_conv(m, THIA_K_CONV, B.c3, ws.act[3], nb, ho, wo, 1, 0, x, true, false, y));
        }
        std::swap(x, y);
        h = ho; w = wo;
    }
    return THIA_OK;
}

// Backbone truncated at exit ep for nb frames; returns the exit-stage tensor (NHWC) in *feat.
int run_backbone(thia_model* m, const uint8_t* frames, int nb, int H, int W, int ep, const void** feat, bool* hf_done = nullptr) {
    Trunk t;
    TRY(run_stem(m, frames, nb, H, W, t));
    const int ns = exit_stages(m, ep);
    for (int s = 0; s < ns; ++s) {
        const Tail tl = stage_tail(m, s, s + 1 == ns ? ep : 0);
        bool applied = false;
        TRY(run_stage(m, s, nb, t, &tl, &applied));
        if (applied) (s + 1 == ns ? t.hf_done : t.c1_done) = true;
    }
    *feat = t.x;
    if (hf_done) *hf_done = t.hf_done;
    return THIA_OK;
}

// Heads of exit ep on nb frames whose exit-stage tensor is `feat`.
int run_heads(thia_model* m, const void* feat, int f0, int nb, int H, int W, int ep, float* out_boxes, float* out_scores,
              int32_t* out_labels, bool hf_ready = false) {
    Workspace& ws = m->ws;
    const ExitUnit& E = m->ex[ep - 1];
    const ExitGeom g = exit_geom(m, ep, H, W);
    const int A = m->anc.n_sizes * m->anc.n_ratios, Ch = head_channels(m, ep), P = m->pool;
    const long nA = (long)g.Hk * g.Wk * A;
    const void* hf = feat;
    if (m->has_lateral) {
        // (hf_ready: the stage's last block has already applied the lateral to its output tile)
        if (!hf_ready) TRY(run_conv(m, THIA_K_RPN, E.lateral, feat, nb, g.Hk, g.Wk, 1, 0, nullptr, false, false, ws.hf));
        hf = ws.hf;
    }
    bool fused_heads = false;
    if (E.head_f && m->fuse_blocks) {
        // 3x3 + ReLU and both 1x1 predictors in one launch: the 256-channel tensor between them never leaves LDS
        ConvArgs a;
        fill_conv_args(m, a, E.rpn_conv, hf, nb, g.Hk, g.Wk, 1, 1, nullptr, true, ws.rpn_t, nullptr, -1, nullptr);
        a.head_w = E.head_f; a.head_b = E.head_fb; a.head_logits = ws.logits; a.head_deltas = ws.deltas; a.head_a = A;
        if (conv_heads_supported(a, m->precision)) {
            Scope sc(m, THIA_K_RPN);
            HIP_TRY(m, launch_conv(a, m->precision, false, m->stream));
            fused_heads = true;
        }
    }
    if (!fused_heads) {
        TRY(run_conv(m, THIA_K_RPN, E.rpn_conv, hf, nb, g.Hk, g.Wk, 1, 1, nullptr, true, false, ws.rpn_t));
        TRY(run_conv(m, THIA_K_RPN, E.rpn_head, ws.rpn_t, nb, g.Hk, g.Wk, 1, 0, nullptr, false, true, ws.logits, ws.deltas, A));
    }
    {
        Scope sc(m, THIA_K_TOPK);
        HIP_TRY(m, launch_rpn_proposals(ws.logits, ws.deltas, nb, nA, m->pre, g.Wk, g.stride, (float)W, (float)H, m->anc, ws.topk,
                                        ws.idx, ws.prop_boxes, ws.prop_n, m->stream));
    }
    {
        Scope sc(m, THIA_K_NMS);
        HIP_TRY(m, launch_nms(ws.prop_boxes, ws.prop_n, nb, m->pre, m->rpn_thr, m->post, ws.mask, ws.keep, ws.roi_n, ws.rois,
                              m->stream));
    }
    {
        Scope sc(m, THIA_K_ROIALIGN);
        HIP_TRY(m, launch_roialign(hf, ws.rois, nb, m->post, g.Hk, g.Wk, Ch, g.stride, P, m->precision, ws.roi_feat, m->stream));
    }
    const int rows = nb * m->post;
    TRY(run_conv(m, THIA_K_FC, E.fc1, ws.roi_feat, rows, 1, 1, 1, 0, nullptr, true, false, ws.h1));
    TRY(run_conv(m, THIA_K_FC, E.fc2, ws.h1, rows, 1, 1, 1, 0, nullptr, true, false, ws.h2));
    TRY(run_conv(m, THIA_K_FC, E.pred, ws.h2, rows, 1, 1, 1, 0, nullptr, false, true, ws.cls, ws.box, m->Kc));
    {
        Scope sc(m, THIA_K_POST);
        HIP_TRY(m, launch_scores_boxes(ws.cls, ws.box, ws.rois, nb, m->post, m->Kc, (float)W, (float)H, ws.cand_scores,
                                       ws.cand_boxes, m->stream));
        HIP_TRY(m, launch_select(ws.cand_scores, ws.cand_boxes, ws.roi_n, nb, m->post, m->Kc, m->score_thr, m->det_thr, m->D,
                                 ws.sel_keys, ws.key_cap, out_boxes, out_scores, out_labels, ws.det_n, m->stream));
    }
    if (m->debug) {
        const size_t esz = m->esz, hw = (size_t)g.Hk * g.Wk;
        TRY(tap_copy(m, THIA_TAP_FEAT, f0, nb, feat));
        TRY(tap_copy(m, THIA_TAP_HEAD_FEAT, f0, nb, hf));
        TRY(tap_copy(m, THIA_TAP_RPN_LOGITS, f0, nb, ws.logits));
        TRY(tap_copy(m, THIA_TAP_RPN_DELTAS, f0, nb, ws.deltas));
        TRY(tap_copy(m, THIA_TAP_TOPK_IDX, f0, nb, ws.idx));
        TRY(tap_copy(m, THIA_TAP_PROP_BOXES, f0, nb, ws.prop_boxes));
        TRY(tap_copy(m, THIA_TAP_PROP_N, f0, nb, ws.prop_n));
        TRY(tap_copy(m, THIA_TAP_ROIS, f0, nb, ws.rois));
        TRY(tap_copy(m, THIA_TAP_ROI_N, f0, nb, ws.roi_n));
        TRY(tap_copy(m, THIA_TAP_ROI_FEAT, f0, nb, ws.roi_feat));
        TRY(tap_copy(m, THIA_TAP_CLS_LOGITS, f0, nb, ws.cls));
        TRY(tap_copy(m, THIA_TAP_BOX_DELTAS, f0, nb, ws.box));
        TRY(tap_copy(m, THIA_TAP_CAND_SCORES, f0, nb, ws.cand_scores));
        TRY(tap_copy(m, THIA_TAP_CAND_BOXES, f0, nb, ws.cand_boxes));
        TRY(tap_copy(m, THIA_TAP_DET_N, f0, nb, ws.det_n));
        (void)esz; (void)hw;
    }
    return THIA_OK;
}

int prepare_taps(thia_model* m, int n, int H, int W, int ep) {
    const ExitGeom g = exit_geom(m, ep, H, W);
    const size_t esz = m->esz, hw = (size_t)g.Hk * g.Wk;
    const int A = m->anc.n_sizes * m->anc.n_ratios, Ch = head_channels(m, ep);
    const size_t post = m->post, Kc = m->Kc;
    TRY(tap_prepare(m, THIA_TAP_FEAT, n, hw * g.C * esz));
    TRY(tap_prepare(m, THIA_TAP_HEAD_FEAT, n, hw * Ch * esz));
    TRY(tap_prepare(m, THIA_TAP_RPN_LOGITS, n, hw * A * 4));
    TRY(tap_prepare(m, THIA_TAP_RPN_DELTAS, n, hw * A * 16));
    TRY(tap_prepare(m, THIA_TAP_TOPK_IDX, n, (size_t)m->pre * 4));
    TRY(tap_prepare(m, THIA_TAP_PROP_BOXES, n, (size_t)m->pre * 16));
    TRY(tap_prepare(m, THIA_TAP_PROP_N, n, 4));
    TRY(tap_prepare(m, THIA_TAP_ROIS, n, post * 16));
    TRY(tap_prepare(m, THIA_TAP_ROI_N, n, 4));
    TRY(tap_prepare(m, THIA_TAP_ROI_FEAT, n, post * m->pool * m->pool * Ch * esz));
    TRY(tap_prepare(m, THIA_TAP_CLS_LOGITS, n, post * Kc * 4));
    TRY(tap_prepare(m, THIA_TAP_BOX_DELTAS, n, post * Kc * 16));
    TRY(tap_prepare(m, THIA_TAP_CAND_SCORES, n, post * Kc * 4));
    TRY(tap_prepare(m, THIA_TAP_CAND_BOXES, n, post * Kc * 16));
    TRY(tap_prepare(m, THIA_TAP_DET_N, n, 4));
    return THIA_OK;
}

int check_frame_args(thia_model* m, const void* frames, int n, int H, int W, const void* ob, const void* os, const void* ol) {
    if (!m) return THIA_E_BADARG;
    if (n < 0) return fail(m, THIA_E_BADARG, "negative frame count");
    if (n > 0 && (!frames || !ob || !os || !ol)) return fail(m, THIA_E_BADARG, "null pointer");
    if (H < 32 || W < 32 || H > 16384 || W > 16384) return fail(m, THIA_E_SHAPE, "frame size must be within 32..16384");
    return THIA_OK;
}

// n frames at exit ep (1..n_exits), micro-batched.  Assumes arguments were validated.
// One micro-batch (nb <= micro-batch frames) on the current lane; f0 = its position in the call (debug taps).
int detect_batch_here(thia_model* m, const uint8_t* frames, int f0, int nb, int H, int W, int ep, float* ob, float* os, int32_t* ol) {
    TRY(ensure_workspace(m, H, W));
    const void* feat = nullptr;
    bool hf_done = false;
    TRY(run_backbone(m, frames, nb, H, W, ep, &feat, &hf_done));
    return run_heads(m, feat, f0, nb, H, W, ep, ob, os, ol, hf_done);
}

int detect_frames(thia_model* m, const uint8_t* frames, int n, int H, int W, int ep, float* ob, float* os, int32_t* ol) {
    if (m->debug) {
        TRY(ensure_workspace(m, H, W));
        TRY(prepare_taps(m, n, H, W, ep));
    }
    LaneScope scope(m);
    TRY(scope.begin());
    const int mb = microbatch_frames(m, H, W), D = m->D;
    for (int f0 = 0; f0 < n; f0 += mb) {
        const int nb = std::min(mb, n - f0);
        int lane = 0;
        if (n > mb || m->lane_depth > 1) TRY(pick_lane(m, &lane));   // a lone micro-batch stays on the caller's stream
        LaneGuard guard(m, lane);
        TRY(detect_batch_here(m, frames + (size_t)f0 * 3 * H * W, f0, nb, H, W, ep, ob + (size_t)f0 * D * 4, os + (size_t)f0 * D,
                              ol + (size_t)f0 * D));
    }
    return scope.join();
}

// n frames through the whole backbone once, every exit's heads applied to its own stage tensor on the way.
// Outputs are exit-major: exit e (1-based) fills the block at (e - 1) * n frames.
int detect_frames_all_exits(thia_model* m, const uint8_t* frames, int n, int H, int W, float* ob, float* os, int32_t* ol) {
    TRY(ensure_workspace(m, H, W));
    const int mb = m->ws.mb, D = m->D;
    const bool debug = m->debug;
    m->debug = false;  // the taps describe one exit; this call records none
    int rc = THIA_OK;
    for (int f0 = 0; f0 < n && rc == THIA_OK; f0 += mb) {
        const int nb = std::min(mb, n - f0);
        Trunk t;
        rc = run_stem(m, frames + (size_t)f0 * 3 * H * W, nb, H, W, t);
        for (int e = 1; e <= m->n_exits && rc == THIA_OK; ++e) {
            if (exit_stages(m, e) > 0) {
                // every stage is followed by the next one here, so the tail layer is the next stage's first 1x1
                const int sidx = exit_stages(m, e) - 1;
                const Tail tl = e < m->n_exits ? stage_tail(m, sidx, 0) : Tail{};
                bool applied = false;
                rc = run_stage(m, sidx, nb, t, &tl, &applied);
                if (applied) t.c1_done = true;
            }
            if (rc != THIA_OK) break;
            const size_t o = (size_t)(e - 1) * n + f0;
            rc = run_heads(m, t.x, f0, nb, H, W, e, ob + o * D * 4, os + o * D, ol + o * D);
        }
    }
    m->debug = debug;
    return rc;
}

// Grow-only device buffer of the model: a larger request replaces it (after waiting for work that may still use it).
template <typename T>
int grow_buffer(thia_model* m, T*& p, size_t& cap, size_t need) {
    if (need <= cap) return THIA_OK;
    if (p) {
        HIP_TRY(m, hipStreamSynchronize(m->stream));
        (void)hipFree(p);
        p = nullptr; cap = 0;
    }
    void* q = nullptr;
    if (hipMalloc(&q, need * sizeof(T)) != hipSuccess) return fail(m, THIA_E_NOMEM, "staging allocation failed");
    p = static_cast<T*>(q);
    cap = need;
    return THIA_OK;
}
int ensure_staging(thia_model* m, thia_model::Staging& st, size_t frame_bytes, size_t rows, size_t flags, size_t opt) {
    TRY(grow_buffer(m, st.frames, st.frames_cap, frame_bytes));
    if (rows > st.out_rows) {
        if (st.ob || st.os || st.ol) {
            HIP_TRY(m, hipStreamSynchronize(m->stream));
            (void)hipFree(st.ob); (void)hipFree(st.os); (void)hipFree(st.ol);
            st.ob = st.os = nullptr; st.ol = nullptr; st.out_rows = 0;
        }
        const size_t D = (size_t)m->D;
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&st.ob), rows * D * 16);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&st.os), rows * D * 4);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&st.ol), rows * D * 4);
        if (e != hipSuccess) {
            (void)hipFree(st.ob); (void)hipFree(st.os); (void)hipFree(st.ol);
            st.ob = st.os = nullptr; st.ol = nullptr;
            return fail(m, THIA_E_NOMEM, std::string("staging outputs: ") + hipGetErrorString(e));
        }
        st.out_rows = rows;
    }
    TRY(grow_buffer(m, st.flags, st.flags_cap, flags));
    TRY(grow_buffer(m, st.opt, st.opt_cap, opt));
    return THIA_OK;
}
void free_staging(thia_model::Staging& st) {
    (void)hipFree(st.frames); (void)hipFree(st.ob); (void)hipFree(st.os); (void)hipFree(st.ol); (void)hipFree(st.flags); (void)hipFree(st.opt);
    st = thia_model::Staging{};
}

// The frames of `spans` (disjoint, any order) at exit ep.  Frames are independent of each other, so chunks of one exit
// share micro-batches: adjacent chunks are joined, and what is left over of chunks shorter than the micro-batch is gathered
// into a staging batch (device-to-device copies of 3 H W bytes per frame), run, and its detections copied to the frames'
// own output positions.  Every frame's result equals that of a stand-alone call on its chunk.
struct Span { int start, len; };
int run_spans(thia_model* m, const uint8_t* frames, int H, int W, int ep, std::vector<Span> spans, float* ob, float* os, int32_t* ol) {
    if (spans.empty()) return THIA_OK;
    std::sort(spans.begin(), spans.end(), [](const Span& a, const Span& b) { return a.start < b.start; });
    std::vector<Span> runs;
    for (const Span& sp : spans) {
        if (sp.len <= 0) continue;
        if (!runs.empty() && runs.back().start + runs.back().len == sp.start) runs.back().len += sp.len;
        else runs.push_back(sp);
    }
    LaneScope scope(m);
    TRY(scope.begin());
    const int mb = microbatch_frames(m, H, W);
    const size_t D = (size_t)m->D, fbytes = (size_t)3 * H * W;
    std::vector<Span> rest;   // what is left of each run after its whole micro-batches
    for (const Span& r : runs) {
        const int whole = r.len / mb * mb;
        if (whole > 0)
            TRY(detect_frames(m, frames + (size_t)r.start * fbytes, whole, H, W, ep, ob + (size_t)r.start * D * 4, os + (size_t)r.start * D,
                              ol + (size_t)r.start * D));
        if (r.len > whole) rest.push_back({r.start + whole, r.len - whole});
    }
    size_t i = 0;
    int off = 0;   // frames of rest[i] already taken
    while (i < rest.size()) {
        std::vector<Span> pieces;
        int total = 0;
        while (i < rest.size() && total < mb) {
            const int take = std::min(mb - total, rest[i].len - off);
            pieces.push_back({rest[i].start + off, take});
            total += take;
            off += take;
            if (off == rest[i].len) { ++i; off = 0; }
        }
        if (pieces.size() == 1) {
            const Span& q = pieces[0];
            TRY(detect_frames(m, frames + (size_t)q.start * fbytes, q.len, H, W, ep, ob + (size_t)q.start * D * 4, os + (size_t)q.start * D,
                              ol + (size_t)q.start * D));
            continue;
        }
        // gather, run and scatter on one lane, with that lane's staging buffers
        int lane = 0;
        TRY(pick_lane(m, &lane));
        LaneGuard guard(m, lane);
        TRY(ensure_staging(m, m->stg, (size_t)mb * fbytes, (size_t)mb, 0, 0));
        int pos = 0;
        for (const Span& q : pieces) {
            HIP_TRY(m, hipMemcpyAsync(m->stg.frames + (size_t)pos * fbytes, frames + (size_t)q.start * fbytes, (size_t)q.len * fbytes,
                                      hipMemcpyDeviceToDevice, m->stream));
            pos += q.len;
        }
        TRY(detect_batch_here(m, m->stg.frames, 0, total, H, W, ep, m->stg.ob, m->stg.os, m->stg.ol));
        pos = 0;
        for (const Span& q : pieces) {
            HIP_TRY(m, hipMemcpyAsync(ob + (size_t)q.start * D * 4, m->stg.ob + (size_t)pos * D * 4, (size_t)q.len * D * 16, hipMemcpyDeviceToDevice, m->stream));
            HIP_TRY(m, hipMemcpyAsync(os + (size_t)q.start * D, m->stg.os + (size_t)pos * D, (size_t)q.len * D * 4, hipMemcpyDeviceToDevice, m->stream));
            HIP_TRY(m, hipMemcpyAsync(ol + (size_t)q.start * D, m->stg.ol + (size_t)pos * D, (size_t)q.len * D * 4, hipMemcpyDeviceToDevice, m->stream));
            pos += q.len;
        }
    }
    return scope.join();
}

void free_estimator(thia_model* m) {
    (void)hipFree(m->est_w1t); (void)hipFree(m->est_b1); (void)hipFree(m->est_w2); (void)hipFree(m->est_b2); (void)hipFree(m->est_pooled);
    m->est_w1t = m->est_b1 = m->est_w2 = m->est_b2 = m->est_pooled = nullptr;
    m->est_hidden = 0; m->est_pooled_cap = 0;
}

// n frames to the last stage once: the estimator reads that stage's tensor, the last exit's units give the reference detections.
int estimate_frames(thia_model* m, const uint8_t* frames, int n, int H, int W, int32_t* opt, float* logits, float* ob, float* os,
                    int32_t* ol) {
    TRY(ensure_workspace(m, H, W));
    const int mb = m->ws.mb, D = m->D, E = m->n_exits;
    const ExitGeom g = exit_geom(m, E, H, W);
    const size_t need = (size_t)mb * g.C * sizeof(float);
    if (need > m->est_pooled_cap) {
        if (m->est_pooled) { HIP_TRY(m, hipStreamSynchronize(m->stream)); (void)hipFree(m->est_pooled); m->est_pooled = nullptr; m->est_pooled_cap = 0; }
        HIP_TRY(m, hipMalloc(reinterpret_cast<void**>(&m->est_pooled), need));
        m->est_pooled_cap = need;
    }
    const bool debug = m->debug;
    m->debug = false;
    int rc = THIA_OK;
    for (int f0 = 0; f0 < n && rc == THIA_OK; f0 += mb) {
        const int nb = std::min(mb, n - f0);
        Trunk t;
        rc = run_stem(m, frames + (size_t)f0 * 3 * H * W, nb, H, W, t);
        for (int s = 0; s < exit_stages(m, E) && rc == THIA_OK; ++s) {
            const Tail tl = s + 1 < exit_stages(m, E) ? stage_tail(m, s, 0) : Tail{};
            bool applied = false;
            rc = run_stage(m, s, nb, t, &tl, &applied);
            if (applied) t.c1_done = true;
        }
        if (rc != THIA_OK) break;
        {
            Scope sc(m, THIA_K_POST);
            const hipError_t e = launch_estimator(t.x, nb, g.Hk * g.Wk, g.C, m->precision, m->est_pooled, m->est_hidden, E, m->est_w1t,
                                                  m->est_b1, m->est_w2, m->est_b2, opt + f0, logits ? logits + (size_t)f0 * E : nullptr,
                                                  m->stream);
            if (e != hipSuccess) { rc = fail_hip(m, e, "launch_estimator"); break; }
        }
        rc = run_heads(m, t.x, f0, nb, H, W, E, ob + (size_t)f0 * D * 4, os + (size_t)f0 * D, ol + (size_t)f0 * D);
    }
    m->debug = debug;
    return rc;
}

}  // namespace

// =================================================================== C ABI
extern "C" {

int thia_load_model(const void* weights, size_t nbytes, int n_exits, thia_model** out) {
    if (!weights || !out) return THIA_E_BADARG;
    *out = nullptr;
    if (nbytes < kHeaderBytes || (nbytes - kHeaderBytes) % 4) return THIA_E_BLOB;
    int32_t h[64];
    float hf[64];
    std::memcpy(h, weights, 256);
    std::memcpy(hf, weights, 256);
    if (h[0] != kMagic || h[1] != 1) return THIA_E_BLOB;
    const int stem_exit = h[38] ? 1 : 0;
    if (h[3] != n_exits || n_exits < 1 || n_exits > 4 + stem_exit) return THIA_E_BLOB;
    thia_model* m = new (std::nothrow) thia_model();
    if (!m) return THIA_E_NOMEM;
    m->precision = h[2];
    m->esz = m->precision ? 2 : 4;
    m->n_exits = n_exits;
    m->stem_exit = stem_exit;
    for (int i = 0; i < 4; ++i) m->blocks_n[i] = h[4 + i];
    m->stem_ch = h[8]; m->has_lateral = h[9]; m->head_ch = h[10];
    m->anc.n_sizes = h[11]; m->anc.n_ratios = h[12];
    m->pre = h[25]; m->post = h[26]; m->rpn_thr = hf[27]; m->pool = h[28]; m->sampling = h[29];
    m->fc_dim = h[30]; m->Kc = h[31]; m->score_thr = hf[32]; m->det_thr = hf[33]; m->D = h[34];
    m->mean = hf[35]; m->stdv = hf[36]; m->base_width = h[37];
    auto bad = [&](int code) { thia_free_model(m); return code; };
    {   // resolve this GPU's copy of the fixed NMS buffer now, so that thia_op_nms_noalloc only ever reads the table
        uint64_t* unused = nullptr;
        if (nms_scratch_ptr(m, &unused) != THIA_OK) return bad(THIA_E_HIP);
    }
    if ((m->precision != 0 && m->precision != 1) || m->anc.n_sizes < 1 || m->anc.n_sizes > 8 || m->anc.n_ratios < 1 ||
        m->anc.n_ratios > 4 || m->pre < 1 || m->pre > 4096 || m->post < 1 || m->post > m->pre || m->Kc < 2 || m->Kc > 256 ||
        m->D < 1 || m->D > 512 || m->pool < 1 || m->pool > 16 || !(m->stdv > 0.f))
        return bad(THIA_E_BLOB);
    // kernel limits: channel counts multiples of 64, 64 stem channels, 2x2 sampling
    if (m->stem_ch != 64 || m->base_width < 64 || m->base_width % 64 || m->head_ch < 64 || m->head_ch % 64 || m->fc_dim < 64 ||
        m->fc_dim % 64 || m->sampling != 2)
        return bad(THIA_E_SHAPE);
    if (m->has_lateral != 0 && m->has_lateral != 1) return bad(THIA_E_BLOB);
    for (int i = 0; i < 8; ++i) m->anc.sizes[i] = hf[13 + i];
    for (int i = 0; i < 4; ++i) m->anc.sqrt_ratios[i] = i < m->anc.n_ratios ? sqrtf(hf[21 + i]) : 1.f;

    BlobReader r{reinterpret_cast<const float*>(static_cast<const char*>(weights) + kHeaderBytes),
                 reinterpret_cast<const float*>(static_cast<const char*>(weights) + nbytes)};
    HostLayer stem;
    if (!take_layer(r, stem, m->stem_ch, 3, 7)) return bad(THIA_E_BLOB);
    {   // stem weights as fp32 [(c*7+ky)*7+kx][64]; bf16 precision keeps bf16-representable values
        std::vector<float> w(147 * 64);
        for (int o = 0; o < 64; ++o)
            for (int t = 0; t < 147; ++t) {
                float v = stem.w[(size_t)o * 147 + t];
                if (m->precision) v = bf16_to_f32(f32_to_bf16(v));
                w[(size_t)t * 64 + o] = v;
            }
        if (hipMalloc(reinterpret_cast<void**>(&m->stem_w), w.size() * 4) != hipSuccess) return bad(THIA_E_NOMEM);
        if (hipMalloc(reinterpret_cast<void**>(&m->stem_b), 64 * 4) != hipSuccess) return bad(THIA_E_NOMEM);
        if (hipMemcpy(m->stem_w, w.data(), w.size() * 4, hipMemcpyHostToDevice) != hipSuccess) return bad(THIA_E_HIP);
        if (hipMemcpy(m->stem_b, stem.b, 64 * 4, hipMemcpyHostToDevice) != hipSuccess) return bad(THIA_E_HIP);
        std::vector<bf16_t> wk((size_t)64 * 22 * 8, (bf16_t)0);
        for (int o = 0; o < 64; ++o)
            for (int r = 0; r < 21; ++r)
                for (int kx = 0; kx < 7; ++kx) wk[((size_t)o * 22 + r) * 8 + kx + 1] = f32_to_bf16(stem.w[(size_t)o * 147 + r * 7 + kx]);
        if (hipMalloc(reinterpret_cast<void**>(&m->stem_wk), wk.size() * 2) != hipSuccess) return bad(THIA_E_NOMEM);
        if (hipMemcpy(m->stem_wk, wk.data(), wk.size() * 2, hipMemcpyHostToDevice) != hipSuccess) return bad(THIA_E_HIP);
    }
    int cin = m->stem_ch;
    for (int s = 0; s < n_exits - stem_exit; ++s) {
        const int w = m->base_width << s;
        if (m->blocks_n[s] < 1 || m->blocks_n[s] > 64) return bad(THIA_E_BLOB);
        m->stage[s].resize(m->blocks_n[s]);
        for (int b = 0; b < m->blocks_n[s]; ++b) {
            Block& B = m->stage[s][b];
            B.stride = (b == 0 && s > 0) ? 2 : 1;  // the stride sits on the 3x3 of a stage's first block
            HostLayer c1, c2, c3, sc;
            if (!take_layer(r, c1, w, cin, 1) || !take_layer(r, c2, w, w, 3) || !take_layer(r, c3, 4 * w, w, 1)) return bad(THIA_E_BLOB);
            int rc = upload_layer(m, c1, nullptr, B.c1);
            if (!rc) rc = upload_layer(m, c2, nullptr, B.c2);
            if (b == 0) {
                if (!take_layer(r, sc, 4 * w, cin, 1)) return bad(THIA_E_BLOB);
                B.has_sc = true;
                B.sc_ci = cin;
                // [W3 | Ws] along K, bias b3 + bs: one contraction over (t2 channels, x channels)
                std::vector<float> wcat((size_t)4 * w * (w + cin)), bcat((size_t)4 * w);
                for (int o = 0; o < 4 * w; ++o) {
                    std::memcpy(&wcat[(size_t)o * (w + cin)], c3.w + (size_t)o * w, sizeof(float) * w);
                    std::memcpy(&wcat[(size_t)o * (w + cin) + w], sc.w + (size_t)o * cin, sizeof(float) * cin);
                    bcat[o] = c3.b[o] + sc.b[o];
                }
                HostLayer cat;
                cat.w = wcat.data(); cat.b = bcat.data(); cat.co = 4 * w; cat.ci = w + cin; cat.k = 1;
                if (!rc) rc = upload_layer(m, cat, nullptr, B.c3);
                if (m->precision == 1 && w == 128 && cin == 256 && !rc) rc = upload_fragments(m, c1, &B.tf);
                if (m->precision == 1 && w == 64 && cin == 64 && B.stride == 1) {   // projection block of the 64-wide stage
                    if (!rc) rc = upload_fragments(m, c1, &B.f1);
                    if (!rc) rc = upload_fragments(m, c2, &B.f2);
                    if (!rc) rc = upload_fragments(m, cat, &B.f3);
                }
            } else {
                if (!rc) rc = upload_layer(m, c3, nullptr, B.c3);
                if (m->precision == 1 && w == 256 && !rc) rc = upload_fragments(m, c3, &B.t3f);
                if (m->precision == 1 && (w == 64 || w == 128)) {   // widths the single-kernel bottleneck is written for
                    if (!rc) rc = upload_fragments(m, c1, &B.f1);
                    if (!rc) rc = upload_fragments(m, c2, &B.f2);
                    if (!rc) rc = upload_fragments(m, c3, &B.f3);
                }
            }
            if (rc) return bad(rc);
            cin = 4 * w;
        }
    }
    const int A = m->anc.n_sizes * m->anc.n_ratios;
    for (int e = 0; e < n_exits; ++e) {
        ExitUnit& E = m->ex[e];
        const int ce = exit_channels(m, e + 1);
        int hc = ce, rc = THIA_OK;
        HostLayer lat, rc3, obj, dl, fc1, fc2, cls, box;
        if (m->has_lateral) {
            if (!take_layer(r, lat, m->head_ch, ce, 1)) return bad(THIA_E_BLOB);
            hc = m->head_ch;
            rc = upload_layer(m, lat, nullptr, E.lateral);
            if (!rc && m->precision == 1 && ce == 256 && hc == 256) rc = upload_fragments(m, lat, &E.lat_f);
        }
        if (!take_layer(r, rc3, hc, hc, 3) || !take_layer(r, obj, A, hc, 1) || !take_layer(r, dl, 4 * A, hc, 1) ||
            !take_layer(r, fc1, m->fc_dim, hc, m->pool) || !take_layer(r, fc2, m->fc_dim, m->fc_dim, 1) ||
            !take_layer(r, cls, m->Kc, m->fc_dim, 1) || !take_layer(r, box, 4 * m->Kc, m->fc_dim, 1))
            return bad(THIA_E_BLOB);
        if (!rc) rc = upload_layer(m, rc3, nullptr, E.rpn_conv);
        if (!rc) rc = upload_layer(m, obj, &dl, E.rpn_head);
        if (!rc && m->precision == 1 && hc == 256 && 5 * A <= 96) {
            std::vector<float> wcat((size_t)96 * hc, 0.f), bcat(96, 0.f);
            std::memcpy(wcat.data(), dl.w, sizeof(float) * 4 * A * hc);
            std::memcpy(wcat.data() + (size_t)4 * A * hc, obj.w, sizeof(float) * A * hc);
            std::memcpy(bcat.data(), dl.b, sizeof(float) * 4 * A);
            std::memcpy(bcat.data() + 4 * A, obj.b, sizeof(float) * A);
            HostLayer cat;
            cat.w = wcat.data(); cat.b = bcat.data(); cat.co = 96; cat.ci = hc; cat.k = 1;
            rc = upload_fragments(m, cat, &E.head_f);
            if (!rc && hipMalloc(reinterpret_cast<void**>(&E.head_fb), 96 * 4) != hipSuccess) rc = THIA_E_NOMEM;
            if (!rc && hipMemcpy(E.head_fb, bcat.data(), 96 * 4, hipMemcpyHostToDevice) != hipSuccess) rc = THIA_E_HIP;
        }
        // FC1 reads ROI features laid out [(ph*P+pw)][c]: the same O,(kh,kw),I repack as a PxP convolution,
        // after which it is a plain matrix product over K = P*P*hc
        if (!rc) rc = upload_layer(m, fc1, nullptr, E.fc1);
        E.fc1.ci = hc * m->pool * m->pool; E.fc1.k = 1;
        if (!rc) rc = upload_layer(m, fc2, nullptr, E.fc2);
        if (!rc) rc = upload_layer(m, cls, &box, E.pred);
        if (rc) return bad(rc);
    }
    if (r.p != r.end) return bad(THIA_E_BLOB);
    *out = m;
    return THIA_OK;
}

void thia_free_model(thia_model* m) {
    if (m) free_estimator(m);
    if (!m) return;
    (void)hipStreamSynchronize(m->stream);
    if (m->lane_stream) (void)hipStreamSynchronize(m->lane_stream);
    free_workspace(m);
    if (m->ws_alt.arena) (void)hipFree(m->ws_alt.arena);
    free_staging(m->stg); free_staging(m->stg_alt); free_staging(m->qry); free_staging(m->qout);
    if (m->ev_fork) (void)hipEventDestroy(m->ev_fork);
    if (m->ev_join) (void)hipEventDestroy(m->ev_join);
    if (m->lane_stream) (void)hipStreamDestroy(m->lane_stream);
    for (auto& t : m->taps) if (t.buf) (void)hipFree(t.buf);
    for (auto e : m->ev_pool) (void)hipEventDestroy(e);
    if (m->stem_w) (void)hipFree(m->stem_w);
    if (m->stem_wk) (void)hipFree(m->stem_wk);
    if (m->stem_b) (void)hipFree(m->stem_b);
    for (int s = 0; s < 4; ++s)
        for (Block& B : m->stage[s]) {
            free_layer(B.c1); free_layer(B.c2); free_layer(B.c3);
            if (B.f1) (void)hipFree(B.f1);
            if (B.f2) (void)hipFree(B.f2);
            if (B.f3) (void)hipFree(B.f3);
            if (B.tf) (void)hipFree(B.tf);
            if (B.t3f) (void)hipFree(B.t3f);
            B.f1 = B.f2 = B.f3 = B.tf = B.t3f = nullptr;
        }
    for (int e = 0; e < 5; ++e) {
        ExitUnit& E = m->ex[e];
        free_layer(E.lateral); free_layer(E.rpn_conv); free_layer(E.rpn_head); free_layer(E.fc1); free_layer(E.fc2); free_layer(E.pred);
        if (E.head_f) (void)hipFree(E.head_f);
        if (E.head_fb) (void)hipFree(E.head_fb);
        if (E.lat_f) (void)hipFree(E.lat_f);
        E.head_f = nullptr; E.head_fb = nullptr; E.lat_f = nullptr;
    }
    delete m;
}

int thia_set_stream(thia_model* m, void* hip_stream) {
    if (!m) return THIA_E_BADARG;
    HIP_TRY(m, hipStreamSynchronize(m->stream));
    if (m->lane_stream) HIP_TRY(m, hipStreamSynchronize(m->lane_stream));
    m->stream = static_cast<hipStream_t>(hip_stream);
    return THIA_OK;
}

int thia_set_lanes(thia_model* m, int lanes) {
    if (!m) return THIA_E_BADARG;
    if (lanes < 1 || lanes > 2) return fail(m, THIA_E_BADARG, "lanes must be 1 or 2");
    m->lanes = lanes;
    return THIA_OK;
}

int thia_set_microbatch(thia_model* m, int frames) {
    if (!m) return THIA_E_BADARG;
    if (frames < 0 || frames > 256) return fail(m, THIA_E_BADARG, "microbatch must be within 0..256");
    m->user_mb = frames;
    return THIA_OK;
}

int thia_get_info(const thia_model* m, thia_info* o) {
    if (!m || !o) return THIA_E_BADARG;
    o->precision = m->precision; o->n_exits = m->n_exits;
    for (int i = 0; i < 4; ++i) o->blocks[i] = m->blocks_n[i];
    o->head_ch = m->head_ch; o->n_anchors = m->anc.n_sizes * m->anc.n_ratios;
    o->pre_nms = m->pre; o->post_nms = m->post; o->pool = m->pool; o->fc_dim = m->fc_dim; o->n_classes = m->Kc;
    o->max_det = m->D; o->microbatch = m->user_mb > 0 ? m->user_mb : m->ws.mb; o->has_lateral = m->has_lateral;
    return THIA_OK;
}

int thia_detect_chunk(thia_model* m, const uint8_t* frames, int n, int H, int W, int ep, float* out_boxes, float* out_scores,
                      int32_t* out_labels) {
    TRY(check_frame_args(m, frames, n, H, W, out_boxes, out_scores, out_labels));
    if (ep < 0 || ep > m->n_exits) return fail(m, THIA_E_BADEP, "exit outside 0..n_exits");
    if (n == 0) return THIA_OK;
    if (ep == 0) {
        HIP_TRY(m, launch_fill_empty(n, m->D, out_boxes, out_scores, out_labels, m->stream));
        return THIA_OK;
    }
    return detect_frames(m, frames, n, H, W, ep, out_boxes, out_scores, out_labels);
}

int thia_detect_all_exits(thia_model* m, const uint8_t* frames, int n, int H, int W, float* out_boxes, float* out_scores,
                          int32_t* out_labels) {
    int rc = check_frame_args(m, frames, n, H, W, out_boxes, out_scores, out_labels);
    if (rc != THIA_OK) return rc;
    if (n == 0) return THIA_OK;
    return detect_frames_all_exits(m, frames, n, H, W, out_boxes, out_scores, out_labels);
}

int thia_run_plan(thia_model* m, const uint8_t* frames, int n_chunks, int chunk_len, int H, int W, const int32_t* chunk_ep,
                  float* out_boxes, float* out_scores, int32_t* out_labels) {
    if (!m) return THIA_E_BADARG;
    if (n_chunks < 0 || chunk_len < 0 || (n_chunks > 0 && !chunk_ep)) return fail(m, THIA_E_BADARG, "bad plan arguments");
    if ((long long)n_chunks * chunk_len > (1ll << 30)) return fail(m, THIA_E_BADARG, "plan too long");
    TRY(check_frame_args(m, frames, n_chunks * chunk_len, H, W, out_boxes, out_scores, out_labels));
    for (int c = 0; c < n_chunks; ++c)
        if (chunk_ep[c] < 0 || chunk_ep[c] > m->n_exits) return fail(m, THIA_E_BADEP, "plan holds an exit outside 0..n_exits");
    if (n_chunks == 0 || chunk_len == 0) return THIA_OK;
    const int D = m->D;
    LaneScope scope(m);
    TRY(scope.begin());
    // group chunks by exit: one group after the other, outputs at the frames' own positions; the chunks of a group share
    // micro-batches (run_spans), and micro-batches alternate between the two lanes across the groups
    for (int ep = 0; ep <= m->n_exits; ++ep) {
        std::vector<Span> spans;
        for (int c = 0; c < n_chunks; ++c) {
            if (chunk_ep[c] != ep) continue;
            const size_t f0 = (size_t)c * chunk_len;
            if (ep == 0) HIP_TRY(m, launch_fill_empty(chunk_len, D, out_boxes + f0 * D * 4, out_scores + f0 * D, out_labels + f0 * D, m->stream));
            else spans.push_back({(int)f0, chunk_len});
        }
        if (ep > 0) TRY(run_spans(m, frames, H, W, ep, spans, out_boxes, out_scores, out_labels));
    }
    return scope.join();
}

int thia_run_chunks(thia_model* m, const uint8_t* frames, int n, int H, int W, int n_chunks, const int32_t* start, const int32_t* len,
                    const int32_t* ep, float* out_boxes, float* out_scores, int32_t* out_labels) {
    if (!m) return THIA_E_BADARG;
    if (n_chunks < 0 || (n_chunks > 0 && (!start || !len || !ep))) return fail(m, THIA_E_BADARG, "bad chunk list");
    TRY(check_frame_args(m, frames, n, H, W, out_boxes, out_scores, out_labels));
    std::vector<std::pair<int, int>> spans;
    for (int c = 0; c < n_chunks; ++c) {
        if (ep[c] < 0 || ep[c] > m->n_exits) return fail(m, THIA_E_BADEP, "chunk list holds an exit outside 0..n_exits");
        if (start[c] < 0 || len[c] < 0 || (long long)start[c] + len[c] > n) return fail(m, THIA_E_BADARG, "chunk outside the frames");
        if (len[c] > 0) spans.emplace_back(start[c], start[c] + len[c]);
    }
    std::sort(spans.begin(), spans.end());
    for (size_t i = 1; i < spans.size(); ++i)
        if (spans[i].first < spans[i - 1].second) return fail(m, THIA_E_BADARG, "chunks overlap");
    if (n == 0) return THIA_OK;
    const int D = m->D;
    LaneScope scope(m);
    TRY(scope.begin());
    // frames no chunk covers, and skipped chunks, get the empty pattern
    int pos = 0;
    for (size_t i = 0; i <= spans.size(); ++i) {
        const int upto = i < spans.size() ? spans[i].first : n;
        if (upto > pos)
            HIP_TRY(m, launch_fill_empty(upto - pos, D, out_boxes + (size_t)pos * D * 4, out_scores + (size_t)pos * D,
                                         out_labels + (size_t)pos * D, m->stream));
        if (i < spans.size()) pos = spans[i].second;
    }
    for (int e = 0; e <= m->n_exits; ++e) {
        std::vector<Span> group;
        for (int c = 0; c < n_chunks; ++c) {
            if (ep[c] != e || len[c] == 0) continue;
            const size_t f0 = (size_t)start[c];
            if (e == 0) HIP_TRY(m, launch_fill_empty(len[c], D, out_boxes + f0 * D * 4, out_scores + f0 * D, out_labels + f0 * D, m->stream));
            else group.push_back({start[c], len[c]});
        }
        if (e > 0) TRY(run_spans(m, frames, H, W, e, group, out_boxes, out_scores, out_labels));
    }
    return scope.join();
}

void thia_planner_defaults(thia_planner_cfg* cfg) {
    if (!cfg) return;
    cfg->precision = 0.8; cfg->recall = 0.8;
    cfg->min_chunk = 100; cfg->final_span = 10;
    cfg->posi_enough = 0.1; cfg->posi_skip = 0.0;
    cfg->reuse_dist = 0; cfg->eval_batch = 32; cfg->use_estimator = 0;
}

int thia_eval_predicate(thia_model* m, const int32_t* labels, const float* scores, int rows, const thia_query* q, uint8_t* flags) {
    if (!m) return THIA_E_BADARG;
    if (rows < 0 || !q || (rows > 0 && (!labels || !scores || !flags))) return fail(m, THIA_E_BADARG, "bad predicate arguments");
    HIP_TRY(m, launch_count_predicate(labels, scores, rows, m->D, q->label, q->min_count, q->min_score, flags, m->stream));
    return THIA_OK;
}

int thia_answer_counts(thia_model* m, const uint8_t* answers, const uint8_t* reference, int n, int32_t* counts) {
    if (!m) return THIA_E_BADARG;
    if (n < 0 || !counts || (n > 0 && (!answers || !reference))) return fail(m, THIA_E_BADARG, "bad metric arguments");
    HIP_TRY(m, launch_answer_counts(answers, reference, n, counts, m->stream));
    return THIA_OK;
}

void thia_metrics_from_counts(const int32_t* c, double* prf) {
    if (!c || !prf) return;
    const double tp = c[0], fp = c[1], fn = c[2];
    prf[0] = tp + fp == 0 ? 1.0 : tp / (tp + fp);
    prf[1] = tp + fn == 0 ? 1.0 : tp / (tp + fn);
    prf[2] = prf[0] + prf[1] == 0 ? 0.0 : 2 * prf[0] * prf[1] / (prf[0] + prf[1]);
}

int thia_set_estimator(thia_model* m, int hidden, const float* w1, const float* b1, const float* w2, const float* b2) {
    if (!m) return THIA_E_BADARG;
    if (hidden < 0 || (hidden > 0 && (!w1 || !b1 || !w2 || !b2))) return fail(m, THIA_E_BADARG, "bad estimator arguments");
    const int E = m->n_exits, Cl = exit_channels(m, E);
    if (hidden > 0 && Cl + hidden + E > 16000) return fail(m, THIA_E_SHAPE, "estimator too wide: channels + hidden + exits must not exceed 16000");
    HIP_TRY(m, hipStreamSynchronize(m->stream));
    free_estimator(m);
    if (hidden == 0) return THIA_OK;
    std::vector<float> w1t((size_t)Cl * hidden);
    for (int j = 0; j < hidden; ++j)
        for (int c = 0; c < Cl; ++c) w1t[(size_t)c * hidden + j] = w1[(size_t)j * Cl + c];
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&m->est_w1t), w1t.size() * 4);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&m->est_b1), (size_t)hidden * 4);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&m->est_w2), (size_t)E * hidden * 4);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&m->est_b2), (size_t)E * 4);
    if (e == hipSuccess) e = hipMemcpy(m->est_w1t, w1t.data(), w1t.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(m->est_b1, b1, (size_t)hidden * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(m->est_w2, w2, (size_t)E * hidden * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(m->est_b2, b2, (size_t)E * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) { free_estimator(m); return fail_hip(m, e, "thia_set_estimator"); }
    m->est_hidden = hidden;
    return THIA_OK;
}

int thia_estimate_exit(thia_model* m, const uint8_t* frames, int n, int H, int W, int32_t* opt_ep, float* logits, float* out_boxes,
                       float* out_scores, int32_t* out_labels) {
    int rc = check_frame_args(m, frames, n, H, W, out_boxes, out_scores, out_labels);
    if (rc != THIA_OK) return rc;
    if (n > 0 && !opt_ep) return fail(m, THIA_E_BADARG, "null pointer");
    if (m->est_hidden == 0) return fail(m, THIA_E_BADARG, "no estimator set (thia_set_estimator)");
    if (n == 0) return THIA_OK;
    return estimate_frames(m, frames, n, H, W, opt_ep, logits, out_boxes, out_scores, out_labels);
}

namespace {
int store_plan(const std::vector<PlanChunk>& plan, int cap, int32_t* start, int32_t* len, int32_t* ep) {
    if ((int)plan.size() > cap) return THIA_E_BADARG;
    for (size_t i = 0; i < plan.size(); ++i) { start[i] = plan[i].start; len[i] = plan[i].len; ep[i] = plan[i].ep; }
    return THIA_OK;
}
}  // namespace

int thia_plan_from_flags(const uint8_t* flags, int n, int n_exits, const thia_planner_cfg* cfg, int cap, int32_t* start, int32_t* len,
                         int32_t* ep, thia_plan_stats* stats, uint8_t* evaluated) {
    if (n < 0 || n_exits < 1 || !cfg || cap < 0 || !stats || (n > 0 && !flags) || (cap > 0 && (!start || !len || !ep))) return THIA_E_BADARG;
    if (planner_cfg_error(*cfg)) return THIA_E_BADARG;
    const int E = n_exits;
    PlanEval eval = [&](const int* fr, int k, uint8_t* out, std::string&) {
        for (int i = 0; i < k; ++i)
            for (int e = 0; e < E; ++e) out[(size_t)i * E + e] = flags[(size_t)fr[i] * E + e] ? 1 : 0;
        return (int)THIA_OK;
    };
    std::vector<PlanChunk> plan;
    std::string err;
    const int rc = plan_core(n, E, *cfg, eval, plan, *stats, evaluated, err);
    if (rc != THIA_OK) return rc;
    return store_plan(plan, cap, start, len, ep);
}

namespace {
int plan_query_impl(thia_model* m, const uint8_t* frames, int n, int H, int W, const thia_query* q, const thia_planner_cfg* cfg,
                    int cap, int32_t* start, int32_t* len, int32_t* ep, thia_plan_stats* stats, uint8_t* evaluated,
                    std::vector<uint8_t>* memo_out) {
    if (!m) return THIA_E_BADARG;
    if (n < 0 || !q || !cfg || cap < 0 || !stats || (n > 0 && !frames) || (cap > 0 && (!start || !len || !ep)))
        return fail(m, THIA_E_BADARG, "bad planner arguments");
    if (const char* why = planner_cfg_error(*cfg)) return fail(m, THIA_E_BADARG, why);
    if (H < 32 || W < 32 || H > 16384 || W > 16384) return fail(m, THIA_E_SHAPE, "frame size must be within 32..16384");
    const bool est = cfg->use_estimator != 0;
    if (est && m->est_hidden == 0) return fail(m, THIA_E_BADARG, "use_estimator without an estimator (thia_set_estimator)");
    const int E = m->n_exits, D = m->D;
    const int kb = cfg->eval_batch > 0 ? cfg->eval_batch : 64;  // staging capacity; larger requests are cut into pieces
    const size_t fbytes = (size_t)3 * H * W;
    // staging (owned by the model, grow-only): gathered frames, every exit's detections for them, the answers
    std::vector<uint8_t> hflags((size_t)E * kb);
    std::vector<int32_t> hopt(kb);
    if (n > 0) TRY(ensure_staging(m, m->qry, fbytes * kb, (size_t)E * kb, (size_t)E * kb, (size_t)kb));
    uint8_t *stage = m->qry.frames, *dflags = m->qry.flags;
    float *ob = m->qry.ob, *os = m->qry.os;
    int32_t *ol = m->qry.ol, *dopt = m->qry.opt;
    PlanEval eval = [&](const int* fr, int k, uint8_t* out, std::string& err) -> int {
        for (int o = 0; o < k; o += kb) {
            const int kk = std::min(kb, k - o);
            for (int i = 0; i < kk; ++i) {
                const hipError_t e1 = hipMemcpyAsync(stage + (size_t)i * fbytes, frames + (size_t)fr[o + i] * fbytes, fbytes,
                                                     hipMemcpyDeviceToDevice, m->stream);
                if (e1 != hipSuccess) { err = std::string("planner gather: ") + hipGetErrorString(e1); return THIA_E_HIP; }
            }
            const int rows = est ? kk : E * kk;
            int rc = est ? estimate_frames(m, stage, kk, H, W, dopt, nullptr, ob, os, ol) : detect_frames_all_exits(m, stage, kk, H, W, ob, os, ol);
            if (rc != THIA_OK) { err = m->err; return rc; }
            hipError_t e2 = launch_count_predicate(ol, os, rows, D, q->label, q->min_count, q->min_score, dflags, m->stream);
            if (e2 == hipSuccess) e2 = hipMemcpyAsync(hflags.data(), dflags, (size_t)rows, hipMemcpyDeviceToHost, m->stream);
            if (e2 == hipSuccess && est) e2 = hipMemcpyAsync(hopt.data(), dopt, (size_t)kk * 4, hipMemcpyDeviceToHost, m->stream);
            if (e2 == hipSuccess) e2 = hipStreamSynchronize(m->stream);
            if (e2 != hipSuccess) { err = std::string("planner predicate: ") + hipGetErrorString(e2); return THIA_E_HIP; }
            for (int i = 0; i < kk; ++i)
                for (int e = 0; e < E; ++e) {
                    // evaluated: exit e+1's own answer (exit-major on the device).  Estimated (Sec. 5.3): exit k is taken to
                    // answer like the reference exactly when k >= OPT_EP, which yields the section's TP, FP and FN sums.
                    const bool ref = hflags[est ? i : (size_t)(E - 1) * kk + i] != 0;
                    out[(size_t)(o + i) * E + e] = est ? ((e + 1 >= hopt[i]) == ref ? 1 : 0) : hflags[(size_t)e * kk + i];
                }
        }
        return THIA_OK;
    };
    std::vector<PlanChunk> plan;
    std::string err;
    const int rc = plan_core(n, E, *cfg, eval, plan, *stats, evaluated, err, memo_out);
    if (rc != THIA_OK) return fail(m, rc, err);
    if (store_plan(plan, cap, start, len, ep) != THIA_OK) return fail(m, THIA_E_BADARG, "plan has more chunks than the capacity given");
    return THIA_OK;
}
}  // namespace

int thia_plan_query(thia_model* m, const uint8_t* frames, int n, int H, int W, const thia_query* q, const thia_planner_cfg* cfg,
                    int cap, int32_t* start, int32_t* len, int32_t* ep, thia_plan_stats* stats, uint8_t* evaluated) {
    return plan_query_impl(m, frames, n, H, W, q, cfg, cap, start, len, ep, stats, evaluated, nullptr);
}

int thia_run_query(thia_model* m, const uint8_t* frames, int n, int H, int W, const thia_query* q, const thia_planner_cfg* cfg,
                   uint8_t* answers, int cap, int32_t* start, int32_t* len, int32_t* ep, thia_plan_stats* stats) {
    if (!m) return THIA_E_BADARG;
    if (n > 0 && !answers) return fail(m, THIA_E_BADARG, "null pointer");
    std::vector<uint8_t> evaluated(n > 0 ? n : 1), memo;
    TRY(plan_query_impl(m, frames, n, H, W, q, cfg, cap, start, len, ep, stats, evaluated.data(), &memo));
    if (n == 0) return THIA_OK;
    // Memoisation carried over from the optimisation to the execution (Sec. 5.2): a frame the planner evaluated already has
    // its answer at every exit (evaluation-based selection), or at the reference exit (estimation-based selection, where the
    // other exits' entries are estimates and are not reused).  Such frames are cut out of their chunks; the remainders
    // share micro-batches like any short chunks.
    const int E = m->n_exits;
    const bool est = cfg->use_estimator != 0;
    std::vector<uint8_t> over((size_t)n, (uint8_t)2);
    std::vector<int32_t> cs, cl, ce;
    for (int c = 0; c < stats->n_chunks; ++c) {
        const int e = ep[c];
        if (e == 0 || (est && e != E)) { cs.push_back(start[c]); cl.push_back(len[c]); ce.push_back(e); continue; }
        int a = start[c];
        for (int f = start[c]; f <= start[c] + len[c]; ++f) {
            const bool cut = f == start[c] + len[c] || evaluated[f];
            if (!cut) continue;
            if (f > a) { cs.push_back(a); cl.push_back(f - a); ce.push_back(e); }
            if (f < start[c] + len[c]) over[f] = memo[(size_t)f * E + (e - 1)] ? 1 : 0;
            a = f + 1;
        }
    }
    // the known answers go up first (the stream is idle: planning ended with a synchronisation), detections of all n
    // frames live in a model-owned, grow-only buffer
    TRY(ensure_staging(m, m->qout, 0, (size_t)n, (size_t)n, 0));
    HIP_TRY(m, hipMemcpyAsync(m->qout.flags, over.data(), (size_t)n, hipMemcpyHostToDevice, m->stream));
    HIP_TRY(m, hipStreamSynchronize(m->stream));
    TRY(thia_run_chunks(m, frames, n, H, W, (int)cs.size(), cs.data(), cl.data(), ce.data(), m->qout.ob, m->qout.os, m->qout.ol));
    TRY(thia_eval_predicate(m, m->qout.ol, m->qout.os, n, q, answers));
    HIP_TRY(m, launch_apply_known_answers(m->qout.flags, n, answers, m->stream));
    return THIA_OK;
}

const char* thia_last_error(const thia_model* m) { return m ? m->err.c_str() : "null model"; }

int thia_set_debug(thia_model* m, int enable) {
    if (!m) return THIA_E_BADARG;
    m->debug = enable != 0;
    return THIA_OK;
}

size_t thia_debug_tap_bytes(const thia_model* m, int which) {
    if (!m || which < 0 || which >= THIA_TAP_COUNT) return 0;
    return m->taps[which].bytes;
}

int thia_debug_tap(thia_model* m, int which, void* dst, size_t nbytes) {
    if (!m || !dst) return THIA_E_BADARG;
    if (which < 0 || which >= THIA_TAP_COUNT) return fail(m, THIA_E_BADARG, "unknown tap");
    const Tap& t = m->taps[which];
    if (!t.buf || t.bytes == 0) return fail(m, THIA_E_BADARG, "tap not recorded (call thia_set_debug first)");
    if (nbytes != t.bytes) return fail(m, THIA_E_BADARG, "tap size mismatch");
    HIP_TRY(m, hipStreamSynchronize(m->stream));
    HIP_TRY(m, hipMemcpy(dst, t.buf, nbytes, hipMemcpyDeviceToHost));
    return THIA_OK;
}

int thia_profile_begin(thia_model* m) {
    if (!m) return THIA_E_BADARG;
    HIP_TRY(m, hipStreamSynchronize(m->stream));
    m->profiling = true;
    m->ev_used = 0;
    return THIA_OK;
}

int thia_profile_read(thia_model* m, float* ms, int32_t* launches) {
    if (!m || !ms || !launches) return THIA_E_BADARG;
    HIP_TRY(m, hipStreamSynchronize(m->stream));
    for (int i = 0; i < THIA_K_COUNT; ++i) { ms[i] = 0.f; launches[i] = 0; }
    for (size_t i = 0; i + 1 < m->ev_used; i += 2) {
        float t = 0.f;
        HIP_TRY(m, hipEventElapsedTime(&t, m->ev_pool[i], m->ev_pool[i + 1]));
        const int c = m->ev_class[i / 2];
        ms[c] += t;
        launches[c] += 1;
    }
    m->ev_used = 0;
    return THIA_OK;
}

int thia_profile_end(thia_model* m) {
    if (!m) return THIA_E_BADARG;
    m->profiling = false;
    m->ev_used = 0;
    return THIA_OK;
}

// ------------------------------------------------------------------ single steps
int thia_op_rpn_proposals(thia_model* m, const float* logits, const float* deltas, int n, int H, int W, int ep, int32_t* out_idx,
                          float* out_boxes, int32_t* out_n) {
    if (!m || !logits || !deltas || !out_idx || !out_boxes || !out_n || n <= 0) return fail(m, THIA_E_BADARG, "bad arguments");
    if (ep < 1 || ep > m->n_exits) return fail(m, THIA_E_BADEP, "exit outside 1..n_exits");
    if (H < 32 || W < 32) return fail(m, THIA_E_SHAPE, "frame too small");
    TRY(ensure_workspace(m, H, W));
    const ExitGeom g = exit_geom(m, ep, H, W);
    const long nA = (long)g.Hk * g.Wk * m->anc.n_sizes * m->anc.n_ratios;
    for (int f0 = 0; f0 < n; f0 += m->ws.mb) {
        const int nb = std::min(m->ws.mb, n - f0);
        HIP_TRY(m, launch_rpn_proposals(logits + (size_t)f0 * nA, deltas + (size_t)f0 * nA * 4, nb, nA, m->pre, g.Wk, g.stride, (float)W,
                                        (float)H, m->anc, m->ws.topk, out_idx + (size_t)f0 * m->pre, out_boxes + (size_t)f0 * m->pre * 4,
                                        out_n + f0, m->stream));
    }
    return THIA_OK;
}

int thia_op_nms(thia_model* m, const float* boxes, const int32_t* counts, int n, int cap, float thr, int max_keep, int32_t* out_keep,
                int32_t* out_n) {
    if (!m || !boxes || !counts || !out_keep || !out_n || n <= 0) return fail(m, THIA_E_BADARG, "bad arguments");
    if (cap < 1 || cap > 4096 || max_keep < 1 || max_keep > 4096) return fail(m, THIA_E_SHAPE, "cap and max_keep must be within 1..4096");
    const int words = (cap + 63) / 64;
    void* mask = nullptr;
    if (hipMalloc(&mask, (size_t)n * cap * words * 8) != hipSuccess) return fail(m, THIA_E_NOMEM, "nms mask allocation failed");
    hipError_t e = launch_nms(boxes, counts, n, cap, thr, max_keep, static_cast<uint64_t*>(mask), out_keep, out_n, nullptr, m->stream);
    hipError_t e2 = hipStreamSynchronize(m->stream);
    (void)hipFree(mask);
    if (e != hipSuccess) return fail_hip(m, e, "launch_nms");
    if (e2 != hipSuccess) return fail_hip(m, e2, "nms sync");
    return THIA_OK;
}

int thia_op_nms_noalloc(thia_model* m, const float* boxes, const int32_t* counts, int n, int cap, float thr, int max_keep,
                        int32_t* out_keep, int32_t* out_n) {
    if (!m || !boxes || !counts || !out_keep || !out_n || n <= 0) return fail(m, THIA_E_BADARG, "bad arguments");
    if (cap < 1 || cap > 4096 || max_keep < 1 || max_keep > 4096) return fail(m, THIA_E_SHAPE, "cap and max_keep must be within 1..4096");
    const size_t words = (size_t)(cap + 63) / 64;
    if ((size_t)n * cap * words > kNmsScratchWords)
        return fail(m, THIA_E_SHAPE, "thia_op_nms_noalloc: n * cap * ceil(cap / 64) exceeds the 1 Mi words (8 MiB) of the fixed overlap-matrix buffer");
    uint64_t* mask = nullptr;
    TRY(nms_scratch_ptr(m, &mask));
    HIP_TRY(m, launch_nms(boxes, counts, n, cap, thr, max_keep, mask, out_keep, out_n, nullptr, m->stream));
    return THIA_OK;
}

int thia_op_roialign(thia_model* m, const void* feat, const float* rois, int n, int Hk, int Wk, int stride, void* out) {
    if (!m || !feat || !rois || !out || n <= 0 || Hk <= 0 || Wk <= 0 || stride <= 0) return fail(m, THIA_E_BADARG, "bad arguments");
    const int Ch = m->has_lateral ? m->head_ch : 0;
    if (!Ch) return fail(m, THIA_E_SHAPE, "thia_op_roialign needs a model with a lateral (fixed head channels)");
    HIP_TRY(m, launch_roialign(feat, rois, n, m->post, Hk, Wk, Ch, stride, m->pool, m->precision, out, m->stream));
    return THIA_OK;
}

int thia_op_select_detections(thia_model* m, const float* scores, const float* boxes, const int32_t* roi_n, int n, float* out_boxes,
                              float* out_scores, int32_t* out_labels, int32_t* out_n) {
    if (!m || !scores || !boxes || !roi_n || !out_boxes || !out_scores || !out_labels || n <= 0) return fail(m, THIA_E_BADARG, "bad arguments");
    const int key_cap = next_pow2(m->post * m->Kc);
    void* keys = nullptr;
    if (hipMalloc(&keys, (size_t)n * key_cap * 8) != hipSuccess) return fail(m, THIA_E_NOMEM, "key allocation failed");
    hipError_t e = launch_select(scores, boxes, roi_n, n, m->post, m->Kc, m->score_thr, m->det_thr, m->D, static_cast<uint64_t*>(keys),
                                 key_cap, out_boxes, out_scores, out_labels, out_n, m->stream);
    hipError_t e2 = hipStreamSynchronize(m->stream);
    (void)hipFree(keys);
    if (e != hipSuccess) return fail_hip(m, e, "launch_select");
    if (e2 != hipSuccess) return fail_hip(m, e2, "select sync");
    return THIA_OK;
}

int thia_op_conv(thia_model* m, const void* in, int n, int H, int W, int Cin, const float* weights, const float* bias, int Cout, int k,
                 int stride, int pad, const void* residual, int relu, int out_f32, void* out) {
    if (!m || !in || !weights || !bias || !out || n <= 0 || H <= 0 || W <= 0 || Cout <= 0 || k <= 0 || stride <= 0 || pad < 0)
        return fail(m, THIA_E_BADARG, "bad arguments");
    if (Cin <= 0 || Cin % 64) return fail(m, THIA_E_SHAPE, "Cin must be a multiple of 64");
    if (conv_out(H, k, stride, pad) <= 0 || conv_out(W, k, stride, pad) <= 0) return fail(m, THIA_E_SHAPE, "empty output");
    HostLayer hl;
    hl.w = weights; hl.b = bias; hl.co = Cout; hl.ci = Cin; hl.k = k;
    Layer L;
    int rc = upload_layer(m, hl, nullptr, L);
    if (rc == THIA_OK) rc = run_conv(m, THIA_K_CONV, L, in, n, H, W, stride, pad, residual, relu != 0, out_f32 != 0, out);
    hipError_t e2 = hipStreamSynchronize(m->stream);
    free_layer(L);
    if (rc != THIA_OK) return rc;
    if (e2 != hipSuccess) return fail_hip(m, e2, "conv sync");
    return THIA_OK;
}

int thia_set_fusion(thia_model* m, int on) {
    if (!m) return THIA_E_BADARG;
    m->fuse_blocks = on != 0;
    m->fuse_always = on == 2;
    return THIA_OK;
}

namespace {
int op_bottleneck_impl(thia_model* m, const void* in, int n, int H, int W, int width, const float* w1, const float* b1, const float* w2,
                       const float* b2, const float* w3, const float* b3, const float* ws, const float* bs, void* out, const float* wt,
                       const float* bt, int tail_n, int tail_relu, void* out_tail) {
    if (!m || !in || !out || !w1 || !b1 || !w2 || !b2 || !w3 || !b3 || n <= 0 || H <= 0 || W <= 0 || in == out || (ws == nullptr) != (bs == nullptr))
        return fail(m, THIA_E_BADARG, "bad arguments");
    if (m->precision != 1) return fail(m, THIA_E_SHAPE, "the single-kernel bottleneck exists for bf16 models only");
    const bool first = ws != nullptr;
    if (width != 64 && !(width == 128 && !first)) return fail(m, THIA_E_SHAPE, "unsupported bottleneck width");
    const int cin = first ? width : 4 * width;
    HostLayer l1, l2, l3;
    l1.w = w1; l1.b = b1; l1.co = width; l1.ci = cin; l1.k = 1;
    l2.w = w2; l2.b = b2; l2.co = width; l2.ci = width; l2.k = 3;
    l3.w = w3; l3.b = b3; l3.co = 4 * width; l3.ci = width; l3.k = 1;
    std::vector<float> wcat, b3v(b3, b3 + 4 * width);
    if (first) {   // [W3 | Ws] along K, summed biases
        wcat.resize((size_t)4 * width * 2 * width);
        for (int o = 0; o < 4 * width; ++o) {
            std::memcpy(&wcat[(size_t)o * 2 * width], w3 + (size_t)o * width, sizeof(float) * width);
            std::memcpy(&wcat[(size_t)o * 2 * width + width], ws + (size_t)o * width, sizeof(float) * width);
            b3v[o] += bs[o];
        }
        l3.w = wcat.data(); l3.ci = 2 * width;
    }
    FusedBlockArgs fa{};
    fa.x = static_cast<const bf16_t*>(in); fa.y = static_cast<bf16_t*>(out);
    fa.N = n; fa.H = H; fa.W = W; fa.first = first ? 1 : 0;
    bf16_t* f[4] = {nullptr, nullptr, nullptr, nullptr};
    float* bias = nullptr;
    auto cleanup = [&]() {
        for (bf16_t* q : f) if (q) (void)hipFree(q);
        if (bias) (void)hipFree(bias);
    };
    int rc = upload_fragments(m, l1, &f[0]);
    if (!rc) rc = upload_fragments(m, l2, &f[1]);
    if (!rc) rc = upload_fragments(m, l3, &f[2]);
    if (!rc && tail_n > 0) {
        HostLayer lt;
        lt.w = wt; lt.b = bt; lt.co = tail_n; lt.ci = 4 * width; lt.k = 1;
        rc = upload_fragments(m, lt, &f[3]);
    }
    if (!rc && hipMalloc(reinterpret_cast<void**>(&bias), ((size_t)6 * width + tail_n) * 4) != hipSuccess) rc = fail(m, THIA_E_NOMEM, "bias allocation failed");
    if (!rc) {
        std::vector<float> hb((size_t)6 * width + tail_n);
        std::memcpy(hb.data(), b1, sizeof(float) * width);
        std::memcpy(hb.data() + width, b2, sizeof(float) * width);
        std::memcpy(hb.data() + 2 * width, b3v.data(), sizeof(float) * 4 * width);
        if (tail_n > 0) std::memcpy(hb.data() + 6 * width, bt, sizeof(float) * tail_n);
        if (hipMemcpy(bias, hb.data(), hb.size() * 4, hipMemcpyHostToDevice) != hipSuccess) rc = fail(m, THIA_E_HIP, "bias upload failed");
    }
    if (rc) { cleanup(); return rc; }
    fa.w1f = f[0]; fa.w2f = f[1]; fa.w3f = f[2];
    fa.b1 = bias; fa.b2 = bias + width; fa.b3 = bias + 2 * width;
    if (tail_n > 0) { fa.wtf = f[3]; fa.bt = bias + 6 * width; fa.z = static_cast<bf16_t*>(out_tail); fa.tail_n = tail_n; fa.tail_relu = tail_relu; }
    hipError_t e = fused_block_supported(fa, width) ? launch_fused_block(fa, width, m->stream) : hipErrorInvalidValue;
    hipError_t e2 = hipStreamSynchronize(m->stream);
    cleanup();
    if (e == hipErrorInvalidValue) return fail(m, THIA_E_SHAPE, "shape not covered by the single-kernel bottleneck");
    if (e != hipSuccess) return fail_hip(m, e, "launch_fused_block");
    if (e2 != hipSuccess) return fail_hip(m, e2, "bottleneck sync");
    return THIA_OK;
}
}  // namespace

int thia_op_bottleneck(thia_model* m, const void* in, int n, int H, int W, int width, const float* w1, const float* b1, const float* w2,
                       const float* b2, const float* w3, const float* b3, const float* ws, const float* bs, void* out) {
    return op_bottleneck_impl(m, in, n, H, W, width, w1, b1, w2, b2, w3, b3, ws, bs, out, nullptr, nullptr, 0, 0, nullptr);
}

int thia_op_bottleneck_tail(thia_model* m, const void* in, int n, int H, int W, const float* w1, const float* b1, const float* w2,
                            const float* b2, const float* w3, const float* b3, const float* wt, const float* bt, int tail_n, int tail_relu,
                            void* out, void* out_tail) {
    if (!m) return THIA_E_BADARG;
    if (!wt || !bt || !out_tail || (tail_n != 128 && tail_n != 256)) return fail(m, THIA_E_BADARG, "bad tail arguments");
    return op_bottleneck_impl(m, in, n, H, W, 64, w1, b1, w2, b2, w3, b3, nullptr, nullptr, out, wt, bt, tail_n, tail_relu, out_tail);
}

int thia_op_stem(thia_model* m, const uint8_t* frames, int n, int H, int W, void* out) {
    if (!m || !frames || !out || n <= 0) return fail(m, THIA_E_BADARG, "bad arguments");
    if (H < 32 || W < 32) return fail(m, THIA_E_SHAPE, "frame too small");
    const int Hs = conv_out(H, 7, 2, 3), Ws = conv_out(W, 7, 2, 3);
    void* tmp = nullptr;
    hipError_t e;
    if (m->precision == 1) {
        e = launch_stem_pool(frames, n, H, W, m->stem_wk, m->stem_b, m->mean, m->stdv, out, m->stream);
    } else {
        if (hipMalloc(&tmp, (size_t)n * Hs * Ws * 64 * m->esz) != hipSuccess) return fail(m, THIA_E_NOMEM, "stem scratch allocation failed");
        e = launch_stem(frames, n, H, W, m->stem_w, m->stem_b, m->mean, m->stdv, tmp, m->stream);
        if (e == hipSuccess) e = launch_maxpool(tmp, n, Hs, Ws, 64, m->precision, out, m->stream);
    }
    hipError_t e2 = hipStreamSynchronize(m->stream);
    if (tmp) (void)hipFree(tmp);
    if (e != hipSuccess) return fail_hip(m, e, "stem launch");
    if (e2 != hipSuccess) return fail_hip(m, e2, "stem sync");
    return THIA_OK;
}

}  // extern "C"
