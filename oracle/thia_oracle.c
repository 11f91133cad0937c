/*
 * CPU oracle for the multi-exit two-stage detector (THIA, arXiv 2102.08481).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path links, loads or calls
 * this file: it exists so that tests, the smoke check and the benchmark's CPU
 * baseline have an independent, plain statement of what the detector computes.
 * It shares no code with the GPU library.
 *
 * What the paper fixes (Sec. 2.1, Sec. 3 "Early Inference", Sec. 4.1-4.2, Table 4,
 * Fig. "EI in Faster-RCNN"): one detector = backbone -> region proposal network
 * (RPN) -> region-of-interest network (ROI) returning category, box, confidence;
 * additional RPN+ROI units with the same structure are attached to earlier
 * backbone stages (exit points, EPs); inference stops at the chosen EP, so the
 * backbone of EP k is a prefix of that of EP k+1; the execution engine receives a
 * plan = list of chunks, each with an EP or "skip".  The paper defers all layer
 * arithmetic to Faster-RCNN on a ResNet backbone; the conventions used here
 * (anchor geometry, delta decoding, IoU, ROIAlign sampling, tie-breaks) are the
 * readings listed in this repository's design notes and in the comments below.
 *
 * Numerics: tensors are fp32; every dot product is accumulated in double and
 * rounded once.  In "bf16" mode weights and stored activations are additionally
 * rounded to bfloat16 (round-to-nearest-even) at the points marked RB below;
 * head outputs (RPN logits/deltas, class logits, box deltas) and all geometry
 * stay fp32.  Geometry that decides integers (IoU tests, orderings) is evaluated
 * in fp32 with singly rounded operations (compile with -ffp-contract=off).
 *
 * Pins (tests/test_oracle_*.py): conv vs 7-loop integer brute force and 1x1 == matmul;
 * maxpool border cases; top-k vs stable full sort; anchors/decoding vs closed
 * forms; NMS vs O(n^2) definition; ROIAlign on constant / linear maps and a
 * hand-computed 2x2 map; softmax invariants; exit-prefix invariant; plan == per
 * chunk calls.  End-to-end detector numbers have no printed example in the paper:
 * parity unpinned for the composed network beyond those per-step pins.
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_MAGIC 0x41494854
#define ORC_HEADER_BYTES 256
#define ORC_MAX_STAGE 4
#define ORC_MAX_EXIT 5

typedef struct {
    const float *w, *b;
    int co, ci, k;
} orc_layer;

typedef struct {
    orc_layer conv1, conv2, conv3, shortcut; /* shortcut.w == NULL -> identity */
    int stride;
} orc_block;

typedef struct {
    orc_layer lateral, rpn_conv, rpn_obj, rpn_delta, fc1, fc2, cls, box;
} orc_exit;

typedef struct orc_model {
    int precision, n_exits, blocks[4], stem_ch, has_lateral, head_ch;
    int n_sizes, n_ratios;
    float sizes[8], ratios[4];
    int pre_nms, post_nms;
    float rpn_nms_thr;
    int pool, sampling, fc_dim, n_classes;
    float score_thr, det_nms_thr;
    int max_det;
    float mean, std;
    int base_width;
    float *store;             /* private copy of all tensors */
    orc_layer stem;
    orc_block *blk[ORC_MAX_STAGE];
    orc_exit ex[ORC_MAX_EXIT];
    /* 1: exit 1 reads the pooled stem output and exit k >= 2 reads conv(k)_x (the paper's five exits, Sec. 4.2,
     * Table 4: EP-1 on the 64-channel stage); 0: exit k reads conv(k+1)_x */
    int stem_exit;
} orc_model;

/* ---------------------------------------------------------------- bf16 (RB) */
float orc_round_bf16(float x) {
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return x; /* NaN unchanged */
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&x, &u, 4);
    return x;
}
static inline float rb(float x, int bf16) { return bf16 ? orc_round_bf16(x) : x; }

/* ------------------------------------------------------------- model loading */
static const float *take(const float **p, size_t n, const float *end) {
    const float *r = *p;
    if ((size_t)(end - r) < n) return NULL;
    *p = r + n;
    return r;
}
static int take_layer(orc_layer *L, int co, int ci, int k, const float **p, const float *end) {
    L->co = co; L->ci = ci; L->k = k;
    L->w = take(p, (size_t)co * ci * k * k, end);
    L->b = take(p, (size_t)co, end);
    return L->w && L->b;
}

void orc_free(orc_model *m) {
    if (!m) return;
    for (int s = 0; s < ORC_MAX_STAGE; ++s) free(m->blk[s]);
    free(m->store);
    free(m);
}

/* precision_override: -1 = as in the header, 0 = fp32, 1 = bf16 storage. */
orc_model *orc_load(const void *blob, size_t nbytes, int precision_override) {
    if (!blob || nbytes < ORC_HEADER_BYTES) return NULL;
    int32_t h[64];
    float hf[64];
    memcpy(h, blob, 256);
    memcpy(hf, blob, 256);
    if (h[0] != ORC_MAGIC || h[1] != 1) return NULL;
    orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
    m->precision = precision_override < 0 ? h[2] : precision_override;
    m->n_exits = h[3];
    for (int i = 0; i < 4; ++i) m->blocks[i] = h[4 + i];
    m->stem_ch = h[8]; m->has_lateral = h[9]; m->head_ch = h[10];
    m->n_sizes = h[11]; m->n_ratios = h[12];
    m->stem_exit = h[38] ? 1 : 0;
    if (m->n_exits < 1 || m->n_exits > 4 + m->stem_exit || m->n_sizes < 1 || m->n_sizes > 8 || m->n_ratios < 1 || m->n_ratios > 4) { free(m); return NULL; }
    for (int i = 0; i < 8; ++i) m->sizes[i] = hf[13 + i];
    for (int i = 0; i < 4; ++i) m->ratios[i] = hf[21 + i];
    m->pre_nms = h[25]; m->post_nms = h[26]; m->rpn_nms_thr = hf[27];
    m->pool = h[28]; m->sampling = h[29]; m->fc_dim = h[30]; m->n_classes = h[31];
    m->score_thr = hf[32]; m->det_nms_thr = hf[33]; m->max_det = h[34];
    m->mean = hf[35]; m->std = hf[36]; m->base_width = h[37];

    size_t nfl = (nbytes - ORC_HEADER_BYTES) / 4;
    m->store = (float *)malloc(nfl * 4 + 4);
    memcpy(m->store, (const char *)blob + ORC_HEADER_BYTES, nfl * 4);
    const float *p = m->store, *end = m->store + nfl;
    int ok = take_layer(&m->stem, m->stem_ch, 3, 7, &p, end);
    int cin = m->stem_ch;
    for (int s = 0; s < m->n_exits - m->stem_exit && ok; ++s) {
        int w = m->base_width << s;
        m->blk[s] = (orc_block *)calloc((size_t)m->blocks[s] + 1, sizeof(orc_block));
        for (int b = 0; b < m->blocks[s] && ok; ++b) {
            orc_block *B = &m->blk[s][b];
            /* stride 2 sits on the 3x3 of the first block of conv3_x..conv5_x */
            B->stride = (b == 0 && s > 0) ? 2 : 1;
            ok = ok && take_layer(&B->conv1, w, cin, 1, &p, end);
            ok = ok && take_layer(&B->conv2, w, w, 3, &p, end);
            ok = ok && take_layer(&B->conv3, 4 * w, w, 1, &p, end);
            if (b == 0) ok = ok && take_layer(&B->shortcut, 4 * w, cin, 1, &p, end);
            cin = 4 * w;
        }
    }
    int A = m->n_sizes * m->n_ratios;
    for (int e = 0; e < m->n_exits && ok; ++e) {
        orc_exit *E = &m->ex[e];
        int st = e - m->stem_exit; /* stage the exit reads; -1 = the pooled stem output */
        int ce = st < 0 ? m->stem_ch : 4 * (m->base_width << st), hc = ce;
        if (m->has_lateral) { ok = ok && take_layer(&E->lateral, m->head_ch, ce, 1, &p, end); hc = m->head_ch; }
        ok = ok && take_layer(&E->rpn_conv, hc, hc, 3, &p, end);
        ok = ok && take_layer(&E->rpn_obj, A, hc, 1, &p, end);
        ok = ok && take_layer(&E->rpn_delta, 4 * A, hc, 1, &p, end);
        ok = ok && take_layer(&E->fc1, m->fc_dim, hc * m->pool * m->pool, 1, &p, end);
        ok = ok && take_layer(&E->fc2, m->fc_dim, m->fc_dim, 1, &p, end);
        ok = ok && take_layer(&E->cls, m->n_classes, m->fc_dim, 1, &p, end);
        ok = ok && take_layer(&E->box, 4 * m->n_classes, m->fc_dim, 1, &p, end);
    }
    if (!ok || p != end) { orc_free(m); return NULL; }
    return m;
}

int orc_precision(const orc_model *m) { return m->precision; }

/* Threads the parallel loops use (for the benchmark's report of the CPU baseline). */
int orc_num_threads(void) { return omp_get_max_threads(); }

/* geometry of exit k (1-based) for an H x W frame: out = floor((n + 2p - k)/s) + 1 */
static int conv_out(int n, int k, int s, int p) { return (n + 2 * p - k) / s + 1; }
void orc_exit_shape(const orc_model *m, int ep, int H, int W, int *C, int *Hk, int *Wk, int *stride) {
    int h = conv_out(conv_out(H, 7, 2, 3), 3, 2, 1), w = conv_out(conv_out(W, 7, 2, 3), 3, 2, 1);
    int st = ep - m->stem_exit; /* bottleneck stages in front of the exit; 0 = the pooled stem output */
    for (int s = 1; s < st; ++s) { h = conv_out(h, 3, 2, 1); w = conv_out(w, 3, 2, 1); }
    *C = st == 0 ? m->stem_ch : 4 * (m->base_width << (st - 1)); *Hk = h; *Wk = w; *stride = st == 0 ? 4 : 4 << (st - 1);
}

/* ------------------------------------------------------------------- steps */

/* x = (u8 - mean)/std, same constants on all channels; RB in bf16 mode. */
void orc_normalize(const uint8_t *in, long count, float mean, float std, int bf16, float *out) {
#pragma omp parallel for
    for (long i = 0; i < count; ++i) out[i] = rb(((float)in[i] - mean) / std, bf16);
}

/*
 * Direct convolution, NCHW input, OIHW weights, zero padding, output size
 * floor((n + 2p - k)/s) + 1:
 *   out[n,co,oy,ox] = act( b[co] + sum_{ci,ky,kx} w[co,ci,ky,kx] * in[n,ci,oy*s-p+ky,ox*s-p+kx] + residual )
 * One output plane is accumulated in double at a time; weights are rounded to
 * bf16 on the fly in bf16 mode (RB), the result is rounded once (fp32, then RB
 * if round_out).
 */
void orc_conv2d(const float *in, int N, int C, int H, int W, const float *w, const float *b, int Co, int kh,
                int kw, int stride, int pad, const float *residual, int relu, int bf16_weights, int round_out,
                float *out) {
    const int Ho = conv_out(H, kh, stride, pad), Wo = conv_out(W, kw, stride, pad);
#pragma omp parallel
    {
        double *acc = (double *)malloc(sizeof(double) * (size_t)Ho * Wo);
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int n = 0; n < N; ++n)
            for (int co = 0; co < Co; ++co) {
                for (long i = 0; i < (long)Ho * Wo; ++i) acc[i] = (double)b[co];
                for (int ci = 0; ci < C; ++ci)
                    for (int ky = 0; ky < kh; ++ky)
                        for (int kx = 0; kx < kw; ++kx) {
                            const double wv = (double)rb(w[(((size_t)co * C + ci) * kh + ky) * kw + kx], bf16_weights);
                            const float *plane = in + ((size_t)n * C + ci) * H * W;
                            /* ox range with 0 <= ox*stride - pad + kx < W */
                            int ox0 = 0;
                            while (ox0 < Wo && ox0 * stride - pad + kx < 0) ++ox0;
                            int ox1 = Wo;
                            while (ox1 > ox0 && (ox1 - 1) * stride - pad + kx >= W) --ox1;
                            for (int oy = 0; oy < Ho; ++oy) {
                                const int iy = oy * stride - pad + ky;
                                if (iy < 0 || iy >= H) continue;
                                const float *row = plane + (size_t)iy * W;
                                const int off = kx - pad;
                                double *arow = acc + (size_t)oy * Wo;
                                if (stride == 1)
                                    for (int ox = ox0; ox < ox1; ++ox) arow[ox] += wv * (double)row[ox + off];
                                else
                                    for (int ox = ox0; ox < ox1; ++ox) arow[ox] += wv * (double)row[ox * stride + off];
                            }
                        }
                float *o = out + ((size_t)n * Co + co) * Ho * Wo;
                const float *r = residual ? residual + ((size_t)n * Co + co) * Ho * Wo : NULL;
                for (long i = 0; i < (long)Ho * Wo; ++i) {
                    double v = acc[i];
                    if (r) v += (double)r[i];
                    if (relu && v < 0.0) v = 0.0;
                    o[i] = rb((float)v, round_out);
                }
            }
        free(acc);
    }
}

/* 3x3 / stride 2 / pad 1 max pooling; padded positions never win. */
void orc_maxpool3x3s2(const float *in, int N, int C, int H, int W, float *out) {
    const int Ho = conv_out(H, 3, 2, 1), Wo = conv_out(W, 3, 2, 1);
#pragma omp parallel for
    for (long p = 0; p < (long)N * C; ++p)
        for (int oy = 0; oy < Ho; ++oy)
            for (int ox = 0; ox < Wo; ++ox) {
                float best = -INFINITY;
                for (int ky = 0; ky < 3; ++ky)
                    for (int kx = 0; kx < 3; ++kx) {
                        int iy = 2 * oy - 1 + ky, ix = 2 * ox - 1 + kx;
                        if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
                        float v = in[((size_t)p * H + iy) * W + ix];
                        if (v > best) best = v;
                    }
                out[((size_t)p * Ho + oy) * Wo + ox] = best;
            }
}

/* Fully connected: out[m,n] = act(b[n] + sum_k in[m,k] w[n,k]). */
void orc_fc(const float *in, int M, int K, const float *w, const float *b, int Nn, int relu, int bf16_weights,
            int round_out, float *out) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < Nn; ++n) {
            double acc = (double)b[n];
            const float *x = in + (size_t)m * K, *ww = w + (size_t)n * K;
            for (int k = 0; k < K; ++k) acc += (double)x[k] * (double)rb(ww[k], bf16_weights);
            if (relu && acc < 0.0) acc = 0.0;
            out[(size_t)m * Nn + n] = rb((float)acc, round_out);
        }
}

/* ---- ordering: (score descending, index ascending); -0 and +0 are equal. */
typedef struct { float s; int32_t i; } orc_si;
static int cmp_si(const void *a, const void *b) {
    const orc_si *x = (const orc_si *)a, *y = (const orc_si *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->i > y->i) - (x->i < y->i);
}

/* First k = min(k, n) entries of the full ordering of `score`. Returns k. */
int orc_topk(const float *score, long n, int k, int32_t *idx, float *val) {
    orc_si *a = (orc_si *)malloc(sizeof(orc_si) * (size_t)(n > 0 ? n : 1));
    for (long i = 0; i < n; ++i) { a[i].s = score[i]; a[i].i = (int32_t)i; }
    qsort(a, (size_t)n, sizeof(orc_si), cmp_si);
    if (k > n) k = (int)n;
    for (int j = 0; j < k; ++j) { idx[j] = a[j].i; val[j] = a[j].s; }
    free(a);
    return k;
}

/*
 * Anchor of flat index i = (y*Wk + x)*A + a, a = size_idx*n_ratios + ratio_idx:
 * centre ((x+0.5)s, (y+0.5)s), width size/sqrt(r), height size*sqrt(r) (r = h/w,
 * area = size^2).  Returned as (cx, cy, w, h).
 */
void orc_anchor(const orc_model *m, int32_t i, int Wk, int stride, float *cxcywh) {
    const int A = m->n_sizes * m->n_ratios;
    const int a = i % A, loc = i / A, x = loc % Wk, y = loc / Wk;
    const float size = m->sizes[a / m->n_ratios], sr = sqrtf(m->ratios[a % m->n_ratios]);
    cxcywh[0] = ((float)x + 0.5f) * (float)stride;
    cxcywh[1] = ((float)y + 0.5f) * (float)stride;
    cxcywh[2] = size / sr;
    cxcywh[3] = size * sr;
}

/*
 * Box-delta decoding with unit weights and the usual size clamp:
 *   cx' = cx + dx*w, cy' = cy + dy*h, w' = w*exp(min(dw, ln(1000/16))), h' likewise;
 * corners cx' -+ w'/2; x clipped to [0, W], y to [0, H].  Returns 1 when the
 * clipped box is non-empty (both sides >= 1e-3 px).
 */
#define ORC_DELTA_CLAMP 4.135166556742356f /* ln(1000/16) */
int orc_decode(const float *cxcywh, const float *d, float W, float H, float *box) {
    float dw = d[2] < ORC_DELTA_CLAMP ? d[2] : ORC_DELTA_CLAMP;
    float dh = d[3] < ORC_DELTA_CLAMP ? d[3] : ORC_DELTA_CLAMP;
    float cx = cxcywh[0] + d[0] * cxcywh[2];
    float cy = cxcywh[1] + d[1] * cxcywh[3];
    float w = cxcywh[2] * expf(dw), h = cxcywh[3] * expf(dh);
    float hw = 0.5f * w, hh = 0.5f * h;
    float x1 = cx - hw, y1 = cy - hh, x2 = cx + hw, y2 = cy + hh;
    x1 = fminf(fmaxf(x1, 0.f), W); x2 = fminf(fmaxf(x2, 0.f), W);
    y1 = fminf(fmaxf(y1, 0.f), H); y2 = fminf(fmaxf(y2, 0.f), H);
    box[0] = x1; box[1] = y1; box[2] = x2; box[3] = y2;
    return (x2 - x1 >= 1e-3f) && (y2 - y1 >= 1e-3f);
}

/*
 * Overlap test of greedy NMS.  Boxes are continuous (no +1).  Division-free:
 *   iw = max(0, min(ax2,bx2) - max(ax1,bx1)), ih likewise, inter = iw*ih,
 *   uni = (areaA + areaB) - inter;  overlapping iff uni > 0 and inter > thr*uni.
 * Every operation is a singly rounded fp32 operation.
 */
int orc_iou_over(const float *a, const float *b, float thr) {
    float iw = fminf(a[2], b[2]) - fmaxf(a[0], b[0]);
    float ih = fminf(a[3], b[3]) - fmaxf(a[1], b[1]);
    iw = fmaxf(iw, 0.f); ih = fmaxf(ih, 0.f);
    float inter = iw * ih;
    float aa = (a[2] - a[0]) * (a[3] - a[1]);
    float ab = (b[2] - b[0]) * (b[3] - b[1]);
    float uni = (aa + ab) - inter;
    float t = thr * uni;
    return uni > 0.f && inter > t;
}

/*
 * Greedy NMS over boxes already in priority order: box i is kept iff no kept
 * j < i (with the same label, when labels != NULL) overlaps it; stops after
 * max_keep kept.  keep[] receives the kept positions in order; returns count.
 */
int orc_nms(const float *boxes, int n, float thr, int max_keep, const int32_t *labels, int32_t *keep) {
    int nk = 0;
    for (int i = 0; i < n && nk < max_keep; ++i) {
        int ok = 1;
        for (int t = 0; t < nk && ok; ++t) {
            int j = keep[t];
            if (labels && labels[j] != labels[i]) continue;
            if (orc_iou_over(boxes + 4 * (size_t)j, boxes + 4 * (size_t)i, thr)) ok = 0;
        }
        if (ok) keep[nk++] = i;
    }
    return nk;
}

/*
 * ROIAlign, continuous coordinates (texel j has centre j + 0.5), fixed
 * `sampling` x `sampling` points per bin, mean of the samples.  For a point
 * (fx, fy) in feature units: u = fx - 0.5, v = fy - 0.5; outside [-1, Wk] x [-1, Hk]
 * contributes 0; otherwise u, v are clamped to [0, Wk-1], [0, Hk-1] and the four
 * neighbours are blended bilinearly.  feat is [C,Hk,Wk] of ONE frame, rois are
 * [n,4] in pixels, out is [n,C,P,P].
 */
void orc_roialign(const float *feat, int C, int Hk, int Wk, const float *rois, int n, int stride, int P, int S,
                  int round_out, float *out) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int r = 0; r < n; ++r)
        for (int c = 0; c < C; ++c) {
            const double sc = 1.0 / (double)stride;
            const double x1 = rois[4 * r] * sc, y1 = rois[4 * r + 1] * sc;
            const double bw = (rois[4 * r + 2] * sc - x1) / P, bh = (rois[4 * r + 3] * sc - y1) / P;
            const float *f = feat + (size_t)c * Hk * Wk;
            for (int ph = 0; ph < P; ++ph)
                for (int pw = 0; pw < P; ++pw) {
                    double sum = 0.0;
                    for (int iy = 0; iy < S; ++iy)
                        for (int ix = 0; ix < S; ++ix) {
                            double fy = y1 + ph * bh + (iy + 0.5) * bh / S;
                            double fx = x1 + pw * bw + (ix + 0.5) * bw / S;
                            double u = fx - 0.5, v = fy - 0.5;
                            if (u < -1.0 || u > (double)Wk || v < -1.0 || v > (double)Hk) continue;
                            if (u < 0) u = 0;
                            if (v < 0) v = 0;
                            if (u > Wk - 1) u = Wk - 1;
                            if (v > Hk - 1) v = Hk - 1;
                            int x0 = (int)floor(u), y0 = (int)floor(v);
                            int xb = x0 + 1 < Wk ? x0 + 1 : Wk - 1, yb = y0 + 1 < Hk ? y0 + 1 : Hk - 1;
                            double lx = u - x0, ly = v - y0;
                            sum += (1 - ly) * ((1 - lx) * f[(size_t)y0 * Wk + x0] + lx * f[(size_t)y0 * Wk + xb]) +
                                   ly * ((1 - lx) * f[(size_t)yb * Wk + x0] + lx * f[(size_t)yb * Wk + xb]);
                        }
                    out[(((size_t)r * C + c) * P + ph) * P + pw] = rb((float)(sum / (S * S)), round_out);
                }
        }
}

/* Row-wise softmax with the row maximum subtracted. */
void orc_softmax(const float *in, int rows, int K, float *out) {
    for (int r = 0; r < rows; ++r) {
        const float *x = in + (size_t)r * K;
        double mx = x[0], s = 0;
        for (int k = 1; k < K; ++k) if (x[k] > mx) mx = x[k];
        for (int k = 0; k < K; ++k) s += exp((double)x[k] - mx);
        for (int k = 0; k < K; ++k) out[(size_t)r * K + k] = (float)(exp((double)x[k] - mx) / s);
    }
}

/*
 * Detection selection for one frame from per-(roi, class) scores [R,Kc] and
 * boxes [R,Kc,4] (class 0 = background, never emitted): candidates j = roi*Kc + c
 * with score > score_thr and a non-empty box, ordered by (score desc, j asc);
 * greedy NMS between same-label candidates; first D survivors.  Unused output
 * slots: box 0, score 0, label -1.  Returns the number of detections.
 */
int orc_select_detections(const float *scores, const float *boxes, int R, int Kc, float score_thr, float nms_thr,
                          int D, float *out_boxes, float *out_scores, int32_t *out_labels) {
    size_t cap = (size_t)R * Kc + 1;
    orc_si *cand = (orc_si *)malloc(sizeof(orc_si) * cap);
    int nc = 0;
    for (int r = 0; r < R; ++r)
        for (int c = 1; c < Kc; ++c) {
            int j = r * Kc + c;
            const float *bx = boxes + 4 * (size_t)j;
            if (!(scores[j] > score_thr)) continue;
            if (!((bx[2] - bx[0] >= 1e-3f) && (bx[3] - bx[1] >= 1e-3f))) continue;
            cand[nc].s = scores[j]; cand[nc].i = j; ++nc;
        }
    qsort(cand, (size_t)nc, sizeof(orc_si), cmp_si);
    float *cb = (float *)malloc(sizeof(float) * 4 * (size_t)(nc + 1));
    int32_t *cl = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nc + 1));
    int32_t *keep = (int32_t *)malloc(sizeof(int32_t) * (size_t)(D + 1));
    for (int t = 0; t < nc; ++t) { memcpy(cb + 4 * t, boxes + 4 * (size_t)cand[t].i, 16); cl[t] = cand[t].i % Kc; }
    int nk = orc_nms(cb, nc, nms_thr, D, cl, keep);
    for (int d = 0; d < D; ++d) {
        if (d < nk) {
            memcpy(out_boxes + 4 * d, cb + 4 * keep[d], 16);
            out_scores[d] = cand[keep[d]].s; out_labels[d] = cl[keep[d]];
        } else {
            memset(out_boxes + 4 * d, 0, 16); out_scores[d] = 0.f; out_labels[d] = -1;
        }
    }
    free(cand); free(cb); free(cl); free(keep);
    return nk;
}

/* ------------------------------------------------------------- whole detector */

/* Optional copies of intermediates; NULL members are skipped. Sizes per call. */
typedef struct {
    float *feat;        /* [n,Ck,Hk,Wk] exit-stage output                       */
    float *head_feat;   /* [n,Ch,Hk,Wk] lateral output (== feat if no lateral)  */
    float *rpn_logits;  /* [n,Hk*Wk*A]   anchor-index order                     */
    float *rpn_deltas;  /* [n,Hk*Wk*A,4]                                        */
    int32_t *topk_idx;  /* [n,pre]                                              */
    int32_t *topk_n;    /* [n]                                                  */
    float *prop_boxes;  /* [n,pre,4] decoded, clipped, empties dropped          */
    int32_t *prop_n;    /* [n]                                                  */
    float *rois;        /* [n,post,4] zero padded                               */
    int32_t *roi_n;     /* [n]                                                  */
    float *roi_feat;    /* [n,post,Ch*P*P], index c*P*P + ph*P + pw             */
    float *cls_logits;  /* [n,post,Kc]                                          */
    float *box_deltas;  /* [n,post,4*Kc]                                        */
    float *cand_scores; /* [n,post,Kc]                                          */
    float *cand_boxes;  /* [n,post,Kc,4]                                        */
    int32_t *det_n;     /* [n]                                                  */
} orc_taps;

static float *falloc(size_t n) { return (float *)malloc(sizeof(float) * (n ? n : 1)); }

static void run_layer(const orc_layer *L, const float *in, int N, int H, int W, int stride, int pad,
                      const float *residual, int relu, int bf16, int round_out, float *out) {
    orc_conv2d(in, N, L->ci, H, W, L->w, L->b, L->co, L->k, L->k, stride, pad, residual, relu, bf16, round_out, out);
}

/*
 * Backbone up to exit `ep`: normalise, stem 7x7/2 + ReLU, maxpool, then the
 * bottleneck stages conv2_x .. conv(ep+1)_x and nothing after them (early
 * inference: later stages are never evaluated).  Returns a malloc'd [n,C,Hk,Wk].
 * If stage_out != NULL, stage_out[s] receives a malloc'd copy of stage s+1's
 * output for every stage run (used to check the prefix property).  With a stem
 * exit, exit 1 stops after the max-pool and exit k runs k - 1 stages.
 */
float *orc_backbone(const orc_model *m, const uint8_t *frames, int n, int H, int W, int ep, float **stage_out) {
    const int bf = m->precision;
    float *x = falloc((size_t)n * 3 * H * W);
    orc_normalize(frames, (long)n * 3 * H * W, m->mean, m->std, bf, x);
    int h = conv_out(H, 7, 2, 3), w = conv_out(W, 7, 2, 3);
    float *y = falloc((size_t)n * m->stem_ch * h * w);
    run_layer(&m->stem, x, n, H, W, 2, 3, NULL, 1, bf, bf, y);
    free(x);
    int hp = conv_out(h, 3, 2, 1), wp = conv_out(w, 3, 2, 1);
    x = falloc((size_t)n * m->stem_ch * hp * wp);
    orc_maxpool3x3s2(y, n, m->stem_ch, h, w, x);
    free(y);
    h = hp; w = wp;
    for (int s = 0; s < ep - m->stem_exit; ++s) {
        for (int b = 0; b < m->blocks[s]; ++b) {
            const orc_block *B = &m->blk[s][b];
            int ho = conv_out(h, 3, B->stride, 1), wo = conv_out(w, 3, B->stride, 1);
            float *t1 = falloc((size_t)n * B->conv1.co * h * w);
            run_layer(&B->conv1, x, n, h, w, 1, 0, NULL, 1, bf, bf, t1);
            float *t2 = falloc((size_t)n * B->conv2.co * ho * wo);
            run_layer(&B->conv2, t1, n, h, w, B->stride, 1, NULL, 1, bf, bf, t2);
            free(t1);
            float *sc = x;
            if (B->shortcut.w) {
                sc = falloc((size_t)n * B->shortcut.co * ho * wo);
                /* the projection shortcut is summed with the residual branch before the block's single
                 * output rounding: it is not a stored activation, so it is not rounded to bf16 */
                run_layer(&B->shortcut, x, n, h, w, B->stride, 0, NULL, 0, bf, 0, sc);
            }
            float *o = falloc((size_t)n * B->conv3.co * ho * wo);
            run_layer(&B->conv3, t2, n, ho, wo, 1, 0, sc, 1, bf, bf, o);
            free(t2);
            if (sc != x) free(sc);
            free(x);
            x = o; h = ho; w = wo;
        }
        if (stage_out) {
            size_t cnt = (size_t)n * (4 * (m->base_width << s)) * h * w;
            stage_out[s] = falloc(cnt);
            memcpy(stage_out[s], x, cnt * 4);
        }
    }
    return x;
}

/*
 * One chunk at one exit (ep in 1..n_exits; ep == 0 = skip: empty outputs).
 * frames: [n,3,H,W] uint8.  out_boxes [n,D,4], out_scores [n,D], out_labels [n,D].
 * Returns 0, or -1 on bad arguments.
 */
int orc_detect(const orc_model *m, const uint8_t *frames, int n, int H, int W, int ep, float *out_boxes,
               float *out_scores, int32_t *out_labels, const orc_taps *taps) {
    if (!m || n < 0 || ep < 0 || ep > m->n_exits) return -1;
    const int D = m->max_det;
    for (long i = 0; i < (long)n * D; ++i) { out_scores[i] = 0.f; out_labels[i] = -1; }
    memset(out_boxes, 0, sizeof(float) * 4 * (size_t)n * D);
    if (ep == 0 || n == 0) return 0;
    static const orc_taps none;
    if (!taps) taps = &none;
    const int bf = m->precision;
    const orc_exit *E = &m->ex[ep - 1];
    int Ck, Hk, Wk, stride;
    orc_exit_shape(m, ep, H, W, &Ck, &Hk, &Wk, &stride);
    const int A = m->n_sizes * m->n_ratios, P = m->pool, Kc = m->n_classes;
    const long HW = (long)Hk * Wk, nA = HW * A;

    float *feat = orc_backbone(m, frames, n, H, W, ep, NULL);
    if (taps->feat) memcpy(taps->feat, feat, sizeof(float) * (size_t)n * Ck * HW);

    /* exit adaptor: 1x1 lateral to head_ch channels, bias, no activation */
    float *hf = feat;
    int Ch = Ck;
    if (m->has_lateral) {
        Ch = m->head_ch;
        hf = falloc((size_t)n * Ch * HW);
        run_layer(&E->lateral, feat, n, Hk, Wk, 1, 0, NULL, 0, bf, bf, hf);
        free(feat);
    }
    if (taps->head_feat) memcpy(taps->head_feat, hf, sizeof(float) * (size_t)n * Ch * HW);

    /* RPN: 3x3 + ReLU, then 1x1 objectness (A) and 1x1 deltas (4A), fp32 outputs */
    float *t = falloc((size_t)n * Ch * HW);
    run_layer(&E->rpn_conv, hf, n, Hk, Wk, 1, 1, NULL, 1, bf, bf, t);
    float *obj = falloc((size_t)n * A * HW), *dl = falloc((size_t)n * 4 * A * HW);
    run_layer(&E->rpn_obj, t, n, Hk, Wk, 1, 0, NULL, 0, bf, 0, obj);
    run_layer(&E->rpn_delta, t, n, Hk, Wk, 1, 0, NULL, 0, bf, 0, dl);
    free(t);

    const int pre = m->pre_nms, post = m->post_nms;
    float *logits = falloc((size_t)nA), *deltas = falloc((size_t)nA * 4);
    int32_t *tidx = (int32_t *)malloc(sizeof(int32_t) * (size_t)(pre + 1));
    float *tval = falloc((size_t)pre), *pbox = falloc((size_t)pre * 4);
    int32_t *keep = (int32_t *)malloc(sizeof(int32_t) * (size_t)(post + 1));
    float *rois = falloc((size_t)post * 4);
    float *rf = falloc((size_t)post * Ch * P * P);
    float *h1 = falloc((size_t)post * m->fc_dim), *h2 = falloc((size_t)post * m->fc_dim);
    float *cl = falloc((size_t)post * Kc), *bd = falloc((size_t)post * 4 * Kc);
    float *cs = falloc((size_t)post * Kc), *cb = falloc((size_t)post * Kc * 4);

    for (int f = 0; f < n; ++f) {
        /* anchor-index order: i = (y*Wk + x)*A + a */
        for (long loc = 0; loc < HW; ++loc)
            for (int a = 0; a < A; ++a) {
                logits[loc * A + a] = obj[((size_t)f * A + a) * HW + loc];
                for (int j = 0; j < 4; ++j)
                    deltas[(loc * A + a) * 4 + j] = dl[((size_t)f * 4 * A + 4 * a + j) * HW + loc];
            }
        if (taps->rpn_logits) memcpy(taps->rpn_logits + (size_t)f * nA, logits, sizeof(float) * (size_t)nA);
        if (taps->rpn_deltas) memcpy(taps->rpn_deltas + (size_t)f * nA * 4, deltas, sizeof(float) * (size_t)nA * 4);

        /* top-k on raw logits, then decode only those, clip, drop empties (order kept) */
        int k = orc_topk(logits, nA, pre, tidx, tval);
        if (taps->topk_idx) {
            for (int j = 0; j < pre; ++j) taps->topk_idx[(size_t)f * pre + j] = j < k ? tidx[j] : -1;
        }
        if (taps->topk_n) taps->topk_n[f] = k;
        int np = 0;
        for (int j = 0; j < k; ++j) {
            float anc[4], bx[4];
            orc_anchor(m, tidx[j], Wk, stride, anc);
            if (orc_decode(anc, deltas + 4 * (size_t)tidx[j], (float)W, (float)H, bx)) { memcpy(pbox + 4 * np, bx, 16); ++np; }
        }
        if (taps->prop_boxes) {
            memset(taps->prop_boxes + (size_t)f * pre * 4, 0, sizeof(float) * 4 * (size_t)pre);
            memcpy(taps->prop_boxes + (size_t)f * pre * 4, pbox, sizeof(float) * 4 * (size_t)np);
        }
        if (taps->prop_n) taps->prop_n[f] = np;

        /* proposal NMS, keep at most `post` */
        int nr = orc_nms(pbox, np, m->rpn_nms_thr, post, NULL, keep);
        memset(rois, 0, sizeof(float) * 4 * (size_t)post);
        for (int j = 0; j < nr; ++j) memcpy(rois + 4 * j, pbox + 4 * keep[j], 16);
        if (taps->rois) memcpy(taps->rois + (size_t)f * post * 4, rois, sizeof(float) * 4 * (size_t)post);
        if (taps->roi_n) taps->roi_n[f] = nr;

        /* ROIAlign on the head feature map of this frame; FC1 input index c*P*P + ph*P + pw */
        orc_roialign(hf + (size_t)f * Ch * HW, Ch, Hk, Wk, rois, nr, stride, P, m->sampling, bf, rf);
        if (taps->roi_feat) {
            memset(taps->roi_feat + (size_t)f * post * Ch * P * P, 0, sizeof(float) * (size_t)post * Ch * P * P);
            memcpy(taps->roi_feat + (size_t)f * post * Ch * P * P, rf, sizeof(float) * (size_t)nr * Ch * P * P);
        }

        /* box head */
        orc_fc(rf, nr, Ch * P * P, E->fc1.w, E->fc1.b, m->fc_dim, 1, bf, bf, h1);
        orc_fc(h1, nr, m->fc_dim, E->fc2.w, E->fc2.b, m->fc_dim, 1, bf, bf, h2);
        orc_fc(h2, nr, m->fc_dim, E->cls.w, E->cls.b, Kc, 0, bf, 0, cl);
        orc_fc(h2, nr, m->fc_dim, E->box.w, E->box.b, 4 * Kc, 0, bf, 0, bd);
        if (taps->cls_logits) {
            memset(taps->cls_logits + (size_t)f * post * Kc, 0, sizeof(float) * (size_t)post * Kc);
            memcpy(taps->cls_logits + (size_t)f * post * Kc, cl, sizeof(float) * (size_t)nr * Kc);
        }
        if (taps->box_deltas) {
            memset(taps->box_deltas + (size_t)f * post * 4 * Kc, 0, sizeof(float) * (size_t)post * 4 * Kc);
            memcpy(taps->box_deltas + (size_t)f * post * 4 * Kc, bd, sizeof(float) * (size_t)nr * 4 * Kc);
        }

        /* scores and per-class boxes */
        orc_softmax(cl, nr, Kc, cs);
        memset(cb, 0, sizeof(float) * (size_t)post * Kc * 4);
        for (int r = 0; r < nr; ++r) {
            const float *q = rois + 4 * r;
            float rw = q[2] - q[0], rh = q[3] - q[1];
            float anc[4] = {q[0] + 0.5f * rw, q[1] + 0.5f * rh, rw, rh};
            for (int c = 1; c < Kc; ++c)
                orc_decode(anc, bd + ((size_t)r * Kc + c) * 4, (float)W, (float)H, cb + ((size_t)r * Kc + c) * 4);
        }
        if (taps->cand_scores) {
            memset(taps->cand_scores + (size_t)f * post * Kc, 0, sizeof(float) * (size_t)post * Kc);
            memcpy(taps->cand_scores + (size_t)f * post * Kc, cs, sizeof(float) * (size_t)nr * Kc);
        }
        if (taps->cand_boxes) memcpy(taps->cand_boxes + (size_t)f * post * Kc * 4, cb, sizeof(float) * (size_t)post * Kc * 4);

        int nd = orc_select_detections(cs, cb, nr, Kc, m->score_thr, m->det_nms_thr, D, out_boxes + (size_t)f * D * 4,
                                       out_scores + (size_t)f * D, out_labels + (size_t)f * D);
        if (taps->det_n) taps->det_n[f] = nd;
    }
    free(logits); free(deltas); free(tidx); free(tval); free(pbox); free(keep); free(rois); free(rf);
    free(h1); free(h2); free(cl); free(bd); free(cs); free(cb); free(obj); free(dl); free(hf);
    return 0;
}

/*
 * Every exit on the same frames (Sec. 5.2, evaluation-based exit selection: all
 * exits are evaluated on each sampled frame).  By definition this is one
 * orc_detect per exit; outputs are exit-major, [n_exits][n][D]...
 */
int orc_detect_all_exits(const orc_model *m, const uint8_t *frames, int n, int H, int W, float *out_boxes,
                         float *out_scores, int32_t *out_labels) {
    if (!m || n < 0) return -1;
    const size_t D = m->max_det;
    for (int ep = 1; ep <= m->n_exits; ++ep) {
        size_t o = (size_t)(ep - 1) * n;
        int rc = orc_detect(m, frames, n, H, W, ep, out_boxes + o * D * 4, out_scores + o * D, out_labels + o * D, NULL);
        if (rc) return rc;
    }
    return 0;
}

/*
 * Plan execution: frames [n_chunks*chunk_len,3,H,W]; chunk c runs at exit
 * chunk_ep[c] (0 = skip).  Each chunk is exactly one orc_detect call.
 */
int orc_run_plan(const orc_model *m, const uint8_t *frames, int n_chunks, int chunk_len, int H, int W,
                 const int32_t *chunk_ep, float *out_boxes, float *out_scores, int32_t *out_labels) {
    const int D = m->max_det;
    for (int c = 0; c < n_chunks; ++c) {
        size_t f0 = (size_t)c * chunk_len;
        int rc = orc_detect(m, frames + f0 * 3 * H * W, chunk_len, H, W, chunk_ep[c], out_boxes + f0 * D * 4,
                            out_scores + f0 * D, out_labels + f0 * D, NULL);
        if (rc) return rc;
    }
    return 0;
}
