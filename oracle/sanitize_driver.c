/*
 * Sanitizer driver for the CPU oracle (TEST INFRASTRUCTURE ONLY, like the rest of oracle/).
 * Built by tests/test_sanitizers.py together with thia_oracle.c under AddressSanitizer and
 * UndefinedBehaviorSanitizer and run as a plain executable: every entry point is called once
 * on a small model (blob and frames are written by the test from the seeded generators), plus
 * the degenerate inputs the steps must survive (nothing to select, k > n, empty chunks, skip).
 * It checks no values - the pins in tests/test_oracle_*.py do that - only that no access is
 * out of bounds, no value is used uninitialised in an undefined way, and nothing leaks.
 * usage: sanitize_driver blob.bin frames.bin n H W
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct orc_model orc_model;
orc_model *orc_load(const void *blob, size_t nbytes, int precision_override);
void orc_free(orc_model *m);
void orc_exit_shape(const orc_model *m, int ep, int H, int W, int *C, int *Hk, int *Wk, int *stride);
int orc_topk(const float *score, long n, int k, int32_t *idx, float *val);
int orc_nms(const float *boxes, int n, float thr, int max_keep, const int32_t *labels, int32_t *keep);
void orc_roialign(const float *feat, int C, int Hk, int Wk, const float *rois, int n, int stride, int P, int S, int round_out, float *out);
void orc_softmax(const float *in, int rows, int K, float *out);
int orc_select_detections(const float *scores, const float *boxes, int R, int Kc, float score_thr, float nms_thr, int D,
                          float *out_boxes, float *out_scores, int32_t *out_labels);
int orc_detect(const orc_model *m, const uint8_t *frames, int n, int H, int W, int ep, float *out_boxes, float *out_scores,
               int32_t *out_labels, const void *taps);
int orc_detect_all_exits(const orc_model *m, const uint8_t *frames, int n, int H, int W, float *out_boxes, float *out_scores,
                         int32_t *out_labels);
int orc_run_plan(const orc_model *m, const uint8_t *frames, int n_chunks, int chunk_len, int H, int W, const int32_t *chunk_ep,
                 float *out_boxes, float *out_scores, int32_t *out_labels);

static void *slurp(const char *path, size_t *n) {
    FILE *f = fopen(path, "rb");
    if (!f) { perror(path); exit(2); }
    fseek(f, 0, SEEK_END);
    *n = (size_t)ftell(f);
    fseek(f, 0, SEEK_SET);
    void *p = malloc(*n ? *n : 1);
    if (fread(p, 1, *n, f) != *n) { fprintf(stderr, "short read\n"); exit(2); }
    fclose(f);
    return p;
}

int main(int argc, char **argv) {
    if (argc != 6) { fprintf(stderr, "usage: %s blob frames n H W\n", argv[0]); return 2; }
    size_t nb, nf;
    void *blob = slurp(argv[1], &nb);
    uint8_t *frames = slurp(argv[2], &nf);
    const int n = atoi(argv[3]), H = atoi(argv[4]), W = atoi(argv[5]);
    if (nf != (size_t)n * 3 * H * W || n < 2) { fprintf(stderr, "frame file does not hold n >= 2 frames\n"); return 2; }
    int32_t hdr[64];
    memcpy(hdr, blob, 256);
    const int E = hdr[3], D = hdr[34];

    /* a truncated blob and a bad magic must be refused, not read past */
    if (orc_load(blob, 100, -1) || orc_load(blob, nb - 4, -1)) { fprintf(stderr, "truncated blob accepted\n"); return 1; }
    for (int prec = 0; prec < 2; ++prec) {
        orc_model *m = orc_load(blob, nb, prec);
        if (!m) { fprintf(stderr, "blob refused\n"); return 1; }
        float *ob = malloc(sizeof(float) * 4 * (size_t)E * n * D), *os = malloc(sizeof(float) * (size_t)E * n * D);
        int32_t *ol = malloc(sizeof(int32_t) * (size_t)E * n * D);
        for (int ep = 0; ep <= E; ++ep)
            if (orc_detect(m, frames, n, H, W, ep, ob, os, ol, NULL)) return 1;
        if (orc_detect(m, frames, 0, H, W, 1, ob, os, ol, NULL)) return 1;            /* no frames */
        if (!orc_detect(m, frames, n, H, W, E + 1, ob, os, ol, NULL)) return 1;        /* bad exit is an error */
        if (orc_detect_all_exits(m, frames, n, H, W, ob, os, ol)) return 1;
        int32_t *plan = malloc(sizeof(int32_t) * n);
        for (int c = 0; c < n; ++c) plan[c] = c % (E + 1);                             /* includes a skipped chunk */
        if (orc_run_plan(m, frames, n, 1, H, W, plan, ob, os, ol)) return 1;
        if (orc_run_plan(m, frames, 0, 1, H, W, plan, ob, os, ol)) return 1;
        int C, Hk, Wk, st;
        orc_exit_shape(m, E, H, W, &C, &Hk, &Wk, &st);
        free(plan); free(ob); free(os); free(ol);
        orc_free(m);
    }

    /* steps on degenerate inputs */
    float sc[5] = {0.5f, -0.0f, 0.0f, 0.5f, -1.f}, val[8];
    int32_t idx[8];
    if (orc_topk(sc, 5, 8, idx, val) != 5 || orc_topk(sc, 0, 3, idx, val) != 0 || orc_topk(sc, 5, 0, idx, val) != 0) return 1;
    float boxes[3 * 4] = {0, 0, 10, 10, 0, 0, 10, 10, 50, 50, 60, 60};
    int32_t keep[4];
    if (orc_nms(boxes, 0, 0.5f, 4, NULL, keep) != 0 || orc_nms(boxes, 3, 0.5f, 4, NULL, keep) != 2 || orc_nms(boxes, 3, 0.5f, 1, NULL, keep) != 1) return 1;
    float feat[2 * 3 * 4];
    for (int i = 0; i < 24; ++i) feat[i] = (float)i;
    float rois[2 * 4] = {-50, -50, 500, 500, 3.999f, 2.999f, 4.0f, 3.0f}, pooled[2 * 2 * 49];
    orc_roialign(feat, 2, 3, 4, rois, 2, 4, 7, 2, 0, pooled);                          /* far outside the map; sub-texel ROI */
    orc_roialign(feat, 2, 3, 4, rois, 0, 4, 7, 2, 1, pooled);
    float logits[2 * 3] = {1e30f, -1e30f, 0.f, 0.f, 0.f, 0.f}, probs[6];
    orc_softmax(logits, 2, 3, probs);
    float cb[2 * 3 * 4];
    memset(cb, 0, sizeof cb);                                                          /* every candidate box empty */
    float db[4 * 4], ds[4];
    int32_t dl[4];
    if (orc_select_detections(probs, cb, 2, 3, 0.05f, 0.5f, 4, db, ds, dl) != 0) return 1;
    if (orc_select_detections(probs, cb, 0, 3, 0.05f, 0.5f, 4, db, ds, dl) != 0) return 1;

    free(blob); free(frames);
    puts("sanitize_driver: ok");
    return 0;
}
