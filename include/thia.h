/*
 * thia.h - C ABI of the MI355X (gfx950) execution engine for a multi-exit two-stage
 * object detector run over chunks of video frames.
 *
 * The method (THIA, arXiv 2102.08481): ONE resident detector (backbone -> region
 * proposal network -> region-of-interest head, Sec. 2.1) carries several exit
 * points (EPs): extra RPN + ROI units attached to earlier backbone stages (Sec. 4.1,
 * Sec. 4.2, Table 4, Fig. "EI in Faster-RCNN").  A query plan is a list of chunks
 * (contiguous frame segments, Sec. 2.2), each assigned an EP or "skip" (Sec. 3,
 * execution engine; Algorithm 1 emits {chunk : EP} pairs).  The engine runs every
 * frame of a chunk through the backbone truncated at the chunk's EP and then through
 * that EP's RPN, proposal decoding, NMS, ROIAlign and box head, and returns per frame
 * the detected objects: category, box, confidence (Sec. 2.1).
 *
 * Conventions common to all calls
 *  - "dev" pointers are device memory on the current HIP device, "host" pointers are
 *    ordinary host memory.  The caller owns every buffer it passes in; the library owns
 *    the weights and its workspace inside thia_model.
 *  - Calls enqueue work on the model's stream (thia_set_stream; default: the null
 *    stream) and return without waiting, unless stated otherwise.  The caller
 *    synchronises before reading outputs.  (Calls that run several micro-batches also
 *    use a second stream inside, joined into the model's stream before they return:
 *    thia_set_lanes.)
 *  - Return value: THIA_OK (0) or a negative THIA_E_* code; thia_last_error() gives a
 *    message.  On an argument error nothing is enqueued and outputs are untouched.
 *  - Exits are numbered 1..n_exits (exit k reads the output of backbone stage
 *    conv(k+1)_x, stride 4 * 2^(k-1)); 0 means "skip the chunk".  A model whose header
 *    sets the stem-exit flag has up to five exits as in the paper's case study (Sec. 4.2,
 *    Table 4): exit 1 reads the pooled stem output (64 channels, stride 4) and exit
 *    k >= 2 reads conv(k)_x.
 *  - Detections: at most D = thia_info.max_det per frame, sorted by descending score.
 *    out_boxes [n,D,4] = (x1,y1,x2,y2) in pixels, out_scores [n,D], out_labels [n,D]
 *    = foreground class 1..n_classes-1.  Unused slots: box 0, score 0, label -1.
 *  - A model must not be used from two threads at once; two calls on the same model
 *    share its workspace and are ordered by the stream.
 */
#ifndef THIA_H
#define THIA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct thia_model thia_model;

enum {
    THIA_OK = 0,
    THIA_E_BADARG = -1, /* null pointer, negative size                               */
    THIA_E_BADEP = -2,  /* exit outside 0..n_exits                                   */
    THIA_E_SHAPE = -3,  /* frame size or channel count the kernels do not support    */
    THIA_E_BLOB = -4,   /* malformed weights blob / n_exits mismatch                 */
    THIA_E_NOMEM = -5,  /* device or host allocation failed                          */
    THIA_E_HIP = -6     /* a HIP runtime call failed                                 */
};

typedef struct thia_info {
    int32_t precision;  /* 0: fp32 tensors; 1: bf16 weights/activations, fp32 accumulate */
    int32_t n_exits;
    int32_t blocks[4];  /* bottleneck blocks of conv2_x..conv5_x                     */
    int32_t head_ch;    /* channels of the map the RPN and ROIAlign read             */
    int32_t n_anchors;  /* anchors per location                                      */
    int32_t pre_nms, post_nms;
    int32_t pool;       /* ROIAlign output side (7)                                  */
    int32_t fc_dim;
    int32_t n_classes;  /* including background (class 0)                            */
    int32_t max_det;    /* D                                                         */
    int32_t microbatch; /* frames processed together (0 = chosen per frame size)     */
    int32_t has_lateral;
} thia_info;

/*
 * Load the single multi-exit model (Sec. 4.1: one model, no model switching).
 * weights: host, nbytes bytes: 256-byte little-endian header (hyper-parameters) then
 * fp32 tensors, conv weights [Cout,Cin,kh,kw], FC weights [out,in] with FC1's input
 * index = c*pool*pool + ph*pool + pw, each weight followed by its bias; order: stem,
 * stages, then per exit lateral (optional), rpn.conv, rpn.obj, rpn.delta, fc1, fc2,
 * cls, box.  n_exits must equal the header's (1..4, or 1..5 with the stem-exit flag,
 * header word 38).  The blob may be freed after the call.
 * Blocking (allocates and uploads).  All channel counts except the 3 input channels
 * and the predictor outputs must be multiples of 64.
 */
int thia_load_model(const void* weights, size_t nbytes, int n_exits, thia_model** out);

/* Waits for the model's stream, then frees weights and workspace. NULL is allowed. */
void thia_free_model(thia_model* m);

/* hip_stream: a hipStream_t (e.g. torch.cuda.current_stream().cuda_stream); NULL = null stream. */
int thia_set_stream(thia_model* m, void* hip_stream);

/* Frames processed together inside a call (workspace grows with it); 0 restores the
 * default.  Results never depend on it: every frame is computed independently. */
int thia_set_microbatch(thia_model* m, int frames);

/* Bottleneck blocks and layer pairs that have a fused kernel variant run through it (on = 1,
 * the default, where the variant pays; on = 2: wherever it applies, also at sizes too small
 * for it to pay) or layer by layer (on = 0).  All give the same tensors up to the
 * accumulation order; the switch exists for measurements and tests. */
int thia_set_fusion(thia_model* m, int on);

/* Micro-batches of one call are independent of each other (Sec. 3: chunks are processed one by one, frames
 * within them batched).  lanes = 2 (the default): a call that runs more than one micro-batch (thia_run_plan,
 * thia_run_chunks, thia_run_query, thia_detect_chunk with more frames than a micro-batch) alternates them
 * between the model's stream and a second stream owned by the model, with a second workspace, so one
 * micro-batch's proposal and selection kernels overlap the next one's convolutions.  The second stream starts
 * after everything queued on the model's stream when the call began, and the model's stream waits for it
 * before the call returns: callers see single-stream ordering, and results do not change.  lanes = 1: one
 * stream, one workspace.  Profiling and debug taps always run on one lane. */
int thia_set_lanes(thia_model* m, int lanes);

int thia_get_info(const thia_model* m, thia_info* out);

/*
 * Run one chunk at one exit (Sec. 3: the engine executes a chunk at the exit the plan
 * chose; Sec. 4.1: inference is short-circuited there, later stages are not run).
 * frames: dev, uint8 [n,3,H,W] (planar RGB), n >= 0.  ep: 1..n_exits, or 0 = skip
 * (outputs are filled with the empty pattern).  Outputs: dev, see above.
 * H, W >= 32.  May (re)allocate workspace when (H, W, microbatch) changes; that
 * first call then blocks.
 */
int thia_detect_chunk(thia_model* m, const uint8_t* frames, int n, int H, int W, int ep,
                      float* out_boxes, float* out_scores, int32_t* out_labels);

/*
 * Run every exit on the same frames in one pass (Sec. 5.2, evaluation-based exit
 * selection: the planner scores all exits on each sampled frame against the reference
 * exit; Sec. 6.8: exits share parameters and the features already computed).  The
 * backbone runs once to the last stage and exit e's units read stage e's tensor on the
 * way, so exit e's result is bit-identical to thia_detect_chunk(..., ep = e) while the
 * earlier stages are evaluated once instead of once per exit.
 * frames: dev uint8 [n,3,H,W].  Outputs: dev, exit-major: out_boxes float32
 * [n_exits,n,D,4], out_scores float32 [n_exits,n,D], out_labels int32 [n_exits,n,D],
 * each exit's block laid out as thia_detect_chunk's.  Debug taps are not recorded.
 * Errors and workspace behaviour as for thia_detect_chunk.
 */
int thia_detect_all_exits(thia_model* m, const uint8_t* frames, int n, int H, int W,
                          float* out_boxes, float* out_scores, int32_t* out_labels);

/*
 * Run a fine-grained plan (Sec. 3; Algorithm 1's output): frames dev uint8
 * [n_chunks*chunk_len,3,H,W]; chunk c = frames [c*chunk_len, (c+1)*chunk_len) runs at
 * exit chunk_ep[c] (host int32 [n_chunks], 0 = skip).  Chunks are grouped by exit and
 * enqueued group by group; outputs are written at the frames' own
 * positions, so out_* are laid out exactly as for n_chunks*chunk_len frames of
 * thia_detect_chunk, and each chunk's slice is bit-identical to a stand-alone call.  Chunks of
 * one exit share micro-batches (frames are independent): adjacent chunks are joined, and the
 * remainders of chunks shorter than the micro-batch are gathered into a staging batch.
 */
int thia_run_plan(thia_model* m, const uint8_t* frames, int n_chunks, int chunk_len, int H, int W,
                  const int32_t* chunk_ep, float* out_boxes, float* out_scores, int32_t* out_labels);

/*
 * Run chunks of any length (the planner's chunks are halves of halves of the video, Sec. 5.2,
 * so they differ in length): frames dev uint8 [n,3,H,W]; chunk c = frames
 * [start[c], start[c]+len[c]) runs at exit ep[c] (0 = skip); start/len/ep host int32
 * [n_chunks]; chunks must lie inside 0..n and must not overlap.  Outputs as for n frames of
 * thia_detect_chunk; frames no chunk covers get the empty pattern.  Grouped by exit like
 * thia_run_plan, and each chunk's slice is bit-identical to a stand-alone call on it.
 */
int thia_run_chunks(thia_model* m, const uint8_t* frames, int n, int H, int W, int n_chunks, const int32_t* start,
                    const int32_t* len, const int32_t* ep, float* out_boxes, float* out_scores, int32_t* out_labels);

/* ---------------------------------------------------------------- query planning
 * Fine-grained planning (Sec. 5.2, Algorithm 1): the video is sampled sparsely, every exit
 * is evaluated on the samples and compared with the last exit (the reference), and a chunk
 * either gets the fastest exit that is accurate enough, is skipped, or is halved and sampled
 * twice as densely.  The query is Table 2's: frames with Count(class) >= t.
 */
typedef struct thia_query {
    int32_t label;     /* class to count (1..n_classes-1)                                   */
    int32_t min_count; /* t: the frame is positive when at least t objects are found        */
    float min_score;   /* detections below this confidence are not counted                  */
} thia_query;

typedef struct thia_planner_cfg {
    double precision, recall; /* P, R an exit must reach on the samples (0.8, 0.8)            */
    int32_t min_chunk;        /* no chunk is shorter than this many frames (100)              */
    int32_t final_span;       /* 1 / final sampling rate: the deepest level samples every     */
                              /* final_span-th frame (rate 0.1 -> 10); level 0 samples every  */
                              /* final_span * 2^ceil(log2(n / min_chunk))-th (the rate bound)  */
    double posi_enough;       /* ratio of positive samples from which a chunk is settled at   */
                              /* the fastest exit                                             */
    double posi_skip;         /* ratio of positive samples up to which a chunk is skipped     */
    int32_t reuse_dist;       /* a memoised frame of the same chunk within this many frames   */
                              /* stands in for a sample (0 = exact reuse only)                */
    int32_t eval_batch;       /* frames evaluated per device batch (0 = all of a level)       */
    int32_t use_estimator;    /* 1: estimation-based exit selection (thia_plan_query only;    */
                              /* needs thia_set_estimator), 0: evaluation-based               */
} thia_planner_cfg;

typedef struct thia_plan_stats {
    int32_t n_chunks;         /* chunks of the plan (also set when the capacity is too small) */
    int32_t frames_evaluated; /* frames on which every exit was run                           */
    int32_t samples_reused;   /* samples answered from memoised frames                        */
    int32_t depth;            /* deepest level reached (0 = the whole video)                  */
    int32_t eval_batches;     /* device batches issued                                        */
} thia_plan_stats;

/* The paper's constants (P = R = 0.8, chunks of at least 100 frames, final rate 0.1) and this
 * library's choices where it names none (posi_enough 0.1, posi_skip 0, reuse_dist 0, eval_batch 32). */
void thia_planner_defaults(thia_planner_cfg* cfg);

/*
 * Count(class) >= t on detection slots: labels dev int32 [rows,D], scores dev float32 [rows,D]
 * (any number of frames, e.g. all exits' outputs at once), flags dev uint8 [rows] (1 = positive).
 */
int thia_eval_predicate(thia_model* m, const int32_t* labels, const float* scores, int rows, const thia_query* q,
                        uint8_t* flags);

/*
 * Accuracy of frame answers relative to the reference exit's (Sec. 6.1: every system is scored
 * against the reference model's answers): answers, reference dev uint8 [n] (as written by
 * thia_eval_predicate), counts dev int32 [3] = true positives, false positives, false negatives.
 */
int thia_answer_counts(thia_model* m, const uint8_t* answers, const uint8_t* reference, int n, int32_t* counts);

/*
 * Precision, recall and F-1 from such counts (host int32 [3] -> host double [3]).  An empty
 * denominator gives 1 for precision / recall (no false claim made, nothing to recall); F-1 is
 * the harmonic mean, 0 when both are 0.
 */
void thia_metrics_from_counts(const int32_t* counts, double* prf);

/*
 * Exit estimator (Sec. 5.3): a two-layer network on the last backbone stage's features names,
 * per frame, the fastest exit that is still right (OPT_EP).  This library's reading of the
 * two layers: features averaged over the positions, hidden = relu(W1 x + b1), logits =
 * W2 hidden + b2, OPT_EP = 1 + arg-max (the faster exit on a tie), all in fp32.
 * thia_set_estimator copies the weights (host float32: w1 [hidden, C], b1 [hidden],
 * w2 [n_exits, hidden], b2 [n_exits], C = channels of the last stage); hidden = 0 removes
 * them.  C + hidden + n_exits must not exceed 16000.
 */
int thia_set_estimator(thia_model* m, int hidden, const float* w1, const float* b1, const float* w2, const float* b2);

/*
 * Reference exit and estimator on the same frames in one backbone pass: opt_ep dev int32 [n]
 * (1..n_exits), logits dev float32 [n, n_exits] or NULL, out_* the last exit's detections as
 * thia_detect_chunk(ep = n_exits) gives them (bit-identical).  The other exits' units are
 * not run: this is what estimation-based planning saves on every sampled frame.
 */
int thia_estimate_exit(thia_model* m, const uint8_t* frames, int n, int H, int W, int32_t* opt_ep, float* logits,
                       float* out_boxes, float* out_scores, int32_t* out_labels);

/*
 * The planner on a table of answers (host only, touches no device): flags host uint8
 * [n,n_exits], flags[f*n_exits+e] = exit e+1's answer on frame f (only sampled rows are read;
 * the last exit is the reference).  Writes the plan in frame order to start/len/ep (host int32,
 * capacity cap chunks; ep 0 = skip) and the counters to stats.  evaluated (host uint8 [n], may
 * be NULL) marks the frames whose row was "evaluated" rather than reused.  Returns
 * THIA_E_BADARG for a bad configuration or when cap is too small (stats->n_chunks = needed).
 */
int thia_plan_from_flags(const uint8_t* flags, int n, int n_exits, const thia_planner_cfg* cfg, int cap, int32_t* start,
                         int32_t* len, int32_t* ep, thia_plan_stats* stats, uint8_t* evaluated);

/*
 * The planner on a video: frames dev uint8 [n,3,H,W].  Each level's unmemoised samples are
 * gathered and run through every exit in one backbone pass (thia_detect_all_exits) in batches
 * of eval_batch frames, the predicate is applied on the device, and only the per-frame answers
 * come back to the host.  Blocks until the plan is known (it synchronises the model's stream
 * once per batch); its staging buffers belong to the model and only ever grow.  Outputs as
 * for thia_plan_from_flags.  Execute the plan with thia_run_chunks.
 * With cfg->use_estimator the samples go through thia_estimate_exit's path instead, and exit
 * k's true/false positives and false negatives are extrapolated as Sec. 5.3 states them:
 * on a frame the reference exit reports positive, exit k counts as a true positive when
 * k >= OPT_EP and as a false negative otherwise; on a negative frame it counts as a false
 * positive when k < OPT_EP.
 */
int thia_plan_query(thia_model* m, const uint8_t* frames, int n, int H, int W, const thia_query* q,
                    const thia_planner_cfg* cfg, int cap, int32_t* start, int32_t* len, int32_t* ep,
                    thia_plan_stats* stats, uint8_t* evaluated);

/*
 * A whole query (Sec. 3: query -> plan -> execution -> frame IDs; Table 2's form "select frameID where
 * Count(class) >= t"): plans with thia_plan_query, executes the plan with thia_run_chunks and applies
 * the predicate to the detections.  frames dev uint8 [n,3,H,W]; answers dev uint8 [n] (1 = the frame
 * satisfies the predicate; frames of skipped chunks are 0).  plan outputs (start/len/ep, capacity cap)
 * and stats as for thia_plan_query; they may be used to see which exit answered which frame.
 * Frames the planner has already evaluated keep the answer computed then (the same kernels on the same frame give the
 * same detections) and are not run again: answers equals thia_run_chunks on the plan followed by thia_eval_predicate.
 * Blocks while planning; the execution and the predicate are enqueued on the model's stream and
 * the call returns without waiting for them.  The detections of the n frames go to a buffer
 * that belongs to the model and only ever grows.
 */
int thia_run_query(thia_model* m, const uint8_t* frames, int n, int H, int W, const thia_query* q,
                   const thia_planner_cfg* cfg, uint8_t* answers, int cap, int32_t* start, int32_t* len,
                   int32_t* ep, thia_plan_stats* stats);

const char* thia_last_error(const thia_model* m);

/* ---------------------------------------------------------------- inspection
 * Intermediates of the most recent thia_detect_chunk (needed to check the tolerances
 * on RPN logits / box deltas, and to feed single steps).  Recording is off by
 * default; thia_set_debug(m, 1) turns it on for later calls (costs copies + memory).
 * thia_debug_tap waits for the stream and copies tap `which` to dst (host).
 * Layouts (n = frames of the call, T = float or bf16 bits (uint16) per precision):
 */
enum {
    THIA_TAP_FEAT = 0,        /* T   [n,Hk,Wk,Ck]       exit stage output, NHWC          */
    THIA_TAP_HEAD_FEAT = 1,   /* T   [n,Hk,Wk,Ch]       lateral output, NHWC             */
    THIA_TAP_RPN_LOGITS = 2,  /* f32 [n,Hk*Wk*A]        index (y*Wk+x)*A + a             */
    THIA_TAP_RPN_DELTAS = 3,  /* f32 [n,Hk*Wk*A,4]                                       */
    THIA_TAP_TOPK_IDX = 4,    /* i32 [n,pre]            anchor indices, best first, -1 pad */
    THIA_TAP_PROP_BOXES = 5,  /* f32 [n,pre,4]          decoded, clipped, empties dropped */
    THIA_TAP_PROP_N = 6,      /* i32 [n]                                                 */
    THIA_TAP_ROIS = 7,        /* f32 [n,post,4]         zero padded                      */
    THIA_TAP_ROI_N = 8,       /* i32 [n]                                                 */
    THIA_TAP_ROI_FEAT = 9,    /* T   [n,post,P*P,Ch]    index (ph*P+pw)*Ch + c           */
    THIA_TAP_CLS_LOGITS = 10, /* f32 [n,post,Kc]                                         */
    THIA_TAP_BOX_DELTAS = 11, /* f32 [n,post,4*Kc]                                       */
    THIA_TAP_CAND_SCORES = 12,/* f32 [n,post,Kc]                                         */
    THIA_TAP_CAND_BOXES = 13, /* f32 [n,post,Kc,4]                                       */
    THIA_TAP_DET_N = 14,      /* i32 [n]                                                 */
    THIA_TAP_COUNT = 15
};
int thia_set_debug(thia_model* m, int enable);
int thia_debug_tap(thia_model* m, int which, void* dst, size_t nbytes);
/* Bytes tap `which` holds for the most recent call (0 if nothing recorded). */
size_t thia_debug_tap_bytes(const thia_model* m, int which);

/* ---------------------------------------------------------------- timing
 * Per-kernel-class device time, measured with HIP events recorded on the model's
 * stream around every launch while profiling is on.  thia_profile_read waits for the
 * stream, sums the elapsed times since thia_profile_begin and fills ms[THIA_K_COUNT]
 * and launches[THIA_K_COUNT] (host).  Profiling adds two event records per launch.
 */
enum {
    THIA_K_STEM = 0, THIA_K_POOL = 1,
    THIA_K_CONV = 2,  /* backbone stages: implicit-GEMM layers and single-kernel blocks (a stage's last block that also
                         applies the exit's lateral to its own output tile counts here as a whole)                     */
    THIA_K_FC = 3, THIA_K_TOPK = 4, THIA_K_NMS = 5, THIA_K_ROIALIGN = 6, THIA_K_POST = 7,
    THIA_K_RPN = 8,   /* exit unit's implicit GEMMs in front of the proposals: lateral, RPN 3x3, RPN predictors        */
    THIA_K_COUNT = 9
};
int thia_profile_begin(thia_model* m);
int thia_profile_read(thia_model* m, float* ms, int32_t* launches);
int thia_profile_end(thia_model* m);

/* ---------------------------------------------------------------- single steps
 * The kernels of the path, callable on caller-provided device tensors, so that each
 * step can be checked against its definition with identical inputs (the orderings and
 * NMS keeps are then exactly determined).  They use the model's hyper-parameters,
 * stream and workspace; all pointers dev unless noted.
 */

/* Step "top-k + decode" of exit ep on an Hk x Wk map of an H x W frame: per frame the
 * k = min(pre_nms, Hk*Wk*A) best logits by (logit desc, index asc), -0 == +0; their
 * anchors are decoded with the deltas, clipped to the frame, and empty boxes
 * (< 1e-3 px) dropped keeping order.  logits [n,Hk*Wk*A], deltas [n,Hk*Wk*A,4];
 * out_idx [n,pre] (-1 padded), out_boxes [n,pre,4] (zero padded), out_n [n]. */
int thia_op_rpn_proposals(thia_model* m, const float* logits, const float* deltas, int n, int H, int W, int ep,
                          int32_t* out_idx, float* out_boxes, int32_t* out_n);

/* Greedy NMS of boxes already in priority order: box i is kept iff no kept j < i has
 * IoU(i,j) > thr (inter > thr * union, fp32, no fused multiply-add); at most max_keep
 * kept.  boxes [n,cap,4], counts [n] (<= cap <= 4096); out_keep [n,max_keep] positions
 * (-1 padded), out_n [n]. */
int thia_op_nms(thia_model* m, const float* boxes, const int32_t* counts, int n, int cap, float thr, int max_keep,
                int32_t* out_keep, int32_t* out_n);

/* thia_op_nms for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments, same kernels, same
 * results, but the k x k overlap bit matrix lives in a fixed 8 MiB device buffer inside the
 * library (one per GPU, resolved when a model is loaded on that GPU, held until the process
 * ends), and the call neither allocates, frees nor waits: it enqueues on the model's stream
 * and returns.  Limit: n * cap * ceil(cap / 64) <= 2^20 (e.g. 32 frames at cap 1000, 16 at
 * cap 2000, 4 at cap 4096); beyond it THIA_E_SHAPE and nothing is enqueued.  Every word of the
 * buffer that a call reads it has written itself, so nothing needs clearing between calls.  All
 * calls on one GPU share the buffer: calls that overlap in time on one GPU (different streams or
 * models) race; calls on one stream are ordered and safe. */
int thia_op_nms_noalloc(thia_model* m, const float* boxes, const int32_t* counts, int n, int cap, float thr,
                        int max_keep, int32_t* out_keep, int32_t* out_n);

/* ROIAlign (P x P bins, 2 x 2 samples, texel centres at j + 0.5) of rois [n,post,4]
 * (pixels) on feat T [n,Hk,Wk,Ch] with the given stride; out T [n,post,P*P,Ch]. */
int thia_op_roialign(thia_model* m, const void* feat, const float* rois, int n, int Hk, int Wk, int stride, void* out);

/* Detection selection: scores [n,post,Kc], boxes [n,post,Kc,4], roi_n [n]: candidates
 * (roi < roi_n, class >= 1, score > score_thr, box non-empty) ordered by (score desc,
 * roi*Kc + class asc), greedy same-class NMS at det_nms_thr, first D.  Outputs as for
 * thia_detect_chunk, plus out_n [n] (may be NULL). */
int thia_op_select_detections(thia_model* m, const float* scores, const float* boxes, const int32_t* roi_n, int n,
                              float* out_boxes, float* out_scores, int32_t* out_labels, int32_t* out_n);

/* One convolution layer of the path on caller tensors: in T [n,H,W,Cin] NHWC, weights
 * host fp32 [Cout,Cin,k,k] (converted and uploaded by the call, which therefore
 * blocks), bias host fp32 [Cout], optional residual T [n,Ho,Wo,Cout], out T or (if
 * out_f32) float [n,Ho,Wo,Cout].  Cin must be a multiple of 64. */
int thia_op_conv(thia_model* m, const void* in, int n, int H, int W, int Cin, const float* weights, const float* bias,
                 int Cout, int k, int stride, int pad, const void* residual, int relu, int out_f32, void* out);

/* One stride-1 bottleneck block (Section 3 backbone; ResNet bottleneck: 1x1 reduce, 3x3,
 * 1x1 expand, + shortcut, ReLU after each layer and after the sum) as a single kernel,
 * bf16 models only.  ws == NULL (identity shortcut):
 *   out = relu(W3 relu(W2 * relu(W1 in + b1) + b2) + b3 + in),   in [n,H,W,4*width];
 * ws != NULL (projection shortcut of a stage's first block):
 *   out = relu(W3 relu(W2 * relu(W1 in + b1) + b2) + b3 + Ws in + bs),   in [n,H,W,width].
 * Zero padding 1 on the 3x3; both intermediates are rounded to bf16 as in the
 * layer-by-layer path; the projection is not rounded before the sum.  in / out: device
 * bf16 NHWC, out [n,H,W,4*width], distinct buffers; weights host fp32 w1 [width,Cin,1,1],
 * w2 [width,width,3,3], w3 [4*width,width,1,1], ws [4*width,width,1,1] and biases
 * (converted and uploaded by the call, which therefore blocks).  THIA_E_SHAPE for a
 * width without a fused variant (64: both forms; 128: identity shortcut only). */
int thia_op_bottleneck(thia_model* m, const void* in, int n, int H, int W, int width, const float* w1, const float* b1,
                       const float* w2, const float* b2, const float* w3, const float* b3, const float* ws,
                       const float* bs, void* out);

/*
 * The same kernel with a tail layer (Sec. 4.2: an exit's unit, or the next stage, reads the
 * stage's output): the 64-wide identity block also applies z = [relu](Wt y + bt), Wt host
 * float32 [tail_n, 256, 1, 1], tail_n = 128 or 256, to its output tile y and writes
 * out_tail dev [n,H,W,tail_n] next to out.  bf16 models only.
 */
int thia_op_bottleneck_tail(thia_model* m, const void* in, int n, int H, int W, const float* w1, const float* b1,
                            const float* w2, const float* b2, const float* w3, const float* b3, const float* wt,
                            const float* bt, int tail_n, int tail_relu, void* out, void* out_tail);

/* Stem of the backbone on frames dev uint8 [n,3,H,W]: normalise, 7x7/2 conv + ReLU,
 * 3x3/2 max-pool; out T [n,Hp,Wp,stem_ch] NHWC. */
int thia_op_stem(thia_model* m, const uint8_t* frames, int n, int H, int W, void* out);

/* ---------------------------------------------------------------- image classifier with exits
 * The paper's generalisation of early inference (Sec. 4.2, "Generalization" and its figure): the same technique on a
 * VGG-16-style image classifier with eight exits.  The backbone is a stack of 3x3 convolutions (zero padding 1,
 * stride 1, ReLU) with 2x2 / stride-2 max-pools after some of them; exit k taps the output of one convolution layer
 * (after its ReLU, before a pool that may follow) and inference stops there: later layers are not run.  The paper does
 * not define the exit's unit; this library's reading: global average pooling over the tapped map, one fully connected
 * layer to the class logits, soft-max; the answer is the arg-max class (the lowest class on a tie) and its probability.
 *
 * weights: host blob, 256-byte little-endian header (word 0 magic 0x43494854, 1 version 1, 2 precision, 3 n_exits
 * (1..8), 4 convolution layers (1..16), 5 input channels (3), 6 classes, 7 pixel mean (float), 8 pixel std (float),
 * 9..24 output channels per layer, 25..40 "a pool follows" per layer, 41..48 tapped layer (1-based) per exit, strictly
 * increasing) followed by fp32 tensors: per layer weight [Cout,Cin,3,3] and bias [Cout], then per exit the unit's weight
 * [classes, C_tap] and bias [classes].  Channel counts must be multiples of 64 (32 for fp32 models) and at most 1024.
 * Calls enqueue on the classifier's stream and return; errors and ownership as for the detector calls above.
 */
typedef struct thia_classifier thia_classifier;
int thia_classifier_load(const void* weights, size_t nbytes, int n_exits, thia_classifier** out);
void thia_classifier_free(thia_classifier* c);
int thia_classifier_set_stream(thia_classifier* c, void* hip_stream);
const char* thia_classifier_last_error(const thia_classifier* c);

/* frames dev uint8 [n,3,H,W]; ep 1..n_exits, or 0 = skip (labels -1, confidence 0).  out_labels dev int32 [n] (class
 * 0..classes-1), out_conf dev float32 [n] (soft-max probability of that class), out_logits dev float32 [n,classes] or
 * NULL.  May (re)allocate its activation buffers when a larger chunk or frame comes along; that call then blocks. */
int thia_classify_chunk(thia_classifier* c, const uint8_t* frames, int n, int H, int W, int ep, int32_t* out_labels,
                        float* out_conf, float* out_logits);

/* Single steps on caller tensors (NHWC, element type per the model's precision), for checking each against its
 * definition: the 2x2 / stride-2 max-pool (a trailing odd row / column is dropped), in [n,H,W,C] -> out [n,H/2,W/2,C];
 * and exit ep's unit on a tapped map feat [n,HW,C_tap]. */
int thia_classifier_op_pool(thia_classifier* c, const void* in, int n, int H, int W, int C, void* out);
int thia_classifier_op_unit(thia_classifier* c, const void* feat, int n, int HW, int ep, int32_t* out_labels, float* out_conf,
                            float* out_logits);

#ifdef __cplusplus
}
#endif
#endif /* THIA_H */
