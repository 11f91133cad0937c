"""Benchmark of the hot path on one MI355X: the four-exit ResNet-50-style detector on a
32-frame batch of synthetic 540x960 traffic frames, swept over exits EP1..EP4.

One "step" = thia_detect_chunk on the resident batch at EP1, EP2, EP3 and EP4 (the whole
hot path at every exit; 4 x 32 frame inferences).  Prints ONE JSON line with the metric, the
roofline of the dominant kernel class and the CPU oracle's rate on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0              # MI355X dense bf16 MFMA peak
CONV_CLASSES = ("conv", "rpn", "fc")   # launches of the implicit-GEMM MFMA kernels: backbone (layers and fused blocks), exit unit, FCs


def conv_out(n, k, s, p):
    return (n + 2 * p - k) // s + 1


def layer_macs(spec, H, W, ep):
    """Algorithmic multiply-accumulates per frame at exit ep: (stem, backbone, lateral+rpn, box head)."""
    h, w = conv_out(H, 7, 2, 3), conv_out(W, 7, 2, 3)
    stem = h * w * spec.stem_ch * 147
    h, w = conv_out(h, 3, 2, 1), conv_out(w, 3, 2, 1)
    back, cin = 0, spec.stem_ch
    for s in range(ep):
        wd = spec.base_width << s
        for b in range(spec.blocks[s]):
            st = 2 if (b == 0 and s > 0) else 1
            ho, wo = conv_out(h, 3, st, 1), conv_out(w, 3, st, 1)
            back += h * w * cin * wd + ho * wo * wd * wd * 9 + ho * wo * wd * 4 * wd
            if b == 0:
                back += ho * wo * cin * 4 * wd
            cin, h, w = 4 * wd, ho, wo
    hc = spec.head_ch if spec.has_lateral else cin
    rpn = h * w * (cin * hc if spec.has_lateral else 0) + h * w * hc * hc * 9 + h * w * hc * 5 * spec.n_anchors
    head = spec.post_nms * (hc * spec.pool ** 2 * spec.fc_dim + spec.fc_dim ** 2 + spec.fc_dim * 5 * spec.n_classes)
    return stem, back, rpn, head


def conv_layer_bytes(spec, H, W, ep, esz=2):
    """Algorithmic HBM bytes per frame of the convolution / FC layers at exit ep, layer by layer and
    unfused: input + output (+ residual) activations once each; weights are negligible and left out.
    (The single-kernel bottleneck blocks move less than this: their intermediates stay in LDS.)"""
    h, w = conv_out(conv_out(H, 7, 2, 3), 3, 2, 1), conv_out(conv_out(W, 7, 2, 3), 3, 2, 1)
    total, cin = 0, spec.stem_ch
    for s in range(ep):
        wd = spec.base_width << s
        for b in range(spec.blocks[s]):
            st = 2 if (b == 0 and s > 0) else 1
            ho, wo = conv_out(h, 3, st, 1), conv_out(w, 3, st, 1)
            total += esz * (h * w * cin + h * w * wd)                       # conv1
            total += esz * (h * w * wd + ho * wo * wd)                      # conv2 (reads every input pixel once)
            total += esz * (ho * wo * wd + 2 * ho * wo * 4 * wd)            # conv3 + residual
            if b == 0:
                total += esz * (ho * wo * cin + ho * wo * 4 * wd)           # shortcut reads the strided pixels only
            cin, h, w = 4 * wd, ho, wo
    hc = spec.head_ch if spec.has_lateral else cin
    A = spec.n_anchors
    if spec.has_lateral:
        total += esz * h * w * (cin + hc)
    total += esz * h * w * 2 * hc + esz * h * w * hc + 4 * h * w * 5 * A   # rpn conv, heads (fp32 out)
    rows = spec.post_nms
    total += esz * rows * (hc * spec.pool ** 2 + spec.fc_dim) + esz * rows * 2 * spec.fc_dim + esz * rows * spec.fc_dim + 4 * rows * 5 * spec.n_classes
    return total


def kernel_sources_sha1():
    """Content hash of the library's kernel sources: the committed counter summary names the sources it was measured on."""
    import hashlib
    d = os.path.join(ROOT, "paper_2102_08481_amd", "csrc")
    h = hashlib.sha1()
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()


def measured_traffic(workload_key):
    """HBM bytes per step of the dominant kernel class from the committed rocprofv3 --pmc summary; None when there is no
    summary or when it was taken on other kernel sources than the ones in this tree (a stale figure is worse than none)."""
    path = os.path.join(ROOT, "profiles", "mfma_kernels_config3_sweep_pmc_fetch_write.txt")
    value, stamp = None, None
    try:
        for line in open(path):
            if line.startswith("TRAFFIC_BYTES_PER_STEP " + workload_key):
                value = float(line.split()[2])
            if line.startswith("KERNEL_SOURCES_SHA1 "):
                stamp = line.split()[1]
    except OSError:
        return None
    return value if stamp == kernel_sources_sha1() else None


def derive_query(labels, scores):
    """A Table-2-style query (Count(class) >= t over detections above a confidence) that is true on about half of the given
    frames.  Random-init predictors put nearly every detection in one class with nearly equal confidence, so the count is
    taken over that class's detections above its median confidence and the threshold is the median such count.
    labels, scores: numpy [n, D] of the reference exit.  Returns (label, t, min_score, ratio of positive frames)."""
    import numpy as np
    label = int(np.bincount(labels[labels > 0].ravel()).argmax())
    min_score = float(np.median(scores[labels == label]))
    cnt = ((labels == label) & (scores >= np.float32(min_score))).sum(axis=1)
    t = max(1, int(np.ceil(np.median(cnt) + 0.5)))
    return label, t, min_score, float((cnt >= t).mean())


def planner_workload(args):
    """Beside the headline metric: query processing time on a long synthetic video, split the way the paper
    splits it (Sec. 6.5): optimisation (the planner's sampling, every exit per sampled frame in one backbone
    pass) and execution (the plan's chunks at their exits), against running the reference exit on every frame."""
    import numpy as np
    import torch
    from paper_2102_08481_amd import planner_cfg, thia_load_model
    from thia_synth import CONFIGS, SceneSpec, make_blob, make_frames, recipe_for

    cfg = CONFIGS[3]
    spec, H, W, N, seg = cfg.model, 540, 960, args.video_frames, 256
    model = thia_load_model(make_blob(spec, cfg.weight_seed, **recipe_for(spec)), spec.n_exits)
    frames = torch.empty((N, 3, H, W), dtype=torch.uint8, device="cuda")
    for i, s0 in enumerate(range(0, N, seg)):         # scenes of 256 frames, alternately sparse and busy
        k = min(seg, N - s0)
        scene = SceneSpec(H, W, k, 1, 3, 16, 60) if i % 2 else SceneSpec(H, W, k, 10, 40, 16, 120)
        frames[s0:s0 + k] = torch.from_numpy(make_frames(scene, cfg.frame_seed + 17 * i)).cuda()
    E = spec.n_exits
    # the query (Table 2's form), chosen on 64 spread frames so that it is neither always nor never true
    sub = frames[:: max(1, N // 64)][:64].contiguous()
    _, sc, lb = model.detect_chunk(sub, E)
    torch.cuda.synchronize()
    label, t, min_score, ratio = derive_query(lb.cpu().numpy(), sc.cpu().numpy())
    pc = planner_cfg()
    model.detect_all_exits(sub[:32].contiguous())     # warm-up: workspace and code objects
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plan, st, ev = model.plan_query(frames, label, t, min_score, pc)
    t1 = time.perf_counter()
    out = model.alloc_outputs(N)
    model.run_chunks(frames[:64], [(0, 64, E)], tuple(o[:64] for o in out))
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    model.run_chunks(frames, plan, out)
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    ans_plan = model.eval_predicate(out[2], out[1], label, t, min_score).bool()
    model.run_chunks(frames, [(0, N, E)], out)
    torch.cuda.synchronize()
    t4 = time.perf_counter()
    ans_ref = model.eval_predicate(out[2], out[1], label, t, min_score).bool()
    tp = int((ans_plan & ans_ref).sum()); fp = int((ans_plan & ~ans_ref).sum()); fn = int((~ans_plan & ans_ref).sum())
    # estimation-based planning (Sec. 5.3) with a random-init two-layer estimator whose outputs are centred on the 64
    # spread frames (there is no labelled data to train it on): what is measured is the cost per sampled frame
    rng = np.random.default_rng(5)
    C_last, hid = 4 * (64 << (E - 1)), 256
    w1, b1 = rng.normal(0, C_last ** -0.5, (hid, C_last)).astype(np.float32), np.zeros(hid, np.float32)
    w2, b2 = rng.normal(0, hid ** -0.5, (E, hid)).astype(np.float32), np.zeros(E, np.float32)
    model.set_estimator(w1, b1, w2, b2)
    _, lg, _ = model.estimate_exit(sub)
    torch.cuda.synchronize()
    model.set_estimator(w1, b1, w2, (-lg.mean(dim=0)).cpu().numpy())
    pe = planner_cfg(use_estimator=1)
    t5 = time.perf_counter()
    plan_e, st_e, _ = model.plan_query(frames, label, t, min_score, pe)
    t6 = time.perf_counter()
    est_ms = 1e3 * (t6 - t5)
    per_exit = {("skip" if e == 0 else f"EP{e}"): int(sum(ln for _, ln, ep in plan if ep == e)) for e in range(E + 1)}
    opt_ms, exe_ms, naive_ms = 1e3 * (t1 - t0), 1e3 * (t3 - t2), 1e3 * (t4 - t3)
    print(json.dumps({
        "metric": "query processing time on a synthetic video: planner (optimisation) + plan execution, vs the reference exit on every frame",
        "value": N / (1e-3 * (opt_ms + exe_ms)), "unit": "frames/s", "n_gpus": 1, "higher_is_better": True, "dtype": "bf16",
        "data": "synthetic", "vs_baseline": None,
        "config": {"workload": f"{N}-frame 540x960 video in 256-frame scenes (alternately busy and sparse), ResNet-50-style 4-exit detector, random-init weights",
                   "query": {"label": label, "min_count": t, "min_score": min_score, "positive_ratio_on_64_spread_frames": ratio},
                   "planner": {"precision": pc.precision, "recall": pc.recall, "min_chunk": pc.min_chunk, "final_span": pc.final_span,
                               "posi_enough": pc.posi_enough, "posi_skip": pc.posi_skip, "reuse_dist": pc.reuse_dist, "eval_batch": pc.eval_batch}},
        "optimise_ms": opt_ms, "execute_ms": exe_ms, "reference_exit_every_frame_ms": naive_ms,
        "speedup_vs_reference_exit": naive_ms / (opt_ms + exe_ms), "planner": st, "frames_per_exit": per_exit,
        "answers_vs_reference": {"precision": tp / max(tp + fp, 1), "recall": tp / max(tp + fn, 1), "positives": tp + fn},
        "optimise_ms_per_sampled_frame": {"evaluation_based": opt_ms / max(st["frames_evaluated"], 1),
                                          "estimation_based": est_ms / max(st_e["frames_evaluated"], 1)},
        "estimation_based": {"optimise_ms": est_ms, "planner": st_e},
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--skip-all-exits", action="store_true", help="leave out the all-exits-in-one-pass timing (for profiler runs)")
    ap.add_argument("--skip-cpu-baseline", action="store_true", help="leave out the oracle timing (for profiler runs)")
    ap.add_argument("--microbatch", type=int, default=0)
    ap.add_argument("--pmc-calibration", action="store_true", help="append one 256 MiB device copy (counter calibration)")
    ap.add_argument("--workload", choices=["sweep", "planner"], default="sweep",
                    help="sweep: the headline metric (default); planner: query planning + execution on a long synthetic video")
    ap.add_argument("--video-frames", type=int, default=2048, help="length of the planner workload's video")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (frames are independent, so more GPUs would each take a share of the chunk); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.workload == "planner":
        return planner_workload(args)

    import numpy as np
    import torch
    from paper_2102_08481_amd import thia_load_model, thia_detect_chunk
    from thia_synth import CONFIGS, make_blob, make_frames, recipe_for

    cfg = CONFIGS[3]
    spec, scene = cfg.model, cfg.scene
    B, H, W = scene.n_frames, scene.height, scene.width
    blob = make_blob(spec, cfg.weight_seed, **recipe_for(spec))
    frames_h = make_frames(scene, cfg.frame_seed)
    model = thia_load_model(blob, spec.n_exits)
    if args.microbatch:
        model.set_microbatch(args.microbatch)
    frames = torch.from_numpy(frames_h).cuda()
    out = model.alloc_outputs(B)
    exits = list(cfg.exits)
    stream = torch.cuda.current_stream()

    def step():
        for ep in exits:
            thia_detect_chunk(model, frames, ep, out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps, inputs resident in HBM, bracketed by device synchronisation.
    # Per-exit times come from events recorded on the stream the kernels run on.
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in exits] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        for i, ep in enumerate(exits):
            ev[k][i][0].record(stream)
            thia_detect_chunk(model, frames, ep, out)
            ev[k][i][1].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    # ---- the same K steps again with the library's HIP events around every kernel launch (two event
    # records per launch, a few per cent slower): per-kernel-class device time for the roofline figure
    # (one exit at a time, so that every class time is also known per exit)
    model.profile_begin()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    prof_exit = {}
    for ep in exits:
        for k in range(args.steps):
            thia_detect_chunk(model, frames, ep, out)
        prof_exit[ep] = model.profile_read()
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    model.profile_end()
    prof = {c: (sum(prof_exit[ep][c][0] for ep in exits), sum(prof_exit[ep][c][1] for ep in exits)) for c in prof_exit[exits[0]]}

    # ---- beside the metric: the same batch with every exit evaluated in ONE backbone pass (what the planner's
    # exit selection needs on its sampled frames); the sweep above pays for the shared stages once per exit
    all_exits_ms = None
    if not args.skip_all_exits:
        out_all = model.detect_all_exits(frames)
        ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        ea.record(stream)
        for k in range(args.steps):
            model.detect_all_exits(frames, out_all)
        eb.record(stream)
        torch.cuda.synchronize()
        all_exits_ms = ea.elapsed_time(eb) / args.steps
        # each exit's frame answers against the last exit's, on the paper's metric (Sec. 6.1: precision / recall / F-1
        # relative to the reference model), for a query derived from the last exit's detections
        E = len(exits)
        qlabel, qt, qscore, qratio = derive_query(out_all[2][E - 1].cpu().numpy(), out_all[1][E - 1].cpu().numpy())
        answers = model.eval_predicate(out_all[2], out_all[1], qlabel, qt, qscore)          # [E, B]
        from paper_2102_08481_amd import metrics_from_counts
        agreement = {"query": {"label": qlabel, "min_count": qt, "min_score": qscore, "positive_ratio_at_reference": qratio}}
        for e in range(E):
            c = model.answer_counts(answers[e].contiguous(), answers[E - 1].contiguous()).cpu().numpy()
            p_, r_, f_ = metrics_from_counts(c)
            agreement[f"EP{e + 1}"] = {"precision": p_, "recall": r_, "f1": f_}

    if args.pmc_calibration:
        # a plain copy of known size, so that a `rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE` run of this command can
        # scale the counters: 256 MiB read + 256 MiB written by one elementwise kernel
        a_ = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        b_ = torch.empty_like(a_)
        a_.zero_()
        torch.cuda.synchronize()
        b_.copy_(a_)
        torch.cuda.synchronize()

    total_s = t1 - t0
    ms_per_step = 1e3 * total_s / args.steps
    per_exit_ms = [float(np.mean([ev[k][i][0].elapsed_time(ev[k][i][1]) for k in range(args.steps)])) for i in range(len(exits))]
    per_exit_fps = {f"EP{ep}": B / (ms * 1e-3) for ep, ms in zip(exits, per_exit_ms)}

    macs = {ep: layer_macs(spec, H, W, ep) for ep in exits}
    conv_flops_step = 2.0 * B * sum(m[1] + m[2] + m[3] for m in macs.values())      # MFMA kernel: backbone + heads + FCs
    conv_ms = sum(prof[c][0] for c in CONV_CLASSES) / args.steps
    conv_launches = sum(prof[c][1] for c in CONV_CLASSES) / args.steps
    achieved = conv_flops_step / (conv_ms * 1e-3) / 1e12
    roofline = {
        "kernel": "implicit-GEMM MFMA kernels: conv_igemm_kernel instantiations + bottleneck_fused kernels (backbone, lateral, RPN, FC)",
        "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
        "traffic": None,   # filled below: bytes per launch from the committed --pmc runs
        "flops_per_step": conv_flops_step, "launches_per_step": conv_launches, "avg_launch_us": 1e3 * conv_ms / max(conv_launches, 1),
        "kernel_ms_per_step": conv_ms,
    }
    # the target's own figure: backbone convolutions alone at the last exit (flops of the stages only; the stem, the
    # exit unit and the box head are neither in the flops nor in the time)
    ep_last = exits[-1]
    bb_ms = prof_exit[ep_last]["conv"][0] / args.steps
    bb_tflops = 2.0 * B * macs[ep_last][1] / (bb_ms * 1e-3) / 1e12
    per_exit_class_ms = {f"EP{ep}": {c: v[0] / args.steps for c, v in prof_exit[ep].items()} for ep in exits}
    per_exit_mfma = {}
    for ep in exits:
        ms_ = sum(prof_exit[ep][c][0] for c in CONV_CLASSES) / args.steps
        per_exit_mfma[f"EP{ep}"] = 2.0 * B * (macs[ep][1] + macs[ep][2] + macs[ep][3]) / (ms_ * 1e-3) / 1e12 / PEAK_BF16_TFLOPS
    class_ms = {k: v[0] / args.steps for k, v in prof.items()}
    alg_bytes_step = float(B * sum(conv_layer_bytes(spec, H, W, ep) for ep in exits))
    roofline["algorithmic_bytes_per_step"] = alg_bytes_step
    tr = measured_traffic("mfma_kernels")
    if tr is not None and not args.microbatch:
        roofline["traffic"] = tr / max(conv_launches, 1)          # per launch, like `achieved`
        roofline["traffic_bytes_per_step"] = tr

    # the two HBM-side steps of the heads, algorithmic bytes over their event time: ROIAlign writes post*P*P*C pooled
    # features per frame (its reads are gathers that mostly hit L2); proposal NMS builds and scans pre*pre bits per frame
    # (a serial greedy chain per frame: latency-bound, the rate is reported, not a bandwidth claim)
    roi_bytes = float(len(exits) * B * spec.post_nms * spec.pool ** 2 * (spec.head_ch if spec.has_lateral else 0) * 2)
    nms_bytes = float(len(exits) * B * spec.pre_nms * ((spec.pre_nms + 63) // 64) * 8)
    hbm_side = {}
    # top-k: the objectness logits (4 bytes per anchor) read once per frame is what the selection needs; the radix
    # select reads them once per pass it takes, so its rate against this figure is below its real read rate
    topk_bytes = 0.0
    for ep in exits:
        h, w = conv_out(conv_out(H, 7, 2, 3), 3, 2, 1), conv_out(conv_out(W, 7, 2, 3), 3, 2, 1)
        for _ in range(ep - 1):
            h, w = conv_out(h, 3, 2, 1), conv_out(w, 3, 2, 1)
        topk_bytes += 4.0 * B * h * w * spec.n_anchors
    for name, nbytes in (("roialign", roi_bytes), ("nms", nms_bytes), ("topk", topk_bytes)):
        ms = class_ms.get(name, 0.0)
        if ms > 0 and nbytes > 0:
            gbs = nbytes / (ms * 1e-3) / 1e9
            hbm_side[name] = {"bound": "hbm", "achieved": gbs, "peak": 8000.0, "unit": "GB/s", "frac": gbs / 8000.0,
                              "algorithmic_bytes_per_step": nbytes, "kernel_ms_per_step": ms}

    result = {
        "metric": "frames/sec per exit point EP1-EP4 @540x960 bf16; MFMA util %; max rel err",
        "value": len(exits) * B * args.steps / total_s, "unit": "frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config 3: ResNet-50-style 4-exit detector, 32 frames 3x540x960, one detect_chunk per exit EP1..EP4 per step",
                   "batch": B, "H": H, "W": W, "microbatch": model.refresh_info().microbatch or None},
        "per_exit_frames_per_s": per_exit_fps,
        "per_exit_ms": {f"EP{ep}": ms for ep, ms in zip(exits, per_exit_ms)},
        "kernel_class_ms_per_step": class_ms,
        "per_exit_kernel_class_ms": per_exit_class_ms,
        "per_exit_mfma_frac": per_exit_mfma,
        "ep4_backbone_mfma_frac": bb_tflops / PEAK_BF16_TFLOPS,
        "ep4_backbone": {"what": f"backbone stage kernels of thia_detect_chunk(ep={ep_last}), {B} frames; flops = 2 x MACs of conv2_x..conv5_x",
                         "kernel_ms": bb_ms, "tflops": bb_tflops, "target_frac": 0.5},
        "instrumented_ms_per_step": 1e3 * (t3 - t2) / args.steps,
        "roofline": roofline,
        "hbm_side_kernels": hbm_side,
    }

    if not args.skip_all_exits:
        # beside the metric: a mixed plan through thia_run_plan (256 frames of the same scene in 8 chunks of 32 at exits
        # 1,4,2,2,3,1,4,3), with the micro-batches alternating between the library's two lanes and on one lane
        from dataclasses import replace
        c4 = CONFIGS[4]
        plan = list(c4.exits)
        pf = torch.from_numpy(make_frames(replace(c4.scene, n_frames=B * len(plan)), c4.frame_seed)).cuda()
        pout = model.alloc_outputs(pf.shape[0])
        plan_ms = {}
        for lanes in (2, 1):
            model.set_lanes(lanes)
            model.run_plan(pf, B, plan, pout)
            ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            ea.record(stream)
            for k in range(args.steps):
                model.run_plan(pf, B, plan, pout)
            eb.record(stream)
            torch.cuda.synchronize()
            plan_ms[lanes] = ea.elapsed_time(eb) / args.steps
        model.set_lanes(2)
        result["mixed_plan"] = {"workload": f"{pf.shape[0]} frames, {len(plan)} chunks of {B} at exits {plan}, one thia_run_plan call",
                                "ms_per_plan": plan_ms[2], "frames_per_s": pf.shape[0] / (plan_ms[2] * 1e-3),
                                "one_lane_ms_per_plan": plan_ms[1]}
        del pf, pout
    if all_exits_ms is not None:
        result["all_exits_one_pass"] = {"ms_per_batch": all_exits_ms, "frames_per_s": B / (all_exits_ms * 1e-3),
                                        "vs_sweep": ms_per_step / all_exits_ms}
        result["answers_vs_last_exit"] = agreement
    if not args.skip_cpu_baseline:
        import oracle
        # max rel err (per tensor: max |gpu - ref| / max |ref|) of the bf16 path's RPN logits and deltas against the fp32
        # oracle, frame 0 at every exit
        o32 = oracle.Model(blob, precision=0)
        model.set_debug(True)
        errs = {}
        for ep in exits:
            model.detect_chunk(frames[:1].contiguous(), ep)
            torch.cuda.synchronize()
            ref = o32.detect(frames_h[:1], ep, taps=["rpn_logits", "rpn_deltas"])
            e_ = 0.0
            for tap in ("rpn_logits", "rpn_deltas"):
                g_ = model.tap(tap).reshape(ref[tap].shape).astype(np.float64)
                e_ = max(e_, float(np.abs(g_ - ref[tap]).max() / np.abs(ref[tap]).max()))
            errs[f"EP{ep}"] = e_
        model.set_debug(False)
        result["max_rel_err"] = {"value": max(errs.values()), "per_exit": errs, "bar": 2e-2,
                                 "what": "bf16 path vs fp32 oracle, RPN logits and box deltas of frame 0, max |gpu - ref| / max |ref| per tensor"}
        orc = oracle.Model(blob)
        tc0 = time.perf_counter()
        n_cpu = 3
        for ep in exits:
            orc.detect(frames_h[:n_cpu], ep)
        tc1 = time.perf_counter()
        result["cpu_baseline"] = {"value": n_cpu * len(exits) / (tc1 - tc0), "unit": "frames/s", "cores": oracle.num_threads(),
                                  "kind": "oracle",
                                  "sample": f"frames 0..{n_cpu - 1} of the batch at each of EP1..EP4 ({n_cpu * len(exits)} frame inferences), bf16-storage oracle"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
