"""Benchmark of the hot path on one MI355X: the four-exit ResNet-50-style detector on a
32-frame batch of synthetic 540x960 traffic frames, swept over exits EP1..EP4.

One "step" = thia_detect_chunk on the resident batch at EP1, EP2, EP3 and EP4 (the whole
hot path at every exit; 4 x 32 frame inferences).  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

RES_GAIN, PRED_STD = 0.25, 0.01        # data-only gains of the synthetic weights
PEAK_BF16_TFLOPS = 2500.0              # MI355X dense bf16 MFMA peak
CONV_CLASSES = ("conv", "fc")          # launches of the implicit-GEMM MFMA kernel


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--skip-cpu-baseline", action="store_true", help="leave out the oracle timing (for profiler runs)")
    ap.add_argument("--microbatch", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (frames are independent; see DESIGN.md for sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2102_08481_amd import thia_load_model, thia_detect_chunk
    from thia_synth import CONFIGS, make_blob, make_frames

    cfg = CONFIGS[3]
    spec, scene = cfg.model, cfg.scene
    B, H, W = scene.n_frames, scene.height, scene.width
    blob = make_blob(spec, cfg.weight_seed, res_gain=RES_GAIN, pred_std=PRED_STD)
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

    # ---- timed region: exactly K steps; per-exit times from events on the stream the kernels run on;
    # per-kernel-class times from the library's own HIP events around every launch
    model.profile_begin()
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
    prof = model.profile_read()
    model.profile_end()

    # the same K steps without the per-launch events: shows what the instrumentation costs
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for k in range(args.steps):
        step()
    torch.cuda.synchronize()
    t3 = time.perf_counter()

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
        "kernel": "conv_igemm_kernel (all instantiations: backbone, lateral, RPN, FC)",
        "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
        "traffic": None,
        "flops_per_step": conv_flops_step, "launches_per_step": conv_launches, "avg_launch_us": 1e3 * conv_ms / max(conv_launches, 1),
        "kernel_ms_per_step": conv_ms,
    }
    class_ms = {k: v[0] / args.steps for k, v in prof.items()}

    result = {
        "metric": "frames/sec per exit point EP1-EP4 @540x960 bf16; MFMA util %; max rel err",
        "value": len(exits) * B * args.steps / total_s, "unit": "frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config 3: ResNet-50-style 4-exit detector, 32 frames 3x540x960, one detect_chunk per exit EP1..EP4 per step",
                   "batch": B, "H": H, "W": W, "microbatch": model.info.microbatch or None},
        "per_exit_frames_per_s": per_exit_fps,
        "per_exit_ms": {f"EP{ep}": ms for ep, ms in zip(exits, per_exit_ms)},
        "kernel_class_ms_per_step": class_ms,
        "uninstrumented_ms_per_step": 1e3 * (t3 - t2) / args.steps,
        "roofline": roofline,
    }

    if not args.skip_cpu_baseline:
        import oracle
        orc = oracle.Model(blob)
        tc0 = time.perf_counter()
        for ep in exits:
            orc.detect(frames_h[:1], ep)
        tc1 = time.perf_counter()
        result["cpu_baseline"] = {"value": len(exits) / (tc1 - tc0), "unit": "frames/s", "cores": os.cpu_count() if not os.environ.get("OMP_NUM_THREADS") else int(os.environ["OMP_NUM_THREADS"]),
                                  "kind": "oracle", "sample": "frame 0 of the batch at each of EP1..EP4 (4 frame inferences), bf16-storage oracle"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
