"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the CPU-side code (no GPU): the C oracle driven through all its
entry points on a small model, and the library's host-side planner logic.  Host code only: the device pass of hipcc is
never instrumented."""
import os
import shutil
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1",
           OMP_NUM_THREADS="4")
ENV.pop("LD_PRELOAD", None)


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-3000:]}\n{r.stderr[-6000:]}"
    return r


def test_oracle_under_asan_and_ubsan(tmp_path):
    from thia_synth import ModelSpec, SceneSpec, make_blob, make_frames, recipe_for
    exe = str(tmp_path / "sanitize_driver")
    _run(["gcc", *SAN, "-fopenmp", "-ffp-contract=off", "-o", exe, os.path.join(ROOT, "oracle", "thia_oracle.c"),
          os.path.join(ROOT, "oracle", "sanitize_driver.c"), "-lm"])
    # four exits at the real channel widths but one block per stage and small frames: seconds under the sanitizers
    spec = ModelSpec(precision=1, blocks=(1, 1, 1, 1), fc_dim=64, pre_nms=60, post_nms=20, n_classes=4, max_det=10)
    H, W, n = 64, 96, 5
    blob = make_blob(spec, 9, **recipe_for(spec))
    frames = make_frames(SceneSpec(H, W, n, 2, 4, 8, 30, noise=8), 9)
    blob.tofile(tmp_path / "blob.bin")
    frames.tofile(tmp_path / "frames.bin")
    r = _run([exe, str(tmp_path / "blob.bin"), str(tmp_path / "frames.bin"), str(n), str(H), str(W)], env=ENV, timeout=600)
    assert "sanitize_driver: ok" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not installed")
def test_planner_host_logic_under_asan_and_ubsan(tmp_path):
    """plan_core (the host half of planner.hip) with the host pass instrumented; the executable makes no HIP call."""
    csrc = os.path.join(ROOT, "paper_2102_08481_amd", "csrc")
    exe = str(tmp_path / "planner_sanitize_driver")
    host_san = []
    for f in SAN[:3]:
        host_san += ["-Xarch_host", f]
    # thia_planner_defaults / thia_metrics_from_counts live in model.hip, which pulls in every kernel file at link time
    srcs = [os.path.join(csrc, f) for f in ("planner.hip", "model.hip", "conv_igemm.hip", "bottleneck_fused.hip", "stem.hip", "rpn.hip", "roi.hip")]
    _run(["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", *host_san, "-o", exe, os.path.join(csrc, "planner_sanitize_driver.cpp"), *srcs], timeout=1500)
    r = _run([exe], env=ENV, timeout=600)
    assert "planner_sanitize_driver: ok" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
