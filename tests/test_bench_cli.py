"""Host-side checks of bench.py that need no GPU: the multi-GPU refusal and the flop counts it prices the
kernels with (against counts written out by hand from the step definitions)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_flop_counts():
    d, T = 128, 16
    # default path, 5 groups: set-up (1/3 + 3 + 2 + 2) d^3, 15 steps of 8 d^3 and one of 6 d^3, 5 solves of 8/3 d^3, K_0 2 d^3
    assert bench.alg_flops(d, T, 5) == pytest.approx((22.0 / 3 + 15 * 8 + 6 + 5 * 8.0 / 3 + 2) * d ** 3)
    assert bench.default_groups(16, "f32") == 5 and bench.default_groups(32, "bf16") == 7
    assert bench.alg_flops_tv(d, T) == pytest.approx(T * (6 * 2 + 1.0 / 3 + 2) * d ** 3)
    assert bench.alg_flops_cxt(16, 16, 8) == 3 * 2 * 16 * 256 + 8 * 5 * 2 * 16 ** 3 == 352256
    assert bench.alg_flops_scan(16, 1) == pytest.approx((12 + 7.0 / 3) * 16 ** 3)


def test_block_and_rollout_flop_counts_and_build_hash():
    C, H, d, r, T = 4096, 16, 16, 16, 8
    # per token: two projections of 2 C H d each, per head the eight maps (5 d + 3 r outputs of d terms) and the solve
    want = 2 * (2 * C * H * d) + H * (2 * d * (5 * d + 3 * r) + 352256)
    assert bench.alg_flops_block(C, H, d, r, T) == want == 9895936
    assert bench.alg_flops_rollout(64, 8) > bench.alg_flops_tv(64, 8) * 0.9   # a Riccati sweep plus the mat-vecs
    # the build script is part of what identifies a build of the kernels
    import hashlib
    h = hashlib.sha256()
    folder = os.path.join(ROOT, "paper_2603_09221_amd", "csrc")
    for path in [os.path.join(folder, n) for n in sorted(os.listdir(folder))] + [os.path.join(ROOT, "paper_2603_09221_amd", "build.py")]:
        with open(path, "rb") as f:
            h.update(os.path.basename(path).encode() + b"\0" + f.read())
    assert bench.source_hash() == h.hexdigest()[:16]
