"""Host-side checks of bench.py that need no GPU: the byte and flop accounting behind `roofline`, and the refusal
of a multi-GPU run."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from paper_2406_02069_amd import synth  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout == ""


def test_algorithmic_bytes_of_the_headline_workload():
    # K once + Q_win per layer: 8 heads x 32768 keys x 128 x 2 B + 32 heads x 32 rows x 128 x 2 B, 32 layers
    w = synth.WORKLOADS[2]
    per_layer = 8 * 32768 * 128 * 2 + 32 * 32 * 128 * 2
    assert bench.kernel_bytes("score_resident", w, [128] * w.L, w.N) == per_layer * 32 == 2155872256
    # one layer: K, Q_win, kept K and V rows read and written, kept indices
    k = 100
    assert bench.layer_bytes(w, k, w.N) == per_layer + 4 * 8 * k * 128 * 2 + 8 * k * 4
    assert bench.kernel_bytes("gather", w, [k, 2 * k], w.N) == 4 * 8 * 3 * k * 128 * 2


def test_matrix_flops_count_every_logit_once():
    w = synth.WORKLOADS[4]   # 8 KV heads x 8 query heads x 64 window queries = 512 rows per key
    assert bench.score_flops(w, w.N) == 2.0 * 512 * 128 * 8 * 32768 * 80


def test_tracked_counter_tables_parse():
    b = bench.tracked("traffic_bytes.txt", "score_resident", "llama3-8b-32k", 128, int)
    assert isinstance(b, int) and 2.15e9 < b < 2.6e9            # measured HBM bytes: at least the algorithmic ones
    f = bench.tracked("pipe_busy.txt", "score_resident:mfma", "llama3-8b-32k", 128, float)
    assert 0.0 < f < 1.0
    assert bench.tracked("traffic_bytes.txt", "score_resident", "no-such-workload", 128, int) is None


@pytest.mark.parametrize("name", ["sweep_loop", "xcd_latency", "poll_behind_loads"])
def test_microbenchmarks_behind_the_profiles_compile_for_gfx950(name, tmp_path):
    # the stand-alone programs whose recorded outputs sit under profiles/ (cross-compiled here; they run on the GPU machine)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    src = os.path.join(ROOT, "tests", "microbench", name + ".hip")
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                        "-packed-fp32-ops", src, "-o", str(tmp_path / name)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    assert os.path.exists(os.path.join(ROOT, "profiles", name + "_microbench.md"))
