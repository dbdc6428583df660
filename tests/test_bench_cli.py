"""Host side of bench.py that needs no GPU: more than one GPU is refused with a message (this build
measures one), and the byte accounting the roofline figures rest on."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    text = p.stdout + p.stderr
    assert "ONE GPU" in text or "one GPU" in text, text
    assert "{" not in p.stdout          # no result line


def test_layer_bytes_counts_every_tensor_once():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    m, k, nc = 1000, 32, 192
    # activations in and out, 2-bit weights (4 per byte), bias + multiplier + shift as int32 per channel
    assert bench.layer_bytes(m, k, nc) == m * k + m * nc + (k // 4) * nc + 12 * nc
    assert bench.layer_bytes(m, k, nc, residual=True) - bench.layer_bytes(m, k, nc) == m * nc
    # a row of 18 input channels packs into 5 bytes
    assert bench.layer_bytes(1, 18, 1) == 18 + 1 + 5 + 12
