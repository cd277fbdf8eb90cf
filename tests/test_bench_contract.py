"""bench.py's accounting and argument contract (no GPU): the byte counts every reported fraction rests on, and
the refusal to run on more than one GPU."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_algorithmic_bytes():
    b = _bench()
    n3 = 4096 * 5376
    # 27B-shaped config, hop by hop: every partial read once (2 B), every wire written once and read once
    # (1 B + 4/256 B each way), the output written once (2 B)
    assert b.chain_bytes(8, n3, 256) == 754_188_288
    assert b.hop_bytes(n3, 256) == 88_768_512 == 44_040_192 + 2 * 22_020_096 + 2 * 344_064
    assert b.fused_bytes(8, n3) == 396_361_728
    # the chain is one quantize, P-1 hops and one dequantize
    quant = n3 * (2 + 1 + 4 / 256)
    assert b.chain_bytes(8, n3, 256) == quant + 7 * b.hop_bytes(n3, 256) + quant
    # the other configs of the list
    assert b.chain_bytes(4, 4096, 256) == 74_240
    assert b.chain_bytes(8, 2048 * 3840, 256) == 269_352_960
    assert b.chain_bytes(16, 64 * 5376, 128) == 23_052_288
    assert [b.chain_bytes(8, 33_554_432, B) for B in (32, 128, 512)] == [1_207_959_552, 1_157_627_904, 1_145_044_992]
    assert b.HBM_PEAK_GBPS == 8000.0


def test_traffic_file_is_read():
    b = _bench()
    t = b.read_traffic()
    assert t is not None and 0.98 * 88_768_512 < t < 1.1 * 88_768_512


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "ONE GPU" in p.stderr and p.stdout.strip() == ""
