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


def test_traffic_file_is_read_only_for_the_library_it_was_made_with():
    """The committed counter summary names the library build it measured; bench.py quotes it for that build only
    (after a change to the kernels the figure is withheld until the profile is made again)."""
    b = _bench()
    with open(b.TRAFFIC_FILE) as f:
        digests = [line.split()[1] for line in f if line.split()[:1] == ["library_digest"]]
    assert len(digests) == 1 and len(digests[0]) == 64, "the profile must name the build it measured"
    t = b.read_traffic(digests[0])
    assert t is not None and 0.98 * 88_768_512 < t < 1.1 * 88_768_512
    assert b.read_traffic("0" * 64) is None


def test_cold_wire_arrangement():
    """Enough interleaved chains that the other chains' wire writes alone, between a wire's write and its read,
    exceed the 256 MB cache."""
    b = _bench()
    n3 = 4096 * 5376
    assert b.wire_bytes(n3, 256) == 22_020_096 + 344_064
    for n, B in ((n3, 256), (2048 * 3840, 256), (33_554_432, 32), (33_554_432, 512)):
        m = b.cold_chains(n, B)
        assert 2 <= m <= 64 and (m - 1) * b.wire_bytes(n, B) >= 1.25 * (256 << 20) > (m - 2) * b.wire_bytes(n, B)
    assert b.cold_chains(n3, 256) == 17
    assert b.cold_chains(64 * 5376, 128) == 0 and b.cold_chains(4096, 256) == 0      # small messages: never cold
    assert b.ends_bytes(8, n3, 256) == 664_731_648
    # all-to-all form: the P-1 wires of one pipeline are written at once, so a few pipelines side by side suffice
    assert b.cold_flat_pipelines(8, n3, 256) == 4 and b.cold_flat_pipelines(8, 2048 * 3840, 256) == 8
    assert b.cold_flat_pipelines(16, 64 * 5376, 128) == 0
    # input sets rotated over: together at least twice the cache (27B shape 2, 12B shape 5, 64 MiB messages 2, small ones capped)
    assert b.input_sets(8, n3) == 2 and b.input_sets(8, 2048 * 3840) == 5 and b.input_sets(8, 33_554_432) == 2
    assert b.input_sets(16, 64 * 5376) == 49 and b.input_sets(4, 4096) == 64


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "ONE GPU" in p.stderr and p.stdout.strip() == ""
