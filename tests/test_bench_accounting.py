"""Host-side checks of bench.py: the byte accounting behind the roofline figures, the traffic
file's guard, and the single-GPU contract.  No GPU needed."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_algorithmic_bytes_of_the_benchmark_cycle():
    # 2^30 f32 in 1,024-element blocks, k = 104,858, 131,072 lost blocks: the scan reads x and
    # c once (2 x 4 GiB) and writes 2^20 float scores; a saved block is read and written once;
    # a lost block is read twice (c and the old x) and written once
    b = bench.algorithmic_bytes(1 << 30, 1024, 4, 4, 4, 104_858, 131_072, 5)
    assert b["scores"] == 2 * 4 * (1 << 30) + 4 * (1 << 20) == 8_594_128_896
    assert b["commit"] == 104_858 * 1024 * 8 + 4 * 104_858 == 859_416_168
    assert b["recover"] == 131_072 * 1024 * 12 + 4 * 131_072 == 1_611_137_024
    assert b["total"] == b["scores"] + b["select"] + b["commit"] + b["recover"]
    # bfloat16 checkpoint of a float32 store: 6 instead of 8 bytes per parameter on the scan
    m = bench.algorithmic_bytes(1 << 30, 1024, 4, 2, 4, 104_858, 131_072, 5)
    assert m["scores"] == 6 * (1 << 30) + 4 * (1 << 20)
    assert m["recover"] == 131_072 * 1024 * (2 + 8) + 4 * 131_072
    # a ragged tail still counts every element once
    r = bench.algorithmic_bytes(25_000_000, 4096, 4, 4, 4, 62, 1145, 5)
    assert r["scores"] == 200_000_000 + 4 * 6104


def test_traffic_figure_is_tied_to_the_kernel_sources():
    path = os.path.join(ROOT, "profiles", bench.TRAFFIC_FILES["flat_f32"])
    fields = dict(line.split(":", 1) for line in open(path) if ":" in line and not line.startswith("#"))
    stored = fields["source_sha256"].strip()
    got = bench.stored_traffic("flat_f32")
    if stored == bench.score_kernel_source_hash():
        assert got == int(fields["traffic_bytes_per_launch"])
        # the counters must not show re-reads: within 1 % of the algorithmic bytes
        assert abs(got - int(fields["algorithmic_bytes_per_launch"])) <= 0.01 * got
    else:
        assert got is None
    assert bench.stored_traffic("lda") is None


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], cwd=ROOT,
                       stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
