"""Host-side pieces of the build and the benchmark that need no GPU: the source hash covers every source of the
library, and the benchmark reads its counter-derived traffic figure from the committed summary only while the
scoring source is the one the counters were taken on."""
import glob
import hashlib
import os

import bench
from paper_2603_17803_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_source_hash_covers_every_source_and_header():
    csrc = os.path.join(ROOT, "paper_2603_17803_amd", "csrc")
    assert sorted(build.SOURCES) == sorted(os.path.basename(p) for p in glob.glob(os.path.join(csrc, "*.hip")))
    assert sorted(build.HEADERS) == sorted(os.path.basename(p) for p in glob.glob(os.path.join(csrc, "*.h")))
    assert len(build.source_hash()) == 32


def test_counter_traffic_is_tied_to_the_scoring_source(tmp_path, monkeypatch):
    # the committed summary: either it matches the scoring source as it is (a figure close to the algorithmic bytes) or it is stale (None)
    got = bench.counter_traffic("long_128k")
    assert got is None or 0.95 * 33818624 <= got <= 1.10 * 33818624
    assert bench.counter_traffic("no_such_workload") is None
    # a summary whose hash is the source's is read, any other hash is refused
    src = os.path.join(ROOT, "paper_2603_17803_amd", "csrc", "score.hip")
    digest = hashlib.sha256(open(src, "rb").read()).hexdigest()
    os.makedirs(tmp_path / "profiles")
    os.makedirs(tmp_path / "paper_2603_17803_amd" / "csrc")
    (tmp_path / "paper_2603_17803_amd" / "csrc" / "score.hip").write_bytes(open(src, "rb").read())
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    f = tmp_path / "profiles" / "score_kernel_w_hbm_traffic.txt"
    f.write_text(f"traffic_bytes_per_launch: 12345\nscore_hip_sha256: {digest}\n")
    assert bench.counter_traffic("w") == 12345
    f.write_text(f"traffic_bytes_per_launch: 12345\nscore_hip_sha256: {'0' * 64}\n")
    assert bench.counter_traffic("w") is None
