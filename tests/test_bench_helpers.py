"""CPU checks of the benchmark's bookkeeping: the algorithmic byte counts it reports and the
figures it reads from the committed counter profiles."""
import os

import bench
from paper_2604_21335_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_algorithmic_bytes_of_the_headline_step():
    w = W.WORKLOADS["qwen25_7b_32k"]
    ab = bench.algorithmic_bytes(w, 4.0)
    # 64 streams x 2048 pages x 512 B of bounds; 128 selected pages of 16 tokens: K rows of 256 B,
    # 4 kept groups of 32 B per token; masks 2 B per token, offset and index 4 B per page each
    assert ab["parts"]["bounds"] == 64 * 2048 * 512 == 67108864
    assert ab["parts"]["K"] == 64 * 128 * 16 * 256 == 33554432
    assert ab["parts"]["V"] == 64 * 128 * 16 * 4 * 32
    assert ab["parts"]["meta"] == 64 * 128 * 16 * 2 + 2 * 64 * 128 * 4
    assert ab["step"] == sum(ab["parts"].values())
    assert ab["score"] == 67108864 + 16 * 28 * 128 * 2 + 64 * 2048 * 4 == 67747840


def test_traffic_is_read_from_the_committed_profiles():
    for name, kernel in (("qwen25_7b_32k", "score_lds_kernel"), ("llama2_7b_4k", "attn_mfma_kernel"),
                         ("llava15_7b_prefix", "attn_mfma_kernel")):
        per_kernel, per_step, src = bench.measured_traffic(name, kernel)
        assert os.path.exists(os.path.join(ROOT, src.split(" @ ")[0]))
        assert src.split(" @ ")[1] not in ("None", "unknown"), "the profile names its source revision"
        w = W.WORKLOADS[name]
        ab = bench.algorithmic_bytes(w, 4.0)
        # counted traffic is at least about the algorithmic bytes and not wildly above them
        assert 0.9 * ab["step"] < per_step < 1.5 * ab["step"], (name, per_step, ab["step"])
        assert 0 < per_kernel <= per_step
    assert bench.measured_traffic("no_such_workload", "x") == (None, None, None)
