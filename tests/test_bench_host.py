"""Host-side logic of bench.py (no GPU): the algorithmic byte / flop accounting and the read-back of the
counter traffic from the committed rocprofv3 summaries."""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_2511_00101_amd import synth  # noqa: E402


def test_algorithmic_work_of_the_decode_heavy_batch():
    """x once, y read + written, A and B of every adapter in use once: 22.8 MB for 256 tokens over 64 rank-16
    adapters of a 4096 -> 4096 projection, and 2 r (d_in + d_out) flops per token."""
    p = synth.config2()
    w = bench.algorithmic_work(p)
    used = len(np.unique(p.batch.token_adapter))
    assert w["tokens"] == 256
    assert w["shrink"] == 256 * 4096 * 2 + used * 16 * 4096 * 2
    assert w["expand"] == 256 * 4096 * 4 + used * 16 * 4096 * 2      # no fine-tune rows, so no saved h
    assert w["total"] == w["shrink"] + w["expand"]
    assert w["flops"] == 256 * 2 * 16 * (4096 + 4096)
    assert 22.0e6 < w["total"] < 23.2e6


def test_algorithmic_work_counts_saved_h_and_skips_dropped_tokens():
    p = synth.config1()
    w = bench.algorithmic_work(p)
    n_ft = int((p.batch.token_kind == 0).sum())
    assert w["tokens"] == p.n_tokens
    assert w["expand"] - (p.n_tokens * p.d_out * 4 + len(np.unique(p.batch.token_adapter)) * 8 * p.d_out * 2) == n_ft * 8 * 4
    q = synth.small_mixed(3, 64, 64, 64, [4, 8], drop_frac=0.25)
    live = (q.batch.token_adapter >= 0) & (q.batch.token_adapter < q.n_adapters) & (q.batch.token_kind <= 2)
    assert bench.algorithmic_work(q)["tokens"] == int(live.sum()) < q.n_tokens


def test_counter_traffic_is_read_from_the_committed_summaries():
    for workload, phase in (("cfg2_decode_heavy", "forward_slab"), ("cfg4_mlp_up", "forward_fused")):
        t = bench.counter_traffic(workload, phase)
        assert t is not None and t > 0
        # what the counters saw is the algorithmic traffic plus re-reads: between 1x and 2x
        maker = synth.config2 if workload.startswith("cfg2") else (lambda: synth.config4("up"))
        alg = bench.algorithmic_work(maker())["total"]
        assert alg <= t <= 2 * alg
    assert bench.counter_traffic("no_such_workload", "expand") is None
    assert bench.counter_traffic("cfg2_decode_heavy", "no_such_phase") is None
