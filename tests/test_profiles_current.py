"""The counter summaries under profiles/ that bench.py reads (executed instruction
count and HBM traffic of the dominant kernel) must belong to the kernel sources in
the tree: each carries a fingerprint of csrc/, and bench.py falls back to the
algorithmic count when it differs."""
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


@pytest.mark.parametrize("tag,kernel", [("workload1", "k_small"), ("workload2", "k_search"),
                                        ("workload3", "k_search"), ("workload3_only_k9", "k_search"),
                                        ("workload4", "k_search"), ("workload5", "k_search")])
def test_counter_summaries_match_the_sources(tag, kernel):
    import bench
    valu, traffic, src = bench._static_counters(tag, kernel)
    assert valu is not None and valu > 0, f"no SQ_INSTS_VALU of {kernel} in profiles/valu_lds_counters_{tag}.txt"
    assert traffic is not None and traffic > 0
    assert src["executed"]["matches_this_build"], (src["executed"]["kernel_sources_sha16"], bench.sources_sha16())
    assert src["traffic"]["matches_this_build"]
    # the reads counted by request size can only be at or below the scaled FETCH_SIZE figure
    assert 0 < src["traffic_by_request_size"] <= traffic * 1.01
