"""Host-side pieces of bench.py that need no GPU: the algorithmic work it prices the stages with, and the
HBM traffic it reads from the tracked profile summary."""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
import workload as W  # noqa: E402


def test_traffic_of_every_call_is_found_in_the_profile_summary():
    # (a renamed kernel or a reshaped table would silently turn roofline.traffic into null)
    for call in ("cc_rope_shift", "cc_select", "cc_sparse_prefill"):
        t = bench.profiled_traffic_bytes(call)
        assert t is not None and t > 1e8, call
    assert bench.profiled_traffic_bytes("cc_no_such_call") is None


def test_algorithmic_work_of_a_small_workload_by_hand():
    w = W.config(2, 0.25)
    sp = w.spec
    work = bench.algorithmic_work(w, cow=True)
    chunk = w.segments[w.segments[:, W.SEG_KIND] == W.KIND_CHUNK]
    n_chunk_tok = int(chunk[:, W.SEG_NTOK].sum())
    # keys only: read + written once, bf16
    assert work["shift_bytes"] == n_chunk_tok * sp.n_kv_heads * sp.head_dim * 2 * 2
    assert bench.algorithmic_work(w, cow=False)["shift_bytes"] == 2 * work["shift_bytes"]
    # score: every token of a chunk that has a prior chunk sees the keys 0..p
    pairs = 0
    for s in chunk:
        st, n = int(s[W.SEG_START]), int(s[W.SEG_NTOK])
        if st > 0:
            pairs += sum(st + t + 1 for t in range(n))
    assert work["score_flops"] == 2.0 * sp.head_dim * sp.n_q_heads * pairs
    # attention: 4 d Hq flops per visible key
    q_pos = np.array([5, 0, 17])
    assert bench.attention_flops(w, q_pos) == 4.0 * sp.head_dim * sp.n_q_heads * (6 + 1 + 18)
