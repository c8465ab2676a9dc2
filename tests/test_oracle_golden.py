"""Regression guard of the oracle: its sampled outputs and gradients on the smallest named
configuration must stay what tests/golden/make_oracle_golden.py (which calls only the oracle)
wrote; and the named workloads must have the shapes the paper's setting fixes (Table S1:
480x832 video, 16x spatial reduction of the latent tokens -> 30 x 52 = 1560 tokens per frame;
chunks of 3 latent frames; a context window of 21 frames = 18 cached + the chunk)."""
import json
import os
import sys

import numpy as np
import pytest

import workloads as wl

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden"))
import make_oracle_golden as gold  # noqa: E402


def test_oracle_reproduces_its_stored_values():
    stored = json.load(open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "oracle_tiny.json")))
    assert [tuple(s) for s in stored["samples"]] == gold.SAMPLES
    for ref in stored["cases"]:
        got = gold.case(ref["sinks"], ref["window_relative"], ref["n_hist"])
        for key in ("out", "dq", "dk", "dv", "lse"):
            np.testing.assert_allclose(got[key], ref[key], rtol=1e-12, atol=1e-14, err_msg=f"{ref} {key}")
        assert got["out_sum"] == pytest.approx(ref["out_sum"], rel=1e-12)
        assert got["dq_abs_sum"] == pytest.approx(ref["dq_abs_sum"], rel=1e-12)
    # the three cases really differ (a sink, and where it sits, changes the result)
    outs = [c["out"] for c in stored["cases"]]
    assert outs[0] != outs[1] and outs[1] != outs[2]


def test_named_workloads_have_the_papers_shapes():
    assert (480 // 16, 832 // 16) == (30, 52)
    for w in (wl.PROD_FWD, wl.GROUP_FWD_APPEND, wl.STREAM_EVICT, wl.RL_BWD, wl.SHARED_PREFIX):
        assert (w.grid_h, w.grid_w, w.tokens_per_frame) == (30, 52, 1560)
        assert (w.heads, w.head_dim, w.chunk_frames, w.n_q) == (12, 128, 3, 4680)
        assert sum(w.rope_pairs) == w.head_dim // 2
    for w in (wl.PROD_FWD, wl.GROUP_FWD_APPEND, wl.RL_BWD):
        assert w.capacity_frames + w.chunk_frames == 21 and w.n_k == 28080 + 4680
    assert (wl.STREAM_EVICT.capacity_frames, wl.STREAM_EVICT.sink_frames) == (12, 1)
    assert (wl.GROUP_FWD_APPEND.batch, wl.RL_BWD.batch, wl.PROD_FWD.batch) == (8, 4, 1)
    t = wl.TINY_FWD
    assert (t.batch, t.heads, t.head_dim, t.tokens_per_frame, t.capacity_frames, t.rope_pairs) == (1, 2, 64, 64, 4, (12, 10, 10))
