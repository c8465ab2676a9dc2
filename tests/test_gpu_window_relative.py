"""GPU parity of window-relative temporal positions (ASTRO_FLAG_WINDOW_RELATIVE): the oracle
rotates every frame at its rank in the attended sequence; the library keeps absolute
positions for window and chunk frames and moves the sinks' keys forward by the number of
evicted frames on every append that evicts (from an un-rotated copy, one rounding).  Both
must give the same outputs and gradients; the slot-position tables (ranks) must match bit
for bit, and the sink slots and the sink copy must hold what the scheme says."""
import numpy as np
import pytest

import workloads as wl
from oracle import rope_angles, rope_rotate, visible_history
from helpers import Lockstep, assert_bf16_close, assert_f32_close, host_f64
from test_gpu_parity import _report

pytestmark = pytest.mark.gpu


def _slot(n, C, S):
    return n if n < C else S + (n - S) % (C - S)


def check_sinks(ls: Lockstep):
    """Sink slot s holds the sink's key rotated at start + s + (frames evicted so far), to the
    storage rounding; the sink copy holds the un-rotated keys bit for bit; values are untouched."""
    import torch
    w = ls.w
    T, C, S = w.tokens_per_frame, w.capacity_frames, w.sink_frames
    tdt = torch.bfloat16 if ls.dtype == "bf16" else torch.float32
    kc = ls.cache.k_storage.view(tdt).view(w.batch, w.heads, C * T, w.head_dim)
    raw = ls.cache.k_sink_storage.view(tdt).view(w.batch, S * T, w.heads, w.head_dim)
    for b in range(w.batch):
        n0 = len(ls.oracle.history[b])
        evicted = max(0, n0 - C)
        for s in range(min(S, n0)):
            kf, _ = ls.oracle.history[b][s]
            np.testing.assert_array_equal(host_f64(raw[b, s * T:(s + 1) * T]), np.asarray(kf, dtype=np.float64))
            phi = rope_angles(ls.oracle.start[b] + s + evicted, w.grid_h, w.grid_w, w.rope_pairs, w.rope_base)
            for h in range(w.heads):
                ref = rope_rotate(np.asarray(kf[:, h:h + 1], dtype=np.float64), phi)[:, 0]
                got = host_f64(kc[b, h, s * T:(s + 1) * T])
                tol = (2.0 ** -8 if ls.dtype == "bf16" else 2e-6) * np.abs(ref) + 1e-6
                assert (np.abs(got - ref) <= tol).all(), (b, s, h)


@pytest.mark.parametrize("D,pairs,C,S,Fc", [(64, (12, 10, 10), 4, 1, 2), (128, (22, 21, 21), 5, 2, 1), (64, (12, 10, 10), 3, 2, 1)])
def test_f32_streaming_fwd_bwd_with_moving_sinks(D, pairs, C, S, Fc):
    w = wl.Workload("wr_f32", 31, 2, 2, D, 3, 5, C, S, Fc, 0, pairs)
    ls = Lockstep(w, dtype="f32", start_frames=[3, 50], window_relative=True)
    shape = (w.batch, w.n_q, w.heads, w.head_dim)
    for step in range(2 * C + 2):
        q, k, v, do = (wl.normal_f32(w.seed, t, shape, step) for t in (wl.T_Q, wl.T_K, wl.T_V, wl.T_DO))
        out, lse = ls.fwd(q, k, v, Fc)
        ro, rl = ls.oracle.attn_fwd(ls.wide(q), ls.wide(k), ls.wide(v), Fc)
        assert_f32_close(host_f64(out), ro, f"step {step} out")
        assert_f32_close(host_f64(lse), rl, f"step {step} lse")
        dq, dk, dv = ls.A.astro_chunk_attn_bwd(ls.cache, ls.dev(q), ls.dev(k), ls.dev(v), out, lse, ls.dev(do), Fc)
        rq, rk, rv = ls.oracle.attn_bwd(ls.wide(q), ls.wide(k), ls.wide(v), ls.wide(do), Fc)
        assert_f32_close(host_f64(dq), rq, f"step {step} dq")
        assert_f32_close(host_f64(dk), rk, f"step {step} dk")
        assert_f32_close(host_f64(dv), rv, f"step {step} dv")
        ls.append(k, v, Fc)
        ls.check_tables()
        check_sinks(ls)
    ls.close()


@pytest.mark.parametrize("D,pairs,gh,gw,B,H,C,S,Fc", [
    (128, (22, 21, 21), 7, 9, 2, 3, 5, 1, 2),    # ragged query and key tails, one sink
    (64, (12, 10, 10), 5, 13, 1, 2, 4, 2, 1),    # two sinks, single-frame chunks
    (128, (22, 21, 21), 16, 20, 1, 2, 3, 1, 2),  # more than one query tile, chunk as long as the window
])
def test_bf16_streaming_fwd_bwd_with_moving_sinks(D, pairs, gh, gw, B, H, C, S, Fc):
    w = wl.Workload("wr_bf16", 32, B, H, D, gh, gw, C, S, Fc, 0, pairs)
    ls = Lockstep(w, start_frames=[5 + 9 * b for b in range(B)], window_relative=True)
    rep = []
    for step in range(C // Fc + 5):
        q, k, v, do = wl.chunk_inputs(w, step, with_dout=True)
        out, lse = ls.fwd(q, k, v, Fc)
        ro, rl = ls.oracle.attn_fwd(ls.wide(q), ls.wide(k), ls.wide(v), Fc)
        assert_bf16_close(host_f64(out), ro, f"step {step} out", rep)
        assert_bf16_close(host_f64(lse), rl, f"step {step} lse", rep)
        dq, dk, dv = ls.A.astro_chunk_attn_bwd(ls.cache, ls.dev(q), ls.dev(k), ls.dev(v), out, lse, ls.dev(do), Fc)
        rq, rk, rv = ls.oracle.attn_bwd(ls.wide(q), ls.wide(k), ls.wide(v), ls.wide(do), Fc)
        assert_bf16_close(host_f64(dq), rq, f"step {step} dq", rep)
        assert_bf16_close(host_f64(dk), rk, f"step {step} dk", rep)
        assert_bf16_close(host_f64(dv), rv, f"step {step} dv", rep)
        ls.append(k, v, Fc)
        ls.check_tables()
        check_sinks(ls)
    _report(rep[-5:])
    ls.close()


def test_bf16_reset_of_one_stream_restarts_its_sinks_and_leaves_the_other_alone():
    w = wl.Workload("wr_reset", 33, 2, 2, 128, 4, 6, 3, 1, 1, 0, (22, 21, 21))
    ls = Lockstep(w, start_frames=[0, 7], window_relative=True)
    rep = []
    for step in range(9):
        if step == 5:   # stream 1 starts over at another frame; its new first frame becomes its sink
            ls.A.astro_kvcache_reset(ls.cache, 1, 100)
            ls.oracle.reset(1, 100)
        q, k, v = wl.chunk_inputs(w, step)
        out, lse = ls.fwd(q, k, v, 1)
        ro, rl = ls.oracle.attn_fwd(ls.wide(q), ls.wide(k), ls.wide(v), 1)
        assert_bf16_close(host_f64(out), ro, f"step {step} out", rep)
        assert_bf16_close(host_f64(lse), rl, f"step {step} lse", rep)
        ls.append(k, v, 1)
        ls.check_tables()
        check_sinks(ls)
    _report(rep[-2:])
    ls.close()


def test_bf16_group_and_non_detached_backward_with_moving_sinks():
    """The group calls see the same moved sinks, and the gradient of a sink's key is turned back
    at the position it is stored at."""
    w = wl.Workload("wr_full", 34, 1, 2, 128, 5, 7, 4, 1, 2, 0, (22, 21, 21))
    ls = Lockstep(w, start_frames=[11], window_relative=True)
    A = ls.A
    T, C, S = w.tokens_per_frame, w.capacity_frames, w.sink_frames
    for step in range(4):   # 8 frames: 4 evicted
        q, k, v = wl.chunk_inputs(w, step)
        ls.append(k, v, 2)
    rep = []
    q, k, v, do = wl.chunk_inputs(w, 9, with_dout=True)
    out, lse = ls.fwd(q, k, v, 2)
    dq, dk, dv, dkc, dvc = A.astro_chunk_attn_bwd_full(ls.cache, ls.dev(q), ls.dev(k), ls.dev(v), out, lse, ls.dev(do), 2)
    rq, rk, rv, extra = ls.oracle.attn_bwd(ls.wide(q), ls.wide(k), ls.wide(v), ls.wide(do), 2, history_grads=True)
    assert_bf16_close(host_f64(dq), rq, "dq", rep)
    assert_bf16_close(host_f64(dk), rk, "dk", rep)
    assert_bf16_close(host_f64(dv), rv, "dv", rep)
    vis = visible_history(len(ls.oracle.history[0]), S, C - S)
    for h in range(w.heads):
        ref_k, ref_v = np.zeros((C * T, w.head_dim)), np.zeros((C * T, w.head_dim))
        for rank, n in enumerate(vis):
            rows = slice(_slot(n, C, S) * T, (_slot(n, C, S) + 1) * T)
            phi = rope_angles(rank, w.grid_h, w.grid_w, w.rope_pairs, w.rope_base)
            ref_k[rows] = rope_rotate(extra[(0, h)]["dk_hist_rot"][rank * T:(rank + 1) * T, None, :], -phi)[:, 0]
            ref_v[rows] = extra[(0, h)]["dv_hist"][rank * T:(rank + 1) * T]
        assert_bf16_close(host_f64(dkc[0, :, h]), ref_k, f"head {h} dk_cache", rep)
        assert_bf16_close(host_f64(dvc[0, :, h]), ref_v, f"head {h} dv_cache", rep)
    # two candidates over the same cache
    G = 2
    q2, k2, v2 = (np.concatenate([x, y], 0) for x, y in zip(wl.chunk_inputs(w, 9), wl.chunk_inputs(w, 10)))
    out2, lse2 = A.astro_group_attn_fwd(ls.cache, ls.dev(q2), ls.dev(k2), ls.dev(v2), 2, G)
    ro2, rl2 = ls.oracle.group_attn_fwd(ls.wide(q2), ls.wide(k2), ls.wide(v2), 2, G)
    assert_bf16_close(host_f64(out2), ro2, "group out", rep)
    assert_bf16_close(host_f64(lse2), rl2, "group lse", rep)
    _report(rep)
    ls.close()


def test_bf16_long_stream_shape_with_one_sink():
    """The long-streaming shape (ring of 12 = 1 sink + 11, 3-frame chunks, 1560-token frames): ten
    chunks, six of them evicting; one head per step against the oracle."""
    w = wl.STREAM_EVICT
    ls = Lockstep(w, start_frames=[0], window_relative=True)
    rep = []
    for step in range(10):
        q, k, v = wl.chunk_inputs(w, step)
        out, lse = ls.fwd(q, k, v, 3)
        h = (5 * step) % w.heads
        qf, kf, vf = (wl.bf16_bits_to_f32(x) for x in (q, k, v))
        ro, rl = ls.oracle.attn_fwd(qf, kf, vf, 3, heads=[h])
        assert_bf16_close(host_f64(out[0, :, h]), ro[0, :, h], f"step {step} head {h} out", rep)
        assert_bf16_close(host_f64(lse[0, h]), rl[0, h], f"step {step} head {h} lse", rep)
        ls.oracle.append(kf, vf, 3)
        ls.A.astro_kvcache_append(ls.cache, ls.dev(k), ls.dev(v), 3)
        ls.check_tables()
        print(f"    step {step}: {rep[-2]}", flush=True)
    check_sinks(ls)
    ls.close()


def test_bf16_production_frames_two_streams_group_backward():
    """1560-token frames, 12 heads; two streams at different points of their life (one still
    filling its ring, one that has evicted many frames), two sinks; two candidates per stream,
    forward and backward on sampled (candidate, head) pairs."""
    import torch
    w = wl.Workload("wr_prod", 35, 2, 12, 128, 30, 52, 8, 2, 3, 0, (22, 21, 21))
    ls = Lockstep(w, start_frames=[0, 40], window_relative=True)
    A, G, Fc = ls.A, 2, 3
    pk, pv = wl.history_frame_pool(w, 6)
    dk, dv = ls.dev(pk), ls.dev(pv)
    fk, fv = wl.bf16_bits_to_f32(pk), wl.bf16_bits_to_f32(pv)
    total = 19
    for n in range(total):
        if n == total - 5:   # stream 0 starts over: it will hold 5 frames (2 sinks + 3), nothing evicted
            A.astro_kvcache_reset(ls.cache, 0, 7)
            ls.oracle.reset(0, 7)
        idx = [wl.pool_index(b, n, 6) for b in range(w.batch)]
        it = torch.tensor(idx, device="cuda:0")
        A.astro_kvcache_append(ls.cache, dk.index_select(0, it).contiguous(), dv.index_select(0, it).contiguous(), 1)
        for b in range(w.batch):
            ls.oracle.append_stream(b, fk[idx[b]], fv[idx[b]], 1)
    ls.check_tables()
    check_sinks(ls)
    assert len(ls.oracle.history[0]) == 5 and len(ls.oracle.history[1]) == 19
    q, k, v, do = (np.concatenate([a, b], 0) for a, b in zip(wl.chunk_inputs(w, 1, with_dout=True),
                                                             wl.chunk_inputs(w, 2, with_dout=True)))
    # candidates are ordered (stream, candidate): rows 0,1 belong to stream 0 and rows 2,3 to stream 1
    order = [0, 2, 1, 3]
    q, k, v, do = (x[order] for x in (q, k, v, do))
    dq_, dk_, dv_, ddo = (ls.dev(x) for x in (q, k, v, do))
    out, lse = A.astro_group_attn_fwd(ls.cache, dq_, dk_, dv_, Fc, G)
    gq, gk, gv = A.astro_group_attn_bwd(ls.cache, dq_, dk_, dv_, out, lse, ddo, Fc, G)
    qf, kf, vf, dof = (wl.bf16_bits_to_f32(x) for x in (q, k, v, do))
    rep = []
    for c, h in [(1, 3), (2, 10)]:
        ro, rl = ls.oracle.group_attn_fwd(qf, kf, vf, Fc, G, candidates=[c], heads=[h])
        rq, rk, rv = ls.oracle.group_attn_bwd(qf, kf, vf, dof, Fc, G, candidates=[c], heads=[h])
        assert_bf16_close(host_f64(out[c, :, h]), ro[c, :, h], f"candidate {c} head {h} out", rep)
        assert_bf16_close(host_f64(lse[c, h]), rl[c, h], f"candidate {c} head {h} lse", rep)
        assert_bf16_close(host_f64(gq[c, :, h]), rq[c, :, h], f"candidate {c} head {h} dq", rep)
        assert_bf16_close(host_f64(gk[c, :, h]), rk[c, :, h], f"candidate {c} head {h} dk", rep)
        assert_bf16_close(host_f64(gv[c, :, h]), rv[c, :, h], f"candidate {c} head {h} dv", rep)
    _report(rep)
    ls.close()
