"""GPU parity of the block-causal mask inside the chunk (desc.block_frames): the chunk's frames
form blocks of k frames and a query sees the chunk keys of its own and of earlier blocks only
(k = 1: frame by frame, Sec. 3.1), through the C ABI against the fp64 oracle.  Frame sizes are
chosen so that block boundaries fall inside key tiles, query tiles and single waves."""
import numpy as np
import pytest

import workloads as wl
from helpers import Lockstep, assert_bf16_close, assert_f32_close, host_f64
from test_gpu_parity import _fill_history, _report

pytestmark = pytest.mark.gpu


def _step(ls, w, Fc, step, check, rep=None, bwd=True):
    if ls.dtype == "bf16":
        q, k, v, do = wl.chunk_inputs(w, step, with_dout=True)
    else:
        shape = (w.batch, w.n_q, w.heads, w.head_dim)
        q, k, v, do = (wl.normal_f32(w.seed, t, shape, step) for t in (wl.T_Q, wl.T_K, wl.T_V, wl.T_DO))
    out, lse = ls.fwd(q, k, v, Fc)
    ro, rl = ls.oracle.attn_fwd(ls.wide(q), ls.wide(k), ls.wide(v), Fc)
    check(host_f64(out), ro, f"step {step} out")
    check(host_f64(lse), rl, f"step {step} lse")
    if bwd:
        dq, dk, dv = ls.A.astro_chunk_attn_bwd(ls.cache, ls.dev(q), ls.dev(k), ls.dev(v), out, lse, ls.dev(do), Fc)
        rq, rk, rv = ls.oracle.attn_bwd(ls.wide(q), ls.wide(k), ls.wide(v), ls.wide(do), Fc)
        check(host_f64(dq), rq, f"step {step} dq")
        check(host_f64(dk), rk, f"step {step} dk")
        check(host_f64(dv), rv, f"step {step} dv")
    ls.append(k, v, Fc)
    ls.check_tables()


@pytest.mark.parametrize("D,pairs,C,S,Fc,bf", [(64, (12, 10, 10), 4, 1, 3, 1), (128, (22, 21, 21), 5, 0, 4, 2), (64, (0, 0, 0), 4, 1, 3, 2)])
def test_f32_debug_path_block_causal(D, pairs, C, S, Fc, bf):
    w = wl.Workload("f32_causal", 21, 2, 2, D, 3, 5, C, S, Fc, 0, pairs)
    ls = Lockstep(w, dtype="f32", start_frames=[3, 50], block_frames=bf)
    for step in range(3):
        _step(ls, w, Fc, step, assert_f32_close)
    ls.close()


@pytest.mark.parametrize("D,pairs,gh,gw,B,H,C,S,Fc,bf", [
    (128, (22, 21, 21), 7, 9, 2, 3, 5, 1, 3, 1),    # 63-token frames: boundaries inside 32- and 64-row tiles
    (64, (12, 10, 10), 5, 13, 1, 2, 6, 0, 4, 2),    # 65-token frames, blocks of two, D 64
    (128, (22, 21, 21), 16, 20, 1, 2, 4, 1, 3, 1),  # 320-token frames: several query tiles per frame
    (128, (0, 0, 0), 2, 3, 1, 1, 5, 0, 5, 1),       # 6-token frames: many blocks inside one wave
    (128, (22, 21, 21), 6, 7, 1, 2, 6, 0, 5, 3),    # blocks of 3 in a chunk of 5: short last block
    # 288-token frames on an empty ring: the forward is split in two key ranges, and for the queries of
    # frame 0 that share a workgroup with queries of frame 1 the second range holds only keys they do not see
    (128, (22, 21, 21), 16, 18, 1, 2, 3, 0, 3, 1),
    (64, (12, 10, 10), 16, 18, 1, 1, 4, 1, 3, 1),
])
def test_bf16_block_causal_streaming_fwd_bwd(D, pairs, gh, gw, B, H, C, S, Fc, bf):
    w = wl.Workload("bf16_causal", 22, B, H, D, gh, gw, C, S, Fc, 0, pairs)
    ls = Lockstep(w, start_frames=[5 + 9 * b for b in range(B)], block_frames=bf)
    rep = []
    check = lambda got, ref, what: assert_bf16_close(got, ref, what, rep)
    for step in range(3):   # empty ring, filling ring, evicting ring
        _step(ls, w, Fc, step, check)
    _report(rep[-5:])
    ls.close()


def test_bf16_block_size_covering_the_chunk_is_the_unmasked_call():
    import torch
    w = wl.Workload("bf16_causal_full", 23, 1, 2, 128, 6, 7, 4, 0, 2, 0, (22, 21, 21))
    res = []
    for bf in (0, 2, 5):
        ls = Lockstep(w, block_frames=bf)
        q, k, v, do = wl.chunk_inputs(w, 0, with_dout=True)
        ls.append(k, v, 2)
        out, lse = ls.fwd(q, k, v, 2)
        grads = ls.A.astro_chunk_attn_bwd(ls.cache, ls.dev(q), ls.dev(k), ls.dev(v), out, lse, ls.dev(do), 2)
        res.append([out, lse, *grads])
        ls.close()
    for other in res[1:]:
        for a, b in zip(res[0], other):
            assert torch.equal(a, b)


def test_bf16_group_and_full_backward_take_the_mask():
    """Candidates over one shared cache and the non-detached backward, frame-causal chunk."""
    w = wl.Workload("bf16_causal_group", 24, 2, 2, 128, 6, 7, 4, 1, 3, 0, (22, 21, 21))
    G = 3
    ls = Lockstep(w, start_frames=[2, 40], block_frames=1)
    for step in range(2):
        _, k, v = wl.chunk_inputs(w, step)
        ls.append(k, v, 3)
    q, k, v, do = wl.group_inputs(w, G, with_dout=True)
    A = ls.A
    out, lse = A.astro_group_attn_fwd(ls.cache, ls.dev(q), ls.dev(k), ls.dev(v), 3, G)
    dq, dk, dv = A.astro_group_attn_bwd(ls.cache, ls.dev(q), ls.dev(k), ls.dev(v), out, lse, ls.dev(do), 3, G)
    ro, rl = ls.oracle.group_attn_fwd(ls.wide(q), ls.wide(k), ls.wide(v), 3, G)
    rq, rk, rv = ls.oracle.group_attn_bwd(ls.wide(q), ls.wide(k), ls.wide(v), ls.wide(do), 3, G)
    rep = []
    for got, ref, name in ((out, ro, "out"), (lse, rl, "lse"), (dq, rq, "dq"), (dk, rk, "dk"), (dv, rv, "dv")):
        assert_bf16_close(host_f64(got), ref, f"group {name}", rep)
    # non-detached backward of a plain chunk on the same cache: the ring rows' gradients
    q1, k1, v1, do1 = wl.chunk_inputs(w, 5, with_dout=True)
    out1, lse1 = ls.fwd(q1, k1, v1, 3)
    got = A.astro_chunk_attn_bwd_full(ls.cache, ls.dev(q1), ls.dev(k1), ls.dev(v1), out1, lse1, ls.dev(do1), 3)
    rq, rk, rv, extra = ls.oracle.attn_bwd(ls.wide(q1), ls.wide(k1), ls.wide(v1), ls.wide(do1), 3, history_grads=True)
    for g_, ref, name in zip(got[:3], (rq, rk, rv), ("dq", "dk", "dv")):
        assert_bf16_close(host_f64(g_), ref, f"full {name}", rep)
    T = w.tokens_per_frame
    dv_cache = host_f64(got[4])
    sf, _, _ = A.astro_kvcache_tables(ls.cache)
    for b in range(w.batch):
        order = sorted(range(w.capacity_frames), key=lambda s: sf[b][s])  # oracle context is in frame order
        for h in range(w.heads):
            ref = extra[(b, h)]["dv_hist"]
            gotv = np.concatenate([dv_cache[b, s * T:(s + 1) * T, h] for s in order], 0)
            assert_bf16_close(gotv, ref, f"full dv_cache b{b} h{h}", rep)
    _report(rep[-6:])
    ls.close()


def test_bf16_production_shape_frame_causal_sampled_pairs():
    """The rl_bwd shape (batch 4, 18 cached frames, 3-frame chunk of 1560-token frames) with
    frame-by-frame causality inside the chunk."""
    w = wl.RL_BWD
    ls = Lockstep(w, max_chunk=3, start_frames=[11, 0, 29, 4], block_frames=1)
    pk, pv = wl.history_frame_pool(w, 6)
    _fill_history(ls, w, pk, pv, 18)
    q, k, v, do = wl.chunk_inputs(w, with_dout=True)
    out, lse = ls.fwd(q, k, v, 3)
    dq, dk, dv = ls.A.astro_chunk_attn_bwd(ls.cache, ls.dev(q), ls.dev(k), ls.dev(v), out, lse, ls.dev(do), 3)
    qf, kf, vf, dof = (wl.bf16_bits_to_f32(x) for x in (q, k, v, do))
    rep = []
    for b, h in [(1, 4), (2, 10)]:
        ro, rl = ls.oracle.attn_fwd(qf, kf, vf, 3, streams=[b], heads=[h])
        assert_bf16_close(host_f64(out[b, :, h]), ro[b, :, h], f"stream {b} head {h} out", rep)
        assert_bf16_close(host_f64(lse[b, h]), rl[b, h], f"stream {b} head {h} lse", rep)
        rq, rk, rv = ls.oracle.attn_bwd(qf, kf, vf, dof, 3, streams=[b], heads=[h])
        assert_bf16_close(host_f64(dq[b, :, h]), rq[b, :, h], f"stream {b} head {h} dq", rep)
        assert_bf16_close(host_f64(dk[b, :, h]), rk[b, :, h], f"stream {b} head {h} dk", rep)
        assert_bf16_close(host_f64(dv[b, :, h]), rv[b, :, h], f"stream {b} head {h} dv", rep)
    _report(rep)
    ls.close()


def test_bf16_production_fwd_batch1_frame_causal_with_key_split():
    """One stream of 12 heads, 18 cached frames + 3-frame chunk, frame-by-frame causality: 444
    workgroups, so the launch is split over the keys (4 ranges) and merged; ranges of chunk keys a
    query does not see weigh 0 in the merge.  Every head on a sample of rows around the frame and
    tile boundaries, three heads in full; outputs pre-filled with NaN."""
    import torch
    w = wl.PROD_FWD
    ls = Lockstep(w, max_chunk=3, start_frames=[7], block_frames=1)
    pk, pv = wl.history_frame_pool(w, 6)
    _fill_history(ls, w, pk, pv, 18)
    q, k, v = wl.chunk_inputs(w)
    out = torch.full((w.batch, w.n_q, w.heads, w.head_dim), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    lse = torch.full((w.batch, w.heads, w.n_q), float("nan"), dtype=torch.float32, device="cuda:0")
    ls.A.astro_chunk_attn_fwd(ls.cache, ls.dev(q), ls.dev(k), ls.dev(v), 3, out, lse)
    torch.cuda.synchronize()
    go, gl = host_f64(out), host_f64(lse)
    assert np.isfinite(go).all() and np.isfinite(gl).all()
    qf, kf, vf = (wl.bf16_bits_to_f32(x) for x in (q, k, v))
    T = w.tokens_per_frame
    rng = np.random.Generator(np.random.Philox(key=[w.seed, 99]))
    edges = [0, 1, 127, 128, T - 1, T, T + 1, 2 * T - 1, 2 * T, 1535, 1536, 1663, 1664, 3 * T - 1]
    rep = []
    for h in range(w.heads):
        rows = np.unique(np.concatenate([edges, rng.integers(0, w.n_q, 100)]))
        ro, rl = ls.oracle.attn_fwd(qf, kf, vf, 3, heads=[h], rows=rows)
        assert_bf16_close(go[0, rows, h], ro[0, rows, h], f"head {h} out (row sample)", rep)
        assert_bf16_close(gl[0, h, rows], rl[0, h, rows], f"head {h} lse (row sample)", rep)
    for h in (0, 6, 11):
        ro, rl = ls.oracle.attn_fwd(qf, kf, vf, 3, heads=[h])
        assert_bf16_close(go[0, :, h], ro[0, :, h], f"head {h} out", rep)
        assert_bf16_close(gl[0, h], rl[0, h], f"head {h} lse", rep)
    _report(rep[-2:])
    ls.close()
