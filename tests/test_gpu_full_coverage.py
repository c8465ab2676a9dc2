"""GPU parity over WHOLE tensors at the production shapes: every (stream, head) pair of the
backward shape (batch 4, 12 heads: the contiguous per-XCD work mapping), every head of the
batch-1 forward (key split active), every pair of the 8-stream forward on a row sample plus one
full pair per stream; and every pair of a 16-pair D = 64 case with ragged frames, a sink and a
wrapped ring.  Outputs are pre-filled with NaN, so a pair or row that no workgroup wrote
fails the finiteness check before any comparison."""
import numpy as np
import pytest

import workloads as wl
from helpers import Lockstep, assert_bf16_close, dev_bf16, host_f64

pytestmark = pytest.mark.gpu


def _fill_history(ls, w, n_pool, n_frames_each):
    import torch
    pk, pv = wl.history_frame_pool(w, n_pool)
    dk, dv = dev_bf16(pk), dev_bf16(pv)
    fk, fv = wl.bf16_bits_to_f32(pk), wl.bf16_bits_to_f32(pv)
    for n in range(n_frames_each):
        idx = [wl.pool_index(b, n, n_pool) for b in range(w.batch)]
        it = torch.tensor(idx, device="cuda:0")
        ls.A.astro_kvcache_append(ls.cache, dk.index_select(0, it).contiguous(), dv.index_select(0, it).contiguous(), 1)
        for b in range(w.batch):
            ls.oracle.append_stream(b, fk[idx[b]], fv[idx[b]], 1)


def _nan_like(shape, dtype):
    import torch
    return torch.full(shape, float("nan"), dtype=dtype, device="cuda:0")


def test_bf16_rl_backward_every_pair():
    """Batch 4 x 12 heads, 18 cached frames detached + 3-frame chunk: out, LSE, dQ, dK_chunk,
    dV_chunk of all 48 pairs against the oracle, element by element."""
    import torch
    w = wl.RL_BWD
    ls = Lockstep(w, max_chunk=3, start_frames=[11, 0, 29, 4])
    _fill_history(ls, w, 6, 18)
    q, k, v, do = wl.chunk_inputs(w, with_dout=True)
    dq_, dk_, dv_ = (_nan_like((w.batch, w.n_q, w.heads, w.head_dim), torch.float32) for _ in range(3))
    out = _nan_like((w.batch, w.n_q, w.heads, w.head_dim), torch.bfloat16)
    lse = _nan_like((w.batch, w.heads, w.n_q), torch.float32)
    q_d, k_d, v_d, do_d = ls.dev(q), ls.dev(k), ls.dev(v), ls.dev(do)
    ls.A.astro_chunk_attn_fwd(ls.cache, q_d, k_d, v_d, 3, out, lse)
    ls.A.astro_chunk_attn_bwd(ls.cache, q_d, k_d, v_d, out, lse, do_d, 3, dq_, dk_, dv_)
    torch.cuda.synchronize()
    got = {n: host_f64(t) for n, t in (("out", out), ("lse", lse), ("dq", dq_), ("dk", dk_), ("dv", dv_))}
    for n, a in got.items():
        assert np.isfinite(a).all(), f"{n}: elements no workgroup wrote"
    qf, kf, vf, dof = (wl.bf16_bits_to_f32(x) for x in (q, k, v, do))
    worst = {n: 0.0 for n in got}
    for b in range(w.batch):
        for h in range(w.heads):
            ro, rl = ls.oracle.attn_fwd(qf, kf, vf, 3, streams=[b], heads=[h])
            rq, rk, rv = ls.oracle.attn_bwd(qf, kf, vf, dof, 3, streams=[b], heads=[h])
            rep = []
            assert_bf16_close(got["out"][b, :, h], ro[b, :, h], f"stream {b} head {h} out", rep)
            assert_bf16_close(got["lse"][b, h], rl[b, h], f"stream {b} head {h} lse", rep)
            assert_bf16_close(got["dq"][b, :, h], rq[b, :, h], f"stream {b} head {h} dq", rep)
            assert_bf16_close(got["dk"][b, :, h], rk[b, :, h], f"stream {b} head {h} dk", rep)
            assert_bf16_close(got["dv"][b, :, h], rv[b, :, h], f"stream {b} head {h} dv", rep)
            for n, line in zip(worst, rep):
                worst[n] = max(worst[n], float(line.split("max_abs=")[1].split()[0]))
        print(f"    stream {b}: 12 heads ok, worst max_abs so far {worst}", flush=True)
    ls.close()


def test_bf16_production_fwd_every_head():
    """Batch 1 (the launch is split over the keys and merged): all 12 heads in full."""
    import torch
    w = wl.PROD_FWD
    ls = Lockstep(w, max_chunk=3, start_frames=[7])
    _fill_history(ls, w, 6, 18)
    q, k, v = wl.chunk_inputs(w)
    out = _nan_like((w.batch, w.n_q, w.heads, w.head_dim), torch.bfloat16)
    lse = _nan_like((w.batch, w.heads, w.n_q), torch.float32)
    ls.A.astro_chunk_attn_fwd(ls.cache, ls.dev(q), ls.dev(k), ls.dev(v), 3, out, lse)
    torch.cuda.synchronize()
    go, gl = host_f64(out), host_f64(lse)
    assert np.isfinite(go).all() and np.isfinite(gl).all()
    qf, kf, vf = (wl.bf16_bits_to_f32(x) for x in (q, k, v))
    rep = []
    for h in range(w.heads):
        ro, rl = ls.oracle.attn_fwd(qf, kf, vf, 3, heads=[h])
        assert_bf16_close(go[0, :, h], ro[0, :, h], f"head {h} out", rep)
        assert_bf16_close(gl[0, h], rl[0, h], f"head {h} lse", rep)
    print("   ", rep[-2], flush=True)
    ls.close()


def test_bf16_grouped_streams_fwd_every_pair():
    """8 streams x 12 heads with different ring phases and frame offsets: every pair on a sample
    of 192 query rows (first, last and random ones), one pair per stream in full."""
    import torch
    w = wl.GROUP_FWD_APPEND
    offs = wl.stream_offsets(w.seed, w.batch, 0, 60)
    starts = [int(100 * b + 3) for b in range(w.batch)]
    ls = Lockstep(w, max_chunk=3, start_frames=starts)
    pk, pv = wl.history_frame_pool(w, 8)
    dk, dv = dev_bf16(pk), dev_bf16(pv)
    fk, fv = wl.bf16_bits_to_f32(pk), wl.bf16_bits_to_f32(pv)
    total = int(offs.max()) + w.capacity_frames
    for n in range(total):
        for b in range(w.batch):
            if total - n == int(offs[b]) + w.capacity_frames:
                ls.A.astro_kvcache_reset(ls.cache, b, starts[b])
                ls.oracle.reset(b, starts[b])
        idx = [wl.pool_index(b, n, 8) for b in range(w.batch)]
        it = torch.tensor(idx, device="cuda:0")
        ls.A.astro_kvcache_append(ls.cache, dk.index_select(0, it).contiguous(), dv.index_select(0, it).contiguous(), 1)
        for b in range(w.batch):
            ls.oracle.append_stream(b, fk[idx[b]], fv[idx[b]], 1)
    ls.check_tables()
    q, k, v = wl.chunk_inputs(w)
    out = _nan_like((w.batch, w.n_q, w.heads, w.head_dim), torch.bfloat16)
    lse = _nan_like((w.batch, w.heads, w.n_q), torch.float32)
    ls.A.astro_chunk_attn_fwd(ls.cache, ls.dev(q), ls.dev(k), ls.dev(v), 3, out, lse)
    torch.cuda.synchronize()
    go, gl = host_f64(out), host_f64(lse)
    assert np.isfinite(go).all() and np.isfinite(gl).all()
    qf, kf, vf = (wl.bf16_bits_to_f32(x) for x in (q, k, v))
    rng = np.random.Generator(np.random.Philox(key=[w.seed, 4242]))
    rep = []
    for b in range(w.batch):
        for h in range(w.heads):
            rows = np.unique(np.concatenate([[0, 1, 127, 128, w.n_q - 129, w.n_q - 1], rng.integers(0, w.n_q, 186)]))
            ro, rl = ls.oracle.attn_fwd(qf, kf, vf, 3, streams=[b], heads=[h], rows=rows)
            assert_bf16_close(go[b, rows, h], ro[b, rows, h], f"stream {b} head {h} out (row sample)", rep)
            assert_bf16_close(gl[b, h, rows], rl[b, h, rows], f"stream {b} head {h} lse (row sample)", rep)
        h = (5 * b + 1) % w.heads
        ro, rl = ls.oracle.attn_fwd(qf, kf, vf, 3, streams=[b], heads=[h])
        assert_bf16_close(go[b, :, h], ro[b, :, h], f"stream {b} head {h} out (full)", rep)
        assert_bf16_close(gl[b, h], rl[b, h], f"stream {b} head {h} lse (full)", rep)
        print(f"    stream {b} ok: {rep[-2]}", flush=True)
    ls.close()


def test_bf16_head_dim_64_every_pair_after_eviction():
    """D = 64 kernels with 16 (stream, head) pairs (the per-XCD mapping), 130-token frames (ragged
    tiles everywhere), one sink frame and a ring that has wrapped: out, LSE, dQ, dK, dV of every
    pair in full."""
    import torch
    w = wl.Workload("d64_every_pair", 31, 2, 8, 64, 10, 13, 6, 1, 2, 0, (12, 10, 10))
    ls = Lockstep(w, max_chunk=2, start_frames=[3, 40])
    _fill_history(ls, w, 5, 9)  # 9 frames into a ring of 6: three evictions behind the sink
    ls.check_tables()
    q, k, v, do = wl.chunk_inputs(w, with_dout=True)
    dq_, dk_, dv_ = (_nan_like((w.batch, w.n_q, w.heads, w.head_dim), torch.float32) for _ in range(3))
    out = _nan_like((w.batch, w.n_q, w.heads, w.head_dim), torch.bfloat16)
    lse = _nan_like((w.batch, w.heads, w.n_q), torch.float32)
    q_d, k_d, v_d, do_d = ls.dev(q), ls.dev(k), ls.dev(v), ls.dev(do)
    ls.A.astro_chunk_attn_fwd(ls.cache, q_d, k_d, v_d, 2, out, lse)
    ls.A.astro_chunk_attn_bwd(ls.cache, q_d, k_d, v_d, out, lse, do_d, 2, dq_, dk_, dv_)
    torch.cuda.synchronize()
    got = {n: host_f64(t) for n, t in (("out", out), ("lse", lse), ("dq", dq_), ("dk", dk_), ("dv", dv_))}
    for n, a in got.items():
        assert np.isfinite(a).all(), f"{n}: elements no workgroup wrote"
    qf, kf, vf, dof = (wl.bf16_bits_to_f32(x) for x in (q, k, v, do))
    ro, rl = ls.oracle.attn_fwd(qf, kf, vf, 2)
    rq, rk, rv = ls.oracle.attn_bwd(qf, kf, vf, dof, 2)
    rep = []
    for b in range(w.batch):
        for h in range(w.heads):
            assert_bf16_close(got["out"][b, :, h], ro[b, :, h], f"stream {b} head {h} out", rep)
            assert_bf16_close(got["lse"][b, h], rl[b, h], f"stream {b} head {h} lse", rep)
            assert_bf16_close(got["dq"][b, :, h], rq[b, :, h], f"stream {b} head {h} dq", rep)
            assert_bf16_close(got["dk"][b, :, h], rk[b, :, h], f"stream {b} head {h} dk", rep)
            assert_bf16_close(got["dv"][b, :, h], rv[b, :, h], f"stream {b} head {h} dv", rep)
    print("   ", rep[-5], flush=True)
    ls.close()
