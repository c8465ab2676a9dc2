"""GPU parity of the non-detached backward: the gradients of the resident ring rows (the
part the detach of Sec. 3.3 drops, the "Clip + Full BP" point of Table 4(a)) against the
oracle's full gradient, slot by slot; the chunk gradients must equal the detached call's."""
import numpy as np
import pytest

import workloads as wl
from oracle import rope_angles, rope_rotate, visible_history
from helpers import Lockstep, assert_bf16_close, host_f64
from test_gpu_parity import _fill_history, _report

pytestmark = pytest.mark.gpu


def _slot(n, C, S):
    return n if n < C else S + (n - S) % (C - S)


def _check_ring_grads(ls, dk_cache, dv_cache, extra, pairs, rep, label):
    """extra[(b, h)] holds the oracle's gradients for the visible frames in frame order."""
    w = ls.w
    T, C, S = w.tokens_per_frame, w.capacity_frames, w.sink_frames
    for b, h in pairs:
        n0 = len(ls.oracle.history[b])
        vis = visible_history(n0, S, C - S)
        if not vis:  # empty cache: nothing may be written
            assert (dk_cache[b, :, h] == 0).all() and (dv_cache[b, :, h] == 0).all()
            continue
        ref_k = np.zeros((C * T, w.head_dim))
        ref_v = np.zeros((C * T, w.head_dim))
        for i, n in enumerate(vis):
            rows = slice(_slot(n, C, S) * T, (_slot(n, C, S) + 1) * T)
            phi = rope_angles(ls.oracle.start[b] + n, w.grid_h, w.grid_w, w.rope_pairs, w.rope_base)
            ref_k[rows] = rope_rotate(extra[(b, h)]["dk_hist_rot"][i * T:(i + 1) * T, None, :], -phi)[:, 0]
            ref_v[rows] = extra[(b, h)]["dv_hist"][i * T:(i + 1) * T]
        assert_bf16_close(host_f64(dk_cache[b, :, h]), ref_k, f"{label} stream {b} head {h} dk_cache", rep)
        assert_bf16_close(host_f64(dv_cache[b, :, h]), ref_v, f"{label} stream {b} head {h} dv_cache", rep)


@pytest.mark.parametrize("D,pairs,gh,gw,B,H,C,S,Fc", [
    (128, (22, 21, 21), 7, 9, 2, 2, 5, 1, 2),   # ragged tails, sink + eviction
    (64, (12, 10, 10), 5, 13, 1, 2, 4, 0, 3),
    (128, (0, 0, 0), 4, 4, 1, 1, 3, 2, 1),      # no rotary, two sinks
])
def test_full_backward_streaming(D, pairs, gh, gw, B, H, C, S, Fc):
    w = wl.Workload("full_bwd_small", 23, B, H, D, gh, gw, C, S, Fc, 0, pairs)
    ls = Lockstep(w, start_frames=[4 + 6 * b for b in range(B)])
    A = ls.A
    rep = []
    for step in range(C // Fc + 3):
        q, k, v, do = wl.chunk_inputs(w, step, with_dout=True)
        out, lse = ls.fwd(q, k, v, Fc)
        dev = [ls.dev(x) for x in (q, k, v)]
        dq0, dk0, dv0 = A.astro_chunk_attn_bwd(ls.cache, *dev, out, lse, ls.dev(do), Fc)
        dq, dk, dv, dkc, dvc = A.astro_chunk_attn_bwd_full(ls.cache, *dev, out, lse, ls.dev(do), Fc)
        for a, b_ in ((dq, dq0), (dk, dk0), (dv, dv0)):
            assert (a == b_).all()
        _, _, _, extra = ls.oracle.attn_bwd(ls.wide(q), ls.wide(k), ls.wide(v), ls.wide(do), Fc, history_grads=True)
        _check_ring_grads(ls, dkc, dvc, extra, [(b, h) for b in range(B) for h in range(H)], rep, f"step {step}")
        # slots that hold no frame yet are left alone (the binding zero-fills what it allocates)
        resident = min(len(ls.oracle.history[0]), C)
        assert (dkc[:, resident * w.tokens_per_frame:] == 0).all() and (dvc[:, resident * w.tokens_per_frame:] == 0).all()
        ls.append(k, v, Fc)
    _report(rep[-4:])
    ls.close()


def test_full_backward_production_shape_sampled_pairs():
    """Batch 4, 18 resident frames (28080 ring rows) + 3-frame chunk."""
    w = wl.RL_BWD
    ls = Lockstep(w, max_chunk=3, start_frames=[11, 0, 29, 4])
    A = ls.A
    pk, pv = wl.history_frame_pool(w, 6)
    _fill_history(ls, w, pk, pv, 18)
    q, k, v, do = wl.chunk_inputs(w, with_dout=True)
    out, lse = ls.fwd(q, k, v, 3)
    dq, dk, dv, dkc, dvc = A.astro_chunk_attn_bwd_full(ls.cache, ls.dev(q), ls.dev(k), ls.dev(v), out, lse, ls.dev(do), 3)
    qf, kf, vf, dof = (wl.bf16_bits_to_f32(x) for x in (q, k, v, do))
    rep = []
    for b, h in [(1, 7)]:
        rq, rk, rv, extra = ls.oracle.attn_bwd(qf, kf, vf, dof, 3, streams=[b], heads=[h], history_grads=True)
        assert_bf16_close(host_f64(dq[b, :, h]), rq[b, :, h], f"stream {b} head {h} dq", rep)
        assert_bf16_close(host_f64(dk[b, :, h]), rk[b, :, h], f"stream {b} head {h} dk", rep)
        _check_ring_grads(ls, dkc, dvc, extra, [(b, h)], rep, "production")
    _report(rep)
    ls.close()


def test_full_backward_is_refused_on_fp32_caches():
    w = wl.Workload("full_bwd_f32", 24, 1, 1, 64, 2, 4, 2, 0, 1, 0, (12, 10, 10))
    ls = Lockstep(w, dtype="f32")
    with pytest.raises(ls.A.AstroError) as e:
        ls.A.astro_chunk_attn_bwd_full_workspace_bytes(ls.cache, 1)
    assert e.value.code == -3
    ls.close()
