"""GPU parity of the group-wise calls (G candidate chunks over one shared, frozen cache,
Sec. 3.2) against the oracle's loop of independent attentions; same gates as the chunk calls."""
import numpy as np
import pytest

import workloads as wl
from helpers import Lockstep, assert_bf16_close, assert_f32_close, host_f64
from test_gpu_parity import _fill_history, _report

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,D,pairs,gh,gw,B,H,C,S,Fc,G", [
    ("f32", 64, (12, 10, 10), 3, 5, 2, 2, 3, 1, 1, 3),
    ("bf16", 128, (22, 21, 21), 7, 9, 2, 3, 4, 1, 2, 3),   # Nq = 126: ragged query and key tails
    ("bf16", 64, (12, 10, 10), 5, 13, 1, 2, 3, 0, 1, 5),
    ("bf16", 128, (22, 21, 21), 6, 6, 8, 1, 2, 0, 1, 8),   # 64 candidates: the most one call takes
])
def test_group_fwd_bwd_streaming(dtype, D, pairs, gh, gw, B, H, C, S, Fc, G):
    w = wl.Workload("group_small", 21, B, H, D, gh, gw, C, S, Fc, 0, pairs)
    ls = Lockstep(w, dtype=dtype, start_frames=[2 + 11 * b for b in range(B)])
    A = ls.A
    close = assert_f32_close if dtype == "f32" else assert_bf16_close
    shape = (B * G, w.n_q, H, D)
    for step in range(C // Fc + 2):
        if dtype == "f32":
            q, k, v, do = (wl.normal_f32(w.seed, t, shape, step) for t in (wl.T_Q, wl.T_K, wl.T_V, wl.T_DO))
        else:
            q, k, v, do = wl.group_inputs(w, G, step, with_dout=True)
        out, lse = A.astro_group_attn_fwd(ls.cache, ls.dev(q), ls.dev(k), ls.dev(v), Fc, G)
        ro, rl = ls.oracle.group_attn_fwd(ls.wide(q), ls.wide(k), ls.wide(v), Fc, G)
        close(host_f64(out), ro, f"step {step} out")
        close(host_f64(lse), rl, f"step {step} lse")
        dq, dk, dv = A.astro_group_attn_bwd(ls.cache, ls.dev(q), ls.dev(k), ls.dev(v), out, lse, ls.dev(do), Fc, G)
        rq, rk, rv = ls.oracle.group_attn_bwd(ls.wide(q), ls.wide(k), ls.wide(v), ls.wide(do), Fc, G)
        close(host_f64(dq), rq, f"step {step} dq")
        close(host_f64(dk), rk, f"step {step} dk")
        close(host_f64(dv), rv, f"step {step} dv")
        # the group call leaves the cache alone; the chosen candidate of every stream is appended
        ls.check_tables()
        pick = [b * G + (step + b) % G for b in range(B)]
        ls.append(np.ascontiguousarray(k[pick]), np.ascontiguousarray(v[pick]), Fc)
        ls.check_tables()
    ls.close()


def test_group_calls_reject_bad_group_sizes():
    import torch
    w = wl.Workload("group_bad", 22, 2, 1, 64, 4, 4, 2, 0, 1, 0, (12, 10, 10))
    ls = Lockstep(w)
    A = ls.A
    with pytest.raises(A.AstroError):
        A.astro_group_attn_workspace_bytes(ls.cache, 1, 0)
    with pytest.raises(A.AstroError):
        A.astro_group_attn_workspace_bytes(ls.cache, 1, 33)  # 2 * 33 candidates > 64
    x = torch.zeros(2 * 33, 16, 1, 64, dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(A.AstroError):
        A.astro_group_attn_fwd(ls.cache, x, x, x, 1, 33, workspace=torch.zeros(1 << 22, dtype=torch.uint8, device="cuda:0"))
    assert A.astro_kvcache_tables(ls.cache)[2] == [0, 0]
    ls.close()


def test_group_shared_prefix_production_shape_sampled_pairs():
    """One stream, 18 cached frames shared by 8 candidate 3-frame chunks (8 x 4680 queries
    over 28080 shared + 4680 own keys), forward and backward, sampled (candidate, head) pairs."""
    w, G = wl.SHARED_PREFIX, 8
    ls = Lockstep(w, max_chunk=3, start_frames=[13])
    A = ls.A
    pk, pv = wl.history_frame_pool(w, 6)
    _fill_history(ls, w, pk, pv, 18)
    q, k, v, do = wl.group_inputs(w, G, with_dout=True)
    dq_, dk_, dv_, ddo = (ls.dev(x) for x in (q, k, v, do))
    out, lse = A.astro_group_attn_fwd(ls.cache, dq_, dk_, dv_, 3, G)
    gq, gk, gv = A.astro_group_attn_bwd(ls.cache, dq_, dk_, dv_, out, lse, ddo, 3, G)
    qf, kf, vf, dof = (wl.bf16_bits_to_f32(x) for x in (q, k, v, do))
    rep = []
    for c, h in [(0, 5), (6, 11)]:
        ro, rl = ls.oracle.group_attn_fwd(qf, kf, vf, 3, G, candidates=[c], heads=[h])
        assert_bf16_close(host_f64(out[c, :, h]), ro[c, :, h], f"candidate {c} head {h} out", rep)
        assert_bf16_close(host_f64(lse[c, h]), rl[c, h], f"candidate {c} head {h} lse", rep)
        rq, rk, rv = ls.oracle.group_attn_bwd(qf, kf, vf, dof, 3, G, candidates=[c], heads=[h])
        assert_bf16_close(host_f64(gq[c, :, h]), rq[c, :, h], f"candidate {c} head {h} dq", rep)
        assert_bf16_close(host_f64(gk[c, :, h]), rk[c, :, h], f"candidate {c} head {h} dk", rep)
        assert_bf16_close(host_f64(gv[c, :, h]), rv[c, :, h], f"candidate {c} head {h} dv", rep)
    _report(rep)
    ls.close()


def test_group_shared_prefix_production_shape_every_candidate():
    """The same 8 candidates over one cache: every (candidate, head) pair of the forward on a
    sample of query rows, outputs pre-filled with NaN; two pairs in full, forward and backward (a
    key's gradient needs every query row of its pair)."""
    import torch
    w, G = wl.SHARED_PREFIX, 8
    ls = Lockstep(w, max_chunk=3, start_frames=[13])
    A = ls.A
    pk, pv = wl.history_frame_pool(w, 6)
    _fill_history(ls, w, pk, pv, 18)
    q, k, v, do = wl.group_inputs(w, G, with_dout=True)
    q_d, k_d, v_d, do_d = (ls.dev(x) for x in (q, k, v, do))
    shape = (G, w.n_q, w.heads, w.head_dim)
    out = torch.full(shape, float("nan"), dtype=torch.bfloat16, device="cuda:0")
    lse = torch.full((G, w.heads, w.n_q), float("nan"), dtype=torch.float32, device="cuda:0")
    gq, gk, gv = (torch.full(shape, float("nan"), dtype=torch.float32, device="cuda:0") for _ in range(3))
    A.astro_group_attn_fwd(ls.cache, q_d, k_d, v_d, 3, G, out, lse)
    A.astro_group_attn_bwd(ls.cache, q_d, k_d, v_d, out, lse, do_d, 3, G, gq, gk, gv)
    torch.cuda.synchronize()
    go, gl = host_f64(out), host_f64(lse)
    for name, t in (("out", go), ("lse", gl), ("dq", host_f64(gq)), ("dk", host_f64(gk)), ("dv", host_f64(gv))):
        assert np.isfinite(t).all(), f"{name}: elements no workgroup wrote"
    qf, kf, vf, dof = (wl.bf16_bits_to_f32(x) for x in (q, k, v, do))
    rng = np.random.Generator(np.random.Philox(key=[w.seed, 777]))
    rep = []
    for c in range(G):
        for h in range(w.heads):
            rows = np.unique(np.concatenate([[0, 127, 128, w.n_q - 1], rng.integers(0, w.n_q, 124)]))
            ro, rl = ls.oracle.group_attn_fwd(qf, kf, vf, 3, G, candidates=[c], heads=[h], rows=rows)
            assert_bf16_close(go[c, rows, h], ro[c, rows, h], f"candidate {c} head {h} out (row sample)", rep)
            assert_bf16_close(gl[c, h, rows], rl[c, h, rows], f"candidate {c} head {h} lse (row sample)", rep)
    for c, h in [(3, 0), (7, 8)]:
        ro, rl = ls.oracle.group_attn_fwd(qf, kf, vf, 3, G, candidates=[c], heads=[h])
        assert_bf16_close(go[c, :, h], ro[c, :, h], f"candidate {c} head {h} out", rep)
        rq, rk, rv = ls.oracle.group_attn_bwd(qf, kf, vf, dof, 3, G, candidates=[c], heads=[h])
        assert_bf16_close(host_f64(gq[c, :, h]), rq[c, :, h], f"candidate {c} head {h} dq", rep)
        assert_bf16_close(host_f64(gk[c, :, h]), rk[c, :, h], f"candidate {c} head {h} dk", rep)
        assert_bf16_close(host_f64(gv[c, :, h]), rv[c, :, h], f"candidate {c} head {h} dv", rep)
    _report(rep[-4:])
    ls.close()
