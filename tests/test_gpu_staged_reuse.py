"""ASTRO_FLAG_REUSE_STAGED: a backward that follows a forward of the same chunk through the same
workspace skips the rotation pre-pass.  The results must be bit-identical to a handle without the
flag, the pre-pass must really be skipped exactly when the call matches, and anything that moves
the chunk (an append, a reset) or changes the call (other tensors, another workspace) must stage
again."""
import numpy as np
import pytest

import workloads as wl
from helpers import dev_bf16

pytestmark = pytest.mark.gpu


def _cache(A, w, reuse):
    c = A.astro_kvcache_create(w.batch, w.heads, w.head_dim, w.grid_h, w.grid_w, w.capacity_frames, w.sink_frames,
                               w.chunk_frames, w.rope_pairs, w.rope_base, reuse_staged=reuse)
    pk, pv = wl.history_frame_pool(w, 3)
    for n in range(2):
        k = dev_bf16(np.stack([pk[(n + b) % 3] for b in range(w.batch)]))
        v = dev_bf16(np.stack([pv[(n + b) % 3] for b in range(w.batch)]))
        A.astro_kvcache_append(c, k, v, 1)
    return c


def _stage_launches(A, fn):
    A.astro_profile_begin()
    res = fn()
    return res, A.astro_profile_end().get("chunk_rope_stage", (0, 0.0))[0]


def test_backward_reuses_what_the_forward_staged_only_when_the_call_matches():
    import torch
    import paper_2603_17051_amd as A
    w = wl.Workload("reuse", 17, 2, 3, 128, 5, 7, 4, 1, 2, 0, (22, 21, 21))
    on, off = _cache(A, w, True), _cache(A, w, False)
    Fc = w.chunk_frames
    q, k, v, do = (dev_bf16(x) for x in wl.chunk_inputs(w, with_dout=True))
    q2 = q.clone()
    ws_on = torch.empty(max(A.astro_chunk_attn_workspace_bytes(on, Fc)), dtype=torch.uint8, device="cuda:0")
    ws_on2 = torch.empty_like(ws_on)
    ws_off = torch.empty_like(ws_on)

    def fwd_bwd(c, ws, qq, ws_bwd=None):
        out, lse = A.astro_chunk_attn_fwd(c, qq, k, v, Fc, workspace=ws)
        return (out, lse) + A.astro_chunk_attn_bwd(c, qq, k, v, out, lse, do, Fc, workspace=ws_bwd if ws_bwd is not None else ws)

    ref, n_off = _stage_launches(A, lambda: fwd_bwd(off, ws_off, q))
    got, n_on = _stage_launches(A, lambda: fwd_bwd(on, ws_on, q))
    assert (n_off, n_on) == (2, 1)
    for a, b in zip(got, ref):
        assert torch.equal(a, b)
    # the same forward again finds its own staging; another q tensor (same values) does not
    _, n = _stage_launches(A, lambda: A.astro_chunk_attn_fwd(on, q, k, v, Fc, workspace=ws_on))
    assert n == 0
    got, n = _stage_launches(A, lambda: fwd_bwd(on, ws_on, q2))
    assert n == 1
    for a, b in zip(got, ref):
        assert torch.equal(a, b)
    # another workspace for the backward: staged again there
    got, n = _stage_launches(A, lambda: fwd_bwd(on, ws_on, q, ws_bwd=ws_on2))
    assert n == 2
    for a, b in zip(got, ref):
        assert torch.equal(a, b)
    # an append moves the chunk's frame positions: the next call stages again, and matches a plain handle
    for c in (on, off):
        A.astro_kvcache_append(c, k, v, Fc)
    ref2, _ = _stage_launches(A, lambda: fwd_bwd(off, ws_off, q))
    got2, n = _stage_launches(A, lambda: fwd_bwd(on, ws_on2, q))
    assert n == 1
    for a, b in zip(got2, ref2):
        assert torch.equal(a, b)
    assert not torch.equal(ref2[0], ref[0])
    # a reset too
    for c in (on, off):
        A.astro_kvcache_reset(c, 0, 5)
    ref3, _ = _stage_launches(A, lambda: fwd_bwd(off, ws_off, q))
    got3, n = _stage_launches(A, lambda: fwd_bwd(on, ws_on2, q))
    assert n == 1
    for a, b in zip(got3, ref3):
        assert torch.equal(a, b)
    torch.cuda.synchronize()
    on.close()
    off.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_reuse_with_candidate_groups_and_on_the_fp32_path(dtype):
    """The same promise for the group calls (3 candidates per stream) and for the fp32 debug path:
    a handle with the flag gives bit-identical results to one without, with one pre-pass per
    forward + backward instead of two."""
    import torch
    import paper_2603_17051_amd as A
    w = wl.Workload("reuse_group", 18, 2, 2, 64, 4, 6, 3, 1, 2, 0, (12, 10, 10))
    G, Fc = 3, w.chunk_frames
    adt = A.ASTRO_BF16 if dtype == "bf16" else A.ASTRO_F32

    def make(reuse):
        c = A.astro_kvcache_create(w.batch, w.heads, w.head_dim, w.grid_h, w.grid_w, w.capacity_frames, w.sink_frames,
                                   Fc, w.rope_pairs, w.rope_base, adt, reuse_staged=reuse)
        shape = (w.batch, w.tokens_per_frame, w.heads, w.head_dim)
        for n in range(2):
            kk, vv = (wl.normal_f32(w.seed, t, shape, n) for t in (wl.T_HIST_K, wl.T_HIST_V))
            if dtype == "bf16":
                kk, vv = dev_bf16(wl.f32_to_bf16_bits(kk)), dev_bf16(wl.f32_to_bf16_bits(vv))
            else:
                kk, vv = torch.from_numpy(kk).to("cuda:0"), torch.from_numpy(vv).to("cuda:0")
            A.astro_kvcache_append(c, kk, vv, 1)
        return c

    shape = (w.batch * G, w.n_q, w.heads, w.head_dim)
    raw = [wl.normal_f32(w.seed, t, shape, 7) for t in (wl.T_Q, wl.T_K, wl.T_V, wl.T_DO)]
    if dtype == "bf16":
        q, k, v, do = (dev_bf16(wl.f32_to_bf16_bits(x)) for x in raw)
    else:
        q, k, v, do = (torch.from_numpy(x).to("cuda:0") for x in raw)
    results, launches = [], []
    for reuse in (False, True):
        c = make(reuse)
        ws = torch.empty(max(A.astro_group_attn_workspace_bytes(c, Fc, G)), dtype=torch.uint8, device="cuda:0")

        def fwd_bwd():
            out, lse = A.astro_group_attn_fwd(c, q, k, v, Fc, G, workspace=ws)
            return (out, lse) + A.astro_group_attn_bwd(c, q, k, v, out, lse, do, Fc, G, workspace=ws)

        res, n = _stage_launches(A, fwd_bwd)
        torch.cuda.synchronize()
        results.append(res)
        launches.append(n)
        c.close()
    assert launches == [2, 1]
    for a, b in zip(*results):
        assert torch.equal(a, b)
