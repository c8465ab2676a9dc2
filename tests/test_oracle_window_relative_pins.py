"""Pins of the oracle's window-relative temporal positions (`window_relative=True`).

Sec. 4.3 says only that a positional-extrapolation method of another paper is used to run
short-clip models on long videos; the definition pinned here is this build's reading: the
temporal position of a frame is its rank in the attended sequence (sinks, resident window
frames oldest first, then the chunk), row and column positions unchanged.  Checked against
(a) a scalar brute force that is handed the ranks, (b) the already pinned absolute-position
path on a FRESH stream that holds exactly the visible frames (their absolute indices then
are the ranks), (c) the shift invariance of rotary scores (no sinks: identical to absolute
positions at any start frame), (d) torch autograd, (e) finite differences, (f) the ranks of
the slot table by brute force."""
import numpy as np
import pytest
import torch

from oracle import RollingCacheOracle
from test_oracle_pins import brute_masked_attention, brute_resident_after, rand, torch_rope


def make(B, H, D, gh, gw, C, S, pairs, start=None, wr=True, bf=None):
    return RollingCacheOracle(B, H, D, gh, gw, C, S, pairs, 10000.0, start_frames=start, window_relative=wr,
                              block_frames=bf)


def fill(orc, rng, nhist):
    hist = []
    for _ in range(nhist):
        k, v = rand(rng, orc.B, orc.T, orc.H, orc.D), rand(rng, orc.B, orc.T, orc.H, orc.D)
        orc.append(k, v, 1)
        hist.append((k, v))
    return hist


@pytest.mark.parametrize("C,S,nhist,Fc", [(3, 1, 7, 2), (4, 2, 9, 1), (2, 0, 5, 2), (3, 1, 2, 1), (3, 2, 0, 2)])
def test_forward_equals_scalar_brute_force_at_rank_positions(C, S, nhist, Fc):
    rng = np.random.default_rng(31)
    B, H, D, gh, gw = 2, 1, 8, 2, 2
    T, pairs, base = gh * gw, (2, 1, 1), 10000.0
    orc = make(B, H, D, gh, gw, C, S, pairs, start=[5, 40])
    hist = fill(orc, rng, nhist)
    q, k, v = (rand(rng, B, Fc * T, H, D) for _ in range(3))
    out, lse = orc.attn_fwd(q, k, v, Fc)
    vis = brute_resident_after(nhist, C, S)
    Nq = Fc * T
    for b in range(B):
        k_ranks = list(range(len(vis) + Fc))       # sinks, window, chunk: 0, 1, 2, ...
        q_ranks = k_ranks[len(vis):]
        K = [list(hist[n][0][b, t, 0]) for n in vis for t in range(T)] + [list(k[b, t, 0]) for t in range(Nq)]
        V = [list(hist[n][1][b, t, 0]) for n in vis for t in range(T)] + [list(v[b, t, 0]) for t in range(Nq)]
        Q = [list(q[b, t, 0]) for t in range(Nq)]
        mask = [[True] * len(K) for _ in range(Nq)]
        O, L = brute_masked_attention(Q, K, V, q_ranks, k_ranks, mask, gh, gw, pairs, base)
        np.testing.assert_allclose(out[b, :, 0], O, atol=1e-12)
        np.testing.assert_allclose(lse[b, 0], L, atol=1e-12)


@pytest.mark.parametrize("C,S,nhist,Fc,bf", [(4, 1, 11, 2, None), (5, 2, 6, 3, 1), (3, 0, 8, 1, None), (4, 3, 4, 2, None)])
def test_equals_absolute_positions_on_a_fresh_stream_of_the_visible_frames(C, S, nhist, Fc, bf):
    """A stream reset to frame 0 and fed exactly the visible frames evicts nothing, and its
    absolute indices are the ranks: the pinned absolute path must give the same outputs and
    gradients."""
    rng = np.random.default_rng(32)
    B, H, D, gh, gw = 1, 2, 8, 2, 3
    T, pairs = gh * gw, (2, 1, 1)
    orc = make(B, H, D, gh, gw, C, S, pairs, start=[17], bf=bf)
    hist = fill(orc, rng, nhist)
    vis = brute_resident_after(nhist, C, S)
    fresh = make(B, H, D, gh, gw, C, S, pairs, start=[0], wr=False, bf=bf)
    for n in vis:
        fresh.append(hist[n][0], hist[n][1], 1)
    q, k, v, do = (rand(rng, B, Fc * T, H, D) for _ in range(4))
    np.testing.assert_allclose(orc.attn_fwd(q, k, v, Fc)[0], fresh.attn_fwd(q, k, v, Fc)[0], atol=1e-13)
    np.testing.assert_allclose(orc.attn_fwd(q, k, v, Fc)[1], fresh.attn_fwd(q, k, v, Fc)[1], atol=1e-13)
    for a, b in zip(orc.attn_bwd(q, k, v, do, Fc), fresh.attn_bwd(q, k, v, do, Fc)):
        np.testing.assert_allclose(a, b, atol=1e-13)


def test_without_sinks_identical_to_absolute_positions_at_any_start_frame():
    """Window and chunk frames are consecutive in both numberings, and rotary scores depend
    on position differences only."""
    rng = np.random.default_rng(33)
    B, H, D, gh, gw, C, Fc = 2, 1, 8, 2, 2, 3, 2
    T, pairs = gh * gw, (2, 1, 1)
    rel = make(B, H, D, gh, gw, C, 0, pairs, start=[3, 1000])
    absolute = make(B, H, D, gh, gw, C, 0, pairs, start=[3, 1000], wr=False)
    for step in range(5):
        q, k, v, do = (rand(rng, B, Fc * T, H, D) for _ in range(4))
        np.testing.assert_allclose(rel.attn_fwd(q, k, v, Fc)[0], absolute.attn_fwd(q, k, v, Fc)[0], atol=1e-9)
        for a, b in zip(rel.attn_bwd(q, k, v, do, Fc), absolute.attn_bwd(q, k, v, do, Fc)):
            np.testing.assert_allclose(a, b, atol=1e-9)
        rel.append(k, v, Fc)
        absolute.append(k, v, Fc)


def test_with_sinks_differs_from_absolute_only_once_frames_are_evicted_and_start_frame_is_irrelevant():
    rng = np.random.default_rng(34)
    B, H, D, gh, gw, C, S, Fc = 1, 1, 8, 2, 2, 3, 1, 1
    T, pairs = gh * gw, (2, 1, 1)
    rel = make(B, H, D, gh, gw, C, S, pairs, start=[0])
    rel_far = make(B, H, D, gh, gw, C, S, pairs, start=[123456])
    absolute = make(B, H, D, gh, gw, C, S, pairs, start=[0], wr=False)
    for step in range(6):
        q, k, v = (rand(rng, B, Fc * T, H, D) for _ in range(3))
        o_rel, o_abs = rel.attn_fwd(q, k, v, Fc)[0], absolute.attn_fwd(q, k, v, Fc)[0]
        np.testing.assert_array_equal(o_rel, rel_far.attn_fwd(q, k, v, Fc)[0])
        if step <= C:   # nothing evicted before the call: ranks are the absolute indices
            np.testing.assert_allclose(o_rel, o_abs, atol=1e-13)
        else:
            assert np.abs(o_rel - o_abs).max() > 1e-3
        for o in (rel, rel_far, absolute):
            o.append(k, v, Fc)


@pytest.mark.parametrize("C,S,nhist", [(3, 1, 6), (4, 2, 3)])
def test_gradients_match_autograd_through_rotation_at_rank_positions(C, S, nhist):
    rng = np.random.default_rng(35)
    B, H, D, gh, gw, Fc = 1, 2, 8, 2, 2, 2
    T, pairs, base = gh * gw, (2, 1, 1), 10000.0
    orc = make(B, H, D, gh, gw, C, S, pairs, start=[9])
    hist = fill(orc, rng, nhist)
    vis = brute_resident_after(nhist, C, S)
    q, k, v, do = (rand(rng, B, Fc * T, H, D) for _ in range(4))
    dq, dk, dv, extra = orc.attn_bwd(q, k, v, do, Fc, history_grads=True)
    from oracle.rolling_attention import rope_angles, rope_rotate
    ranks_h = list(range(len(vis)))
    ranks_c = [len(vis) + i for i in range(Fc)]
    for h in range(H):
        tq, tk, tv = (torch.tensor(x[0, :, h], dtype=torch.float64, requires_grad=True) for x in (q, k, v))
        # un-rotated cached keys as leaves: the gradient of the non-detached variant is w.r.t. them
        th_k = torch.tensor(np.concatenate([hist[n][0][0, :, h] for n in vis], 0), dtype=torch.float64, requires_grad=True)
        th_v = torch.tensor(np.concatenate([hist[n][1][0, :, h] for n in vis], 0), dtype=torch.float64, requires_grad=True)
        kr = torch.cat([torch_rope(th_k, ranks_h, gh, gw, pairs, base), torch_rope(tk, ranks_c, gh, gw, pairs, base)], 0)
        s_ = torch_rope(tq, ranks_c, gh, gw, pairs, base) @ kr.T / np.sqrt(D)
        o = torch.softmax(s_, -1) @ torch.cat([th_v, tv], 0)
        o.backward(torch.tensor(do[0, :, h]))
        np.testing.assert_allclose(dq[0, :, h], tq.grad.numpy(), atol=1e-11)
        np.testing.assert_allclose(dk[0, :, h], tk.grad.numpy(), atol=1e-11)
        np.testing.assert_allclose(dv[0, :, h], tv.grad.numpy(), atol=1e-11)
        for i in range(len(vis)):   # cached rows: gradient w.r.t. the rotated key, turned back at the rank
            phi = rope_angles(i, gh, gw, pairs, base)
            got = rope_rotate(extra[(0, h)]["dk_hist_rot"][i * T:(i + 1) * T, None, :], -phi)[:, 0]
            np.testing.assert_allclose(got, th_k.grad.numpy()[i * T:(i + 1) * T], atol=1e-11)
        np.testing.assert_allclose(extra[(0, h)]["dv_hist"], th_v.grad.numpy(), atol=1e-11)


def test_gradients_match_central_finite_differences():
    rng = np.random.default_rng(36)
    B, H, D, gh, gw, C, S, Fc = 1, 1, 4, 1, 2, 3, 1, 2
    T, pairs = gh * gw, (1, 0, 1)
    orc = make(B, H, D, gh, gw, C, S, pairs, start=[2])
    fill(orc, rng, 5)
    q, k, v, do = (rand(rng, B, Fc * T, H, D) for _ in range(4))
    grads = orc.attn_bwd(q, k, v, do, Fc)
    eps = 1e-6
    for which, g in zip(range(3), grads):
        for idx in [(0, 0, 0, 0), (0, 1, 0, 2), (0, Fc * T - 1, 0, D - 1)]:
            args = [q.copy(), k.copy(), v.copy()]
            args[which][idx] += eps
            up = (orc.attn_fwd(*args, Fc)[0] * do).sum()
            args[which][idx] -= 2 * eps
            dn = (orc.attn_fwd(*args, Fc)[0] * do).sum()
            assert abs((up - dn) / (2 * eps) - g[idx]) < 1e-7


@pytest.mark.parametrize("C,S", [(4, 1), (5, 2), (3, 0)])
def test_slot_positions_are_the_ranks_of_the_resident_frames(C, S):
    rng = np.random.default_rng(37)
    B, H, D, gh, gw = 1, 1, 4, 1, 1
    orc = make(B, H, D, gh, gw, C, S, (0, 0, 0), start=[50])
    for n_total in range(1, 3 * C):
        k = rand(rng, B, 1, H, D)
        orc.append(k, k, 1)
        slot_frame, slot_pos, next_n = orc.table_arrays()
        resident = brute_resident_after(n_total, C, S)        # stream-local numbers, ascending
        for slot in range(C):
            f = int(slot_frame[0, slot])
            if f < 0:
                assert slot_pos[0, slot] == -1
            else:
                assert slot_pos[0, slot] == resident.index(f - 50)
        assert sorted(int(p) for p in slot_pos[0] if p >= 0) == list(range(len(resident)))
