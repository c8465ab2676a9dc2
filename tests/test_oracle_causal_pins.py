"""Pins of the oracle's finer block-causal mask inside the chunk (`block_frames`): the
frames of a chunk form blocks of k frames, and a query sees the chunk keys of its own and
of earlier blocks only -- with k = 1 the frame-by-frame factorisation p(x_i | x_<i) of
Sec. 3.1 evaluated for several frames in one call (teacher forcing).  Checked against
(a) a scalar brute force with the visibility rule written out per frame,
(b) the already pinned unmasked path fed one block at a time with appends in between,
(c) a closed form that reads out the visible frames, (d) torch autograd through a masked
softmax, (e) finite differences."""
import math

import numpy as np
import pytest
import torch

from oracle import RollingCacheOracle
from test_oracle_pins import brute_masked_attention, brute_resident_after, rand, torch_rope


def make(B, H, D, gh, gw, C, S, pairs, start, bf):
    return RollingCacheOracle(B, H, D, gh, gw, C, S, pairs, 10000.0, start_frames=start, block_frames=bf)


def fill(orc, rng, nhist):
    hist = []
    for _ in range(nhist):
        k, v = rand(rng, orc.B, orc.T, orc.H, orc.D), rand(rng, orc.B, orc.T, orc.H, orc.D)
        orc.append(k, v, 1)
        hist.append((k, v))
    return hist


def frame_rule(Nq, T, nh, bf):
    """mask[i][j]: history keys always; chunk key of frame fj iff its block is not later."""
    return [[j < nh or ((j - nh) // T) // bf <= (i // T) // bf for j in range(nh + Nq)] for i in range(Nq)]


@pytest.mark.parametrize("C,S,nhist,Fc,bf", [(3, 1, 5, 3, 1), (2, 0, 1, 3, 2), (2, 0, 0, 2, 1), (4, 1, 2, 4, 2), (3, 0, 4, 4, 3)])
def test_block_causal_forward_equals_scalar_brute_force(C, S, nhist, Fc, bf):
    rng = np.random.default_rng(21)
    B, H, D, gh, gw = 2, 1, 8, 2, 2
    T, pairs, base, start = gh * gw, (2, 1, 1), 10000.0, [4, 9]
    orc = make(B, H, D, gh, gw, C, S, pairs, start, bf)
    hist = fill(orc, rng, nhist)
    q, k, v = (rand(rng, B, Fc * T, H, D) for _ in range(3))
    out, lse = orc.attn_fwd(q, k, v, Fc)
    vis = brute_resident_after(nhist, C, S)
    nh, Nq = len(vis) * T, Fc * T
    for b in range(B):
        cf = [start[b] + nhist + i for i in range(Fc)]
        K = [list(hist[n][0][b, t, 0]) for n in vis for t in range(T)] + [list(k[b, t, 0]) for t in range(Nq)]
        V = [list(hist[n][1][b, t, 0]) for n in vis for t in range(T)] + [list(v[b, t, 0]) for t in range(Nq)]
        Q = [list(q[b, t, 0]) for t in range(Nq)]
        O, L = brute_masked_attention(Q, K, V, cf, [start[b] + n for n in vis] + cf, frame_rule(Nq, T, nh, bf),
                                      gh, gw, pairs, base)
        np.testing.assert_allclose(out[b, :, 0], O, atol=1e-12)
        np.testing.assert_allclose(lse[b, 0], L, atol=1e-12)


@pytest.mark.parametrize("nhist,Fc,bf", [(0, 3, 1), (2, 3, 1), (1, 4, 2), (3, 3, 2)])
def test_block_causal_chunk_equals_block_by_block_streaming_when_nothing_is_evicted(nhist, Fc, bf):
    # with room for every frame, frame block m of the chunk sees exactly what a chunk made of
    # that block alone would see after the earlier blocks have been appended
    rng = np.random.default_rng(22)
    B, H, D, gh, gw, C = 1, 2, 8, 2, 3, 16
    T, pairs = gh * gw, (2, 1, 1)
    masked = make(B, H, D, gh, gw, C, 0, pairs, [3], bf)
    stream = make(B, H, D, gh, gw, C, 0, pairs, [3], None)
    for _ in range(nhist):
        kf, vf = rand(rng, B, T, H, D), rand(rng, B, T, H, D)
        masked.append(kf, vf, 1)
        stream.append(kf, vf, 1)
    q, k, v, do = (rand(rng, B, Fc * T, H, D) for _ in range(4))
    out, lse = masked.attn_fwd(q, k, v, Fc)
    dq, dk, dv = masked.attn_bwd(q, k, v, do, Fc)
    for f0 in range(0, Fc, bf):
        n = min(bf, Fc - f0)
        rows = slice(f0 * T, (f0 + n) * T)
        o1, l1 = stream.attn_fwd(q[:, rows], k[:, rows], v[:, rows], n)
        np.testing.assert_allclose(out[:, rows], o1, atol=1e-13)
        np.testing.assert_allclose(lse[:, :, rows], l1, atol=1e-13)
        # dQ of a block is that of the streaming call (queries of later blocks do not enter it)
        dq1, _, _ = stream.attn_bwd(q[:, rows], k[:, rows], v[:, rows], do[:, rows], n)
        np.testing.assert_allclose(dq[:, rows], dq1, atol=1e-13)
        stream.append(k[:, rows], v[:, rows], n)
    # the last block's keys are seen by the last block only: their gradients are the streaming call's
    n_last = Fc - (Fc - 1) // bf * bf
    rows = slice((Fc - n_last) * T, Fc * T)
    ref = make(B, H, D, gh, gw, C, 0, pairs, [3], None)
    ref.history = [list(h[:nhist + Fc - n_last]) for h in stream.history]
    for t in ref.tables:
        for _ in range(nhist + Fc - n_last):
            t.append_frame()
    _, dk1, dv1 = ref.attn_bwd(q[:, rows], k[:, rows], v[:, rows], do[:, rows], n_last)
    np.testing.assert_allclose(dk[:, rows], dk1, atol=1e-13)
    np.testing.assert_allclose(dv[:, rows], dv1, atol=1e-13)


def test_zero_queries_read_out_the_visible_frames_per_query_frame():
    # Q = 0 -> uniform weights; V = one-hot of the frame a key belongs to -> O is the
    # indicator of the visible frames divided by their number
    B, H, gh, gw, C, S, nhist, Fc, bf = 1, 1, 2, 2, 3, 1, 5, 4, 2
    T = gh * gw
    n_ids = nhist + Fc
    D = 2 * ((n_ids + 1) // 2)
    orc = RollingCacheOracle(B, H, D, gh, gw, C, S, (0, 0, 0), 10000.0, block_frames=bf)
    def onehot(f):
        x = np.zeros((B, T, H, D)); x[..., f] = 1.0
        return x
    for n in range(nhist):
        orc.append(np.ones((B, T, H, D)), onehot(n), 1)
    v = np.concatenate([onehot(nhist + i) for i in range(Fc)], axis=1)
    out, _ = orc.attn_fwd(np.zeros((B, Fc * T, H, D)), np.ones((B, Fc * T, H, D)), v, Fc)
    resident = [0, 3, 4]                      # sink + the last two of frames 1..4
    for i in range(Fc):
        seen = resident + [nhist + j for j in range(Fc) if j // bf <= i // bf]
        expect = np.zeros(D); expect[seen] = 1.0 / len(seen)
        np.testing.assert_allclose(out[0, i * T:(i + 1) * T, 0], np.tile(expect, (T, 1)), atol=1e-15)


def test_block_size_of_the_whole_chunk_or_more_is_the_unmasked_call():
    rng = np.random.default_rng(23)
    B, H, D, gh, gw, C, S, Fc = 2, 2, 8, 2, 2, 3, 1, 3
    T = gh * gw
    q, k, v, do = (rand(rng, B, Fc * T, H, D) for _ in range(4))
    res = []
    for bf in (None, Fc, Fc + 2):
        orc = make(B, H, D, gh, gw, C, S, (2, 1, 1), [0, 7], bf)
        fill(orc, np.random.default_rng(24), 4)
        res.append(orc.attn_fwd(q, k, v, Fc) + orc.attn_bwd(q, k, v, do, Fc))
    for other in res[1:]:
        for a, b in zip(res[0], other):
            np.testing.assert_array_equal(a, b)


@pytest.mark.parametrize("C,S,nhist,Fc,bf", [(3, 1, 4, 3, 1), (2, 0, 0, 3, 2), (2, 0, 3, 4, 2)])
def test_block_causal_gradients_equal_autograd_of_a_masked_softmax(C, S, nhist, Fc, bf):
    rng = np.random.default_rng(25)
    B, H, D, gh, gw = 1, 2, 8, 2, 2
    T, pairs, base, start = gh * gw, (2, 1, 1), 10000.0, [3]
    orc = make(B, H, D, gh, gw, C, S, pairs, start, bf)
    hist = fill(orc, rng, nhist)
    q, k, v, do = (rand(rng, B, Fc * T, H, D) for _ in range(4))
    dq, dk, dv = orc.attn_bwd(q, k, v, do, Fc)
    vis = brute_resident_after(nhist, C, S)
    Nq, nh = Fc * T, len(vis) * T
    cf = [start[0] + nhist + i for i in range(Fc)]
    visible = torch.tensor(frame_rule(Nq, T, nh, bf))
    for h in range(H):
        tq, tk, tv = (torch.tensor(x[0, :, h], dtype=torch.float64, requires_grad=True) for x in (q, k, v))
        hk = [torch_rope(torch.tensor(hist[n][0][0, :, h]), [start[0] + n], gh, gw, pairs, base) for n in vis]
        hv = [torch.tensor(hist[n][1][0, :, h]) for n in vis]
        kk = torch.cat(hk + [torch_rope(tk, cf, gh, gw, pairs, base)], 0)
        vv = torch.cat(hv + [tv], 0)
        s = torch_rope(tq, cf, gh, gw, pairs, base) @ kk.T / math.sqrt(D)
        o = torch.softmax(s.masked_fill(~visible, -math.inf), -1) @ vv
        o.backward(torch.tensor(do[0, :, h]))
        np.testing.assert_allclose(dq[0, :, h], tq.grad.numpy(), atol=1e-12)
        np.testing.assert_allclose(dk[0, :, h], tk.grad.numpy(), atol=1e-12)
        np.testing.assert_allclose(dv[0, :, h], tv.grad.numpy(), atol=1e-12)


def test_block_causal_gradients_match_finite_differences():
    rng = np.random.default_rng(26)
    B, H, D, gh, gw, C, S, nhist, Fc, bf = 1, 1, 4, 1, 2, 2, 0, 3, 3, 1
    T = gh * gw
    orc = make(B, H, D, gh, gw, C, S, (1, 0, 1), [2], bf)
    fill(orc, rng, nhist)
    q, k, v, do = (rand(rng, B, Fc * T, H, D) for _ in range(4))
    grads = orc.attn_bwd(q, k, v, do, Fc)

    def loss(q_, k_, v_):
        return float((orc.attn_fwd(q_, k_, v_, Fc)[0] * do).sum())

    eps = 1e-6
    for which, g in enumerate(grads):
        for idx in [(0, 0, 0, 0), (0, T, 0, 1), (0, 2 * T + 1, 0, 3), (0, Fc * T - 1, 0, 2)]:
            args = [q.copy(), k.copy(), v.copy()]
            args[which][idx] += eps
            up = loss(*args)
            args[which][idx] -= 2 * eps
            dn = loss(*args)
            np.testing.assert_allclose(g[idx], (up - dn) / (2 * eps), rtol=2e-6, atol=1e-9)


def test_group_calls_take_the_same_mask():
    rng = np.random.default_rng(27)
    B, H, D, gh, gw, C, S, Fc, G, bf = 2, 1, 8, 2, 2, 3, 1, 3, 2, 1
    T = gh * gw
    orc = make(B, H, D, gh, gw, C, S, (2, 1, 1), [0, 5], bf)
    fill(orc, rng, 4)
    q, k, v, do = (rand(rng, B * G, Fc * T, H, D) for _ in range(4))
    out, lse = orc.group_attn_fwd(q, k, v, Fc, G)
    grads = orc.group_attn_bwd(q, k, v, do, Fc, G)
    for g in range(G):
        sel = [b * G + g for b in range(B)]
        o1, l1 = orc.attn_fwd(q[sel], k[sel], v[sel], Fc)
        np.testing.assert_array_equal(out[sel], o1)
        np.testing.assert_array_equal(lse[sel], l1)
        for a, b_ in zip(grads, orc.attn_bwd(q[sel], k[sel], v[sel], do[sel], Fc)):
            np.testing.assert_array_equal(a[sel], b_)
