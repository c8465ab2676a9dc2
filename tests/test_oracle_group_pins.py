"""Pins of the oracle's group-wise candidate attention (Sec. 3.2: G candidate chunks are
generated from one shared, frozen rolling cache).  The oracle writes it as a loop of
independent attentions; here it is checked against ONE attention over the history and all
candidates' chunks at once, with a mask that hides the other candidates' chunks: by scalar
brute force for the forward, by torch autograd for the gradients."""
import math

import numpy as np
import pytest
import torch

from test_oracle_pins import brute_masked_attention, brute_resident_after, make, rand, torch_rope


def _setup(rng, B, H, D, gh, gw, C, S, pairs, start, nhist, Fc, G):
    T = gh * gw
    orc = make(B, H, D, gh, gw, C, S, pairs, start=start)
    hist = []
    for _ in range(nhist):
        k, v = rand(rng, B, T, H, D), rand(rng, B, T, H, D)
        orc.append(k, v, 1)
        hist.append((k, v))
    q, k, v, do = (rand(rng, B * G, Fc * T, H, D) for _ in range(4))
    return orc, hist, q, k, v, do


@pytest.mark.parametrize("C,S,nhist,Fc,G", [(3, 1, 5, 1, 3), (2, 0, 1, 2, 2), (2, 0, 0, 1, 2)])
def test_group_forward_equals_one_masked_attention_over_all_candidates(C, S, nhist, Fc, G):
    rng = np.random.default_rng(5)
    B, H, D, gh, gw = 2, 1, 8, 2, 2
    T, pairs, base, start = gh * gw, (2, 1, 1), 10000.0, [4, 9]
    orc, hist, q, k, v, _ = _setup(rng, B, H, D, gh, gw, C, S, pairs, start, nhist, Fc, G)
    out, lse = orc.group_attn_fwd(q, k, v, Fc, G)
    vis = brute_resident_after(nhist, C, S)
    Nq = Fc * T
    for b in range(B):
        chunk_frames = [start[b] + nhist + i for i in range(Fc)]
        K = [list(hist[n][0][b, t, 0]) for n in vis for t in range(T)]
        V = [list(hist[n][1][b, t, 0]) for n in vis for t in range(T)]
        k_frames = [start[b] + n for n in vis]
        Q = []
        for g in range(G):
            c = b * G + g
            K += [list(k[c, t, 0]) for t in range(Nq)]
            V += [list(v[c, t, 0]) for t in range(Nq)]
            Q += [list(q[c, t, 0]) for t in range(Nq)]
            k_frames += chunk_frames
        nh = len(vis) * T
        mask = [[j < nh or (j - nh) // Nq == i // Nq for j in range(len(K))] for i in range(len(Q))]
        O, L = brute_masked_attention(Q, K, V, chunk_frames * G, k_frames, mask, gh, gw, pairs, base)
        for g in range(G):
            c = b * G + g
            np.testing.assert_allclose(out[c, :, 0], O[g * Nq:(g + 1) * Nq], atol=1e-12)
            np.testing.assert_allclose(lse[c, 0], L[g * Nq:(g + 1) * Nq], atol=1e-12)


@pytest.mark.parametrize("C,S,nhist,Fc,G", [(3, 1, 4, 2, 3), (2, 0, 0, 1, 2)])
def test_group_gradients_equal_autograd_of_the_masked_attention_with_history_detached(C, S, nhist, Fc, G):
    rng = np.random.default_rng(6)
    B, H, D, gh, gw = 1, 2, 8, 2, 2
    T, pairs, base, start = gh * gw, (2, 1, 1), 10000.0, [3]
    orc, hist, q, k, v, do = _setup(rng, B, H, D, gh, gw, C, S, pairs, start, nhist, Fc, G)
    dq, dk, dv = orc.group_attn_bwd(q, k, v, do, Fc, G)
    vis = brute_resident_after(nhist, C, S)
    Nq = Fc * T
    cf = [start[0] + nhist + i for i in range(Fc)]
    for h in range(H):
        tq, tk, tv = (torch.tensor(x[:, :, h].reshape(G * Nq, D), dtype=torch.float64, requires_grad=True) for x in (q, k, v))
        hk = [torch_rope(torch.tensor(hist[n][0][0, :, h]), [start[0] + n], gh, gw, pairs, base) for n in vis]
        hv = [torch.tensor(hist[n][1][0, :, h]) for n in vis]
        kk = torch.cat(hk + [torch_rope(tk, cf * G, gh, gw, pairs, base)], 0)
        vv = torch.cat(hv + [tv], 0)
        nh = len(vis) * T
        s = torch_rope(tq, cf * G, gh, gw, pairs, base) @ kk.T / math.sqrt(D)
        i = torch.arange(G * Nq)[:, None] // Nq
        j = torch.arange(nh + G * Nq)[None, :]
        visible = (j < nh) | ((j - nh) // Nq == i)
        o = torch.softmax(s.masked_fill(~visible, -math.inf), -1) @ vv
        o.backward(torch.tensor(do[:, :, h].reshape(G * Nq, D)))
        np.testing.assert_allclose(dq[:, :, h].reshape(G * Nq, D), tq.grad.numpy(), atol=1e-12)
        np.testing.assert_allclose(dk[:, :, h].reshape(G * Nq, D), tk.grad.numpy(), atol=1e-12)
        np.testing.assert_allclose(dv[:, :, h].reshape(G * Nq, D), tv.grad.numpy(), atol=1e-12)


def test_group_of_one_is_the_plain_call_and_candidates_do_not_see_each_other():
    rng = np.random.default_rng(7)
    B, H, D, gh, gw, C, S, Fc, G = 2, 2, 8, 2, 3, 3, 1, 1, 3
    orc, _, q, k, v, do = _setup(rng, B, H, D, gh, gw, C, S, (2, 1, 1), [0, 5], 4, Fc, G)
    out, lse = orc.group_attn_fwd(q, k, v, Fc, G)
    grads = orc.group_attn_bwd(q, k, v, do, Fc, G)
    for g in range(G):
        sel = [b * G + g for b in range(B)]
        o1, l1 = orc.attn_fwd(q[sel], k[sel], v[sel], Fc)
        np.testing.assert_array_equal(out[sel], o1)
        np.testing.assert_array_equal(lse[sel], l1)
        for a, b_ in zip(grads, orc.attn_bwd(q[sel], k[sel], v[sel], do[sel], Fc)):
            np.testing.assert_array_equal(a[sel], b_)
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[1], k2[1], v2[1] = 7.0, -3.0, 2.0  # another candidate of stream 0
    out2, _ = orc.group_attn_fwd(q2, k2, v2, Fc, G)
    np.testing.assert_array_equal(out2[0], out[0])
    np.testing.assert_array_equal(out2[2:], out[2:])
