"""Pins for the fp64 oracle: everything here checks oracle/ against something
other than itself -- brute force written out with python loops and complex
arithmetic, closed forms, invariants, a library SDPA + autograd, and finite
differences.  CPU only.

The paper prints no worked numeric example for this path (it has no attention
formula at all), so there is no paper-value fixture; the definitions pinned
are those of Sec. 3.2 (sinks + rolling window), Sec. 3.3 (detached history)
and the readings stated in the oracle's module docstring.
"""
import cmath
import math

import numpy as np
import pytest
import torch

from oracle import RollingCacheOracle, RingTableSim, rope_angles, rope_rotate, visible_history


# ----------------------------------------------------------------------------
# an independent brute force, scalar loops only
# ----------------------------------------------------------------------------

def brute_rope(vec, frame, row, col, pairs, base):
    """Rotate one D-vector using complex multiplication, pair by pair."""
    n_t, n_h, n_w = pairs
    out = list(vec)
    for i in range(n_t + n_h + n_w):
        if i < n_t:
            pos, j, n = frame, i, n_t
        elif i < n_t + n_h:
            pos, j, n = row, i - n_t, n_h
        else:
            pos, j, n = col, i - n_t - n_h, n_w
        ang = pos * (1.0 / (base ** (j / n)))
        z = complex(vec[2 * i], vec[2 * i + 1]) * cmath.exp(1j * ang)
        out[2 * i], out[2 * i + 1] = z.real, z.imag
    return out


def brute_masked_attention(Q, K, V, q_frames, k_frames, mask, gh, gw, pairs, base):
    """Q [Nq][D] with absolute frame per query frame block, K/V [Nk][D]; mask[i][j]
    says whether query i sees key j.  All python floats."""
    T = gh * gw
    D = len(Q[0])

    def rot(X, frames):
        res = []
        for n, x in enumerate(X):
            f = frames[n // T]
            t = n % T
            res.append(brute_rope(x, f, t // gw, t % gw, pairs, base))
        return res

    Qr, Kr = rot(Q, q_frames), rot(K, k_frames)
    O, L = [], []
    for i, qv in enumerate(Qr):
        s = []
        for j, kv in enumerate(Kr):
            if mask[i][j]:
                s.append((j, sum(a * b for a, b in zip(qv, kv)) / math.sqrt(D)))
        z = sum(math.exp(x) for _, x in s)
        o = [0.0] * D
        for j, x in s:
            w = math.exp(x) / z
            for d in range(D):
                o[d] += w * V[j][d]
        O.append(o)
        L.append(math.log(z))
    return np.array(O), np.array(L)


def brute_resident_after(n_total, capacity, sinks):
    """Frame numbers resident after appending frames 0..n_total-1 one by one into
    a store of `capacity` frames that drops the oldest non-sink frame when full."""
    resident = []
    for n in range(n_total):
        if len(resident) == capacity:
            victims = [m for m in resident if m >= sinks]
            resident.remove(min(victims))
        resident.append(n)
    return sorted(resident)


def make(B, H, D, gh, gw, C, S, pairs, seed=0, start=None):
    return RollingCacheOracle(B, H, D, gh, gw, C, S, pairs, 10000.0, start_frames=start)


def rand(rng, *shape):
    return rng.standard_normal(shape)


# ----------------------------------------------------------------------------
# rotary embedding
# ----------------------------------------------------------------------------

def test_rope_matches_complex_rotation_per_token():
    rng = np.random.default_rng(1)
    gh, gw, H, D, pairs = 3, 4, 2, 12, (2, 2, 2)
    x = rand(rng, gh * gw, H, D)
    y = rope_rotate(x, rope_angles(5, gh, gw, pairs, 10000.0))
    for t in range(gh * gw):
        for h in range(H):
            ref = brute_rope(list(x[t, h]), 5, t // gw, t % gw, pairs, 10000.0)
            np.testing.assert_allclose(y[t, h], ref, rtol=0, atol=1e-13)


def test_rope_angle_values_and_axis_assignment():
    # frequencies are base**(-j/n_axis): j=0 -> 1, so the first pair of each axis
    # turns by exactly the position; the last pair by position*base**(-(n-1)/n)
    phi = rope_angles(7, 2, 3, (2, 3, 1), 100.0)
    assert phi.shape == (6, 6)
    t = 1 * 3 + 2  # row 1, col 2
    np.testing.assert_allclose(phi[t], [7.0, 7.0 * 100 ** -0.5, 1.0, 100 ** (-1 / 3), 100 ** (-2 / 3), 2.0], rtol=1e-15)
    assert rope_angles(0, 2, 3, (2, 3, 1), 100.0)[0].tolist() == [0.0] * 6


def test_rope_is_norm_preserving_identity_at_origin_and_invertible():
    rng = np.random.default_rng(2)
    gh, gw, pairs = 4, 5, (4, 2, 2)
    x = rand(rng, gh * gw, 3, 16)
    phi = rope_angles(9, gh, gw, pairs, 10000.0)
    y = rope_rotate(x, phi)
    n_in = x[..., 0::2] ** 2 + x[..., 1::2] ** 2
    n_out = y[..., 0::2] ** 2 + y[..., 1::2] ** 2
    np.testing.assert_allclose(n_out, n_in, rtol=1e-13)
    y0 = rope_rotate(x, rope_angles(0, gh, gw, pairs, 10000.0))
    np.testing.assert_array_equal(y0[0], x[0])  # frame 0, row 0, col 0
    np.testing.assert_allclose(rope_rotate(y, -phi), x, atol=1e-14)
    assert np.abs(y - x).max() > 0.1  # it does rotate


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(3)
    gh, gw, pairs, D = 2, 2, (2, 1, 1), 8
    q = rand(rng, gh * gw, 1, D)
    k = rand(rng, gh * gw, 1, D)
    s1 = rope_rotate(q, rope_angles(10, gh, gw, pairs, 50.0))[:, 0] @ rope_rotate(k, rope_angles(7, gh, gw, pairs, 50.0))[:, 0].T
    s2 = rope_rotate(q, rope_angles(110, gh, gw, pairs, 50.0))[:, 0] @ rope_rotate(k, rope_angles(107, gh, gw, pairs, 50.0))[:, 0].T
    np.testing.assert_allclose(s1, s2, atol=1e-11)


# ----------------------------------------------------------------------------
# visible set and ring tables
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("C,S", [(1, 0), (3, 0), (4, 1), (5, 2), (6, 5), (12, 1), (7, 3)])
def test_visible_history_equals_fifo_store_with_sinks(C, S):
    for n0 in range(0, 4 * C + 3):
        assert visible_history(n0, S, C - S) == brute_resident_after(n0, C, S)


@pytest.mark.parametrize("C,S,Fc", [(4, 0, 1), (4, 1, 3), (6, 2, 3), (12, 1, 3), (5, 0, 5)])
def test_attend_then_append_equals_append_first_into_larger_store(C, S, Fc):
    # what the chunk sees = residents of a C-frame store + the chunk itself
    #                     = residents of a (C+Fc)-frame store after the chunk went in
    for n0 in range(0, 3 * C + 2):
        seen = visible_history(n0, S, C - S) + list(range(n0, n0 + Fc))
        assert seen == brute_resident_after(n0 + Fc, C + Fc, S)


@pytest.mark.parametrize("C,S", [(1, 0), (4, 0), (4, 1), (12, 1), (18, 0), (21, 3), (5, 4)])
def test_ring_table_sim_invariants(C, S):
    sim = RingTableSim(C, S, start_frame=100)
    for n in range(5 * C + 7):
        slot = sim.append_frame()
        assert 0 <= slot < C
        frames = sim.slot_frame()
        resident = sorted(f - 100 for f in frames if f >= 0)
        assert resident == brute_resident_after(n + 1, C, S)
        # sinks never move
        for s in range(min(S, n + 1)):
            assert frames[s] == 100 + s
        assert sim.slot_pos() == frames
        # closed form of the slot a frame number lands in
        expect = n if n < C else (S + (n - S) % (C - S))
        assert slot == expect


# ----------------------------------------------------------------------------
# forward vs brute force
# ----------------------------------------------------------------------------

def stream_through_oracle(orc, Ks, Vs, Qs, Fc):
    """Feed chunks one by one: attend, then append.  Returns per-chunk (O, LSE)."""
    outs = []
    for q, k, v in zip(Qs, Ks, Vs):
        outs.append(orc.attn_fwd(q, k, v, Fc))
        orc.append(k, v, Fc)
    return outs


@pytest.mark.parametrize("C,S,start", [(64, 0, 0), (3, 1, 0), (4, 0, 11), (2, 1, 5)])
def test_streaming_equals_block_causal_masked_attention_over_whole_sequence(C, S, start):
    rng = np.random.default_rng(10 + C)
    B, H, D, gh, gw, Fc, nchunks = 1, 2, 8, 2, 2, 2, 4
    pairs = (2, 1, 1)
    T = gh * gw
    orc = make(B, H, D, gh, gw, C, S, pairs, start=[start])
    Qs = [rand(rng, B, Fc * T, H, D) for _ in range(nchunks)]
    Ks = [rand(rng, B, Fc * T, H, D) for _ in range(nchunks)]
    Vs = [rand(rng, B, Fc * T, H, D) for _ in range(nchunks)]
    outs = stream_through_oracle(orc, Ks, Vs, Qs, Fc)
    Kall = np.concatenate(Ks, 1)
    Vall = np.concatenate(Vs, 1)
    nfr = Fc * nchunks
    k_frames = [start + n for n in range(nfr)]
    for c in range(nchunks):
        n0 = c * Fc
        resident = brute_resident_after(n0, C, S)
        for h in range(H):
            mask = []
            for i in range(Fc * T):
                row = []
                for j in range(nfr * T):
                    fn = j // T
                    row.append((fn in resident) or (n0 <= fn < n0 + Fc))
                mask.append(row)
            O, L = brute_masked_attention(
                Qs[c][0, :, h].tolist(), Kall[0, :, h].tolist(), Vall[0, :, h].tolist(),
                [start + n0 + i for i in range(Fc)], k_frames, mask, gh, gw, pairs, 10000.0)
            np.testing.assert_allclose(outs[c][0][0, :, h], O, atol=1e-12)
            np.testing.assert_allclose(outs[c][1][0, h], L, atol=1e-12)


def test_eviction_equals_masking_and_big_ring_equals_full_causal():
    # with C >= all frames nothing is ever masked: every earlier frame is visible
    # (plain block-causal); with a small ring some are not, and the outputs differ
    rng = np.random.default_rng(4)
    B, H, D, gh, gw, Fc = 2, 1, 8, 2, 3, 1
    T = gh * gw
    pairs = (2, 1, 1)
    big = make(B, H, D, gh, gw, 50, 0, pairs)
    small = make(B, H, D, gh, gw, 3, 1, pairs)
    differs = False
    for c in range(7):
        q, k, v = (rand(rng, B, Fc * T, H, D) for _ in range(3))
        ob, _ = big.attn_fwd(q, k, v, Fc)
        os_, _ = small.attn_fwd(q, k, v, Fc)
        if c <= 3:
            np.testing.assert_allclose(ob, os_, atol=1e-13)  # ring not yet overflowing
        else:
            differs |= np.abs(ob - os_).max() > 1e-3
        big.append(k, v, Fc)
        small.append(k, v, Fc)
    assert differs


def test_softmax_rows_sum_to_one_and_lse_consistent():
    rng = np.random.default_rng(5)
    B, H, D, gh, gw, Fc = 1, 2, 16, 2, 2, 2
    T = gh * gw
    orc = make(B, H, D, gh, gw, 3, 1, (4, 2, 2))
    for _ in range(4):
        k, v = rand(rng, B, T, H, D), rand(rng, B, T, H, D)
        orc.append(k, v, 1)
    q, k, v = (rand(rng, B, Fc * T, H, D) for _ in range(3))
    o, lse, probs = orc.attn_fwd(q, k, v, Fc, return_probs=True)
    for (b, h), p in probs.items():
        assert p.shape == (Fc * T, (3 + Fc) * T)
        np.testing.assert_allclose(p.sum(1), 1.0, atol=1e-14)
        assert (p > 0).all()


def test_zero_query_gives_mean_of_visible_values_and_reads_out_visible_frames():
    # V = one-hot of the frame number: with Q = 0 the output is uniform over the
    # visible tokens, so O[d] = T/(Nk) for visible frame d and 0 for evicted ones
    B, H, gh, gw, Fc, C, S = 1, 1, 2, 2, 2, 5, 2
    D = 32
    T = gh * gw
    pairs = (8, 4, 4)
    orc = make(B, H, D, gh, gw, C, S, pairs, start=[3])
    rng = np.random.default_rng(6)

    def onehot_frames(first, count):
        v = np.zeros((B, count * T, H, D))
        for i in range(count):
            v[:, i * T:(i + 1) * T, :, first + i] = 1.0
        return v

    n = 0
    for step in range(6):
        q = np.zeros((B, Fc * T, H, D))
        k = rand(rng, B, Fc * T, H, D)
        v = onehot_frames(n, Fc)
        o, lse = orc.attn_fwd(q, k, v, Fc)
        vis = brute_resident_after(n, C, S) + list(range(n, n + Fc))
        expect = np.zeros(D)
        expect[vis] = 1.0 / len(vis)
        np.testing.assert_allclose(o[0, :, 0], np.broadcast_to(expect, (Fc * T, D)), atol=1e-15)
        np.testing.assert_allclose(lse[0, 0], math.log(len(vis) * T), atol=1e-13)
        orc.append(k, v, Fc)
        n += Fc


def test_constant_values_pass_through():
    rng = np.random.default_rng(7)
    B, H, D, gh, gw = 1, 2, 8, 2, 2
    T = gh * gw
    orc = make(B, H, D, gh, gw, 2, 0, (2, 1, 1))
    row = rand(rng, D)
    for _ in range(3):
        orc.append(rand(rng, B, T, H, D), np.broadcast_to(row, (B, T, H, D)).copy(), 1)
    q, k = rand(rng, B, T, H, D), rand(rng, B, T, H, D)
    o, _ = orc.attn_fwd(q, k, np.broadcast_to(row, (B, T, H, D)).copy(), 1)
    np.testing.assert_allclose(o, np.broadcast_to(row, o.shape), atol=1e-14)


def test_frame_shift_invariance_of_outputs_and_gradients():
    rng = np.random.default_rng(8)
    B, H, D, gh, gw, Fc, C, S = 2, 2, 16, 2, 2, 2, 3, 1
    T = gh * gw
    pairs = (4, 2, 2)
    a = make(B, H, D, gh, gw, C, S, pairs, start=[0, 4])
    b = make(B, H, D, gh, gw, C, S, pairs, start=[37, 1000])
    for _ in range(5):
        k, v = rand(rng, B, T, H, D), rand(rng, B, T, H, D)
        a.append(k, v, 1)
        b.append(k, v, 1)
    q, k, v, do = (rand(rng, B, Fc * T, H, D) for _ in range(4))
    oa, la = a.attn_fwd(q, k, v, Fc)
    ob, lb = b.attn_fwd(q, k, v, Fc)
    np.testing.assert_allclose(oa, ob, atol=1e-10)
    np.testing.assert_allclose(la, lb, atol=1e-10)
    for ga, gb in zip(a.attn_bwd(q, k, v, do, Fc), b.attn_bwd(q, k, v, do, Fc)):
        np.testing.assert_allclose(ga, gb, atol=1e-9)


# ----------------------------------------------------------------------------
# library routine: SDPA and autograd in fp64 on the CPU
# ----------------------------------------------------------------------------

def test_no_rope_empty_cache_is_plain_sdpa_with_autograd_gradients():
    rng = np.random.default_rng(9)
    B, H, D, gh, gw, Fc = 2, 3, 16, 2, 3, 2
    T = gh * gw
    orc = make(B, H, D, gh, gw, 4, 1, (0, 0, 0))
    q, k, v, do = (rand(rng, B, Fc * T, H, D) for _ in range(4))
    o, lse = orc.attn_fwd(q, k, v, Fc)
    tq, tk, tv = (torch.tensor(x.transpose(0, 2, 1, 3), dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    to = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)
    np.testing.assert_allclose(o, to.detach().numpy().transpose(0, 2, 1, 3), atol=1e-13)
    to.backward(torch.tensor(do.transpose(0, 2, 1, 3)))
    dq, dk, dv = orc.attn_bwd(q, k, v, do, Fc)
    for mine, ref in ((dq, tq), (dk, tk), (dv, tv)):
        np.testing.assert_allclose(mine, ref.grad.numpy().transpose(0, 2, 1, 3), atol=1e-12)
    tl = torch.logsumexp(tq.detach() @ tk.detach().transpose(-1, -2) / math.sqrt(D), -1)
    np.testing.assert_allclose(lse, tl.numpy(), atol=1e-12)


def torch_rope(x, frames, gh, gw, pairs, base):
    """x [N, D] torch fp64; complex-multiplication rotary, differentiable."""
    T = gh * gw
    N, D = x.shape
    n_t, n_h, n_w = pairs
    ang = torch.zeros(N, D // 2, dtype=torch.float64)
    for n in range(N):
        f, t = frames[n // T], n % T
        pos = [f] * n_t + [t // gw] * n_h + [t % gw] * n_w
        idx = list(range(n_t)) + list(range(n_h)) + list(range(n_w))
        cnt = [n_t] * n_t + [n_h] * n_h + [n_w] * n_w
        for i in range(D // 2):
            ang[n, i] = pos[i] * base ** (-idx[i] / cnt[i])
    z = torch.view_as_complex(x.reshape(N, D // 2, 2).contiguous()) * torch.polar(torch.ones_like(ang), ang)
    return torch.view_as_real(z).reshape(N, D)


@pytest.mark.parametrize("C,S,nhist", [(3, 1, 5), (4, 0, 2), (2, 0, 0)])
def test_gradients_with_detached_history_match_autograd_through_rope(C, S, nhist):
    rng = np.random.default_rng(11)
    B, H, D, gh, gw, Fc = 1, 2, 8, 2, 2, 2
    T = gh * gw
    pairs, base, start = (2, 1, 1), 10000.0, 6
    orc = make(B, H, D, gh, gw, C, S, pairs, start=[start])
    hist = []
    for _ in range(nhist):
        k, v = rand(rng, B, T, H, D), rand(rng, B, T, H, D)
        orc.append(k, v, 1)
        hist.append((k, v))
    q, k, v, do = (rand(rng, B, Fc * T, H, D) for _ in range(4))
    dq, dk, dv, extra = orc.attn_bwd(q, k, v, do, Fc, history_grads=True)
    vis = brute_resident_after(nhist, C, S)
    for h in range(H):
        tq, tk, tv = (torch.tensor(x[0, :, h], dtype=torch.float64, requires_grad=True) for x in (q, k, v))
        cf = [start + nhist + i for i in range(Fc)]
        parts_k = [torch_rope(torch.tensor(hist[n][0][0, :, h]), [start + n], gh, gw, pairs, base) for n in vis]
        parts_v = [torch.tensor(hist[n][1][0, :, h]) for n in vis]
        hk = [p.clone().requires_grad_(True) for p in parts_k]
        hv = [p.clone().requires_grad_(True) for p in parts_v]
        kk = torch.cat(hk + [torch_rope(tk, cf, gh, gw, pairs, base)], 0)
        vv = torch.cat(hv + [tv], 0)
        s = torch_rope(tq, cf, gh, gw, pairs, base) @ kk.T / math.sqrt(D)
        o = torch.softmax(s, -1) @ vv
        o.backward(torch.tensor(do[0, :, h]))
        np.testing.assert_allclose(dq[0, :, h], tq.grad.numpy(), atol=1e-12)
        np.testing.assert_allclose(dk[0, :, h], tk.grad.numpy(), atol=1e-12)
        np.testing.assert_allclose(dv[0, :, h], tv.grad.numpy(), atol=1e-12)
        # the chunk's gradients are the chunk rows of the full gradient; the
        # history rows exist too but are simply not returned (detached)
        if vis:
            np.testing.assert_allclose(extra[(0, h)]["dk_hist_rot"], torch.cat([t.grad for t in hk]).numpy(), atol=1e-12)
            np.testing.assert_allclose(extra[(0, h)]["dv_hist"], torch.cat([t.grad for t in hv]).numpy(), atol=1e-12)
        # each row of dS sums to zero
        np.testing.assert_allclose(extra[(0, h)]["ds"].sum(1), 0.0, atol=1e-13)


def test_gradients_match_central_finite_differences():
    rng = np.random.default_rng(12)
    B, H, D, gh, gw, Fc, C, S = 1, 1, 8, 2, 2, 1, 2, 1
    T = gh * gw
    pairs = (2, 1, 1)

    def build():
        o = make(B, H, D, gh, gw, C, S, pairs, start=[2])
        r = np.random.default_rng(99)
        for _ in range(4):
            o.append(rand(r, B, T, H, D), rand(r, B, T, H, D), 1)
        return o

    orc = build()
    q, k, v, w = (rand(rng, B, Fc * T, H, D) for _ in range(4))

    def loss(q_, k_, v_):
        return float((orc.attn_fwd(q_, k_, v_, Fc)[0] * w).sum())

    grads = orc.attn_bwd(q, k, v, w, Fc)
    eps = 1e-6
    for which, g in enumerate(grads):
        for idx in [(0, 0, 0, 0), (0, 1, 0, 3), (0, 3, 0, 7), (0, 2, 0, 4)]:
            args = [q.copy(), k.copy(), v.copy()]
            args[which][idx] += eps
            up = loss(*args)
            args[which][idx] -= 2 * eps
            dn = loss(*args)
            fd = (up - dn) / (2 * eps)
            assert abs(fd - g[idx]) <= 1e-7 * max(1.0, abs(fd)), (which, idx, fd, g[idx])


# ----------------------------------------------------------------------------
# planted mistakes must be caught (run against mutated copies, CPU only)
# ----------------------------------------------------------------------------

def test_pins_catch_a_transposed_pair_layout():
    # a half-split ("rotate-half") pair layout instead of adjacent pairs gives
    # the same scores but different gradients w.r.t. un-rotated inputs: the
    # complex-rotation pin must tell the two apart
    rng = np.random.default_rng(13)
    x = rand(rng, 4, 1, 8)
    phi = rope_angles(3, 2, 2, (2, 1, 1), 10000.0)
    good = rope_rotate(x, phi)
    half = x.copy()
    c, s = np.cos(phi)[:, None, :], np.sin(phi)[:, None, :]
    half[..., :4] = x[..., :4] * c - x[..., 4:] * s
    half[..., 4:] = x[..., :4] * s + x[..., 4:] * c
    ref = np.array([brute_rope(list(x[t, 0]), 3, t // 2, t % 2, (2, 1, 1), 10000.0) for t in range(4)])
    assert np.abs(good[:, 0] - ref).max() < 1e-13
    assert np.abs(half[:, 0] - ref).max() > 1e-2
