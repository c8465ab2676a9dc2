"""Pins for the parts of the oracle's state handling and test conveniences that the attention
pins do not reach: a per-stream reset in the middle of a run, the row-subset option of the
forward, and the bf16 rounding used by the kernels' rounding model (and by the oracle's diagnostic
switch that rounds the cached rotated keys).  CPU only."""
import numpy as np
import pytest
import torch

from oracle import RollingCacheOracle, rope_angles, rope_rotate, round_to_bf16, visible_history


def _rand(rng, *shape):
    return rng.standard_normal(shape)


@pytest.mark.parametrize("C,S,Fc,window_relative", [(3, 1, 2, False), (4, 0, 1, False), (3, 1, 1, True)])
def test_reset_of_one_stream_equals_a_fresh_stream_fed_the_later_frames(C, S, Fc, window_relative):
    """Sec. 3.2: a stream's context is a function of the frames appended since it started.  After
    reset(b, start) stream b must behave exactly like stream b of a NEW oracle that starts at
    `start` and is fed only the frames appended after the reset (outputs, LSE, gradients, tables),
    while the other stream -- which keeps its history -- is untouched by the reset."""
    B, H, D, gh, gw = 2, 2, 16, 2, 3
    pairs = (4, 2, 2)
    T = gh * gw
    rng = np.random.default_rng(7)
    a = RollingCacheOracle(B, H, D, gh, gw, C, S, pairs, 10000.0, [3, 40], window_relative=window_relative)
    frames = [(_rand(rng, B, Fc * T, H, D), _rand(rng, B, Fc * T, H, D)) for _ in range(7)]
    n_before, new_start = 4, 11
    for k, v in frames[:n_before]:          # enough to wrap the ring of both streams
        a.append(k, v, Fc)
    a.reset(1, new_start)
    for k, v in frames[n_before:]:
        a.append(k, v, Fc)
    # stream 1 of `fresh` never saw the early frames; stream 0 of `kept` never saw a reset
    fresh = RollingCacheOracle(B, H, D, gh, gw, C, S, pairs, 10000.0, [3, new_start], window_relative=window_relative)
    for k, v in frames[n_before:]:
        fresh.append_stream(1, k[1], v[1], Fc)
    kept = RollingCacheOracle(B, H, D, gh, gw, C, S, pairs, 10000.0, [3, 40], window_relative=window_relative)
    for k, v in frames:
        kept.append_stream(0, k[0], v[0], Fc)
    q, kc, vc, do = (_rand(rng, B, Fc * T, H, D) for _ in range(4))
    out, lse = a.attn_fwd(q, kc, vc, Fc)
    dq, dk, dv = a.attn_bwd(q, kc, vc, do, Fc)
    for orc, b in ((fresh, 1), (kept, 0)):
        ro, rl = orc.attn_fwd(q, kc, vc, Fc, streams=[b])
        rq, rk, rv = orc.attn_bwd(q, kc, vc, do, Fc, streams=[b])
        for got, ref in ((out, ro), (dq, rq), (dk, rk), (dv, rv)):
            np.testing.assert_allclose(got[b], ref[b], rtol=0, atol=1e-13)
        np.testing.assert_allclose(lse[b], rl[b], rtol=0, atol=1e-13)
        sf, sp, nn = a.table_arrays()
        rf, rp, rn = orc.table_arrays()
        assert sf[b].tolist() == rf[b].tolist() and sp[b].tolist() == rp[b].tolist() and nn[b] == rn[b]
    # and the reset really changed something: without it stream 1 would see other frames at other positions
    never = RollingCacheOracle(B, H, D, gh, gw, C, S, pairs, 10000.0, [3, 40], window_relative=window_relative)
    for k, v in frames:
        never.append(k, v, Fc)
    no, _ = never.attn_fwd(q, kc, vc, Fc, streams=[1])
    assert np.abs(no[1] - out[1]).max() > 1e-3
    # tables of the reset stream count from zero again
    assert a.table_arrays()[2][1] == (len(frames) - n_before) * Fc
    assert a.tables[1].slot_frame()[0] == new_start


def test_reset_of_all_streams():
    B, H, D, gh, gw, C, S = 2, 1, 8, 2, 2, 2, 0
    rng = np.random.default_rng(8)
    a = RollingCacheOracle(B, H, D, gh, gw, C, S, (2, 1, 1), 10000.0, [1, 2])
    for _ in range(3):
        a.append(_rand(rng, B, 4, H, D), _rand(rng, B, 4, H, D), 1)
    a.reset(-1, 9)
    assert a.table_arrays()[2].tolist() == [0, 0] and (a.table_arrays()[0] == -1).all()
    q, k, v = (_rand(rng, B, 4, H, D) for _ in range(3))
    out, _ = a.attn_fwd(q, k, v, 1)
    fresh = RollingCacheOracle(B, H, D, gh, gw, C, S, (2, 1, 1), 10000.0, [9, 9])
    ref, _ = fresh.attn_fwd(q, k, v, 1)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-14)


def test_row_subset_of_the_forward_is_the_full_forward_at_those_rows():
    """A query's output depends on no other query (softmax is per row), so computing a subset of
    the rows must give exactly the rows of the whole result -- also under causal blocks, where the
    visible keys differ from row to row."""
    B, H, D, gh, gw, C, S, Fc = 1, 2, 16, 2, 3, 3, 1, 3
    rng = np.random.default_rng(9)
    for block in (None, 1, 2):
        a = RollingCacheOracle(B, H, D, gh, gw, C, S, (4, 2, 2), 10000.0, [5], block_frames=block)
        for _ in range(4):
            a.append(_rand(rng, B, gh * gw, H, D), _rand(rng, B, gh * gw, H, D), 1)
        q, k, v = (_rand(rng, B, Fc * gh * gw, H, D) for _ in range(3))
        full_o, full_l = a.attn_fwd(q, k, v, Fc)
        rows = np.array([0, 5, 6, 11, 17])
        sub_o, sub_l = a.attn_fwd(q, k, v, Fc, rows=rows)
        np.testing.assert_array_equal(sub_o[:, rows], full_o[:, rows])
        np.testing.assert_array_equal(sub_l[:, :, rows], full_l[:, :, rows])
        others = np.setdiff1d(np.arange(Fc * gh * gw), rows)
        assert np.isnan(sub_o[:, others]).all() and np.isnan(sub_l[:, :, others]).all()
        # the subset's rows do not depend on the other queries' values at all
        q2 = q.copy()
        q2[:, others] = 123.0
        sub2_o, _ = a.attn_fwd(q2, k, v, Fc, rows=rows)
        np.testing.assert_array_equal(sub2_o[:, rows], sub_o[:, rows])


def test_row_subset_of_the_group_forward_is_the_full_group_forward_at_those_rows():
    B, H, D, gh, gw, C, S, Fc, G = 1, 2, 16, 2, 3, 3, 1, 2, 3
    rng = np.random.default_rng(12)
    a = RollingCacheOracle(B, H, D, gh, gw, C, S, (4, 2, 2), 10000.0, [5], block_frames=1)
    for _ in range(4):
        a.append(_rand(rng, B, gh * gw, H, D), _rand(rng, B, gh * gw, H, D), 1)
    q, k, v = (_rand(rng, B * G, Fc * gh * gw, H, D) for _ in range(3))
    full_o, full_l = a.group_attn_fwd(q, k, v, Fc, G)
    rows = np.array([1, 6, 11])
    sub_o, sub_l = a.group_attn_fwd(q, k, v, Fc, G, rows=rows)
    np.testing.assert_array_equal(sub_o[:, rows], full_o[:, rows])
    np.testing.assert_array_equal(sub_l[:, :, rows], full_l[:, :, rows])
    assert np.isnan(sub_o[:, [0, 2, 7]]).all()


def test_round_to_bf16_matches_the_library_conversion_bit_for_bit():
    """Against torch's float32 -> bfloat16 conversion (round to nearest, ties to even) on random
    values, exact ties in both directions, values next to ties, subnormals, the largest finite
    bf16 and the first value that rounds up to infinity."""
    rng = np.random.default_rng(10)
    x = rng.standard_normal(200_000).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 200_000).astype(np.float32)
    def bits(u):
        return np.array(u, dtype=np.uint32).view(np.float32)
    special = bits([
        0x3F808000,  # 1 + 2^-8: tie, even mantissa below -> rounds down to 1
        0x3F818000,  # tie, odd mantissa below -> rounds up
        0x3F807FFF, 0x3F808001, 0xBF808000, 0xBF818000,
        0x00000001, 0x00008000, 0x00018000, 0x007FFFFF, 0x80008000,   # fp32 subnormals around bf16 subnormal ties
        0x7F7F0000,  # largest finite bf16
        0x7F7F7FFF,  # still rounds to it
        0x7F7F8000,  # tie at the top: rounds to +inf
        0x00000000, 0x80000000,
    ])
    x = np.concatenate([x, special])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = round_to_bf16(x.astype(np.float64)).astype(np.float32)
    np.testing.assert_array_equal(got.view(np.uint32), want.view(np.uint32))
    # values that are already bf16 pass unchanged, and rounding is idempotent
    np.testing.assert_array_equal(round_to_bf16(want.astype(np.float64)), want.astype(np.float64))


def test_cache_rounding_switch_rounds_exactly_the_rotated_cached_keys():
    """The diagnostic switch must change one thing only: the rotated keys of the visible HISTORY
    are rounded to bf16 (the library conversion is the reference); cached values, the chunk's own
    keys and the queries stay as they are."""
    B, H, D, gh, gw, C, S = 1, 2, 16, 2, 3, 3, 1
    rng = np.random.default_rng(11)
    plain = RollingCacheOracle(B, H, D, gh, gw, C, S, (4, 2, 2), 10000.0, [4])
    rounded = RollingCacheOracle(B, H, D, gh, gw, C, S, (4, 2, 2), 10000.0, [4], cache_rounding=True)
    for _ in range(5):
        k, v = _rand(rng, B, gh * gw, H, D), _rand(rng, B, gh * gw, H, D)
        plain.append(k, v, 1)
        rounded.append(k, v, 1)
    for h in range(H):
        kp, vp = plain._context(0, h)
        kr, vr = rounded._context(0, h)
        want = torch.from_numpy(kp).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
        np.testing.assert_array_equal(kr, want)
        np.testing.assert_array_equal(vr, vp)
        assert np.abs(kr - kp).max() > 0
    q, k, v = (_rand(rng, B, gh * gw, H, D) for _ in range(3))
    o_p, _ = plain.attn_fwd(q, k, v, 1)
    o_r, _ = rounded.attn_fwd(q, k, v, 1)
    # the effect on the output is of the size of one bf16 rounding of the scores' operands
    d = np.abs(o_p - o_r).max()
    assert 0 < d < 2e-2
