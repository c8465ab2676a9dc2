"""CPU tests of the C-ABI library: it loads, exports every declared symbol,
rejects bad arguments without changing state, and its host slot tables follow
the naive ring simulation of the oracle (Sec. 3.2).  No GPU, no compute calls."""
import ctypes
import os
import re

import pytest

import paper_2603_17051_amd as A
from paper_2603_17051_amd import binding
from oracle import RingTableSim


def test_library_exports_every_symbol_the_header_declares(repo_root):
    header = open(os.path.join(repo_root, "include", "astro.h")).read()
    declared = set(re.findall(r"\b(astro_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTED)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_error_codes_have_text():
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert isinstance(A.astro_strerror(code), str) and A.astro_strerror(code)


def test_cache_bytes():
    d = A.make_desc(2, 12, 128, 30, 52, 18, 0, 3, (22, 21, 21))
    kb, vb = A.astro_kvcache_bytes(d)
    assert kb == vb == 2 * 12 * 18 * 1560 * 128 * 2
    d = A.make_desc(1, 2, 64, 8, 8, 4, 0, 1, (12, 10, 10), dtype=A.ASTRO_F32)
    assert A.astro_kvcache_bytes(d)[0] == 2 * 4 * 64 * 64 * 4


GOOD = dict(batch=1, heads=2, head_dim=64, grid_h=8, grid_w=8, capacity_frames=4, sink_frames=1,
            max_chunk_frames=2, rope_pairs=(12, 10, 10))


@pytest.mark.parametrize("change,code", [
    (dict(batch=0), A.binding.ASTRO_ERR_INVALID_ARG),
    (dict(batch=65), A.binding.ASTRO_ERR_INVALID_ARG),
    (dict(heads=0), A.binding.ASTRO_ERR_INVALID_ARG),
    (dict(head_dim=96), A.binding.ASTRO_ERR_UNSUPPORTED),
    (dict(grid_h=0), A.binding.ASTRO_ERR_INVALID_ARG),
    (dict(capacity_frames=0), A.binding.ASTRO_ERR_INVALID_ARG),
    (dict(capacity_frames=257), A.binding.ASTRO_ERR_INVALID_ARG),
    (dict(sink_frames=4), A.binding.ASTRO_ERR_INVALID_ARG),
    (dict(sink_frames=-1), A.binding.ASTRO_ERR_INVALID_ARG),
    (dict(max_chunk_frames=0), A.binding.ASTRO_ERR_INVALID_ARG),
    (dict(max_chunk_frames=4), A.binding.ASTRO_ERR_INVALID_ARG),  # > window of 3
    (dict(rope_pairs=(12, 10, 9)), A.binding.ASTRO_ERR_INVALID_ARG),
    (dict(rope_pairs=(-1, 23, 10)), A.binding.ASTRO_ERR_INVALID_ARG),
    (dict(rope_base=1.0), A.binding.ASTRO_ERR_INVALID_ARG),
    (dict(dtype=7), A.binding.ASTRO_ERR_UNSUPPORTED),
    (dict(block_frames=-1), A.binding.ASTRO_ERR_INVALID_ARG),
])
def test_create_rejects_bad_descriptors(change, code):
    args = dict(GOOD)
    args.update(change)
    with pytest.raises(A.AstroError) as e:
        A.astro_kvcache_create(host_only=True, **args)
    assert e.value.code == code


def test_any_non_negative_causal_block_size_is_accepted():
    for bf in (0, 1, 2, 100):
        A.astro_kvcache_create(host_only=True, block_frames=bf, **GOOD).close()


def test_create_needs_storage_unless_host_only():
    d = A.make_desc(1, 2, 64, 8, 8, 4, 1, 2, (12, 10, 10))
    h = ctypes.c_void_p(None)
    assert binding.library().astro_kvcache_create(ctypes.byref(d), ctypes.byref(h)) == binding.ASTRO_ERR_INVALID_ARG
    assert h.value is None
    assert binding.library().astro_kvcache_create(None, ctypes.byref(h)) == binding.ASTRO_ERR_INVALID_ARG
    assert binding.library().astro_kvcache_create(ctypes.byref(d), None) == binding.ASTRO_ERR_INVALID_ARG


def test_null_handles_are_rejected():
    lib = binding.library()
    assert lib.astro_kvcache_destroy(None) == binding.ASTRO_ERR_INVALID_ARG
    assert lib.astro_kvcache_reset(None, 0, 0) == binding.ASTRO_ERR_INVALID_ARG
    assert lib.astro_kvcache_append(None, None, None, 1, None) == binding.ASTRO_ERR_INVALID_ARG
    assert lib.astro_kvcache_tables(None, None, None, None) == binding.ASTRO_ERR_INVALID_ARG
    assert lib.astro_chunk_attn_workspace_bytes(None, 1, None, None) == binding.ASTRO_ERR_INVALID_ARG
    assert lib.astro_chunk_attn_fwd(None, None, None, None, 1, None, None, None, 0, None) == binding.ASTRO_ERR_INVALID_ARG
    assert lib.astro_chunk_attn_bwd(None, None, None, None, None, None, None, 1, None, None, None, None, 0,
                                    None) == binding.ASTRO_ERR_INVALID_ARG


def test_errors_leave_state_unchanged_and_host_only_handles_refuse_compute():
    c = A.astro_kvcache_create(host_only=True, **GOOD)
    A.astro_kvcache_append(c, n_frames=2)
    before = A.astro_kvcache_tables(c)
    lib = binding.library()
    assert lib.astro_kvcache_append(c.handle, None, None, 0, None) == binding.ASTRO_ERR_INVALID_ARG
    assert lib.astro_kvcache_append(c.handle, None, None, 3, None) == binding.ASTRO_ERR_INVALID_ARG  # > max chunk
    assert lib.astro_kvcache_reset(c.handle, 1, 0) == binding.ASTRO_ERR_INVALID_ARG  # no such stream
    assert lib.astro_kvcache_reset(c.handle, 0, -5) == binding.ASTRO_ERR_INVALID_ARG
    assert lib.astro_chunk_attn_fwd(c.handle, None, None, None, 1, None, None, None, 0, None) == binding.ASTRO_ERR_BAD_STATE
    assert A.astro_kvcache_tables(c) == before
    # frame indices must stay in int32
    A.astro_kvcache_reset(c, 0, 2**31 - 2)
    assert lib.astro_kvcache_append(c.handle, None, None, 2, None) == binding.ASTRO_ERR_BAD_STATE
    assert A.astro_kvcache_tables(c)[2] == [0]
    c.close()


def test_workspace_sizes_are_reported():
    c = A.astro_kvcache_create(host_only=True, **GOOD)
    f, b = A.astro_chunk_attn_workspace_bytes(c, 2)
    rot = 1 * 2 * 2 * 64 * 64 * 2  # B*H*Nq*D*2 bytes
    tab = 256                      # (cos, sin) of the temporal pairs per chunk frame: 2 * 12 * 8 bytes, 256-aligned
    # rotated Q and K_chunk and the temporal table, plus -- for a shape that cannot fill the chip --
    # room for the results of up to 8 key-range splits (bf16 output rows and fp32 log-sum-exps)
    assert f == 2 * rot + tab + 8 * (1 * 2 * 2 * 64) * (64 * 2 + 4)
    # backward: the row terms (Delta, LSE*log2e) instead; the bf16 kernels write the gradients
    # un-rotated themselves, so no rotated fp32 copies
    assert b == 2 * rot + tab + 2 * (1 * 2 * 2 * 64) * 4
    with pytest.raises(A.AstroError):
        A.astro_chunk_attn_workspace_bytes(c, 3)
    c.close()


def test_group_workspace_scales_with_the_group_and_bad_groups_are_rejected():
    c = A.astro_kvcache_create(host_only=True, **GOOD)
    f1, b1 = A.astro_chunk_attn_workspace_bytes(c, 2)
    assert A.astro_group_attn_workspace_bytes(c, 2, 1) == (f1, b1)
    f4, b4 = A.astro_group_attn_workspace_bytes(c, 2, 4)
    assert f4 >= 4 * (f1 - 256) and b4 >= 4 * (b1 - 1024)
    # enough work for two rounds of workgroups on 256 CUs: no split, so no room for its results
    big = A.astro_kvcache_create(host_only=True, **dict(GOOD, batch=64, heads=32, grid_h=32, grid_w=32, head_dim=128, rope_pairs=(22, 21, 21)))
    assert A.astro_chunk_attn_workspace_bytes(big, 1)[0] == 2 * 64 * 32 * 1024 * 128 * 2 + 64 * 1 * 22 * 8
    big.close()
    for bad in (0, -1, binding.ASTRO_MAX_BATCH + 1):
        with pytest.raises(A.AstroError) as e:
            A.astro_group_attn_workspace_bytes(c, 2, bad)
        assert e.value.code == binding.ASTRO_ERR_INVALID_ARG
    # a host-only handle refuses the compute call itself
    lib = binding.library()
    assert lib.astro_group_attn_fwd(c.handle, None, None, None, 2, 2, None, None, None, 0, None) == binding.ASTRO_ERR_BAD_STATE
    c.close()


def test_window_relative_flag_sink_storage_and_unknown_flags():
    lib = binding.library()
    # sizes: un-rotated keys of the S sink frames, only when the sinks can move
    d = A.make_desc(2, 12, 128, 30, 52, 12, 1, 3, (22, 21, 21), flags=binding.ASTRO_FLAG_WINDOW_RELATIVE)
    assert A.binding.astro_kvcache_sink_bytes(d) == 2 * 1 * 1560 * 12 * 128 * 2
    for desc in (A.make_desc(2, 12, 128, 30, 52, 12, 1, 3, (22, 21, 21)),                                    # flag off
                 A.make_desc(2, 12, 128, 30, 52, 12, 0, 3, (22, 21, 21), flags=binding.ASTRO_FLAG_WINDOW_RELATIVE),  # no sinks
                 A.make_desc(2, 12, 128, 30, 52, 12, 1, 3, (0, 32, 32), flags=binding.ASTRO_FLAG_WINDOW_RELATIVE),   # no frame pairs
                 A.make_desc(2, 12, 128, 30, 52, 12, 1, 3, (0, 0, 0), flags=binding.ASTRO_FLAG_WINDOW_RELATIVE)):
        assert A.binding.astro_kvcache_sink_bytes(desc) == 0
    assert lib.astro_kvcache_sink_bytes(None, None) == binding.ASTRO_ERR_INVALID_ARG
    # a device handle whose sinks move needs the sink storage (fake, never dereferenced pointers: creation
    # is refused before anything touches the device)
    d.k_storage = d.v_storage = ctypes.c_void_p(256)
    h = ctypes.c_void_p(None)
    assert lib.astro_kvcache_create(ctypes.byref(d), ctypes.byref(h)) == binding.ASTRO_ERR_INVALID_ARG
    assert h.value is None
    d.flags = 8
    assert lib.astro_kvcache_sink_bytes(ctypes.byref(d), ctypes.byref(ctypes.c_size_t(0))) == binding.ASTRO_ERR_INVALID_ARG


@pytest.mark.parametrize("C,S,Fc,start", [(1, 0, 1, 0), (4, 0, 1, 0), (4, 1, 3, 7), (12, 1, 3, 0), (18, 0, 3, 41),
                                          (21, 3, 3, 0), (5, 4, 1, 2), (7, 2, 5, 1000), (256, 3, 11, 5)])
@pytest.mark.parametrize("window_relative", [False, True])
def test_tables_follow_the_naive_ring_simulation(C, S, Fc, start, window_relative):
    B = 3
    c = A.astro_kvcache_create(B, 1, 64, 2, 2, C, S, Fc, host_only=True, window_relative=window_relative)
    starts = [start + 10 * b for b in range(B)]
    sims = [RingTableSim(C, S, s) for s in starts]
    for b, s in enumerate(starts):
        A.astro_kvcache_reset(c, b, s)
    steps = 0
    n = 0
    while n < 3 * C + 2 * Fc and steps < 400:
        k = 1 + (steps * 7) % Fc
        A.astro_kvcache_append(c, n_frames=k)
        for sim in sims:
            for _ in range(k):
                sim.append_frame()
        sf, sp, nn = A.astro_kvcache_tables(c)
        assert sf == [sim.slot_frame() for sim in sims]
        assert sp == [sim.slot_pos(window_relative) for sim in sims]
        assert nn == [sim.next_n for sim in sims]
        n += k
        steps += 1
    # reset of one stream leaves the others alone
    A.astro_kvcache_reset(c, 1, 5)
    sf, _, nn = A.astro_kvcache_tables(c)
    assert sf[1] == [-1] * C and nn[1] == 0
    assert sf[0] == sims[0].slot_frame() and sf[2] == sims[2].slot_frame()
    c.close()
