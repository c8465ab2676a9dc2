"""The attention calls under HIP graph capture: forward + backward over a fixed cache are captured
once (inputs, outputs and workspace preallocated; the library allocates nothing and takes the
stream it is given) and replayed with new inputs.  Every replay is compared bit for bit with an
eager call on the same inputs, with eager work and synchronisations between the replays, and one
of them with the oracle.  The append is not captured: it advances host tables."""
import numpy as np
import pytest

import workloads as wl
from helpers import Lockstep, assert_bf16_close, host_f64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("window_relative", [False, True])
def test_forward_and_backward_replayed_from_a_graph_equal_eager_calls(window_relative):
    import torch
    w = wl.Workload("graph_small", 41, 2, 2, 128, 6, 10, 3, 1, 2, 0, (22, 21, 21))
    ls = Lockstep(w, start_frames=[0, 9], window_relative=window_relative)
    A, Fc = ls.A, w.chunk_frames
    for step in range(3):   # 6 frames into a ring of 3: evictions have happened
        _, k, v = wl.chunk_inputs(w, step)
        ls.append(k, v, Fc)
    shape = (w.batch, w.n_q, w.heads, w.head_dim)
    dev = "cuda:0"
    q, k, v, do = (torch.zeros(shape, dtype=torch.bfloat16, device=dev) for _ in range(4))
    out = torch.empty_like(q)
    lse = torch.empty((w.batch, w.heads, w.n_q), dtype=torch.float32, device=dev)
    dq, dk, dv = (torch.empty(shape, dtype=torch.float32, device=dev) for _ in range(3))
    ws = torch.empty(max(A.astro_chunk_attn_workspace_bytes(ls.cache, Fc)), dtype=torch.uint8, device=dev)

    def load(step):
        host = wl.chunk_inputs(w, step, with_dout=True)
        for dst, src in zip((q, k, v, do), host):
            dst.copy_(ls.dev(src))
        return host

    load(10)
    # warm up on a side stream, as capture needs, then capture
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        A.astro_chunk_attn_fwd(ls.cache, q, k, v, Fc, out, lse, ws)
        A.astro_chunk_attn_bwd(ls.cache, q, k, v, out, lse, do, Fc, dq, dk, dv, ws)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        A.astro_chunk_attn_fwd(ls.cache, q, k, v, Fc, out, lse, ws)
        A.astro_chunk_attn_bwd(ls.cache, q, k, v, out, lse, do, Fc, dq, dk, dv, ws)

    rep = []
    for i, step in enumerate((11, 12, 13, 11)):
        host = load(step)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (out, lse, dq, dk, dv)]
        # eager work between the replays: the same calls with buffers of their own
        e_out, e_lse = A.astro_chunk_attn_fwd(ls.cache, q, k, v, Fc)
        e_dq, e_dk, e_dv = A.astro_chunk_attn_bwd(ls.cache, q, k, v, e_out, e_lse, do, Fc)
        torch.cuda.synchronize()
        for name, a, b in zip(("out", "lse", "dq", "dk", "dv"), got, (e_out, e_lse, e_dq, e_dk, e_dv)):
            assert torch.equal(a, b), f"replay {i} (inputs of step {step}): {name} differs from the eager call"
        if i == 1:
            wide = [ls.wide(x) for x in host]
            ro, rl = ls.oracle.attn_fwd(*wide[:3], Fc)
            rq, rk, rv = ls.oracle.attn_bwd(*wide, Fc)
            for name, a, b in zip(("out", "lse", "dq", "dk", "dv"), got, (ro, rl, rq, rk, rv)):
                assert_bf16_close(host_f64(a), b, f"replay {i} {name} vs oracle", rep)
    ls.close()
