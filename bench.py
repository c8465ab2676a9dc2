#!/usr/bin/env python3
"""Benchmark of the rolling-cache chunk-attention hot path on one MI355X.

A step = one pass of the whole hot path over one batch of synthetic input:
chunk attention forward over the resident ring + the chunk, backward with the
cached context detached, then the KV append of the chunk (rotary fused, ring
eviction).  Inputs are resident in HBM before the timed region.  Prints ONE
JSON line (metric, roofline of the dominant kernel, oracle timed on the host).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E peak


def flops_fwd(w) -> float:
    """4*Nq*Nk*D*H*B: the QK^T and PV contractions."""
    return 4.0 * w.n_q * w.n_k * w.head_dim * w.heads * w.batch


def flops_bwd(w) -> float:
    """(6*Nq*Nk_cache + 10*Nq*Nq)*D*H*B: dP, dQ (+ S recompute counted once) over the
    cached keys, all five contractions over the chunk's own keys; rotary, the second
    S/dP recompute on chunk columns and staging are not counted."""
    nk_cache = w.n_k - w.n_q
    return (6.0 * w.n_q * nk_cache + 10.0 * w.n_q * w.n_q) * w.head_dim * w.heads * w.batch


def append_bytes(w) -> float:
    """read K, V + write K, V of the chunk (bf16); eviction moves nothing."""
    return 4.0 * w.n_q * w.heads * w.head_dim * 2 * w.batch


# algorithmic flops of one launch of each attention kernel
def kernel_flops(name: str, w) -> float:
    per = w.head_dim * w.heads * w.batch
    if name == "attn_fwd_bf16":
        return flops_fwd(w)
    if name == "attn_bwd_dq_bf16":      # S, dP, dQ over all visible keys
        return 6.0 * w.n_q * w.n_k * per
    if name == "attn_bwd_dkv_bf16":     # dK, dV over the chunk's keys (its S/dP recompute not counted)
        return 4.0 * w.n_q * w.n_q * per
    return 0.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="rl_bwd")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-full", action="store_true",
                    help="time the oracle on the WHOLE step (every stream and head) instead of the bounded sample")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--no-calibration", action="store_true")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for counter runs (rocprofv3 --pmc): one calibration copy of 1 GiB, then three forwards over 8 "
                         "independent caches, then three forwards of 8 candidates over ONE shared cache, and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (streams and heads shard "
              "without any exchange between GPUs)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2603_17051_amd as A
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = wl.WORKLOADS[args.workload]

    def dev_bf16(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)

    def make_cache(w, block_frames=0, reuse_staged=False):
        cache = A.astro_kvcache_create(w.batch, w.heads, w.head_dim, w.grid_h, w.grid_w, w.capacity_frames,
                                       w.sink_frames, w.chunk_frames, w.rope_pairs, w.rope_base,
                                       block_frames=block_frames, reuse_staged=reuse_staged)
        pk, pv = wl.history_frame_pool(w, 4)
        dk, dv = dev_bf16(pk), dev_bf16(pv)
        for n in range(min(w.resident_frames, w.capacity_frames)):
            idx = torch.tensor([wl.pool_index(b, n, 4) for b in range(w.batch)], device=dev)
            A.astro_kvcache_append(cache, dk.index_select(0, idx).contiguous(), dv.index_select(0, idx).contiguous(), 1)
        return cache

    if args.traffic_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).zero_()
        dst = torch.empty_like(src)
        A.astro_calib_copy(src, dst)
        del src, dst
        for name, G in (("group_fwd_append", 1), ("shared_prefix", 8)):
            we = wl.WORKLOADS[name]
            ce = make_cache(we)
            qe, ke, ve = (dev_bf16(x) for x in (wl.chunk_inputs(we) if G == 1 else wl.group_inputs(we, G)))
            oe = torch.empty_like(qe)
            le = torch.empty((we.batch * G, we.heads, we.n_q), dtype=torch.float32, device=dev)
            wse = torch.empty(A.astro_group_attn_workspace_bytes(ce, we.chunk_frames, G)[0], dtype=torch.uint8, device=dev)
            for _ in range(3):
                A.astro_group_attn_fwd(ce, qe, ke, ve, we.chunk_frames, G, oe, le, wse)
            torch.cuda.synchronize()
            ce.close()
        print(json.dumps({"traffic_probe": "calib_copy x1, attn_fwd x3 over 8 independent caches, attn_fwd x3 of 8 candidates over one cache"}))
        return 0

    # ---- main workload: fwd + bwd + append ---------------------------------------
    # The handle may reuse what a forward staged when the backward that follows it gets the same
    # chunk and workspace (the re-forward + backward of gradient checkpointing).  Each step works
    # on one of three distinct input sets (3 x 460 MB), so neither the attention kernels nor the
    # append find their sources in the 256 MB last-level cache from the step before.
    cache = make_cache(w, reuse_staged=True)
    n_sets = 3
    sets = [tuple(dev_bf16(x) for x in wl.chunk_inputs(w, step=s, with_dout=True)) for s in range(n_sets)]
    q = sets[0][0]
    out = torch.empty_like(q)
    lse = torch.empty((w.batch, w.heads, w.n_q), dtype=torch.float32, device=dev)
    dq, dk_, dv_ = (torch.empty(q.shape, dtype=torch.float32, device=dev) for _ in range(3))
    fwd_b, bwd_b = A.astro_chunk_attn_workspace_bytes(cache, w.chunk_frames)
    ws = torch.empty(max(fwd_b, bwd_b), dtype=torch.uint8, device=dev)
    Fc = w.chunk_frames

    def step(i):
        q, k, v, do = sets[i % n_sets]
        A.astro_chunk_attn_fwd(cache, q, k, v, Fc, out, lse, ws)
        A.astro_chunk_attn_bwd(cache, q, k, v, out, lse, do, Fc, dq, dk_, dv_, ws)
        A.astro_kvcache_append(cache, k, v, Fc)

    for i in range(args.warmup):
        step(i)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step(args.warmup + i)
        marks[i + 1].record()   # on the stream the library launches on (torch's current stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    per_step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    median_ms = per_step_ms[len(per_step_ms) // 2] if args.steps % 2 else 0.5 * (per_step_ms[args.steps // 2 - 1] + per_step_ms[args.steps // 2])
    step_flops = flops_fwd(w) + flops_bwd(w)
    value = step_flops / (ms_per_step * 1e-3) / 1e12

    # ---- per-kernel HIP-event timing over the same step (separate pass) ------------
    A.astro_profile_begin()
    for i in range(args.steps):
        step(i)
    ktimes = A.astro_profile_end()
    kernels = {}
    for name, (launches, total_ms) in ktimes.items():
        avg = total_ms / launches
        ent = {"launches": launches, "avg_ms": round(avg, 4)}
        fl = kernel_flops(name, w)
        if fl:
            ent["tflops"] = round(fl / (avg * 1e-3) / 1e12, 1)
            ent["frac_bf16_mfma_peak"] = round(fl / (avg * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4)
        if name == "kv_append_rope":
            ent["gbs"] = round(append_bytes(w) / (avg * 1e-3) / 1e9, 1)
            ent["frac_hbm_peak"] = round(append_bytes(w) / (avg * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
        kernels[name] = ent
    dominant = max((n for n in ktimes if kernel_flops(n, w)), key=lambda n: ktimes[n][1])
    d_avg = ktimes[dominant][1] / ktimes[dominant][0]
    achieved = kernel_flops(dominant, w) / (d_avg * 1e-3) / 1e12
    # HBM bytes per launch of that kernel: NOT measured by this run (counters need rocprofv3); taken
    # from the committed summary of the rocprofv3 --pmc runs of this command, and labelled as such
    traffic, traffic_source = None, None
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic_rl_bwd.json")) as f:
            prof = json.load(f)
        ent = prof["kernels"].get(dominant) if args.workload == "rl_bwd" else None
        if ent:
            traffic = ent["fetch_bytes"] + ent["write_bytes"]
            traffic_source = "profiles/hbm_traffic_rl_bwd.json: " + prof.get("source", "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs")
    except (OSError, ValueError, KeyError):
        pass
    roofline = {"kernel": dominant, "bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_BF16_MFMA_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_MFMA_TFLOPS, 4), "traffic": traffic,
                "traffic_source": traffic_source, "avg_launch_ms": round(d_avg, 4)}

    result = {
        "metric": "chunk-attn fwd+bwd TFLOP/s (algorithmic flops, bf16 MFMA, fp32 accumulate)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "median_ms_per_step": round(median_ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: B{w.batch} H{w.heads} D{w.head_dim} T{w.tokens_per_frame} "
                               f"ring {w.capacity_frames} frames full, chunk {w.chunk_frames} frames "
                               f"(Nq={w.n_q}, Nk={w.n_k}); step = attn fwd + bwd (cache detached; it reuses the rotated Q / K_chunk "
                               f"its forward staged, ASTRO_FLAG_REUSE_STAGED) + KV append; {n_sets} input sets in rotation",
                   "flops_per_step": step_flops, "frac_bf16_mfma_peak": round(value / PEAK_BF16_MFMA_TFLOPS, 4)},
        "roofline": roofline,
        "kernels": kernels,
    }
    cache.close()
    del q, sets, out, lse, dq, dk_, dv_, ws

    # ---- extras: forward-only shapes and the append at batch 8 ----------------------
    if not args.no_extras:
        extras = {}
        for name in ("prod_fwd", "group_fwd_append"):
            we = wl.WORKLOADS[name]
            ce = make_cache(we)
            qe, ke, ve = (dev_bf16(x) for x in wl.chunk_inputs(we))
            oe = torch.empty_like(qe)
            le = torch.empty((we.batch, we.heads, we.n_q), dtype=torch.float32, device=dev)
            wse = torch.empty(A.astro_chunk_attn_workspace_bytes(ce, we.chunk_frames)[0], dtype=torch.uint8, device=dev)
            for _ in range(3):
                A.astro_chunk_attn_fwd(ce, qe, ke, ve, we.chunk_frames, oe, le, wse)
            torch.cuda.synchronize()
            n = 20
            t0 = time.perf_counter()
            for _ in range(n):
                A.astro_chunk_attn_fwd(ce, qe, ke, ve, we.chunk_frames, oe, le, wse)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / n
            ent = {"fwd_ms": round(ms, 4), "fwd_tflops": round(flops_fwd(we) / (ms * 1e-3) / 1e12, 1),
                   "frac_bf16_mfma_peak": round(flops_fwd(we) / (ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4)}
            if name == "group_fwd_append":
                # rotate over distinct source buffers (> 256 MB in flight) so the append is not cache resident
                srcs = [(dev_bf16(a), dev_bf16(b)) for a, b in
                        (wl.chunk_inputs(we, step=s)[1:3] for s in range(1, 4))]
                for i in range(3):
                    A.astro_kvcache_append(ce, srcs[i % 3][0], srcs[i % 3][1], we.chunk_frames)
                A.astro_profile_begin()
                for i in range(18):
                    A.astro_kvcache_append(ce, srcs[i % 3][0], srcs[i % 3][1], we.chunk_frames)
                la, tot = A.astro_profile_end()["kv_append_rope"]
                ent["append_ms"] = round(tot / la, 4)
                ent["append_gbs"] = round(append_bytes(we) / (tot / la * 1e-3) / 1e9, 1)
                ent["append_frac_hbm_peak"] = round(ent["append_gbs"] / PEAK_HBM_GBS, 4)
                del srcs
            extras[name] = ent
            ce.close()
            del qe, ke, ve, oe, le, wse
        # the batch-1 forward with frame-by-frame causality inside the chunk: 444 workgroups, split over the keys
        we = wl.WORKLOADS["prod_fwd"]
        ce = make_cache(we, block_frames=1)
        qe, ke, ve = (dev_bf16(x) for x in wl.chunk_inputs(we))
        oe = torch.empty_like(qe)
        le = torch.empty((we.batch, we.heads, we.n_q), dtype=torch.float32, device=dev)
        wse = torch.empty(A.astro_chunk_attn_workspace_bytes(ce, we.chunk_frames)[0], dtype=torch.uint8, device=dev)
        for _ in range(3):
            A.astro_chunk_attn_fwd(ce, qe, ke, ve, we.chunk_frames, oe, le, wse)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(20):
            A.astro_chunk_attn_fwd(ce, qe, ke, ve, we.chunk_frames, oe, le, wse)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / 20
        T_, Fc_ = we.tokens_per_frame, we.chunk_frames
        fl = 4.0 * (we.n_q * (we.n_k - we.n_q) + T_ * T_ * Fc_ * (Fc_ + 1) / 2.0) * we.head_dim * we.heads * we.batch
        extras["prod_fwd_frame_causal"] = {"fwd_ms": round(ms, 4), "fwd_tflops": round(fl / (ms * 1e-3) / 1e12, 1),
                                           "frac_bf16_mfma_peak": round(fl / (ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4)}
        ce.close()
        del qe, ke, ve, oe, le, wse
        # group-wise candidates over one shared, frozen cache (8 candidate chunks, one stream)
        we, G = wl.WORKLOADS["shared_prefix"], 8
        ce = make_cache(we)
        qe, ke, ve, de = (dev_bf16(x) for x in wl.group_inputs(we, G, with_dout=True))
        oe = torch.empty_like(qe)
        le = torch.empty((we.batch * G, we.heads, we.n_q), dtype=torch.float32, device=dev)
        gq, gk, gv = (torch.empty(qe.shape, dtype=torch.float32, device=dev) for _ in range(3))
        wse = torch.empty(max(A.astro_group_attn_workspace_bytes(ce, we.chunk_frames, G)), dtype=torch.uint8, device=dev)

        def group_step():
            A.astro_group_attn_fwd(ce, qe, ke, ve, we.chunk_frames, G, oe, le, wse)
            A.astro_group_attn_bwd(ce, qe, ke, ve, oe, le, de, we.chunk_frames, G, gq, gk, gv, wse)

        for _ in range(2):
            group_step()
        torch.cuda.synchronize()
        n = 10
        t0 = time.perf_counter()
        for _ in range(n):
            group_step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / n
        fl = G * (flops_fwd(we) + flops_bwd(we))
        A.astro_profile_begin()
        group_step()
        kt = A.astro_profile_end()
        fwd_ms = kt["attn_fwd_bf16"][1] / kt["attn_fwd_bf16"][0]
        extras["shared_prefix_group8"] = {
            "fwd_bwd_ms": round(ms, 4), "fwd_bwd_tflops": round(fl / (ms * 1e-3) / 1e12, 1),
            "frac_bf16_mfma_peak": round(fl / (ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4),
            "fwd_kernel_ms": round(fwd_ms, 4), "fwd_kernel_tflops": round(G * flops_fwd(we) / (fwd_ms * 1e-3) / 1e12, 1)}
        ce.close()
        del qe, ke, ve, de, oe, le, gq, gk, gv, wse
        # backward with and without the detach (the paper's "Clip + Full BP" comparison point), config-5 shape
        we = wl.WORKLOADS["rl_bwd"]
        ce = make_cache(we)
        qe, ke, ve, de = (dev_bf16(x) for x in wl.chunk_inputs(we, with_dout=True))
        oe, le = A.astro_chunk_attn_fwd(ce, qe, ke, ve, we.chunk_frames)
        g3 = [torch.empty(qe.shape, dtype=torch.float32, device=dev) for _ in range(3)]
        ring_shape = (we.batch, we.capacity_frames * we.tokens_per_frame, we.heads, we.head_dim)
        gk, gv = (torch.zeros(ring_shape, dtype=torch.float32, device=dev) for _ in range(2))
        wsf = torch.empty(A.astro_chunk_attn_bwd_full_workspace_bytes(ce, we.chunk_frames), dtype=torch.uint8, device=dev)
        times = {}
        for label, fn in (("detached", lambda: A.astro_chunk_attn_bwd(ce, qe, ke, ve, oe, le, de, we.chunk_frames, *g3, wsf)),
                          ("full", lambda: A.astro_chunk_attn_bwd_full(ce, qe, ke, ve, oe, le, de, we.chunk_frames, *g3, gk, gv, wsf))):
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(10):
                fn()
            torch.cuda.synchronize()
            times[label] = (time.perf_counter() - t0) * 1e3 / 10
        full_flops = 10.0 * we.n_q * we.n_k * we.head_dim * we.heads * we.batch  # all five products over all keys
        extras["backward_detached_vs_full"] = {
            "detached_ms": round(times["detached"], 4), "full_ms": round(times["full"], 4),
            "detached_tflops": round(flops_bwd(we) / (times["detached"] * 1e-3) / 1e12, 1),
            "full_tflops": round(full_flops / (times["full"] * 1e-3) / 1e12, 1),
            "full_over_detached_time": round(times["full"] / times["detached"], 3),
            "extra_gradient_bytes": int(2 * np.prod(ring_shape) * 4)}
        ce.close()
        del qe, ke, ve, de, oe, le, g3, gk, gv, wsf
        # frame-by-frame causality inside the chunk (block_frames = 1), config-5 shape: a query sees the
        # chunk keys of its own and earlier frames, T*T*Fc*(Fc+1)/2 of the Nq*Nq chunk pairs
        ce = make_cache(we, block_frames=1)
        qe, ke, ve, de = (dev_bf16(x) for x in wl.chunk_inputs(we, with_dout=True))
        oe = torch.empty_like(qe)
        le = torch.empty((we.batch, we.heads, we.n_q), dtype=torch.float32, device=dev)
        g3 = [torch.empty(qe.shape, dtype=torch.float32, device=dev) for _ in range(3)]
        wse = torch.empty(max(A.astro_chunk_attn_workspace_bytes(ce, we.chunk_frames)), dtype=torch.uint8, device=dev)

        def causal_step():
            A.astro_chunk_attn_fwd(ce, qe, ke, ve, we.chunk_frames, oe, le, wse)
            A.astro_chunk_attn_bwd(ce, qe, ke, ve, oe, le, de, we.chunk_frames, *g3, wse)

        for _ in range(2):
            causal_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            causal_step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / 10
        A.astro_profile_begin()
        for _ in range(5):
            causal_step()
        kt = {n: t / l for n, (l, t) in A.astro_profile_end().items()}
        T_, Fc_ = we.tokens_per_frame, we.chunk_frames
        pairs = T_ * T_ * Fc_ * (Fc_ + 1) / 2.0
        per = we.head_dim * we.heads * we.batch
        fl = ((4.0 + 6.0) * we.n_q * (we.n_k - we.n_q) + (4.0 + 10.0) * pairs) * per
        extras["frame_causal_fwd_bwd"] = {
            "fwd_bwd_ms": round(ms, 4), "fwd_bwd_tflops": round(fl / (ms * 1e-3) / 1e12, 1),
            "frac_bf16_mfma_peak": round(fl / (ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4),
            "fwd_kernel_ms": round(kt["attn_fwd_bf16"], 4), "dq_kernel_ms": round(kt["attn_bwd_dq_bf16"], 4),
            "dkv_kernel_ms": round(kt["attn_bwd_dkv_bf16"], 4)}
        ce.close()
        del qe, ke, ve, de, oe, le, g3, wse
        # window-relative temporal positions at the long-streaming shape (ring of 12 = 1 sink + 11, batch 1):
        # every evicting append also rotates the sink's keys again (2 x 4.8 MB); forward on the same cache
        we = wl.WORKLOADS["stream_evict"]
        ce = A.astro_kvcache_create(we.batch, we.heads, we.head_dim, we.grid_h, we.grid_w, we.capacity_frames,
                                    we.sink_frames, we.chunk_frames, we.rope_pairs, we.rope_base, window_relative=True)
        srcs = [tuple(dev_bf16(x) for x in wl.chunk_inputs(we, step=s)) for s in range(3)]
        for i in range(6):   # fills the ring and starts evicting
            A.astro_kvcache_append(ce, srcs[i % 3][1], srcs[i % 3][2], we.chunk_frames)
        oe = torch.empty_like(srcs[0][0])
        le = torch.empty((we.batch, we.heads, we.n_q), dtype=torch.float32, device=dev)
        wse = torch.empty(A.astro_chunk_attn_workspace_bytes(ce, we.chunk_frames)[0], dtype=torch.uint8, device=dev)
        A.astro_profile_begin()
        for i in range(12):
            qe, ke, ve = srcs[i % 3]
            A.astro_chunk_attn_fwd(ce, qe, ke, ve, we.chunk_frames, oe, le, wse)
            A.astro_kvcache_append(ce, ke, ve, we.chunk_frames)
        kt = {k_: t / n_ for k_, (n_, t) in A.astro_profile_end().items()}
        sink_bytes = 2 * we.batch * we.sink_frames * we.tokens_per_frame * we.heads * we.head_dim * 2
        extras["window_relative_stream"] = {
            "fwd_kernel_ms": round(kt["attn_fwd_bf16"], 4), "append_ms": round(kt["kv_append_rope"], 4),
            "sink_rerotate_ms": round(kt["sink_rerotate"], 4),
            "sink_rerotate_gbs": round(sink_bytes / (kt["sink_rerotate"] * 1e-3) / 1e9, 1)}
        ce.close()
        del srcs, oe, le, wse
        # smallest shape (config 1: one 64-token frame over a ring of 4), forward + backward: eager calls against one HIP graph replay
        we = wl.WORKLOADS["tiny_fwd"]
        ce = make_cache(we)
        qe, ke, ve, de = (dev_bf16(x) for x in wl.chunk_inputs(we, with_dout=True))
        oe = torch.empty_like(qe)
        le = torch.empty((we.batch, we.heads, we.n_q), dtype=torch.float32, device=dev)
        g3 = [torch.empty(qe.shape, dtype=torch.float32, device=dev) for _ in range(3)]
        wse = torch.empty(max(A.astro_chunk_attn_workspace_bytes(ce, we.chunk_frames)), dtype=torch.uint8, device=dev)

        def tiny_step():
            A.astro_chunk_attn_fwd(ce, qe, ke, ve, we.chunk_frames, oe, le, wse)
            A.astro_chunk_attn_bwd(ce, qe, ke, ve, oe, le, de, we.chunk_frames, *g3, wse)

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            tiny_step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            tiny_step()
        times = {}
        for label, fn in (("eager", tiny_step), ("graph", graph.replay)):
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
            n = 200
            t0 = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            times[label] = (time.perf_counter() - t0) * 1e6 / n
        extras["tiny_fwd_bwd_graph"] = {"eager_us": round(times["eager"], 1), "graph_replay_us": round(times["graph"], 1)}
        del graph
        ce.close()
        del qe, ke, ve, de, oe, le, g3, wse
        # fused clip-level loss: 24 (one group) and 192 candidate clips of 3 latent frames 16 x 60 x 104, bf16
        for n_clips in (24, 192):
            shape = (n_clips, 3 * 16 * 60 * 104)
            vs = [torch.randn(shape, device=dev, dtype=torch.float32).to(torch.bfloat16) for _ in range(4)]
            adv = torch.randn(n_clips, device=dev)
            msk = (torch.arange(n_clips, device=dev) % 5 == 0).to(torch.int32)
            l3 = torch.empty(3, device=dev)
            gr = torch.empty(shape, dtype=torch.float32, device=dev)
            wsn = torch.empty(A.astro_nft_loss_workspace_bytes(*shape), dtype=torch.uint8, device=dev)
            for _ in range(3):
                A.astro_nft_loss(*vs, adv, msk, 1.0, 1.0, 0.1, l3, gr, wsn)
            A.astro_profile_begin()
            for _ in range(20):
                A.astro_nft_loss(*vs, adv, msk, 1.0, 1.0, 0.1, l3, gr, wsn)
            la, tot = A.astro_profile_end()["nft_loss"]
            nbytes = shape[0] * shape[1] * (4 * 2 + 4)  # four bf16 tensors read, fp32 gradient written
            extras[f"nft_loss_{n_clips}_clips"] = {"ms": round(tot / la, 4), "gbs": round(nbytes / (tot / la * 1e-3) / 1e9, 1),
                                                  "frac_hbm_peak": round(nbytes / (tot / la * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
            del vs, gr, wsn
        result["extras"] = extras

    # ---- what the chip sustains on MFMAs alone and on a plain copy (context for the peaks) -----
    if not args.no_calibration:
        wgs, iters = 512, 4000
        sink = torch.empty(wgs * 256, dtype=torch.float32, device=dev)
        calib = {}
        for label, ops in (("normal", dev_bf16(wl.normal_bf16(wl.BASE_SEED, 99, (8 * 256 * 8,)))),
                           ("zeros", torch.zeros(8 * 256 * 8, dtype=torch.bfloat16, device=dev))):
            A.astro_calib_mfma(ops, wgs, iters, sink)
            A.astro_profile_begin()
            for _ in range(3):
                A.astro_calib_mfma(ops, wgs, iters, sink)
            la, tot = A.astro_profile_end()["calib_mfma_bf16"]
            calib[f"mfma_only_tflops_{label}_operands"] = round(wgs * 4 * iters * 16 * 32768.0 / (tot / la * 1e-3) / 1e12, 1)
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).zero_()
        dst = torch.empty_like(src)
        A.astro_calib_copy(src, dst)
        A.astro_profile_begin()
        for _ in range(5):
            A.astro_calib_copy(src, dst)
        la, tot = A.astro_profile_end()["calib_copy"]
        calib["copy_gbs_read_plus_write"] = round(2.0 * (1 << 30) / (tot / la * 1e-3) / 1e9, 1)
        result["calibration"] = calib
        del src, dst, sink

    # ---- the fp64 oracle on the host cores, bounded sample of the same workload -----
    if not args.no_cpu_baseline:
        from oracle import RollingCacheOracle
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        # bounded sample (about 10-20 s of host time): 8 heads of one stream; --cpu-baseline-full: the whole step
        n_streams, n_heads = (w.batch, w.heads) if args.cpu_baseline_full else (1, min(w.heads, 8))
        orc = RollingCacheOracle(n_streams, n_heads, w.head_dim, w.grid_h, w.grid_w, w.capacity_frames, w.sink_frames,
                                 w.rope_pairs, w.rope_base)
        w1 = w.scaled(batch=n_streams, heads=n_heads)
        pk, pv = wl.history_frame_pool(w1, 4)
        fk, fv = wl.bf16_bits_to_f32(pk), wl.bf16_bits_to_f32(pv)
        for n in range(min(w.resident_frames, w.capacity_frames)):
            for b in range(n_streams):
                orc.append_stream(b, fk[wl.pool_index(b, n, 4)], fv[wl.pool_index(b, n, 4)], 1)
        qf, kf, vf, dof = (wl.bf16_bits_to_f32(x) for x in wl.chunk_inputs(w1, with_dout=True))
        t0 = time.perf_counter()
        orc.attn_fwd(qf, kf, vf, w.chunk_frames)
        orc.attn_bwd(qf, kf, vf, dof, w.chunk_frames)
        sec = time.perf_counter() - t0
        fl = flops_fwd(w1) + flops_bwd(w1)
        what = ("the whole step: every stream and head of the workload" if args.cpu_baseline_full
                else f"{n_heads} heads of one stream of the workload")
        result["cpu_baseline"] = {"value": round(fl / sec / 1e12, 5), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
                                  "sample": f"{what}, forward + backward, {fl / 1e9:.1f} GFLOP algorithmic in "
                                            f"{sec:.2f} s (fp64 numpy, {cores} BLAS threads)"}

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
