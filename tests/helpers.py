"""Shared helpers of the GPU parity tests: feed the HIP library and the fp64
oracle the same seeded inputs in lockstep and compare."""
from __future__ import annotations

import numpy as np

import workloads as wl
from oracle import RollingCacheOracle

# contract: max abs error on outputs and gradients for bf16 N(0,1) inputs
BF16_ABS_TOL = 2e-2
# The abs bound is larger than the signal at production key counts (outputs have std ~
# sqrt(e/Nk)), so errors are also gated relative to the reference.  The bounds are 2 x what a
# CPU model of the kernels' bf16 roundings (tests/bf16_model.py) lands from the fp64 definition on
# N(0,1) inputs (rms/rms 3.6e-3, max/max 6.9e-3 at the smallest named shape and a mid-size one;
# tests/test_error_gates.py recomputes them and checks these constants).  The largest error is
# normalised by the largest reference entry, not by rms(ref): max/rms moves with the SHAPE of the
# reference's distribution (causal blocks leave late keys with small gradients, which lowers
# rms(ref) and leaves the largest error where it was: 8.7e-2 on a correct dK against 3.3e-2 on the
# unmasked case), so no single bound on it is both tight and passable; it is reported only.
BF16_RMS_OVER_RMS = 7.2e-3   # rms(err) / rms(ref)
BF16_MAX_OVER_MAX = 1.4e-2   # max |err| / max |ref|
F32_ABS_TOL = 1e-5
# inputs outside the N(0,1) contract (large logits, keys with a large common offset): the error
# may be this many times what the rounding model lands on the SAME inputs
MODEL_FACTOR = 2.0


def dev_bf16(bits: np.ndarray, device="cuda:0"):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def dev_f32(x: np.ndarray, device="cuda:0"):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device)


def host_f64(t) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def err_stats(got: np.ndarray, ref: np.ndarray):
    """(max abs err, max abs err / max abs ref, rms(err) / rms(ref)) over finite ref entries."""
    mask = np.isfinite(ref)
    assert mask.any()
    e = got[mask] - ref[mask]
    assert np.isfinite(e).all(), "non-finite values in the GPU result"
    rms_ref = float(np.sqrt(np.mean(ref[mask] ** 2)))
    max_ref = float(np.abs(ref[mask]).max())
    return float(np.abs(e).max()), float(np.abs(e).max() / max_ref), float(np.sqrt(np.mean(e ** 2)) / rms_ref)


def assert_bf16_close(got, ref, what: str, report=None):
    """The N(0,1) contract plus the normalised gates."""
    mx, mx_n, rms_n = err_stats(got, ref)
    mask = np.isfinite(ref)
    mx_r = mx / float(np.sqrt(np.mean(ref[mask] ** 2)))
    if report is not None:
        report.append(f"{what}: max_abs={mx:.3e} max/max={mx_n:.3e} max/rms={mx_r:.3e} rms/rms={rms_n:.3e}")
    assert mx <= BF16_ABS_TOL, f"{what}: max abs err {mx} > {BF16_ABS_TOL}"
    assert mx_n <= BF16_MAX_OVER_MAX, f"{what}: max err / max |ref| = {mx_n}"
    assert rms_n <= BF16_RMS_OVER_RMS, f"{what}: rms err / rms(ref) = {rms_n}"


def assert_within_model(got, ref, model, what: str, report=None):
    """For inputs outside the N(0,1) contract (the absolute bound does not apply): the error
    against the fp64 reference must stay within the normalised gates, or, where the bf16 rounding
    model on the SAME inputs says those cannot hold (a rounded dS meeting keys with a large common
    offset, rotated keys at large logits), within MODEL_FACTOR times the model's error; plus a floor
    for what the model leaves out (fp32 accumulation of the products, fp32 exp2).  One realisation
    of the model's largest error is itself noisy, hence the 'or'."""
    assert np.isfinite(got).all(), f"{what}: non-finite values in the GPU result"
    e, em = got - ref, model - ref
    floor = 2e-5 * max(1.0, float(np.abs(ref).max()))
    mx, mx_m = float(np.abs(e).max()), float(np.abs(em).max())
    rms, rms_m = float(np.sqrt(np.mean(e ** 2))), float(np.sqrt(np.mean(em ** 2)))
    mx_gate = max(MODEL_FACTOR * mx_m, BF16_MAX_OVER_MAX * float(np.abs(ref).max())) + floor
    rms_gate = max(MODEL_FACTOR * rms_m, BF16_RMS_OVER_RMS * float(np.sqrt(np.mean(ref ** 2)))) + floor
    if report is not None:
        report.append(f"{what}: max_abs={mx:.3e} (model {mx_m:.3e}, gate {mx_gate:.3e}) rms={rms:.3e} (model {rms_m:.3e}, gate {rms_gate:.3e})")
    assert mx <= mx_gate, f"{what}: max abs err {mx}, rounding model {mx_m}, gate {mx_gate}"
    assert rms <= rms_gate, f"{what}: rms err {rms}, rounding model {rms_m}, gate {rms_gate}"


def assert_f32_close(got, ref, what: str):
    mx, _, _ = err_stats(got, ref)
    assert mx <= F32_ABS_TOL, f"{what}: max abs err {mx} > {F32_ABS_TOL}"


class Lockstep:
    """One GPU cache and one oracle fed the same frames."""

    def __init__(self, w: wl.Workload, dtype="bf16", start_frames=None, max_chunk=None, device="cuda:0",
                 block_frames=0, window_relative=False):
        import paper_2603_17051_amd as A
        self.A = A
        self.w = w
        self.dtype = dtype
        self.device = device
        self.cache = A.astro_kvcache_create(
            w.batch, w.heads, w.head_dim, w.grid_h, w.grid_w, w.capacity_frames, w.sink_frames,
            max_chunk or w.chunk_frames, w.rope_pairs, w.rope_base,
            A.ASTRO_BF16 if dtype == "bf16" else A.ASTRO_F32, device=device, block_frames=block_frames,
            window_relative=window_relative)
        self.oracle = RollingCacheOracle(w.batch, w.heads, w.head_dim, w.grid_h, w.grid_w, w.capacity_frames,
                                         w.sink_frames, w.rope_pairs, w.rope_base, start_frames,
                                         block_frames=block_frames or None, window_relative=window_relative)
        if start_frames is not None:
            for b, s in enumerate(start_frames):
                A.astro_kvcache_reset(self.cache, b, int(s))

    # inputs are bf16 bit patterns (uint16) for dtype bf16, float32 arrays for f32
    def dev(self, x):
        return dev_bf16(x, self.device) if self.dtype == "bf16" else dev_f32(x, self.device)

    def wide(self, x):
        return wl.bf16_bits_to_f64(x) if self.dtype == "bf16" else np.asarray(x, dtype=np.float64)

    def append(self, k, v, n_frames):
        self.A.astro_kvcache_append(self.cache, self.dev(k), self.dev(v), n_frames)
        self.oracle.append(self.wide(k), self.wide(v), n_frames)

    def check_tables(self):
        sf, sp, nn = self.A.astro_kvcache_tables(self.cache)
        osf, osp, onn = self.oracle.table_arrays()
        assert sf == osf.tolist(), (sf, osf.tolist())
        assert sp == osp.tolist()
        assert nn == onn.tolist()
        return sf

    def fwd(self, q, k, v, n_frames):
        out, lse = self.A.astro_chunk_attn_fwd(self.cache, self.dev(q), self.dev(k), self.dev(v), n_frames)
        return out, lse

    def close(self):
        self.cache.close()
