"""The normalised error gates of the GPU parity tests are derived, not picked: a CPU model that
rounds to bf16 where the kernels do (rotated Q / K, the probabilities and dS that enter a matrix
product, the stored output) and is otherwise the fp64 oracle shows how far from the fp64
definition such an implementation lands on N(0,1) inputs.  The gates must be at most twice that
(so a real defect of a few percent cannot hide) and not below it (so a correct kernel passes)."""
import numpy as np
import pytest

import workloads as wl
from oracle import RollingCacheOracle
from bf16_model import model_fwd_bwd, normalised_errors
import helpers


def _model_errors(w, n_hist):
    orc = RollingCacheOracle(w.batch, w.heads, w.head_dim, w.grid_h, w.grid_w, w.capacity_frames, w.sink_frames,
                             w.rope_pairs, w.rope_base, [5] * w.batch)
    pk, pv = wl.history_frame_pool(w, 4)
    fk, fv = wl.bf16_bits_to_f64(pk), wl.bf16_bits_to_f64(pv)
    for n in range(n_hist):
        orc.append_stream(0, fk[n % 4], fv[n % 4], 1)
    q, k, v, do = (wl.bf16_bits_to_f64(x) for x in wl.chunk_inputs(w, with_dout=True))
    Fc = w.chunk_frames
    ro, rl = orc.attn_fwd(q, k, v, Fc, streams=[0], heads=[0])
    rq, rk, rv = orc.attn_bwd(q, k, v, do, Fc, streams=[0], heads=[0])
    m = model_fwd_bwd(orc, q, k, v, do, Fc, 0, 0)
    refs = (ro[0, :, 0], rl[0, 0], rq[0, :, 0], rk[0, :, 0], rv[0, :, 0])
    out = {}
    for name, g, r in zip(("out", "lse", "dq", "dk", "dv"), m, refs):
        mx, mx_rms, rms_rms = normalised_errors(g, r)
        out[name] = dict(max_abs=mx, max_over_rms=mx_rms, rms_over_rms=rms_rms, max_over_max=mx / float(np.abs(r).max()))
    return out


@pytest.fixture(scope="module")
def model_errors():
    tiny = _model_errors(wl.TINY_FWD, 4)                                                              # 64 x 320, D 64
    mid = _model_errors(wl.Workload("mid", 21, 1, 2, 128, 16, 20, 6, 0, 2, 6, (22, 21, 21)), 6)       # 640 x 2560, D 128
    return tiny, mid


def test_gates_are_between_one_and_two_times_the_rounding_model(model_errors):
    worst = {k: max(e[n][k] for e in model_errors for n in ("out", "dq", "dk", "dv"))
             for k in ("rms_over_rms", "max_over_max")}
    for gate, key in ((helpers.BF16_RMS_OVER_RMS, "rms_over_rms"), (helpers.BF16_MAX_OVER_MAX, "max_over_max")):
        assert worst[key] < gate <= 2.05 * worst[key], (key, gate, worst[key])


def test_contract_bound_is_far_above_the_rounding_model_on_unit_gaussians(model_errors):
    # max abs 2e-2 (outputs, gradients, LSE) leaves a wide margin on N(0,1) inputs ...
    for e in model_errors:
        for n in e:
            assert e[n]["max_abs"] < helpers.BF16_ABS_TOL / 5
    # ... which is why it cannot be the only gate: an all-zero output would pass it at 2560 keys
    assert 0.03 < np.sqrt(np.e / 2560) < 2 * helpers.BF16_ABS_TOL


def test_model_reduces_to_the_oracle_when_nothing_is_rounded(monkeypatch):
    """With the rounding switched off the model must reproduce the oracle to fp64 accuracy: its
    own algebra (the five products, the row terms, the un-rotation) adds nothing."""
    import bf16_model
    monkeypatch.setattr(bf16_model, "round_to_bf16", lambda x: np.asarray(x, dtype=np.float64))
    w = wl.Workload("mid", 21, 1, 2, 64, 5, 7, 3, 1, 2, 3, (12, 10, 10))
    e = _model_errors(w, 3)
    for n in e:
        assert e[n]["max_abs"] < 1e-12, (n, e[n])
