"""Writes tests/golden/oracle_tiny.json: sampled outputs and gradients of the fp64 oracle on
the smallest named configuration (one 64-token frame over a full ring of 4 frames, 2 heads,
head dim 64, rotary 12/10/10; Sec. 3.2 rolling cache, Sec. 3.3 detached backward), with and
without window-relative positions and a sink.  Calls only `oracle/` and the seeded input module.
The stored numbers are a regression guard for the oracle itself (its independent pins are the
tests/test_oracle_*.py files): an accidental change of its arithmetic shows up here first.

    python tests/golden/make_oracle_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import workloads as wl  # noqa: E402
from oracle import RollingCacheOracle  # noqa: E402

SAMPLES = [(0, 0, 0, 0), (0, 17, 1, 5), (0, 63, 0, 63), (0, 40, 1, 32)]


def case(sinks: int, window_relative: bool, n_hist: int):
    w = wl.TINY_FWD
    orc = RollingCacheOracle(w.batch, w.heads, w.head_dim, w.grid_h, w.grid_w, w.capacity_frames, sinks,
                             w.rope_pairs, w.rope_base, start_frames=[3], window_relative=window_relative)
    pk, pv = wl.history_frame_pool(w, 4)
    fk, fv = wl.bf16_bits_to_f64(pk), wl.bf16_bits_to_f64(pv)
    for n in range(n_hist):
        orc.append(fk[n % 4][None], fv[n % 4][None], 1)
    q, k, v, do = (wl.bf16_bits_to_f64(x) for x in wl.chunk_inputs(w, with_dout=True))
    out, lse = orc.attn_fwd(q, k, v, 1)
    dq, dk, dv = orc.attn_bwd(q, k, v, do, 1)
    pick = lambda a: [float(a[i]) for i in SAMPLES]
    return {"sinks": sinks, "window_relative": window_relative, "n_hist": n_hist,
            "out": pick(out), "dq": pick(dq), "dk": pick(dk), "dv": pick(dv),
            "lse": [float(lse[0, 0, 0]), float(lse[0, 1, 63])],
            "out_sum": float(out.sum()), "dq_abs_sum": float(np.abs(dq).sum())}


if __name__ == "__main__":
    cases = [case(0, False, 4), case(1, False, 7), case(1, True, 7)]
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_tiny.json")
    with open(path, "w") as f:
        json.dump({"samples": SAMPLES, "cases": cases}, f, indent=1)
    print("wrote", path)
