"""CPU model of WHERE the bf16 kernels round, built from the oracle's own pieces in fp64.

It is not a second oracle and no GPU result is ever compared with it: it answers "how far from
the pure fp64 definition must an implementation land that keeps bf16 operands for the matrix
products", which is what the normalised error gates of the GPU parity tests are derived from
(gate <= 2 x the model's error on the same kind of input).

Roundings modelled (everything else in fp64):
  * rotated queries (multiplied by log2(e)/sqrt(D) before the rounding, so that their products with
    the keys are exponents of 2), rotated chunk keys and rotated cached keys are stored as bf16;
  * the probabilities that enter the P V product are bf16 (and the row sum is taken over the
    rounded values); the output is stored as bf16;
  * backward: S is recomputed from the bf16 rotated operands, Delta = <dO, O> uses the bf16 output,
    dS = P o (dP - Delta) is rounded to bf16 before dS K and dS^T Q, P is rounded to bf16 before
    P^T dO, and P itself is taken relative to the LSE the forward produced.
"""
from __future__ import annotations

import numpy as np

from oracle import RollingCacheOracle, rope_rotate
from oracle.rolling_attention import round_to_bf16


def model_fwd_bwd(orc: RollingCacheOracle, q, k_chunk, v_chunk, dout, n_frames: int, b: int, h: int):
    """(out, lse, dq, dk, dv) of one (stream, head) pair with the kernels' roundings; inputs are the
    same un-rotated fp64 arrays the oracle gets.  Whole-chunk block (no causal blocks)."""
    D = orc.D
    scale = 1.0 / np.sqrt(np.float64(D))
    log2e, ln2 = 1.0 / np.log(2.0), np.log(2.0)
    phi = orc._chunk_phi(b, n_frames)
    qt = round_to_bf16(scale * log2e * rope_rotate(np.asarray(q[b, :, h:h + 1, :], dtype=np.float64), phi)[:, 0])
    kc = round_to_bf16(rope_rotate(np.asarray(k_chunk[b, :, h:h + 1, :], dtype=np.float64), phi)[:, 0])
    kh, vh = orc._context(b, h)
    kt = np.concatenate([round_to_bf16(kh), kc], 0)
    nh = kh.shape[0]
    vv = np.concatenate([vh, np.asarray(v_chunk[b, :, h, :], dtype=np.float64)], 0)
    do = np.asarray(dout[b, :, h, :], dtype=np.float64)
    # forward, in exponents of 2
    s2 = qt @ kt.T
    m2 = s2.max(axis=1, keepdims=True)
    p_b = round_to_bf16(np.exp2(s2 - m2))
    z = p_b.sum(axis=1, keepdims=True)
    out = round_to_bf16((p_b @ vv) / z)
    lse = ((m2 + np.log2(z)) * ln2)[:, 0]
    # backward
    p = np.exp2(s2 - lse[:, None] * log2e)
    delta = (do * out).sum(axis=1, keepdims=True)
    dp = do @ vv.T
    ds_b = round_to_bf16(p * (dp - delta))
    dqt = scale * (ds_b @ kt)
    # the key-side kernel multiplies the bf16 probabilities it also uses for P^T dO
    pk_b = round_to_bf16(p[:, nh:])
    dsk_b = round_to_bf16(pk_b * (dp[:, nh:] - delta))
    dkt = ln2 * (dsk_b.T @ qt)   # the stored queries carry log2(e)/sqrt(D)
    dv = pk_b.T @ do
    dq = rope_rotate(dqt[:, None, :], -phi)[:, 0]
    dk = rope_rotate(dkt[:, None, :], -phi)[:, 0]
    return out, lse, dq, dk, dv


def normalised_errors(got: np.ndarray, ref: np.ndarray):
    """(max |err|, max |err| / rms(ref), rms(err) / rms(ref))"""
    e = got - ref
    rms_ref = float(np.sqrt(np.mean(ref ** 2)))
    return float(np.abs(e).max()), float(np.abs(e).max() / rms_ref), float(np.sqrt(np.mean(e ** 2)) / rms_ref)
