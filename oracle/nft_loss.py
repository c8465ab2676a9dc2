"""fp64 CPU oracle of the clip-level forward-process RL loss.  TEST INFRASTRUCTURE ONLY.

Follows Sec. 3.1 (implicit positive / negative policies, eq. (1); policy loss, eq. (2)),
Sec. 3.3 (advantage normalisation r~ = clip(A / A_max) / 2 + 0.5) and Sec. 3.4 (KL penalty
applied only to the masked, high-uncertainty samples; total L = L_policy + lambda_KL L_KL),
in the form Alg. 1, Phase 2 states them.  Written as the formulas, one numpy expression
per line; no blocking, no fusion.

Readings where the paper leaves a choice:
* ||.||^2 is the sum of squares over ONE sample's elements; the mini-batch is averaged
  over its samples (the paper writes the loss for one sample);
* clip(.) carries no bounds in the paper: [-1, 1] is taken, which is what makes
  r~ land in [0, 1] as Sec. 3.1 requires;
* the regression target is an input (eq. (2) calls it v_target, Alg. 1 writes x_0);
* L_KL = (1/|M|) sum over masked samples of ||v_theta - v_ref||^2, 0 when none is masked.
"""
from __future__ import annotations

import numpy as np


def normalized_reward(advantage: np.ndarray, a_max: float) -> np.ndarray:
    """r~_i = clip(A_i / A_max, -1, 1) / 2 + 0.5  (Sec. 3.3)."""
    a = np.asarray(advantage, dtype=np.float64)
    return np.clip(a / np.float64(a_max), -1.0, 1.0) / 2.0 + 0.5


def nft_loss(v_theta, v_old, v_ref, target, advantage, a_max, kl_mask, beta, lambda_kl):
    """Inputs [n, ...] (any trailing shape), advantage [n], kl_mask [n] of 0/1.
    Returns (loss, policy_loss, kl_loss, grad) with grad = dL/dv_theta, same shape as v_theta."""
    vt, vo, vr, tg = (np.asarray(x, dtype=np.float64) for x in (v_theta, v_old, v_ref, target))
    n = vt.shape[0]
    flat = lambda x: x.reshape(n, -1)
    r = normalized_reward(advantage, a_max)[:, None]
    m = np.asarray(kl_mask, dtype=np.float64)[:, None]
    beta, lam = np.float64(beta), np.float64(lambda_kl)
    v_pos = (1.0 - beta) * flat(vo) + beta * flat(vt)          # eq. (1)
    v_neg = (1.0 + beta) * flat(vo) - beta * flat(vt)
    e_pos, e_neg = v_pos - flat(tg), v_neg - flat(tg)
    per_sample = r[:, 0] * (e_pos ** 2).sum(1) + (1.0 - r[:, 0]) * (e_neg ** 2).sum(1)   # eq. (2)
    policy = per_sample.sum() / n
    n_masked = m.sum()
    d_ref = flat(vt) - flat(vr)
    kl = (m[:, 0] * (d_ref ** 2).sum(1)).sum() / n_masked if n_masked > 0 else 0.0
    loss = policy + lam * kl
    # dv+/dv_theta = beta, dv-/dv_theta = -beta
    grad = (2.0 * beta / n) * (r * e_pos - (1.0 - r) * e_neg)
    if n_masked > 0:
        grad = grad + (2.0 * lam / n_masked) * m * d_ref
    return float(loss), float(policy), float(kl), grad.reshape(vt.shape)
