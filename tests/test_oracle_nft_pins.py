"""Pins of the loss oracle: torch autograd of the loss written independently, closed forms
of eq. (1)-(2), and the special cases the text fixes (r~ in [0,1], no masked sample)."""
import numpy as np
import pytest
import torch

from oracle import nft_loss, normalized_reward


def _inputs(rng, n=5, shape=(3, 4)):
    vt, vo, vr, tg = (rng.standard_normal((n,) + shape) for _ in range(4))
    adv = rng.standard_normal(n) * 2.0
    mask = (rng.random(n) < 0.5).astype(np.float64)
    mask[0] = 1.0
    return vt, vo, vr, tg, adv, mask


def test_normalized_reward_maps_advantages_into_unit_interval():
    r = normalized_reward(np.array([-10.0, -2.0, -1.0, 0.0, 0.5, 2.0, 7.0]), 2.0)
    np.testing.assert_allclose(r, [0.0, 0.0, 0.25, 0.5, 0.625, 1.0, 1.0])


@pytest.mark.parametrize("beta,lam", [(1.0, 0.0), (0.3, 0.7), (1.0, 2.5)])
def test_loss_and_gradient_match_torch_autograd(beta, lam):
    rng = np.random.default_rng(1)
    vt, vo, vr, tg, adv, mask = _inputs(rng)
    a_max = 1.5
    loss, pol, kl, grad = nft_loss(vt, vo, vr, tg, adv, a_max, mask, beta, lam)
    t = lambda x: torch.tensor(x, dtype=torch.float64)
    tvt = t(vt).requires_grad_(True)
    r = torch.clamp(t(adv) / a_max, -1, 1) / 2 + 0.5
    total = 0.0
    for i in range(vt.shape[0]):  # per sample, as the paper states the loss
        vp = beta * tvt[i] + (1 - beta) * t(vo)[i]
        vn = (1 + beta) * t(vo)[i] - beta * tvt[i]
        total = total + (r[i] * ((vp - t(tg)[i]) ** 2).sum() + (1 - r[i]) * ((vn - t(tg)[i]) ** 2).sum()) / vt.shape[0]
    klt = sum(((tvt[i] - t(vr)[i]) ** 2).sum() for i in range(vt.shape[0]) if mask[i] == 1.0) / mask.sum()
    (total + lam * klt).backward()
    assert loss == pytest.approx(float((total + lam * klt).detach()), rel=1e-13)
    assert pol == pytest.approx(float(total.detach()), rel=1e-13)
    assert kl == pytest.approx(float(klt.detach()), rel=1e-13)
    np.testing.assert_allclose(grad, tvt.grad.numpy(), atol=1e-13)


def test_neutral_reward_closed_form():
    """With r~ = 1/2 the two terms combine: ||v_old - t||^2 + beta^2 ||v_theta - v_old||^2."""
    rng = np.random.default_rng(2)
    vt, vo, vr, tg, _, _ = _inputs(rng, n=4)
    beta = 0.6
    _, pol, kl, _ = nft_loss(vt, vo, vr, tg, np.zeros(4), 1.0, np.zeros(4), beta, 3.0)
    expect = (((vo - tg) ** 2).sum() + beta ** 2 * ((vt - vo) ** 2).sum()) / 4
    assert pol == pytest.approx(expect, rel=1e-13)
    assert kl == 0.0  # nothing masked: no penalty, and no division by zero


def test_extreme_rewards_select_one_branch_and_on_policy_point():
    rng = np.random.default_rng(3)
    vt, vo, vr, tg, _, _ = _inputs(rng, n=3)
    beta = 1.0  # the paper's setting: v+ = v_theta, v- = 2 v_old - v_theta
    _, pol_pos, _, g_pos = nft_loss(vt, vo, vr, tg, np.full(3, 9.0), 1.0, np.zeros(3), beta, 0.0)
    assert pol_pos == pytest.approx(((vt - tg) ** 2).sum() / 3, rel=1e-13)
    np.testing.assert_allclose(g_pos, 2 * (vt - tg) / 3, atol=1e-13)
    _, pol_neg, _, g_neg = nft_loss(vt, vo, vr, tg, np.full(3, -9.0), 1.0, np.zeros(3), beta, 0.0)
    assert pol_neg == pytest.approx(((2 * vo - vt - tg) ** 2).sum() / 3, rel=1e-13)
    np.testing.assert_allclose(g_neg, -2 * (2 * vo - vt - tg) / 3, atol=1e-13)
    # at v_theta = v_old both implicit policies coincide with v_old, whatever beta is
    _, pol_on, _, _ = nft_loss(vo, vo, vr, tg, rng.standard_normal(3), 1.0, np.zeros(3), 0.37, 0.0)
    assert pol_on == pytest.approx(((vo - tg) ** 2).sum() / 3, rel=1e-13)


def test_kl_term_touches_only_masked_samples():
    rng = np.random.default_rng(4)
    vt, vo, vr, tg, adv, _ = _inputs(rng, n=4)
    mask = np.array([0.0, 1.0, 0.0, 1.0])
    _, _, kl, g = nft_loss(vt, vo, vr, tg, adv, 1.0, mask, 1.0, 2.0)
    _, _, _, g0 = nft_loss(vt, vo, vr, tg, adv, 1.0, np.zeros(4), 1.0, 2.0)
    assert kl == pytest.approx((((vt - vr)[[1, 3]]) ** 2).sum() / 2, rel=1e-13)
    np.testing.assert_array_equal(g[[0, 2]], g0[[0, 2]])
    np.testing.assert_allclose(g[[1, 3]] - g0[[1, 3]], 2 * 2.0 * (vt - vr)[[1, 3]] / 2, atol=1e-13)


def test_gradient_matches_finite_differences():
    rng = np.random.default_rng(5)
    vt, vo, vr, tg, adv, mask = _inputs(rng, n=3, shape=(2, 2))
    args = (vo, vr, tg, adv, 1.3, mask, 0.8, 0.4)
    _, _, _, grad = nft_loss(vt, *args)
    h = 1e-6
    for idx in [(0, 0, 0), (1, 1, 0), (2, 0, 1)]:
        up, dn = vt.copy(), vt.copy()
        up[idx] += h
        dn[idx] -= h
        fd = (nft_loss(up, *args)[0] - nft_loss(dn, *args)[0]) / (2 * h)
        assert grad[idx] == pytest.approx(fd, rel=1e-6, abs=1e-9)
