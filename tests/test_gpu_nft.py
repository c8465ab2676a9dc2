"""GPU parity of the fused clip-level loss against the fp64 oracle: same inputs (bf16 bit
patterns widened exactly, or fp32), gradient element by element, the three loss values."""
import numpy as np
import pytest

import workloads as wl
from oracle import nft_loss
from helpers import dev_bf16, dev_f32, host_f64

pytestmark = pytest.mark.gpu

# fp32 arithmetic on both dtypes: a gradient element is a sum of a few products (relative 1e-6),
# a loss value a sum of up to 1e7 squares accumulated in fp32 per thread, fp64 across blocks
GRAD_REL, LOSS_REL = 2e-6, 2e-5


def _case(n, shape, dtype, seed, masked):
    full = (n,) + shape
    raw = [wl.normal_f32(seed, t, full) for t in (wl.T_Q, wl.T_K, wl.T_V, wl.T_DO)]
    raw[0] = raw[1] + 0.3 * raw[0]  # the current policy stays near the old one
    raw[2] = raw[1] + 0.1 * raw[2]
    adv = wl.normal_f32(seed, wl.T_OFFSETS, (n,)) * 1.5
    mask = np.zeros(n, dtype=np.int32)
    mask[list(masked)] = 1
    if dtype == "bf16":
        bits = [wl.f32_to_bf16_bits(x) for x in raw]
        return [dev_bf16(b) for b in bits], [wl.bf16_bits_to_f64(b) for b in bits], adv, mask
    return [dev_f32(x) for x in raw], [x.astype(np.float64) for x in raw], adv, mask


@pytest.mark.parametrize("dtype,n,shape,masked,beta,lam", [
    ("f32", 3, (2, 6), (1,), 1.0, 0.5),
    ("bf16", 5, (40,), (0, 3), 0.7, 2.0),
    ("bf16", 4, (3, 16, 20, 26), (), 1.0, 1.0),              # nothing masked; 24960 elements: two blocks per sample, ragged
    ("bf16", 24, (3, 16, 60, 104), (2, 5, 11, 23), 1.0, 0.1),   # 24 candidate clips of 3 latent frames (16 x 60 x 104)
    ("bf16", 1024, (24,), (0, 17, 1023), 1.0, 0.3),            # the most samples the main launch prepares for itself
    ("bf16", 1500, (16,), (3, 700, 1499), 0.9, 0.3),           # above it: separate prepare launch
])
def test_nft_loss_and_gradient(dtype, n, shape, masked, beta, lam):
    import torch
    import paper_2603_17051_amd as A
    dev, wide, adv, mask = _case(n, shape, dtype, wl.BASE_SEED + 31, masked)
    a_max = 1.2
    loss, grad = A.astro_nft_loss(*dev, dev_f32(adv), torch.from_numpy(mask).to("cuda:0"), a_max, beta, lam)
    torch.cuda.synchronize()
    ref = nft_loss(*wide, adv.astype(np.float64), a_max, mask, beta, lam)
    got = host_f64(loss)
    for k in range(3):
        assert got[k] == pytest.approx(ref[k], rel=LOSS_REL, abs=1e-30), ("loss", k)
    g, rg = host_f64(grad), ref[3]
    assert np.isfinite(g).all()
    assert np.abs(g - rg).max() <= GRAD_REL * np.abs(rg).max()


def test_nft_loss_rejects_bad_calls():
    import torch
    import paper_2603_17051_amd as A
    x = torch.zeros(2, 12, dtype=torch.bfloat16, device="cuda:0")   # 12 elements: not a multiple of 8
    adv = torch.zeros(2, device="cuda:0")
    m = torch.zeros(2, dtype=torch.int32, device="cuda:0")
    with pytest.raises(A.AstroError):
        A.astro_nft_loss(x, x, x, x, adv, m, 1.0, 1.0, 0.0)
    y = torch.zeros(2, 16, dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(A.AstroError):
        A.astro_nft_loss(y, y, y, y, adv, m, 0.0, 1.0, 0.0)          # a_max must be positive
    with pytest.raises(A.AstroError):
        A.astro_nft_loss(y, y, y, y, adv, m, 1.0, 1.0, 0.0, workspace=torch.zeros(256, dtype=torch.uint8, device="cuda:0"))
