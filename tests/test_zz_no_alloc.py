"""The entry point that allocates nothing (astro_nft_loss_static: the library's static device
array is the scratch) against astro_nft_loss on the same inputs, through the C ABI: two calls in a
row on one GPU, the second with a smaller input, so that what the first call left in the shared
array cannot leak into the second.  Both entry points run the same kernels in the same order, so
the results must be bit-identical."""
import ctypes

import numpy as np
import pytest

import workloads as wl
from helpers import dev_bf16, dev_f32

pytestmark = pytest.mark.gpu


def _inputs(n, elems, seed, masked):
    import torch
    raw = [wl.normal_f32(seed, t, (n, elems)) for t in (wl.T_Q, wl.T_K, wl.T_V, wl.T_DO)]
    raw[0] = raw[1] + 0.3 * raw[0]
    raw[2] = raw[1] + 0.1 * raw[2]
    tensors = [dev_bf16(wl.f32_to_bf16_bits(x)) for x in raw]
    adv = dev_f32(wl.normal_f32(seed, wl.T_OFFSETS, (n,)) * 1.5)
    mask = np.zeros(n, dtype=np.int32)
    mask[list(masked)] = 1
    return tensors, adv, torch.from_numpy(mask).to("cuda:0")


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    import torch
    import paper_2603_17051_amd as A
    from paper_2603_17051_amd import binding
    lib = binding.library()
    limit = A.astro_nft_loss_static_bytes()
    assert limit == 1 << 20
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    # first call: 40 samples of 40000 elements (3 blocks per sample, ragged last block);
    # second call: 7 samples of 4104 elements (one block per sample)
    for n, elems, masked in ((40, 40000, (0, 3, 39)), (7, 4104, (2,))):
        tensors, adv, mask = _inputs(n, elems, wl.BASE_SEED + 77 + n, masked)
        assert A.astro_nft_loss_workspace_bytes(n, elems) <= limit
        ref_loss, ref_grad = A.astro_nft_loss(*tensors, adv, mask, 1.2, 0.8, 0.4)
        loss = torch.full((3,), float("nan"), device="cuda:0")
        grad = torch.full((n, elems), float("nan"), device="cuda:0")
        rc = lib.astro_nft_loss_static(*(P(t) for t in tensors), P(adv), P(mask), n, elems, binding.ASTRO_BF16,
                                       1.2, 0.8, 0.4, P(loss), P(grad), stream)
        assert rc == binding.ASTRO_OK
        torch.cuda.synchronize()
        assert torch.isfinite(loss).all() and torch.isfinite(grad).all()
        assert torch.equal(loss, ref_loss), (n, loss.tolist(), ref_loss.tolist())
        assert torch.equal(grad, ref_grad), n


def test_static_scratch_entry_point_rejects_sizes_beyond_its_array():
    import torch
    import paper_2603_17051_amd as A
    from paper_2603_17051_amd import binding
    lib = binding.library()
    n, elems = 4096, 64 * 16384   # 4096 samples x 64 blocks x 3 sums x 4 B = 3 MiB of partial sums
    assert A.astro_nft_loss_workspace_bytes(n, elems) > A.astro_nft_loss_static_bytes()
    x = torch.zeros(8, dtype=torch.bfloat16, device="cuda:0")   # never read: the size check comes first
    f = torch.zeros(8, device="cuda:0")
    m = torch.zeros(8, dtype=torch.int32, device="cuda:0")
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = lib.astro_nft_loss_static(P(x), P(x), P(x), P(x), P(f), P(m), n, elems, binding.ASTRO_BF16, 1.0, 1.0, 0.0,
                                   P(f), P(f), None)
    assert rc == binding.ASTRO_ERR_WORKSPACE
    torch.cuda.synchronize()
