"""GPU check of the entry point that allocates nothing (mtmc_ppo_clip_loss_static): its per-workgroup partial
sums live in a static device array of the library instead of a caller's workspace.  Same kernels as
mtmc_ppo_clip_loss, so the four outputs must be identical, on two calls in a row that share the array, the
second one smaller (fewer partial sums: stale entries of the first call stay behind it and must not be read)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import mtmc_oracle as oracle
from paper_2511_20100_amd import inputs


def test_static_scratch_entry_point_equals_the_workspace_one():
    import torch
    from paper_2511_20100_amd import mtmc
    dev = lambda x: torch.from_numpy(x).cuda()
    out = torch.empty(4, dtype=torch.float64, device="cuda")
    for n, masked in [(1_500_037, True), (1000, False), (1, False)]:   # 1024 partial sums, then 1, then 1
        new, old, adv, mask = inputs.make_ppo_samples(n, seed=11)
        d_new, d_old, d_adv, d_mask = dev(new), dev(old), dev(adv), dev(mask) if masked else None
        ref = mtmc.mtmc_ppo_clip_loss(d_new, d_old, d_adv, 0.2, d_mask).cpu().numpy()
        got = mtmc.mtmc_ppo_clip_loss_static(d_new, d_old, d_adv, 0.2, d_mask, out=out).cpu().numpy()
        assert np.array_equal(got, ref), (n, got, ref)
        want = oracle.ppo_clip_loss(new, old, adv, 0.2, mask if masked else None)
        assert got[3] == want[3] and np.abs(got[:3] - np.array(want[:3])).max() <= 1e-9
    # the first n samples of larger buffers: a smaller input right after a larger one, same device buffers
    new, old, adv, mask = inputs.make_ppo_samples(300_000, seed=5)
    d_new, d_old, d_adv = dev(new), dev(old), dev(adv)
    big = mtmc.mtmc_ppo_clip_loss_static(d_new, d_old, d_adv, 0.1, out=out).cpu().numpy()
    small = mtmc.mtmc_ppo_clip_loss_static(d_new, d_old, d_adv, 0.1, n=5000, out=out).cpu().numpy()
    assert np.array_equal(big, mtmc.mtmc_ppo_clip_loss(d_new, d_old, d_adv, 0.1).cpu().numpy())
    assert np.array_equal(small, mtmc.mtmc_ppo_clip_loss(d_new[:5000].contiguous(), d_old[:5000].contiguous(),
                                                         d_adv[:5000].contiguous(), 0.1).cpu().numpy())


def test_static_scratch_entry_point_rejects_what_it_cannot_take():
    import torch
    from paper_2511_20100_amd import mtmc
    x = torch.zeros(8, dtype=torch.float32, device="cuda")
    out = torch.empty(4, dtype=torch.float64, device="cuda")
    with pytest.raises(mtmc.MtmcError, match="MTMC_PPO_STATIC_MAX_SAMPLES"):
        # only the size is checked before the error: no kernel runs on these 8-element buffers
        mtmc._check(mtmc._lib.mtmc_ppo_clip_loss_static(x.data_ptr(), x.data_ptr(), x.data_ptr(), None,
                                                       mtmc.MTMC_PPO_STATIC_MAX_SAMPLES + 1, 0.2, out.data_ptr(), None))
    with pytest.raises(mtmc.MtmcError, match="clip_eps"):
        mtmc.mtmc_ppo_clip_loss_static(x, x, x, 1.5, out=out)
