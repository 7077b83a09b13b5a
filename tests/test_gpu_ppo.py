"""GPU parity of the clipped PPO surrogate against the oracle (both sum in double; only the order differs)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import mtmc_oracle as oracle
from paper_2511_20100_amd import inputs

TOL = 1e-9  # absolute, on values of order 1: double sums of up to ~1e6 terms in different orders


@pytest.mark.parametrize("n", [1, 7, 1000, 4096, 1024 * 1024 + 37, 5_000_011])
@pytest.mark.parametrize("masked", [False, True])
def test_ppo_matches_oracle(n, masked):
    import torch
    from paper_2511_20100_amd import mtmc
    new, old, adv, mask = inputs.make_ppo_samples(n, seed=n % 97)
    dev = lambda x: torch.from_numpy(x).cuda()
    out = mtmc.mtmc_ppo_clip_loss(dev(new), dev(old), dev(adv), 0.2, dev(mask) if masked else None).cpu().numpy()
    again = mtmc.mtmc_ppo_clip_loss(dev(new), dev(old), dev(adv), 0.2, dev(mask) if masked else None).cpu().numpy()
    assert np.array_equal(out, again)  # fixed summation order
    ref = oracle.ppo_clip_loss(new, old, adv, 0.2, mask if masked else None)
    assert out[3] == ref[3]
    assert np.abs(out[:3] - np.array(ref[:3])).max() <= TOL, (out, ref)
    if n >= 1000:
        assert 0.0 < out[1] < 1.0  # the case has clipped and unclipped samples


def test_ppo_edge_cases():
    import torch
    from paper_2511_20100_amd import mtmc
    new, old, adv, mask = inputs.make_ppo_samples(300, seed=3)
    dev = lambda x: torch.from_numpy(x).cuda()
    none = mtmc.mtmc_ppo_clip_loss(dev(new), dev(old), dev(adv), 0.2, dev(np.zeros(300, dtype=np.int32))).cpu().numpy()
    assert np.all(none == 0.0)
    same = mtmc.mtmc_ppo_clip_loss(dev(old), dev(old), dev(adv), 0.2).cpu().numpy()
    assert abs(same[0] + adv.astype(np.float64).mean()) < 1e-12 and same[1] == 0.0 and same[2] == 0.0 and same[3] == 300
    wide = mtmc.mtmc_ppo_clip_loss(dev(new), dev(old), dev(adv), 0.0).cpu().numpy()  # eps 0: everything clipped to r = 1 or below
    ref = oracle.ppo_clip_loss(new, old, adv, 0.0)
    assert np.abs(wide[:3] - np.array(ref[:3])).max() <= TOL
    with pytest.raises(mtmc.MtmcError, match="clip_eps"):
        mtmc.mtmc_ppo_clip_loss(dev(new), dev(old), dev(adv), 1.5)


def test_measurement_probes_run_and_report_their_work():
    """The two probes behind the `attainable` figures of the benchmark: the streaming read touches nothing but its
    sink, the matrix-instruction loop returns the flops of its launch and overwrites its output with finite sums."""
    import torch
    from paper_2511_20100_amd import mtmc
    src = torch.ones(64 << 20, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    mtmc.mtmc_read_probe(src, sink)
    out = torch.full((8 * 256,), float("nan"), dtype=torch.float32, device="cuda")
    flops = mtmc.mtmc_mfma_probe(out, 8, 100)
    torch.cuda.synchronize()
    assert int(sink.item()) == 0 and bool((src == 1).all())
    assert flops == 8 * 4 * 16 * 100 * 2 * 32 * 32 * 16
    assert bool(torch.isfinite(out).all()) and float(out.abs().max()) > 0.0
