"""Host logic of the rollout that takes in prompts as it runs (no GPU): which prompts join the batch at one look.
The invariants a wrong plan would break on the device: a slot whose sequence still runs is never given away, two
prompts never get the same slot or the same region of shared prompt pages, a region that a running sequence
reads is never handed out, and the count is the largest the free slots, free regions, remaining prompts and the
prefill's capacity allow - or zero while it is worth waiting for more."""
import numpy as np
import pytest

from paper_2511_20100_amd import mtmc


def brute(live, slot_region, n_regions, ns, left, max_at_once, wait_for):
    free = [s for s in range(len(live)) if not live[s]]
    used = {int(slot_region[s]) for s in range(len(live)) if live[s]}
    free_regions = [r for r in range(n_regions) if r not in used]
    k = min(len(free) // ns, len(free_regions), left, max_at_once)
    if k <= 0 or (k < min(left, wait_for, max_at_once) and any(live)):
        k = 0
    return k, free[:k * ns], free_regions[:k]


@pytest.mark.parametrize("seed", range(40))
def test_plans_agree_with_brute_force_and_keep_the_invariants(seed):
    rng = np.random.default_rng(seed)
    ns = int(rng.choice([1, 2, 8, 24]))
    places = max(1, 128 // ns)
    n_slots = places * ns
    n_regions = int(rng.integers(places, 4 * places + 1))
    live = (rng.random(n_slots) < rng.choice([0.0, 0.3, 0.8, 0.97, 1.0])).astype(np.int32)
    slot_region = rng.integers(0, n_regions, n_slots).astype(np.int32)
    left = int(rng.integers(0, 40))
    max_at_once = int(rng.integers(1, 17))
    wait_for = int(rng.integers(1, 9))
    slots, regions = mtmc.mtmc_admission_plan(live, slot_region, n_regions, ns, left, max_at_once, wait_for)
    k, want_slots, want_regions = brute(live, slot_region, n_regions, ns, left, max_at_once, wait_for)
    assert slots.shape == (k, ns) and regions.shape == (k,)
    assert slots.reshape(-1).tolist() == want_slots and regions.tolist() == want_regions
    flat = slots.reshape(-1)
    assert len(set(flat.tolist())) == flat.size and not live[flat].any()
    assert len(set(regions.tolist())) == regions.size
    assert not (set(regions.tolist()) & {int(r) for r in slot_region[live == 1]})


def test_waits_for_a_few_prompts_unless_nothing_runs_or_few_are_left():
    ns, n_regions = 8, 64
    slot_region = (np.arange(128) // ns).astype(np.int32)
    live = np.ones(128, dtype=np.int32)
    live[8:16] = 0                                      # one prompt's slots are free
    plan = lambda **kw: mtmc.mtmc_admission_plan(live, slot_region, n_regions, ns, kw.get("left", 10), 16, kw.get("wait", 4))
    assert plan()[0].shape[0] == 0                      # worth waiting: 1 < min(10, 4)
    assert plan(wait=1)[0].tolist() == [list(range(8, 16))]
    assert plan(left=1)[0].shape[0] == 1                # the last prompt does not wait
    live[:] = 0
    s, r = plan()                                       # nothing runs: as many as a prefill takes
    assert s.shape[0] == 10 and r.tolist() == list(range(10))
    live[:] = 1
    assert plan(left=0)[0].shape[0] == 0 and plan()[0].shape[0] == 0


def test_a_region_still_read_by_one_straggler_is_not_handed_out():
    ns = 8
    slot_region = (np.arange(128) // ns).astype(np.int32)      # 16 regions, all in use at the start
    live = np.zeros(128, dtype=np.int32)
    live[::8] = 1                                              # one straggler per prompt: 112 free slots, no free region
    s, r = mtmc.mtmc_admission_plan(live, slot_region, 16, ns, 10, 16, 1)
    assert s.shape[0] == 0
    s, r = mtmc.mtmc_admission_plan(live, slot_region, 19, ns, 10, 16, 1)   # three spare regions
    assert s.shape[0] == 3 and r.tolist() == [16, 17, 18]
    assert not live[s.reshape(-1)].any()


def test_bad_arguments_are_rejected():
    one = np.zeros(4, dtype=np.int32)
    with pytest.raises(mtmc.MtmcError):
        mtmc.mtmc_admission_plan(one, one, 0, 1, 1, 1, 1)
    with pytest.raises(mtmc.MtmcError):
        mtmc.mtmc_admission_plan(one, one, 2, 0, 1, 1, 1)


def test_never_waits_for_more_than_one_prefill_takes():
    ns = 8
    slot_region = (np.arange(128) // ns).astype(np.int32)
    live = np.ones(128, dtype=np.int32)
    live[:16] = 0                                       # two prompts' slots are free, a prefill takes two (long prompts)
    s, r = mtmc.mtmc_admission_plan(live, slot_region, 64, ns, 10, 2, 4)
    assert s.shape[0] == 2
