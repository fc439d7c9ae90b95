"""Pins for the oracle's rebalancing policy: the paper's defaults, each edge of
Fig. 2, trigger placement (only inside a failing allocate), the operation-count
throttle, the no-donor fallback (static-partition behaviour) and the config
validation named under Limitations."""
import os

import numpy as np
import pytest

from oracle import avmp_oracle as orc
from gen import inputs
from tests import helpers

TINY = helpers.oracle_shape(inputs.TINY)
UK, US = TINY.unit_bytes(0), TINY.unit_bytes(1)          # 16 KiB pages, 8 KiB blocks


def _pools(kv, ssm):
    return orc.Pools(TINY, kv * UK + ssm * US, kv, ssm, with_data=False)


def test_defaults_are_the_papers():
    want = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "policy_defaults.txt")) as f:
        for ln in f:
            if ln.strip() and not ln.startswith("#"):
                k, v = ln.split()
                want[k] = float(v)
    pol = orc.Policy()
    assert {k: float(getattr(pol, k)) for k in want} == want


def test_invalid_thresholds_are_rejected():
    p = _pools(4, 4)
    for lo, hi in ((0.3, 0.3), (0.4, 0.3), (-0.1, 0.3), (0.05, 1.5)):
        with pytest.raises(ValueError):
            orc.Rebalancer(p, orc.Policy(threshold_low=lo, threshold_high=hi))
    with pytest.raises(ValueError):
        orc.Rebalancer(p, orc.Policy(migration_batch_size=0))


def test_capacity_error_with_a_slack_donor_migrates_and_retries():
    p = _pools(20, 40)                       # SSM pool has slack
    rb = orc.Rebalancer(p, orc.Policy(migration_batch_size=4, min_rebalance_interval_ops=1000))
    assert rb.allocate(0, 20)[0] == orc.OK   # KV full now; no handler ran
    assert (rb.state, rb.rebalance_count, p.migrations) == (orc.BALANCED, 0, 0)
    code, hs, moved = rb.allocate(0, 3)      # fails -> handler -> migrate 8 blocks = 4 pages -> retry ok
    assert code == orc.OK and len(hs) == 3 and moved == 8
    assert p.stats()["capacity"] == (24, 32)
    assert (rb.state, rb.rebalance_count, rb.oom_events) == (orc.BALANCED, 1, 0)
    assert p.capacity_errors == 1            # the raw failure that triggered the handler


def test_migration_step_is_bounded_by_batch_size_and_donor_free_units():
    p = _pools(10, 40)
    rb = orc.Rebalancer(p, orc.Policy(migration_batch_size=4, min_rebalance_interval_ops=0))
    rb.allocate(0, 10)
    code, hs, moved = rb.allocate(0, 9)      # needs 9, one step gives only 4: retry fails
    assert (code, moved) == (orc.ERR_CAPACITY, 8) and rb.oom_events == 1
    assert p.stats()["capacity"] == (14, 32)
    # donor nearly empty of free units: the step shrinks to what it can give
    p2 = _pools(10, 10)
    rb2 = orc.Rebalancer(p2, orc.Policy(migration_batch_size=4, min_rebalance_interval_ops=0))
    rb2.allocate(0, 10)
    rb2.allocate(1, 6)                       # 4 of 10 blocks free = 0.4 > 0.3
    code, hs, moved = rb2.allocate(0, 1)
    assert (code, moved) == (orc.OK, 4) and p2.stats()["capacity"] == (12, 6)


def test_throttle_counts_logical_operations():
    p = _pools(10, 200)
    rb = orc.Rebalancer(p, orc.Policy(migration_batch_size=1, min_rebalance_interval_ops=50))
    rb.allocate(0, 10)
    assert rb.allocate(0, 1)[2] == 2         # first rebalance: 2 blocks = 1 page
    first = rb.last_rebalance_op
    n_fail = 0
    while p.ops - first < 50 - 1:            # every failing allocate in the window is refused
        code, hs, moved = rb.allocate(0, 1)
        assert (code, moved) == (orc.ERR_CAPACITY, 0)
        n_fail += 1
    assert n_fail > 10 and rb.rebalance_count == 1
    assert rb.state == orc.KV_PRESSURED      # stays pressured while throttled
    assert rb.allocate(0, 1)[2] == 2 and rb.rebalance_count == 2
    assert p.ops - first >= 50


def test_no_donor_behaves_as_a_static_partition():
    rng = np.random.default_rng(4)
    p = _pools(12, 10)
    rb = orc.Rebalancer(p, orc.Policy(min_rebalance_interval_ops=0))
    # keep the SSM pool above 70 % occupancy so it is never a donor
    _, keep = p.alloc(1, 8)
    used, cap, live = [0, 8], [12, 10], []
    for _ in range(600):
        if rng.random() < 0.6 or not live:
            n = int(rng.integers(1, 4))
            code, hs, moved = rb.allocate(0, n)
            ok = used[0] + n <= cap[0]
            assert moved == 0 and code == (orc.OK if ok else orc.ERR_CAPACITY)
            if ok:
                used[0] += n
                live.extend(hs)
        else:
            h = live.pop(int(rng.integers(0, len(live))))
            p.free([h])
            used[0] -= 1
    assert p.migrations == 0 and rb.oom_events > 20
    assert p.stats()["capacity"] == (12, 10)


def test_fig2_edges():
    pol = orc.Policy(threshold_low=0.25, threshold_high=0.5, migration_batch_size=1,
                     min_rebalance_interval_ops=0)
    # BALANCED stays BALANCED if the failing pool is not under threshold_low
    p = _pools(8, 8)
    rb = orc.Rebalancer(p, pol)
    rb.allocate(0, 5)                        # 3 of 8 free = 0.375 >= 0.25
    assert rb.allocate(0, 4)[0] == orc.ERR_CAPACITY and rb.state == orc.BALANCED and p.migrations == 0
    # BALANCED -> KV_PRESSURED, no donor (SSM free 0.5 is not > 0.5): stays pressured
    rb.allocate(0, 2)                        # 1 of 8 free
    rb.allocate(1, 4)                        # SSM free fraction exactly 0.5
    assert rb.allocate(0, 2)[0] == orc.ERR_CAPACITY and rb.state == orc.KV_PRESSURED
    # "free recovers": KV frees up, the next handler run (an SSM failure) sees it
    _, hs = p.alloc(1, 4)                    # SSM now full
    p.free([orc.encode_handle(0, v) for v in range(5)])      # KV free 6/8
    assert rb.allocate(1, 1)[0] == orc.OK    # SSM fails, KV is a donor now
    assert rb.state == orc.BALANCED and p.migrations == 1     # KV_PRESSURED->BALANCED->SSM_PRESSURED->REBALANCING->BALANCED
    # SSM_PRESSURED -> REBALANCING -> BALANCED symmetric case with the other donor
    p2 = _pools(8, 2)
    rb2 = orc.Rebalancer(p2, pol)
    rb2.allocate(1, 2)
    code, hs, moved = rb2.allocate(1, 1)     # 1 page = 2 blocks, B = 1 block -> ceil(8K/16K) = 1 page
    assert (code, moved) == (orc.OK, 1) and p2.stats()["capacity"] == (7, 4)


def test_migrations_happen_only_inside_failing_allocations():
    rng = np.random.default_rng(9)
    p = _pools(16, 16)
    rb = orc.Rebalancer(p, orc.Policy(migration_batch_size=2, min_rebalance_interval_ops=20))
    live = []
    for _ in range(3000):
        before = (p.migrations, p.capacity_errors)
        if rng.random() < 0.55 or not live:
            pool = int(rng.random() < 0.3)
            code, hs, moved = rb.allocate(pool, int(rng.integers(1, 4)))
            live.extend(hs)
            if p.migrations != before[0]:
                assert moved > 0 and p.capacity_errors > before[1]
        else:
            p.free([live.pop(int(rng.integers(0, len(live))))])
            assert p.migrations == before[0]
        st = p.stats()
        assert st["capacity"][0] * UK + st["capacity"][1] * US + st["gap_bytes"] == p.usable
    assert rb.rebalance_count == p.migrations > 3


def test_a_gap_that_holds_the_step_is_used_without_a_donor():
    """Bytes between the pools belong to nobody: when they already hold the B units a
    step gives, the step takes them from there, with no donor and no copy, but as a
    rebalance like any other (counted, throttled)."""
    pol = orc.Policy(migration_batch_size=4, min_rebalance_interval_ops=30)
    # arena with room for 5 pages and half a page more than the pools take
    p = orc.Pools(TINY, 10 * UK + 10 * US + 5 * UK + US, 10, 10, with_data=False)
    rb = orc.Rebalancer(p, pol)
    rb.allocate(0, 10)
    rb.allocate(1, 9)                        # SSM 1 of 10 free: never a donor
    code, hs, moved = rb.allocate(0, 2)      # KV fails; the gap holds 5 >= 4 pages
    assert (code, len(hs), moved) == (orc.OK, 2, 0)
    st = p.stats()
    assert st["capacity"] == (15, 10) and st["gap_bytes"] == US      # every whole page of the gap, remainder kept
    assert (p.migrations, p.units_copied, p.bytes_migrated, rb.rebalance_count) == (1, 0, 0, 1)
    assert rb.state == orc.BALANCED and rb.oom_events == 0
    # the next step is throttled like after any rebalance, and then finds no whole step in the gap
    rb.allocate(0, 3)
    assert rb.allocate(0, 1)[0] == orc.ERR_CAPACITY and rb.rebalance_count == 1
    while p.ops - rb.last_rebalance_op < 30 - 1:
        assert rb.allocate(0, 1) == (orc.ERR_CAPACITY, [], 0)
    assert rb.allocate(0, 1) == (orc.ERR_CAPACITY, [], 0)            # gap 8 KiB < 4 pages, SSM no donor: static
    assert p.stats()["capacity"] == (15, 10) and rb.rebalance_count == 1


def test_a_step_from_the_gap_is_throttled_like_any_other():
    pol = orc.Policy(migration_batch_size=1, min_rebalance_interval_ops=40)
    p = orc.Pools(TINY, 4 * UK + 4 * US + US, 4, 4, with_data=False)         # gap: one block
    rb = orc.Rebalancer(p, pol)
    rb.allocate(0, 4)                        # KV full: never a donor
    rb.allocate(1, 4)
    assert rb.allocate(1, 1)[0] == orc.OK and rb.rebalance_count == 1 and p.stats()["capacity"] == (4, 5)
    # put a block's worth back into the gap by hand, inside the throttle window
    p.free([orc.encode_handle(1, 4)])
    assert p.migrate(1, 1).recipient_gain == 0 and p.gap == US
    assert rb.allocate(1, 1) == (orc.ERR_CAPACITY, [], 0) and rb.rebalance_count == 1
    while p.ops - rb.last_rebalance_op < 40 - 1:
        assert rb.allocate(1, 1)[0] == orc.ERR_CAPACITY
    assert rb.allocate(1, 1)[0] == orc.OK and rb.rebalance_count == 2 and p.gap == 0


def test_a_gap_short_of_the_step_still_counts_towards_it():
    """With less than B units in the gap the donor gives the difference, as before."""
    pol = orc.Policy(migration_batch_size=4, min_rebalance_interval_ops=0)
    p = orc.Pools(TINY, 10 * UK + 40 * US + 3 * UK, 10, 40, with_data=False)    # gap: 3 pages
    rb = orc.Rebalancer(p, pol)
    rb.allocate(0, 10)
    code, hs, moved = rb.allocate(0, 1)      # 4 pages wanted, 3 in the gap: 2 blocks = 1 page from SSM
    assert (code, moved) == (orc.OK, 2) and p.stats()["capacity"] == (14, 38) and p.gap == 0
