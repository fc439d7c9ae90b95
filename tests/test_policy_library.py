"""The library's rebalancing policy (avmp_alloc_auto on metadata-only pools)
against the oracle's, call by call, plus the qualitative direction the paper
reports: with a slack donor, capacity errors drop relative to a static split."""
import numpy as np
import pytest

from oracle import avmp_oracle as orc
from paper_2605_22416_amd import binding as av
from gen import inputs
from tests import helpers


def _pair(spec, kv_cap, ssm_cap, seed, policy):
    rng = np.random.default_rng(seed)
    arena = kv_cap * spec.kv_page_bytes + ssm_cap * spec.ssm_block_bytes
    ranks = [rng.permutation(arena // spec.kv_page_bytes).astype(np.uint32),
             rng.permutation(arena // spec.ssm_block_bytes).astype(np.uint32)]
    op = orc.Pools(helpers.oracle_shape(spec), arena, kv_cap, ssm_cap, slot_rank=ranks, with_data=False)
    cfg, keep = av.make_config(spec.dtype, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                               spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate, kv_cap, ssm_cap,
                               slot_rank=ranks)
    rc, lp = av.avmp_pools_create(cfg, None, arena)
    assert rc == av.AVMP_OK
    rb = orc.Rebalancer(op, orc.Policy(**policy))
    assert av.avmp_policy_set(lp, **policy) == av.AVMP_OK
    return op, rb, lp


def test_policy_validation_matches():
    spec = inputs.TINY
    op, rb, lp = _pair(spec, 4, 4, 0, dict())
    for lo, hi, b in ((0.3, 0.3, 128), (0.5, 0.3, 128), (-0.1, 0.3, 128), (0.05, 1.5, 128), (0.05, 0.3, 0)):
        assert av.avmp_policy_set(lp, lo, hi, b, 1000) == av.AVMP_ERR_INVALID_ARG
        with pytest.raises(ValueError):
            orc.Rebalancer(op, orc.Policy(lo, hi, b, 1000))
    assert av.avmp_policy_state(lp)["state"] == av.AVMP_BALANCED
    av.avmp_pools_destroy(lp)


@pytest.mark.parametrize("seed,policy", [
    (1, dict(threshold_low=0.05, threshold_high=0.30, migration_batch_size=4, min_rebalance_interval_ops=40)),
    (2, dict(threshold_low=0.2, threshold_high=0.4, migration_batch_size=1, min_rebalance_interval_ops=0)),
    (3, dict(threshold_low=0.05, threshold_high=0.30, migration_batch_size=128, min_rebalance_interval_ops=1000)),
])
def test_alloc_auto_matches_the_oracle_call_by_call(seed, policy):
    spec = inputs.TINY
    op, rb, lp = _pair(spec, 40, 24, seed, policy)
    rng = np.random.default_rng(seed + 100)
    live = []
    phase_len = 1500
    for step in range(4 * phase_len):
        kv_heavy = (step // phase_len) % 2 == 0          # the mix shifts, as in the paper's motivation
        if rng.random() < 0.56 or not live:
            pool = int(rng.random() < (0.15 if kv_heavy else 0.7))
            n = int(rng.integers(1, 5))
            oc, oh, om = rb.allocate(pool, n)
            lc, lh, lm = av.avmp_alloc_auto(lp, pool, n)
            assert (oc, om) == (lc, lm)
            if oc == orc.OK:
                assert list(lh) == oh
                live.extend(oh)
        else:
            k = int(rng.integers(1, min(4, len(live)) + 1))
            hs = [live.pop(int(rng.integers(0, len(live)))) for _ in range(k)]
            assert op.free(hs) == av.avmp_free(lp, hs) == orc.OK
        if step % 100 == 0:
            assert av.avmp_stats(lp) == op.stats()
            st = av.avmp_policy_state(lp)
            assert (st["state"], st["rebalance_count"], st["oom_events"]) == \
                (rb.state, rb.rebalance_count, rb.oom_events)
            assert st["has_rebalanced"] == (rb.last_rebalance_op is not None)
            if rb.last_rebalance_op is not None:
                assert st["last_rebalance_op"] == rb.last_rebalance_op
    assert av.avmp_stats(lp) == op.stats()
    assert rb.oom_events > 0
    if policy["min_rebalance_interval_ops"] < 1000:
        assert rb.rebalance_count > 3
    av.avmp_pools_destroy(lp)


def _run_trace(lp, auto, seed, n_ops=6000, target_live=70):
    """About target_live units stay allocated while the page : block mix of new
    requests shifts every 1500 operations (total demand fits the arena, the static
    split does not fit the KV-heavy phases); returns the count of failed allocations."""
    rng = np.random.default_rng(seed)
    live, failed = [], 0
    for step in range(n_ops):
        kv_heavy = (step // 1500) % 2 == 0
        if len(live) < target_live and rng.random() < 0.7:
            pool = int(rng.random() < (0.1 if kv_heavy else 0.6))
            if auto:
                rc, hs, _ = av.avmp_alloc_auto(lp, pool, 1)
            else:
                rc, hs = av.avmp_alloc(lp, pool, 1)
            if rc == av.AVMP_OK:
                live.extend(hs)
            else:
                failed += 1
        elif live:
            av.avmp_free(lp, [live.pop(int(rng.integers(0, len(live))))])
    return failed


def test_dynamic_rebalancing_lowers_capacity_errors_on_a_shifting_mix():
    """Direction only (the paper's OOM counts need its harness and are not
    reproduced): same trace, same arena split, static versus dynamic."""
    spec = inputs.TINY
    policy = dict(threshold_low=0.05, threshold_high=0.30, migration_batch_size=8,
                  min_rebalance_interval_ops=100)
    fails = {}
    for auto in (False, True):
        op, rb, lp = _pair(spec, 48, 48, 5, policy)
        fails[auto] = _run_trace(lp, auto, seed=6)
        if auto:
            assert av.avmp_policy_state(lp)["rebalance_count"] > 0
        else:
            assert av.avmp_stats(lp)["migrations"] == 0
        av.avmp_pools_destroy(lp)
    assert fails[True] < fails[False], fails


def test_trace_driver_dynamic_split_has_fewest_capacity_errors_across_workloads():
    """The serving-trace driver on the three workload shapes: each static split is
    right for some shapes and wrong for others, the dynamic one follows the load.
    Direction only, on synthetic arrivals (the paper's counts are not reproduced)."""
    from paper_2605_22416_amd import trace_driver
    totals = {"static 0.5": 0, "static 0.9": 0, "dynamic": 0}
    per = {}
    for workload in ("uniform_short", "mixed_long", "agentic_burst"):
        for name, dynamic, share in (("static 0.5", False, 0.5), ("static 0.9", False, 0.9),
                                     ("dynamic", True, 0.5)):
            errs = sum(trace_driver.run_trace(workload, s, dynamic, share, ticks=1500)["capacity_errors"]
                       for s in range(2))
            totals[name] += errs
            per[(workload, name)] = errs
    assert totals["dynamic"] < totals["static 0.5"] and totals["dynamic"] < totals["static 0.9"], totals
    # and it never does worse than the split it started from
    for workload in ("uniform_short", "mixed_long", "agentic_burst"):
        assert per[(workload, "dynamic")] <= 1.1 * per[(workload, "static 0.5")], per


def test_a_step_out_of_the_gap_matches_the_oracle():
    """An arena larger than the two pools: the first capacity error is served from the
    gap (no donor exists), the following ones are throttled, then the static behaviour."""
    spec = inputs.TINY
    kv_cap, ssm_cap = 10, 10
    arena = kv_cap * spec.kv_page_bytes + ssm_cap * spec.ssm_block_bytes + 5 * spec.kv_page_bytes + 4096
    policy = dict(threshold_low=0.05, threshold_high=0.30, migration_batch_size=4, min_rebalance_interval_ops=25)
    op = orc.Pools(helpers.oracle_shape(spec), arena, kv_cap, ssm_cap, with_data=False)
    cfg, keep = av.make_config(spec.dtype, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                               spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate, kv_cap, ssm_cap)
    rc, lp = av.avmp_pools_create(cfg, None, arena)
    assert rc == av.AVMP_OK and av.avmp_policy_set(lp, **policy) == av.AVMP_OK
    rb = orc.Rebalancer(op, orc.Policy(**policy))
    calls = [(0, 10), (1, 9), (0, 2), (0, 3)] + [(0, 1)] * 40
    for pool, n in calls:
        oc, oh, om = rb.allocate(pool, n)
        lc, lh, lm = av.avmp_alloc_auto(lp, pool, n)
        assert (oc, om) == (lc, lm) and (oc != orc.OK or list(lh) == oh)
        assert av.avmp_stats(lp) == op.stats()
        st = av.avmp_policy_state(lp)
        assert (st["state"], st["rebalance_count"], st["oom_events"]) == (rb.state, rb.rebalance_count, rb.oom_events)
    assert av.avmp_stats(lp)["capacity"] == (15, 10) and rb.rebalance_count == 1 and rb.oom_events > 30
    av.avmp_pools_destroy(lp)
