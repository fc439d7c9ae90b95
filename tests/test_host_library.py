"""CPU-side tests of the native library: the C ABI loads and exports what the
header declares, and its host logic (metadata-only pools: tables and counters,
no device) reproduces the oracle's handles, codes and counters bit for bit."""
import os
import re

import numpy as np
import pytest

from oracle import avmp_oracle as orc
from paper_2605_22416_amd import binding as av
from gen import inputs
from tests import helpers

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "avmp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(avmp_[a-z_]+)\s*\(", text)))
    assert {"avmp_pools_create", "avmp_alloc", "avmp_free", "avmp_migrate", "avmp_decode_step"} <= set(names)
    for n in names:
        assert hasattr(av.lib, n), "libavmp.so does not export " + n
        assert hasattr(av, n), "binding has no function named " + n


def _lib_pools(spec, arena_bytes, kv_cap, ssm_cap, ranks):
    cfg, keep = av.make_config(spec.dtype, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                               spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate, kv_cap, ssm_cap,
                               slot_rank=ranks, state_dtype=spec.state_dtype,
                               conv_kernel=spec.conv_kernel, pad_ssm_to_kv_page=spec.pad_ssm_to_kv_page)
    rc, p = av.avmp_pools_create(cfg, None, arena_bytes)
    assert rc == av.AVMP_OK, av.avmp_last_error()
    return p


def test_geometry_matches_the_size_formulas():
    for spec, kvb, ssb in ((inputs.TINY, 16384, 8192), (inputs.JAMBA_MINI, 65536, 4194304)):
        cfg, _ = av.make_config(spec.dtype, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                                spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate, 1, 1)
        rc, g = av.avmp_geometry(cfg, 10 * ssb + 77)
        assert rc == av.AVMP_OK
        assert tuple(g.unit_bytes) == (kvb, ssb)
        assert g.usable_bytes == (10 * ssb + 77) // 128 * 128
        assert tuple(g.max_slots) == (g.usable_bytes // kvb, g.usable_bytes // ssb)


def test_geometry_with_a_convolution_window():
    for spec in (inputs.with_conv(inputs.TINY, 3), inputs.with_conv(inputs.JAMBA_MINI, 4),
                 inputs.with_conv(inputs.with_state_dtype(inputs.JAMBA_MINI, "bf16"), 2)):
        cfg, _ = av.make_config(spec.dtype, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                                spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate, 1, 1,
                                state_dtype=spec.state_dtype, conv_kernel=spec.conv_kernel)
        rc, g = av.avmp_geometry(cfg, 1 << 30)
        assert rc == av.AVMP_OK
        assert g.unit_bytes[1] == spec.ssm_block_bytes == \
            helpers.oracle_shape(spec).unit_bytes(orc.POOL_SSM)
        assert g.unit_bytes[1] > spec.ssm_state_bytes
    base = dict(dtype="bf16", n_q_heads=4, n_kv_heads=2, head_dim=64, ssm_heads=4, ssm_headdim=32,
                ssm_dstate=16, kv_capacity=1, ssm_capacity=1)
    for bad in (dict(conv_kernel=1), dict(conv_kernel=5), dict(conv_kernel=4, ssm_headdim=3),
                dict(conv_kernel=4, dtype="f32", ssm_heads=1, ssm_headdim=6)):
        cfg, _ = av.make_config(**{**base, **bad})
        assert av.avmp_geometry(cfg, 1 << 30)[0] == av.AVMP_ERR_INVALID_ARG
    cfg, _ = av.make_config(**{**base, "conv_kernel": 4})
    assert av.avmp_geometry(cfg, 1 << 30)[0] == av.AVMP_OK


def test_padded_unified_geometry_reports_native_and_padded_sizes():
    """The unified-pool sizing mode against the hand-evaluated sizes, and what it costs."""
    import os
    specs = {"tiny_fp32": inputs.TINY, "jamba_mini_like": inputs.JAMBA_MINI}
    rows = [ln.split() for ln in open(os.path.join(os.path.dirname(__file__), "golden", "padded_unified_sizes.txt"))
            if ln.strip() and not ln.startswith("#")]
    for name, state_dtype, k, page, native, padded in rows:
        spec = specs[name]
        for pad in (False, True):
            cfg, _ = av.make_config(spec.dtype, spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.ssm_heads,
                                    spec.ssm_headdim, spec.ssm_dstate, 1, 1, state_dtype=state_dtype,
                                    conv_kernel=int(k), pad_ssm_to_kv_page=pad)
            rc, g = av.avmp_geometry(cfg, 1 << 30)
            assert rc == av.AVMP_OK
            assert (g.unit_bytes[0], g.ssm_native_bytes) == (int(page), int(native))
            assert g.unit_bytes[1] == (int(padded) if pad else int(native))
            assert g.max_slots[1] == (1 << 30) // g.unit_bytes[1]
    cfg.ssm_pad_to_kv_page = 2
    assert av.avmp_geometry(cfg, 1 << 30)[0] == av.AVMP_ERR_INVALID_ARG


def test_create_rejects_bad_configs():
    spec = inputs.TINY
    ok = dict(dtype="f32", n_q_heads=4, n_kv_heads=2, head_dim=64, ssm_heads=4, ssm_headdim=32,
              ssm_dstate=16, kv_capacity=4, ssm_capacity=2)
    arena = 4 * spec.kv_page_bytes + 2 * spec.ssm_block_bytes
    for bad in (dict(n_q_heads=3), dict(head_dim=66), dict(ssm_dstate=24), dict(kv_capacity=5),
                dict(page_tokens=32), dict(n_kv_heads=0)):
        cfg, _ = av.make_config(**{**ok, **bad})
        rc, p = av.avmp_pools_create(cfg, None, arena)
        assert rc == av.AVMP_ERR_INVALID_ARG and p is None
    cfg, keep = av.make_config(**ok, slot_rank=[np.zeros(arena // spec.kv_page_bytes, dtype=np.uint32), None])
    assert av.avmp_pools_create(cfg, None, arena)[0] == av.AVMP_ERR_INVALID_ARG   # not a permutation
    cfg, _ = av.make_config(**ok)
    rc, p = av.avmp_pools_create(cfg, None, arena)
    assert rc == av.AVMP_OK
    # metadata-only pools refuse device entry points loudly
    assert av.avmp_flush(p) == av.AVMP_ERR_DEVICE
    st, keep = av.make_step(0, [], 1, *([None] * 11))
    assert av.avmp_decode_step(p, st) == av.AVMP_ERR_DEVICE
    assert av.avmp_pools_destroy(p) == av.AVMP_OK


def _check_same(op, lp):
    assert av.avmp_stats(lp) == op.stats()


@pytest.mark.parametrize("seed,conv,n_ops,pad", [(1, 0, 50000, False), (2, 0, 40000, False), (3, 3, 12000, False),
                                                  (4, 3, 12000, True)])
def test_random_traces_match_the_oracle_bit_for_bit(seed, conv, n_ops, pad):
    # with a 3-tap convolution window the block is 9472 bytes: units that divide nothing evenly;
    # padded to whole pages it becomes 16384 bytes
    spec = inputs.with_conv(inputs.TINY, conv) if conv else inputs.TINY
    if pad:
        spec = inputs.with_padded_blocks(spec)
    rng = np.random.default_rng(seed)
    kv_cap, ssm_cap = 37, 11
    arena = kv_cap * spec.kv_page_bytes + ssm_cap * spec.ssm_block_bytes + 128 * 5
    ranks = [rng.permutation(arena // spec.kv_page_bytes).astype(np.uint32),
             rng.permutation(arena // spec.ssm_block_bytes).astype(np.uint32)]
    op = orc.Pools(helpers.oracle_shape(spec), arena, kv_cap, ssm_cap, slot_rank=ranks, with_data=False)
    lp = _lib_pools(spec, arena, kv_cap, ssm_cap, ranks)
    live = {0: [], 1: []}
    n_cap = n_mig = n_bad = n_gap = 0
    for step in range(n_ops):
        u = rng.random()
        pool = int(rng.integers(0, 2))
        if u < 0.50:
            n = int(rng.integers(1, 6))
            oc, oh = op.alloc(pool, n)
            lc, lh = av.avmp_alloc(lp, pool, n)
            assert oc == lc
            if oc == orc.OK:
                assert list(lh) == oh
                live[pool].extend(oh)
            else:
                n_cap += 1
        elif u < 0.90:
            if not live[0] and not live[1]:
                continue
            both = live[0] + live[1]                       # a free call may mix pools
            k = int(rng.integers(1, min(6, len(both)) + 1))
            hs = [both[i] for i in rng.choice(len(both), size=k, replace=False)]
            if rng.random() < 0.05:
                hs.append(hs[0] if rng.random() < 0.5 else int(rng.integers(0, 1 << 32)))
            oc = op.free(hs)
            assert av.avmp_free(lp, hs) == oc
            if oc == orc.OK:
                for h in hs:
                    live[h >> 30].remove(h)
            else:
                n_bad += 1
        elif u < 0.97:
            n = int(rng.integers(1, 7))
            if rng.random() < 0.15:                        # the gap's whole units to one pool
                ores = op.absorb_gap(pool)
                lc, lres = av.avmp_absorb_gap(lp, pool)
                n_gap += lc == av.AVMP_OK
            else:
                ores = op.migrate(pool, n)
                lc, lres = av.avmp_migrate(lp, pool, n)
            assert lc == ores.code
            if lc == av.AVMP_OK:
                n_mig += 1
                assert (lres.units_copied, lres.recipient_gain, lres.bytes_wasted) == \
                    (ores.units_copied, ores.recipient_gain, ores.bytes_wasted)
        else:
            assert av.avmp_alloc(lp, 2, 1)[0] == op.alloc(2, 1)[0] == orc.ERR_INVALID_ARG
            assert av.avmp_migrate(lp, pool, 0)[0] == op.migrate(pool, 0).code == orc.ERR_INVALID_ARG
            assert av.avmp_absorb_gap(lp, 2)[0] == op.absorb_gap(2).code == orc.ERR_INVALID_ARG
        if step % 50 == 0:
            _check_same(op, lp)
            for h in live[0] + live[1]:
                rc, pl, sl, off = av.avmp_resolve(lp, h)
                assert rc == av.AVMP_OK and (pl, sl, off) == op.resolve(h)
    _check_same(op, lp)
    assert n_cap > 100 and n_mig > 100 and n_bad > 50 and (n_gap > 5 or pad)   # equal units leave no whole unit in the gap
    assert av.avmp_resolve(lp, 0xFFFFFFFF)[0] == av.AVMP_ERR_INVALID_HANDLE
    av.avmp_pools_destroy(lp)


def test_capacity_scale_workload_cut_to_a_sixteenth_matches_the_oracle():
    """The capacity-scale workload's shape at a sixteenth of its size (32 requests of
    U[1024,8192] tokens and one of 16384, pools at 1.7x demand, seeded placement), where
    the oracle's linear scans still finish: every allocation, then migration batches of 4,
    64 and 1024 pages (a sixteenth of 64, 1024 and 16384), handle by handle."""
    spec = inputs.JAMBA_MINI
    rng = np.random.default_rng(1005)
    ctx = np.concatenate([rng.integers(1024, 8193, size=32), [16384]]).astype(np.uint32)
    sc = inputs.make_scenario(spec, "capacity", len(ctx), seed=1005, ctx=ctx, headroom=1.7)
    op, kv, ssm = helpers.build_oracle(sc, with_data=False)
    lp = _lib_pools(spec, sc.arena_bytes, sc.kv_capacity, sc.ssm_capacity, sc.slot_rank)
    for pool, n, tag in helpers.alloc_order(sc):
        lc, lh = av.avmp_alloc(lp, pool, n)
        assert lc == av.AVMP_OK
        want = kv[tag[1], tag[2], :n] if tag[0] == "kv" else ssm[:, tag[1]]
        assert np.array_equal(lh, want)
    _check_same(op, lp)
    handles = np.concatenate([kv[kv != 0xFFFFFFFF], ssm.reshape(-1)])
    for n in (4, 64, 1024):
        ores = op.migrate(0, n)
        lc, lres = av.avmp_migrate(lp, 0, n)
        assert lc == ores.code == orc.OK
        assert (lres.units_copied, lres.recipient_gain, lres.bytes_wasted) == \
            (ores.units_copied, ores.recipient_gain, ores.bytes_wasted) and ores.units_copied > 0
        _check_same(op, lp)
        for h in handles[:: 7]:
            assert av.avmp_resolve(lp, int(h))[1:] == op.resolve(int(h))
    av.avmp_pools_destroy(lp)


def test_jamba_shaped_allocation_order_matches_the_oracle():
    spec = inputs.scaled_down(inputs.JAMBA_MINI, 1)
    sc = inputs.make_scenario(spec, "uniform_short", 16, seed=1002)
    op, kv, ssm = helpers.build_oracle(sc, with_data=False)
    lp = _lib_pools(spec, sc.arena_bytes, sc.kv_capacity, sc.ssm_capacity, sc.slot_rank)
    kv2, ssm2 = helpers.empty_handle_tables(sc)
    for pool, n, tag in helpers.alloc_order(sc):
        rc, hs = av.avmp_alloc(lp, pool, n)
        assert rc == av.AVMP_OK
        helpers.place_handles(kv2, ssm2, tag, hs)
    assert np.array_equal(kv, kv2) and np.array_equal(ssm, ssm2)
    for h in list(kv2[0, 3, : sc.n_pages[3]]) + list(ssm2[:, 5]):
        assert av.avmp_resolve(lp, int(h))[1:] == op.resolve(int(h))
    _check_same(op, lp)
    av.avmp_pools_destroy(lp)


def test_bench_refuses_more_than_one_gpu():
    """The path is a one-GPU path: the benchmark says so instead of running."""
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode == 2
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""
