"""Pins for the oracle's handle codec, table, allocate/free and migration.

Each test checks the oracle against something fixed outside it: the paper's
worked example, hand-evaluated size formulas, a two-integer capacity model
(the paper's finding that the table-backed allocator without migration is
OOM-for-OOM identical to a static dual pool), conservation laws of migration,
brute force on tiny pools.
"""
import os

import numpy as np
import pytest

from oracle import avmp_oracle as orc
from gen import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def _shape(spec):
    return orc.Shape(spec.dtype, spec.page_tokens, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                     spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate, spec.state_dtype,
                     spec.conv_kernel, spec.pad_ssm_to_kv_page)


TINY = _shape(inputs.TINY)
JAMBA = _shape(inputs.JAMBA_MINI)


def rank_with_first(n, first):
    """A permutation rank[] of n slots whose lowest ranks go to `first`, in order."""
    rest = [s for s in range(n) if s not in first]
    order = list(first) + rest
    rank = np.empty(n, dtype=np.int64)
    rank[order] = np.arange(n)
    return rank


# ---- P1: handle codec and Fig. 1's worked example ---------------------------
def test_handle_is_32_bit_tagged():
    assert orc.encode_handle(orc.POOL_KV, 0) == 0
    assert orc.encode_handle(orc.POOL_SSM, 0) == 0x40000000
    assert orc.encode_handle(orc.POOL_SSM, 5) == 0x40000005
    assert orc.encode_handle(3, orc.PAGE_ID_MASK) == orc.INVALID_HANDLE
    rng = np.random.default_rng(7)
    for pool, vid in zip(rng.integers(0, 4, 1 << 16), rng.integers(0, 1 << 30, 1 << 16)):
        h = orc.encode_handle(int(pool), int(vid))
        assert 0 <= h < (1 << 32)
        assert orc.decode_handle(h) == (int(pool), int(vid))
    with pytest.raises(ValueError):
        orc.encode_handle(0, 1 << 30)


def test_fig1_worked_example():
    want = {r[0]: (r[1], int(r[2])) for r in _rows("fig1_translation.txt")}
    unit_kv, unit_ssm = TINY.unit_bytes(0), TINY.unit_bytes(1)
    arena = 8 * unit_kv + 3 * unit_ssm
    n_kv, n_ssm = arena // unit_kv, arena // unit_ssm
    p = orc.Pools(TINY, arena, 8, 3, slot_rank=[rank_with_first(n_kv, [3, 7]),
                                                 rank_with_first(n_ssm, [1])])
    _, (h0,) = p.alloc(orc.POOL_KV, 1)
    _, (h1,) = p.alloc(orc.POOL_SSM, 1)
    _, (h2,) = p.alloc(orc.POOL_KV, 1)
    got = {}
    for name, h in (("h_0", h0), ("h_1", h1), ("h_2", h2)):
        pool, slot, off = p.resolve(h)
        got[name] = ("KV" if pool == orc.POOL_KV else "SSM", slot)
        # the offset is inside the tagged store's region
        if pool == orc.POOL_KV:
            assert off == slot * unit_kv
        else:
            assert off == p.usable - (slot + 1) * unit_ssm
    assert got == want
    # tags dispatch to different stores: same page_id, different pool
    assert orc.decode_handle(h0)[1] == orc.decode_handle(h1)[1] == 0
    assert p.resolve(h0)[0] != p.resolve(h1)[0]


# ---- P2: unit sizes and alignment -------------------------------------------
def test_unit_sizes_closed_form():
    specs = {"tiny_fp32": inputs.TINY, "jamba_mini_like": inputs.JAMBA_MINI}
    for r in _rows("unit_sizes.txt"):
        spec = specs[r[0]]
        sh = _shape(spec)
        assert [sh.page_tokens, sh.n_kv_heads, sh.head_dim, sh.elem_bytes, sh.ssm_heads,
                sh.ssm_headdim, sh.ssm_dstate] == [int(v) for v in r[1:8]]
        assert sh.unit_bytes(orc.POOL_KV) == int(r[8])
        assert sh.unit_bytes(orc.POOL_SSM) == int(r[9])
        # the input generator's own size arithmetic agrees with the fixture too
        assert spec.kv_page_bytes == int(r[8]) and spec.ssm_block_bytes == int(r[9])


def test_padded_unified_sizes_closed_form():
    """The unified-pool sizing mode: the block grows to whole attention pages, nothing else."""
    specs = {"tiny_fp32": inputs.TINY, "jamba_mini_like": inputs.JAMBA_MINI}
    for name, state_dtype, k, page, native, padded in _rows("padded_unified_sizes.txt"):
        spec = specs[name]
        if state_dtype != "f32":
            spec = inputs.with_state_dtype(spec, state_dtype)
        if int(k):
            spec = inputs.with_conv(spec, int(k))
        plain, pad = _shape(spec), _shape(inputs.with_padded_blocks(spec))
        assert plain.unit_bytes(orc.POOL_KV) == pad.unit_bytes(orc.POOL_KV) == int(page)
        assert plain.unit_bytes(orc.POOL_SSM) == pad.native_ssm_bytes() == int(native)
        assert pad.unit_bytes(orc.POOL_SSM) == int(padded) and int(padded) % int(page) == 0
        # the generator's size arithmetic agrees
        assert inputs.with_padded_blocks(spec).ssm_block_bytes == int(padded)
        assert inputs.with_padded_blocks(spec).ssm_native_bytes == int(native)
    # with padding a budget holds fewer blocks: same arena, capacities by the padded unit
    sh = _shape(inputs.with_padded_blocks(inputs.TINY))
    p = orc.Pools(sh, 4 * 16384 + 4 * 16384, 4, 4, with_data=False)
    assert p.unit[1] == 16384 and p.gap == 0
    assert p.migrate(0, 1).recipient_gain == 1          # a page buys one padded block, not two


def test_alignment_rules():
    # odd shapes: units round up to 16 B, slab anchors to 128 B
    sh = orc.Shape("bf16", 16, 3, 1, 9, 1, 3, 5)
    assert sh.unit_bytes(0) % 16 == 0 and sh.unit_bytes(0) >= 16 * 2 * 9 * 2
    assert sh.unit_bytes(1) % 16 == 0 and sh.unit_bytes(1) >= 15 * 4
    p = orc.Pools(sh, 100000 + 77, 20, 30)
    assert p.usable % 128 == 0 and p.usable <= 100077
    for pool in (0, 1):
        for s in range(p.capacity[pool]):
            assert p.byte_offset(pool, s) % 16 == 0
            assert 0 <= p.byte_offset(pool, s) <= p.usable - p.unit[pool]
    # regions never overlap: top of KV region <= bottom of SSM region
    assert p.capacity[0] * p.unit[0] + p.gap == p.usable - p.capacity[1] * p.unit[1]


# ---- P6: allocate/free outcomes equal a two-counter model ---------------------
def _random_trace(p, rng, n_ops, pools=(0, 1), max_n=5):
    """Drive p with a random alloc/free trace; yield (op, code, payload)."""
    live = {0: [], 1: []}
    for _ in range(n_ops):
        pool = int(rng.choice(pools))
        if rng.random() < 0.55 or not live[pool]:
            n = int(rng.integers(1, max_n + 1))
            code, hs = p.alloc(pool, n)
            live[pool].extend(hs)
            yield ("alloc", pool, n, code, tuple(hs))
        else:
            k = int(rng.integers(1, min(max_n, len(live[pool])) + 1))
            idx = rng.choice(len(live[pool]), size=k, replace=False)
            hs = [live[pool][i] for i in idx]
            for i in sorted(idx, reverse=True):
                live[pool].pop(int(i))
            yield ("free", pool, k, p.free(hs), tuple(hs))


def test_static_mode_equals_two_counter_model():
    rng = np.random.default_rng(11)
    unit_kv, unit_ssm = TINY.unit_bytes(0), TINY.unit_bytes(1)
    cap = [13, 6]
    arena = cap[0] * unit_kv + cap[1] * unit_ssm
    prng = np.random.default_rng(5)
    p = orc.Pools(TINY, arena, cap[0], cap[1],
                  slot_rank=[prng.permutation(arena // unit_kv), prng.permutation(arena // unit_ssm)],
                  with_data=False)
    used = [0, 0]
    n_err = 0
    for op, pool, n, code, hs in _random_trace(p, rng, 4000):
        if op == "alloc":
            if used[pool] + n <= cap[pool]:
                assert code == orc.OK and len(hs) == n
                used[pool] += n
            else:
                assert code == orc.ERR_CAPACITY and hs == ()
                n_err += 1
        else:
            assert code == orc.OK
            used[pool] -= n
        st = p.stats()
        assert st["live"] == tuple(used)
        assert st["free"] == (cap[0] - used[0], cap[1] - used[1])
        assert st["capacity_errors"] == n_err
    assert n_err > 50          # the trace really exercised the failure path


def test_alloc_picks_lowest_vid_and_best_ranked_slot_bruteforce():
    rng = np.random.default_rng(3)
    unit_kv, unit_ssm = TINY.unit_bytes(0), TINY.unit_bytes(1)
    arena = 9 * unit_kv + 4 * unit_ssm
    ranks = [rng.permutation(arena // unit_kv), rng.permutation(arena // unit_ssm)]
    p = orc.Pools(TINY, arena, 9, 4, slot_rank=ranks, with_data=False)
    mapped = [dict(), dict()]            # independent model: vid -> slot
    for op, pool, n, code, hs in _random_trace(p, rng, 1500, max_n=3):
        if op == "alloc" and code == orc.OK:
            for h in hs:
                tag, vid = h >> 30, h & 0x3FFFFFFF
                assert tag == pool
                free_vids = [v for v in range(p.max_vid[pool]) if v not in mapped[pool]]
                assert vid == free_vids[0]
                taken = set(mapped[pool].values())
                free_slots = [s for s in range(p.capacity[pool]) if s not in taken]
                best = min(free_slots, key=lambda s: ranks[pool][s])
                assert p.resolve(h)[1] == best
                mapped[pool][vid] = best
        elif op == "free":
            for h in hs:
                del mapped[pool][h & 0x3FFFFFFF]
    # every live handle resolves to a distinct slot
    for pool in (0, 1):
        assert len(set(mapped[pool].values())) == len(mapped[pool])


def test_invalid_calls_change_nothing():
    unit_kv, unit_ssm = TINY.unit_bytes(0), TINY.unit_bytes(1)
    p = orc.Pools(TINY, 4 * unit_kv + 2 * unit_ssm, 4, 2, with_data=False)
    _, hs = p.alloc(0, 2)
    before = (p.stats(), p.slot_of[0].copy(), p.slot_of[1].copy())

    def unchanged(ops_delta):
        st = p.stats()
        want = dict(before[0])
        want["ops"] += ops_delta
        assert st == want
        assert np.array_equal(p.slot_of[0], before[1]) and np.array_equal(p.slot_of[1], before[2])

    assert p.alloc(0, 0) == (orc.ERR_INVALID_ARG, [])
    assert p.alloc(2, 1) == (orc.ERR_INVALID_ARG, [])
    assert p.free([]) == orc.ERR_INVALID_ARG
    unchanged(0)
    assert p.free([orc.encode_handle(0, 3)]) == orc.ERR_INVALID_HANDLE        # never allocated
    assert p.free([hs[0], hs[0]]) == orc.ERR_INVALID_HANDLE                   # duplicate in one call
    assert p.free([hs[0], orc.encode_handle(1, 0)]) == orc.ERR_INVALID_HANDLE  # one bad spoils all
    assert p.free([orc.INVALID_HANDLE]) == orc.ERR_INVALID_HANDLE
    assert p.free([orc.encode_handle(2, 0)]) == orc.ERR_INVALID_HANDLE        # unknown pool tag
    unchanged(5)
    assert p.free([hs[0]]) == orc.OK
    assert p.free([hs[0]]) == orc.ERR_INVALID_HANDLE                          # stale handle
    assert p.resolve(hs[0]) is None and p.resolve(hs[1]) is not None


# ---- P7: migration -------------------------------------------------------------
def _snapshot(p, handles):
    return {h: (p.resolve(h), bytes(p.unit_view(h))) for h in handles}


def test_tiny_migration_four_pages_become_eight_blocks():
    sc = inputs.make_scenario(inputs.TINY, "tiny", 4, seed=1001, headroom=1.0,
                              ctx=[16, 16, 16, 16])
    unit_kv, unit_ssm = TINY.unit_bytes(0), TINY.unit_bytes(1)
    arena = 64 * unit_kv + 8 * unit_ssm
    p = orc.Pools(TINY, arena, 64, 8)
    r = p.migrate(orc.POOL_KV, 4)
    assert r.code == orc.OK
    assert (r.units_copied, r.recipient_gain, r.bytes_wasted) == (0, 8, 0)
    assert p.stats()["capacity"] == (60, 16)
    assert p.stats()["bytes_migrated"] == 4 * 16384
    assert sc.batch == 4


def test_migration_preserves_contents_and_handles():
    rng = np.random.default_rng(21)
    unit_kv, unit_ssm = TINY.unit_bytes(0), TINY.unit_bytes(1)
    arena = 40 * unit_kv + 10 * unit_ssm + 128 * 3       # some initial gap too
    ranks = [rng.permutation(arena // unit_kv), rng.permutation(arena // unit_ssm)]
    p = orc.Pools(TINY, arena, 40, 10, slot_rank=ranks)
    p.arena[:] = rng.integers(0, 256, size=p.usable, dtype=np.uint8)
    _, kv = p.alloc(0, 30)
    _, ss = p.alloc(1, 7)
    for h in kv + ss:
        p.unit_view(h)[:] = rng.integers(0, 256, size=p.unit_view(h).size, dtype=np.uint8)
    p.free(kv[::3])
    kv = [h for i, h in enumerate(kv) if i % 3]
    usable = p.usable

    def conserved():
        st = p.stats()
        assert st["capacity"][0] * unit_kv + st["capacity"][1] * unit_ssm + st["gap_bytes"] == usable

    conserved()
    for donor, n in ((0, 9), (1, 2), (0, 5), (1, 3), (0, 1)):
        snap = _snapshot(p, kv + ss)
        st0 = p.stats()
        r = p.migrate(donor, n)
        assert r.code == orc.OK
        st1 = p.stats()
        recip = 1 - donor
        avail = st0["gap_bytes"] + n * p.unit[donor]
        assert st1["capacity"][donor] == st0["capacity"][donor] - n
        assert st1["capacity"][recip] == st0["capacity"][recip] + avail // p.unit[recip]
        assert r.bytes_wasted == avail % p.unit[recip] == st1["gap_bytes"]
        assert st1["live"] == st0["live"]
        conserved()
        for h in kv + ss:
            pool, slot, off = p.resolve(h)
            assert slot < p.capacity[pool]                      # nothing left above the new capacity
            assert bytes(p.unit_view(h)) == snap[h][1]          # byte-identical contents
            if snap[h][0][1] < p.capacity[pool] and pool == donor:
                assert slot == snap[h][0][1] or snap[h][0][1] >= st1["capacity"][donor]
        # moved units are exactly the live ones that sat in the vacated range, ascending
        vacated = [snap[h][0][1] for h in kv + ss
                   if snap[h][0][0] == donor and snap[h][0][1] >= st1["capacity"][donor]]
        assert [m[0] for m in r.moves] == sorted(vacated)
        assert r.units_copied == len(vacated)
        # all resolved slots distinct per pool
        for pool, hs in ((0, kv), (1, ss)):
            slots = [p.resolve(h)[1] for h in hs]
            assert len(set(slots)) == len(slots)


def test_failed_migration_is_a_no_op_and_round_trip_restores_capacity():
    unit_kv, unit_ssm = TINY.unit_bytes(0), TINY.unit_bytes(1)
    arena = 20 * unit_kv + 5 * unit_ssm
    p = orc.Pools(TINY, arena, 20, 5)
    _, kv = p.alloc(0, 15)
    snap = _snapshot(p, kv)
    st0 = p.stats()
    assert p.migrate(0, 6).code == orc.ERR_CAPACITY          # only 5 free
    assert p.migrate(0, 21).code == orc.ERR_CAPACITY         # more than the pool holds
    assert p.migrate(0, 0).code == orc.ERR_INVALID_ARG
    assert p.migrate(2, 1).code == orc.ERR_INVALID_ARG
    st1 = p.stats()
    st0["ops"] += 2                                          # the two refused calls still count as ops
    assert st1 == st0
    assert _snapshot(p, kv) == snap
    # an odd number of pages leaves a remainder; going back picks it up again
    r = p.migrate(0, 3)                                      # 3 pages = 48 KiB -> 6 blocks of 8 KiB
    assert (r.recipient_gain, r.bytes_wasted) == (6, 0)
    r = p.migrate(1, 5)                                      # 5 blocks = 40 KiB -> 2 pages + 8 KiB waste
    assert (r.recipient_gain, r.bytes_wasted) == (2, 8192)
    r = p.migrate(1, 1)                                      # 8 KiB + 8 KiB gap -> 1 page, waste 0
    assert (r.recipient_gain, r.bytes_wasted) == (1, 0)
    assert p.stats()["capacity"] == (20, 5)
    assert p.stats()["bytes_wasted"] == 8192
    assert _snapshot(p, kv).keys() == snap.keys()
    for h in kv:
        assert bytes(p.unit_view(h)) == snap[h][1]


def test_counter_model_holds_with_new_capacities_after_migration():
    rng = np.random.default_rng(5)
    unit_kv, unit_ssm = TINY.unit_bytes(0), TINY.unit_bytes(1)
    p = orc.Pools(TINY, 16 * unit_kv + 6 * unit_ssm, 16, 6, with_data=False)
    assert p.alloc(1, 7)[0] == orc.ERR_CAPACITY
    assert p.migrate(0, 4).code == orc.OK                     # +8 blocks
    cap = list(p.stats()["capacity"])
    assert cap == [12, 14]
    used = [0, 0]
    for op, pool, n, code, hs in _random_trace(p, rng, 1500):
        if op == "alloc":
            ok = used[pool] + n <= cap[pool]
            assert code == (orc.OK if ok else orc.ERR_CAPACITY)
            used[pool] += n if ok else 0
        else:
            used[pool] -= n


# ---- P8: determinism -------------------------------------------------------------
def test_same_trace_twice_is_identical():
    unit_kv, unit_ssm = TINY.unit_bytes(0), TINY.unit_bytes(1)
    arena = 30 * unit_kv + 9 * unit_ssm
    logs = []
    for _ in range(2):
        prng = np.random.default_rng(77)
        p = orc.Pools(TINY, arena, 30, 9, slot_rank=[prng.permutation(arena // unit_kv),
                                                      prng.permutation(arena // unit_ssm)],
                      with_data=False)
        rng = np.random.default_rng(9)
        log = []
        for i, ev in enumerate(_random_trace(p, rng, 1200)):
            log.append(ev)
            if i % 200 == 199:
                r = p.migrate(i // 200 % 2, 2)
                log.append((r.code, r.units_copied, r.recipient_gain, r.bytes_wasted, tuple(r.moves)))
        log.append(tuple(sorted(p.stats().items())))
        logs.append(log)
    assert logs[0] == logs[1]


def test_absorb_gap_closed_forms_and_round_trip():
    """The gap's whole units go to the pool that asks; the remainder stays; nothing else moves."""
    uk, us = TINY.unit_bytes(0), TINY.unit_bytes(1)          # 16 KiB, 8 KiB
    extra = 3 * uk + us // 2
    p = orc.Pools(TINY, 6 * uk + 4 * us + extra, 6, 4, with_data=False)
    assert p.gap == extra - extra % 128 or p.gap == extra     # usable is the arena rounded down to 128
    g0 = p.gap
    _, live = p.alloc(0, 6)
    before = p.stats()
    assert p.absorb_gap(2).code == orc.ERR_INVALID_ARG and p.stats() == before     # bad pool: not even counted
    r = p.absorb_gap(0)
    assert (r.code, r.units_copied, r.recipient_gain, r.bytes_wasted) == (orc.OK, 0, g0 // uk, g0 % uk)
    st = p.stats()
    assert st["capacity"] == (6 + g0 // uk, 4) and st["gap_bytes"] == g0 % uk
    assert st["capacity"][0] * uk + st["capacity"][1] * us + st["gap_bytes"] == p.usable
    assert (st["migrations"], st["units_copied"], st["bytes_migrated"], st["bytes_wasted"]) == (1, 0, 0, g0 % uk)
    assert st["ops"] == before["ops"] + 1
    # exactly the gained pages can be allocated now, in the slots just above the old capacity
    code, hs = p.alloc(0, g0 // uk)
    assert code == orc.OK and sorted(p.resolve(h)[1] for h in hs) == list(range(6, 6 + g0 // uk))
    assert p.alloc(0, 1)[0] == orc.ERR_CAPACITY
    assert [p.resolve(h)[1] for h in live] == list(range(6))                        # nobody moved
    # a gap smaller than one unit: refused, nothing changes but the operation counter
    before = p.stats()
    r = p.absorb_gap(0)
    after = p.stats()
    assert r.code == orc.ERR_CAPACITY and {**after, "ops": before["ops"]} == before
    # what a migration leaves over can be taken back: one block to the page pool leaves 8 KiB in the gap
    q = orc.Pools(TINY, 4 * uk + 4 * us, 4, 4, with_data=False)
    assert q.migrate(1, 1).recipient_gain == 0 and q.gap == us and q.stats()["capacity"] == (4, 3)
    assert q.absorb_gap(1).recipient_gain == 1 and q.gap == 0 and q.stats()["capacity"] == (4, 4)
