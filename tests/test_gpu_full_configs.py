"""GPU parity at the workloads' full sizes, in the launch configuration bench.py
times.  The oracle cannot walk these arenas whole, so outputs are checked on
sampled requests it computes one by one (a request's outputs depend on its own
units only, and unit contents are a pure function of the seed), and the
integer side is checked against the oracle's metadata-only pools where those
finish in seconds, else through properties that hold at any size."""
import numpy as np
import pytest

from oracle import avmp_oracle as orc
from oracle.sampled import RequestReference
from gen import inputs
from tests import helpers

pytestmark = pytest.mark.gpu

TOL = 2e-3      # bf16 in / fp32 accumulate


def _session(sc, **kw):
    import torch
    from paper_2605_22416_amd.session import DeviceSession
    torch.cuda.empty_cache()
    return DeviceSession(sc, **kw)


def _first_layers(inp, n_attn, n_ssm):
    """Step inputs restricted to the first layers of each kind (A has no batch axis)."""
    return {k: (v[:n_attn] if k == "q" else v[:n_ssm]) for k, v in inp.items()}


def _check_sample(ses, refs, inp, o, y, what, conv=None, tol_state=TOL, tol_y=TOL):
    """refs: request -> RequestReference, built on the full model or on its first layers."""
    for r, ref in refs.items():
        na, ns = ref.spec.n_attn, ref.spec.n_ssm
        ro, ry = ref.step(_first_layers(inp, na, ns),
                          None if conv is None else (conv[0][:ns], conv[1][:ns]))
        eo = helpers.rel_err_rows(o[:na, r], ro).max() if ro.size else 0.0
        ey = helpers.rel_err_rows(y[:ns, r], ry).max()
        assert np.isfinite(o[:, r]).all() and np.isfinite(y[:, r]).all()
        assert eo <= TOL and ey <= tol_y, "%s request %d: attention %.3g ssm %.3g" % (what, r, eo, ey)
        for ls in sorted({0, ns - 1}):
            got = ses.states(ls, [r])[0]
            assert helpers.rel_err_rows(got, ref.state(ls)).max() <= tol_state, "%s state r=%d" % (what, r)


def _sample(sc, k, rng, always=()):
    picks = set(int(i) for i in always)
    picks.add(int(np.argmin(sc.ctx)))
    picks.add(int(np.argmax(sc.ctx)))
    while len(picks) < k:
        picks.add(int(rng.integers(0, sc.batch)))
    return sorted(picks)


def _check_handles_resolve_everywhere(ses, handles):
    """Host resolve and device translation agree, slots are distinct and below capacity."""
    from paper_2605_22416_amd import binding as av
    hs = np.asarray(handles, dtype=np.uint32).reshape(-1)
    dev = ses.translate(hs)
    st = av.avmp_stats(ses.p)
    seen = set()
    for h, off in zip(hs, dev):
        rc, pool, slot, hoff = av.avmp_resolve(ses.p, int(h))
        assert rc == av.AVMP_OK and off == hoff
        assert slot < st["capacity"][pool] and (pool, slot) not in seen
        seen.add((pool, slot))


def test_jamba_batch64_uniform_short_full_size():
    """Config 2, exactly as bench.py runs it: two steps, sampled requests."""
    from paper_2605_22416_amd import binding as av
    spec = inputs.JAMBA_MINI
    sc = inputs.make_scenario(spec, "uniform_short", 64, seed=1002)
    ses = _session(sc, fill_byte=None)
    ses.fill(threads=16)
    op, kv, ssm = helpers.build_oracle(sc, with_data=False)       # integer side, whole config
    assert np.array_equal(ses.kv, kv) and np.array_equal(ses.ssm, ssm)
    assert av.avmp_stats(ses.p) == op.stats()
    rng = np.random.default_rng(0)
    sample = _sample(sc, 6, rng)
    refs = {r: RequestReference(spec, sc.seed, r, int(sc.ctx[r])) for r in sample}
    for step in range(2):
        inp = inputs.step_inputs(spec, sc.batch, sc.seed, step=step)
        o, y = ses.step(inp)
        _check_sample(ses, refs, inp, o, y, "cfg2 step %d" % step)
    ses.close()


@pytest.mark.parametrize("state_dtype,conv_kernel", [("f32", 4), ("bf16", 0), ("bf16", 4)])
def test_jamba_batch64_variants_of_the_ssm_block(state_dtype, conv_kernel):
    """Config 2's batch, contexts and head shapes (one block of 1 attention + 7 SSM
    layers) with the block variants: state stored as bf16, a 4-tap convolution
    window, both.  Three steps, sampled requests.

    With a bf16 state the stored codes of the two sides part by one ulp where the
    exact value sits on a rounding tie (fp32 against float64 arithmetic).  So that
    every step is held to the 2e-3 bar on its own, one set of references is re-based
    before each later step: its blocks are loaded with the bytes the GPU has stored,
    and that step's y must then agree within 2e-3 and its state within one bf16 ulp.
    A second set is never re-based and bounds the drift over the steps (state one
    ulp of the row maximum per step taken, y one ulp)."""
    base = inputs.scaled_down(inputs.JAMBA_MINI, 1)
    spec = inputs.with_state_dtype(base, state_dtype) if state_dtype != "f32" else base
    if conv_kernel:
        spec = inputs.with_conv(spec, conv_kernel)
    sc = inputs.make_scenario(spec, "uniform_short", 64, seed=1002)
    ses = _session(sc, fill_byte=None)
    ses.fill(threads=16)
    conv = inputs.conv_weights(spec, sc.seed) if conv_kernel else None
    rng = np.random.default_rng(5)
    sample = _sample(sc, 5, rng)
    free_run = {r: RequestReference(spec, sc.seed, r, int(sc.ctx[r])) for r in sample}
    rebased = {r: RequestReference(spec, sc.seed, r, int(sc.ctx[r])) for r in sample} \
        if state_dtype == "bf16" else None
    ulp = 2.0 ** -7
    for step in range(3):
        inp = inputs.step_inputs(spec, sc.batch, sc.seed, step=step)
        if rebased is not None and step > 0:
            for r, ref in rebased.items():
                for ls in range(spec.n_ssm):
                    ref.load_block(ls, ses.read_unit(int(ses.ssm[ls, r])))
        o, y = ses.step(inp, conv=conv)
        what = "%s conv %d step %d" % (state_dtype, conv_kernel, step)
        _check_sample(ses, free_run, inp, o, y, what + " (drift)", conv=conv,
                      tol_state=TOL if state_dtype == "f32" else ulp * (step + 1),
                      tol_y=TOL if state_dtype == "f32" or step == 0 else ulp)
        if rebased is not None:
            _check_sample(ses, rebased, inp, o, y, what + " (from the stored state)", conv=conv,
                          tol_state=ulp, tol_y=TOL)
    ses.close()


@pytest.mark.parametrize("state_dtype,batch,conv_kernel", [
    ("f32", 112, 4),      # 1024-thread recurrence kernel, convolution as a launch of its own
    ("bf16", 112, 4),     # a head per workgroup, convolution inside
    ("bf16", 232, 4),     # two heads per workgroup of 1024 threads, convolution inside
    ("bf16", 160, 0),     # a head per workgroup, arithmetic before the state loads
    ("bf16", 232, 0),     # two heads per workgroup, arithmetic before the state loads
])
def test_long_launches_of_the_recurrence_kernels(state_dtype, batch, conv_kernel):
    """Batches of 112 ... 232 requests at the Jamba head shapes (1 attention + 7 SSM layers):
    launches long enough for the forms of the recurrence kernels that short launches do not
    reach.  Four steps, so that a convolution window's rows for B and C, which every workgroup
    of a request reads and the last of them moves on, turn over completely; sampled requests,
    windows compared byte for byte after every step."""
    base = inputs.scaled_down(inputs.JAMBA_MINI, 1)
    spec = inputs.with_state_dtype(base, state_dtype) if state_dtype != "f32" else base
    if conv_kernel:
        spec = inputs.with_conv(spec, conv_kernel)
    sc = inputs.make_scenario(spec, "uniform_short", batch, seed=1006)
    ses = _session(sc, fill_byte=0xFF)
    rng = np.random.default_rng(6)
    sample = _sample(sc, 5, rng, always=[0, sc.batch - 1])
    ses.fill(threads=16, requests=sample)
    conv = inputs.conv_weights(spec, sc.seed) if conv_kernel else None
    refs = {r: RequestReference(spec, sc.seed, r, int(sc.ctx[r])) for r in sample}
    a, n = spec.ssm_state_bytes, spec.conv_window_bytes
    ulp = 2.0 ** -7
    for step in range(4):
        inp = inputs.step_inputs(spec, sc.batch, sc.seed, step=step)
        if state_dtype == "bf16" and step > 0:       # each step judged from the state the GPU stored
            for r, ref in refs.items():
                for ls in range(spec.n_ssm):
                    ref.load_block(ls, ses.read_unit(int(ses.ssm[ls, r])))
        o, y = ses.step(inp, conv=conv)
        _check_sample(ses, refs, inp, o, y, "%s state, batch %d, conv %d, step %d" % (state_dtype, batch, conv_kernel, step),
                      conv=conv, tol_state=TOL if state_dtype == "f32" else ulp)
        for r, ref in refs.items():
            for ls in range(spec.n_ssm if conv_kernel else 0):
                assert np.array_equal(ses.read_unit(int(ses.ssm[ls, r]))[a: a + n],
                                      ref.pools.unit_view(int(ref.ssm[ls, 0]))[a: a + n]), \
                    "window of layer %d request %d after step %d" % (ls, r, step)
    ses.close()


def test_mixed_long_batch32_with_migration_there_and_back():
    """Config 3: long-context mix, KV pool at 95 % occupancy; 1024 pages of
    capacity move to the SSM pool between two steps and come back before a third."""
    from paper_2605_22416_amd import binding as av
    spec = inputs.JAMBA_MINI
    sc = inputs.make_scenario(spec, "mixed_long", 32, seed=1003, occupancy=0.95)
    ses = _session(sc, fill_byte=None)
    ses.fill(threads=16)
    op, kv, ssm = helpers.build_oracle(sc, with_data=False)
    assert np.array_equal(ses.kv, kv) and np.array_equal(ses.ssm, ssm)
    rng = np.random.default_rng(1)
    sample = _sample(sc, 4, rng)
    refs = {r: RequestReference(spec, sc.seed, r, int(sc.ctx[r])) for r in sample}
    watch = np.concatenate([ses.kv[:, r, : sc.n_pages[r]].reshape(-1) for r in sample] + [ses.ssm.reshape(-1)])
    cap0 = av.avmp_stats(ses.p)["capacity"]
    for step, mig in enumerate(((0, 1024), (1, 16), None)):
        inp = inputs.step_inputs(spec, sc.batch, sc.seed, step=step)
        o, y = ses.step(inp)
        _check_sample(ses, refs, inp, o, y, "cfg3 step %d" % step)
        if mig is None:
            break
        ores = op.migrate(*mig)
        rc, res = av.avmp_migrate(ses.p, *mig)
        assert rc == ores.code == orc.OK
        assert (res.units_copied, res.recipient_gain, res.bytes_wasted) == \
            (ores.units_copied, ores.recipient_gain, ores.bytes_wasted)
        assert av.avmp_stats(ses.p) == op.stats()
        _check_handles_resolve_everywhere(ses, watch)
        for h in watch[:: 97]:
            assert av.avmp_resolve(ses.p, int(h))[1:] == op.resolve(int(h))
        if step == 0:
            assert res.units_copied > 800          # the pool is 95 % full: most vacated slots were live
    assert av.avmp_stats(ses.p)["capacity"] == cap0      # there and back restores the split exactly
    ses.close()


def test_agentic_burst_batch256_churn_and_migration():
    """Config 4: 256 requests, half newly admitted with zeroed SSM blocks; a
    seeded churn of 512 handles and a 512-page migration precede the step."""
    from paper_2605_22416_amd import binding as av
    spec = inputs.JAMBA_MINI
    sc = inputs.make_scenario(spec, "agentic_burst", 256, seed=1004)
    ses = _session(sc, fill_byte=0xFF)          # anything not written reads as NaN
    op, kv, ssm = helpers.build_oracle(sc, with_data=False)
    assert np.array_equal(ses.kv, kv) and np.array_equal(ses.ssm, ssm)
    rng = np.random.default_rng(2)
    fresh_one = int(np.flatnonzero(sc.fresh)[3])
    sample = _sample(sc, 5, rng, always=[fresh_one])
    ses.fill(threads=16, requests=sample)
    refs = {r: RequestReference(spec, sc.seed, r, int(sc.ctx[r]), bool(sc.fresh[r])) for r in sample}
    # requests that finished earlier still hold pages: 384 ghost pages + 32 ghost blocks
    ghosts = []
    for pool, n in ((0, 384), (1, 32)):
        oc, oh = op.alloc(pool, n)
        lc, lh = av.avmp_alloc(ses.p, pool, n)
        assert oc == lc == orc.OK and list(lh) == oh
        ghosts.extend(oh)
    for step in range(2):
        # churn: 256 handles freed, 256 allocated (7/8 KV pages, 1/8 SSM blocks)
        drop = [ghosts.pop(int(rng.integers(0, len(ghosts)))) for _ in range(256)]
        assert op.free(drop) == av.avmp_free(ses.p, drop) == orc.OK
        for pool, n in ((0, 224), (1, 32)):
            oc, oh = op.alloc(pool, n)
            lc, lh = av.avmp_alloc(ses.p, pool, n)
            assert oc == lc == orc.OK and list(lh) == oh
            ghosts.extend(oh)
        donor, n = ((0, 512), (1, 8))[step]
        ores = op.migrate(donor, n)
        rc, res = av.avmp_migrate(ses.p, donor, n)
        assert rc == ores.code == orc.OK
        assert (res.units_copied, res.recipient_gain) == (ores.units_copied, ores.recipient_gain)
        assert av.avmp_stats(ses.p) == op.stats()
        inp = inputs.step_inputs(spec, sc.batch, sc.seed, step=step)
        o, y = ses.step(inp)
        _check_sample(ses, refs, inp, o, y, "cfg4 step %d" % step)
    ses.close()


def _expected_fresh_allocation(sc):
    """Closed form of the scenario's allocation sequence on fresh pools: the k-th unit a pool
    hands out gets virtual id k and the slot of k-th lowest rank below the pool's capacity.
    Returns per pool (handle tables as the session lays them out, slot of every id)."""
    spec = sc.spec
    slot_of = []
    for pool, cap in ((0, sc.kv_capacity), (1, sc.ssm_capacity)):
        below = np.arange(cap, dtype=np.int64)
        slot_of.append(below[np.argsort(sc.slot_rank[pool][:cap], kind="stable")])
    kv = np.full((spec.n_attn, sc.batch, sc.max_pages), 0xFFFFFFFF, dtype=np.uint32)
    ssm = np.zeros((spec.n_ssm, sc.batch), dtype=np.uint32)
    next_id = [0, 0]
    for r in range(sc.batch):
        n = int(sc.n_pages[r])
        for la in range(spec.n_attn):
            kv[la, r, :n] = np.arange(next_id[0], next_id[0] + n, dtype=np.uint32)      # tag 0
            next_id[0] += n
        ssm[:, r] = (1 << 30) | np.arange(next_id[1], next_id[1] + spec.n_ssm, dtype=np.uint32)
        next_id[1] += spec.n_ssm
    return kv, ssm, [slot_of[0][: next_id[0]].copy(), slot_of[1][: next_id[1]].copy()]


def _expected_migration(slot_of_kv, rank, cap, n):
    """The copy rule on the KV pool in closed form: live slots at or above the new capacity,
    ascending, move to the free slots below it of lowest rank, best rank first."""
    newcap = cap - n
    live = np.zeros(cap, dtype=bool)
    live[slot_of_kv] = True
    src = np.flatnonzero(live[newcap:]) + newcap
    free = np.flatnonzero(~live[:newcap])
    dst = free[np.argsort(rank[free], kind="stable")[: len(src)]]
    remap = np.arange(cap, dtype=np.int64)
    remap[src] = dst
    return remap[slot_of_kv], len(src)


def test_capacity_scale_pools_200gb_long_contexts_and_migration_sweep():
    """Config 5: pools filling about 200 GB, batch 512 + 4 requests of 262144 tokens.
    Every handle the 3.4 M allocations returned and every slot behind it (device
    translation of all of them) against the closed form for fresh pools; sampled
    outputs; then the migration sweep of 64, 1024 and 16384 pages, after each of
    which the whole device table must equal the copy rule evaluated in numpy.  (The
    262144-token requests have the next test to themselves.)"""
    import torch
    from paper_2605_22416_amd import binding as av
    free_b, total_b = torch.cuda.mem_get_info()
    if total_b < 250e9:
        pytest.skip("needs a 288 GB device")
    spec = inputs.JAMBA_MINI
    sc = inputs.make_scenario(spec, "capacity", 512, seed=1005, headroom=1.7)
    assert 190e9 < sc.arena_bytes < 215e9
    ses = _session(sc, fill_byte=0)
    # ---- allocation: handles and slots, all of them ------------------------------------------
    want_kv, want_ssm, slot_of = _expected_fresh_allocation(sc)
    assert np.array_equal(ses.kv, want_kv) and np.array_equal(ses.ssm, want_ssm)
    usable = sc.arena_bytes // 128 * 128
    all_kv = np.arange(len(slot_of[0]), dtype=np.uint32)
    all_ssm = (1 << 30) | np.arange(len(slot_of[1]), dtype=np.uint32)

    def check_device_table(what):
        got = ses.translate(all_kv)
        assert np.array_equal(got, slot_of[0].astype(np.uint64) * np.uint64(spec.kv_page_bytes)), what
        got = ses.translate(all_ssm)
        assert np.array_equal(got, np.uint64(usable) - (slot_of[1].astype(np.uint64) + np.uint64(1))
                              * np.uint64(spec.ssm_block_bytes)), what
    check_device_table("after allocation")
    for h in np.concatenate([all_kv[:: 100003], all_ssm[:: 1009]]):       # the host table, sampled
        rc, pool, slot, off = av.avmp_resolve(ses.p, int(h))
        assert rc == av.AVMP_OK and slot == slot_of[pool][int(h) & 0x3FFFFFFF]
    # ---- one decode step, sampled requests -----------------------------------------------------
    rng = np.random.default_rng(3)
    sample = [int(np.argmin(sc.ctx)), int(rng.integers(0, 512)), int(rng.integers(0, 512))]
    ses.fill(threads=16, requests=sample)
    inp = inputs.step_inputs(spec, sc.batch, sc.seed)
    watch = np.concatenate([ses.kv[:, r, : sc.n_pages[r]].reshape(-1)[:: 11] for r in sample]
                           + [ses.ssm[:, sample].reshape(-1)])
    before = {int(h): ses.read_unit(int(h)).copy() for h in watch[:: 7]}
    o, y = ses.step(inp)
    refs = {r: RequestReference(spec, sc.seed, r, int(sc.ctx[r])) for r in sample}
    _check_sample(ses, refs, inp, o, y, "cfg5")
    # ---- the migration sweep --------------------------------------------------------------------
    for n in (64, 1024, 16384):
        st0 = av.avmp_stats(ses.p)
        rc, res = av.avmp_migrate(ses.p, 0, n)
        assert rc == av.AVMP_OK
        st1 = av.avmp_stats(ses.p)
        avail = st0["gap_bytes"] + n * spec.kv_page_bytes
        assert st1["capacity"] == (st0["capacity"][0] - n, st0["capacity"][1] + avail // spec.ssm_block_bytes)
        assert res.bytes_wasted == avail % spec.ssm_block_bytes == st1["gap_bytes"]
        assert st1["capacity"][0] * spec.kv_page_bytes + st1["capacity"][1] * spec.ssm_block_bytes \
            + st1["gap_bytes"] == usable
        slot_of[0], moved = _expected_migration(slot_of[0], sc.slot_rank[0], st0["capacity"][0], n)
        assert st1["live"] == st0["live"] and res.units_copied == moved and 0 < moved <= n
        check_device_table("after migrating %d pages" % n)
        for h in watch:
            rc, pool, slot, off = av.avmp_resolve(ses.p, int(h))
            assert rc == av.AVMP_OK and slot == slot_of[pool][int(h) & 0x3FFFFFFF]
    for h, data in before.items():
        if (h >> 30) == 0:            # KV pages are read-only in a step; SSM blocks were updated by it
            assert np.array_equal(ses.read_unit(h), data)
    # the step after the migrations reproduces the attention rows bit for bit
    o2, y2 = ses.step(inp)
    assert np.array_equal(o2[:, sample], o[:, sample])
    assert av.avmp_migrate(ses.p, 0, 1 << 29)[0] == av.AVMP_ERR_CAPACITY     # refused, nothing changes
    assert av.avmp_stats(ses.p)["capacity"] == st1["capacity"]
    ses.close()


def test_capacity_scale_262144_token_request_on_every_attention_layer():
    """Config 5's launch configuration (batch 512 + 4 x 262144 tokens, 198 GB arena); one
    of the 262144-token requests is checked against the oracle on all four attention
    layers, one layer at a time (the oracle needs about 10 s and 10 GB per layer at that
    length), each with the SSM layer that follows it in the model."""
    import torch
    free_b, total_b = torch.cuda.mem_get_info()
    if total_b < 250e9:
        pytest.skip("needs a 288 GB device")
    spec = inputs.JAMBA_MINI
    sc = inputs.make_scenario(spec, "capacity", 512, seed=1005, headroom=1.7)
    ses = _session(sc, fill_byte=0)
    longest = int(np.argmax(sc.ctx)) + 2            # the third of the four
    assert sc.ctx[longest] == 262144
    ses.fill(threads=16, requests=[longest])
    inp = inputs.step_inputs(spec, sc.batch, sc.seed)
    o, y = ses.step(inp)
    for la in range(spec.n_attn):
        one = inputs.ModelSpec("layer%d" % la, spec.dtype, spec.page_tokens, spec.n_q_heads,
                               spec.n_kv_heads, spec.head_dim, spec.ssm_heads, spec.ssm_headdim,
                               spec.ssm_dstate, (inputs.ATTN, inputs.SSM), spec.scale_inputs)
        ls = 7 * la + 4                             # the SSM layer right behind attention layer la
        ref = RequestReference(one, sc.seed, longest, 262144, attn_ordinals=[la], ssm_ordinals=[ls])
        cut = {k: (v[la: la + 1] if k == "q" else v[ls: ls + 1]) for k, v in inp.items()}
        ro, ry = ref.step(cut)
        eo = helpers.rel_err_rows(o[la, longest], ro[0]).max()
        ey = helpers.rel_err_rows(y[ls, longest], ry[0]).max()
        assert np.isfinite(o[la, longest]).all()
        assert eo <= TOL and ey <= TOL, \
            "262144 tokens, attention layer %d: %.3g, ssm layer %d: %.3g" % (la, eo, ls, ey)
        assert helpers.rel_err_rows(ses.states(ls, [longest])[0], ref.state(0)).max() <= TOL
        del ref
    ses.close()
