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
    window, both.  Three steps, sampled requests.  With a bf16 state the stored
    codes of the two sides part by one ulp where the exact value sits on a rounding
    tie (fp32 against float64 arithmetic), so from the second step on both start
    from slightly different states: the state is then compared to one bf16 ulp
    (2^-7) of its row maximum per step taken, and y to one ulp."""
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
    refs = {r: RequestReference(spec, sc.seed, r, int(sc.ctx[r])) for r in sample}
    for step in range(3):
        inp = inputs.step_inputs(spec, sc.batch, sc.seed, step=step)
        o, y = ses.step(inp, conv=conv)
        _check_sample(ses, refs, inp, o, y, "%s conv %d step %d" % (state_dtype, conv_kernel, step),
                      conv=conv, tol_state=TOL if state_dtype == "f32" else 2.0 ** -7 * (step + 1),
                      tol_y=TOL if state_dtype == "f32" or step == 0 else 2.0 ** -7)
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


def test_capacity_scale_pools_200gb_long_contexts_and_migration_sweep():
    """Config 5: pools filling about 200 GB, batch 512 + 4 requests of 262144
    tokens.  Sampled outputs (one of the 262144-token requests among them), then
    the migration sweep of 64, 1024 and 16384 pages with contents and translation
    checked after each."""
    import torch
    from paper_2605_22416_amd import binding as av
    free_b, total_b = torch.cuda.mem_get_info()
    if total_b < 250e9:
        pytest.skip("needs a 288 GB device")
    spec = inputs.JAMBA_MINI
    sc = inputs.make_scenario(spec, "capacity", 512, seed=1005, headroom=1.7)
    assert 190e9 < sc.arena_bytes < 215e9
    ses = _session(sc, fill_byte=0)
    rng = np.random.default_rng(3)
    longest = int(np.argmax(sc.ctx))
    assert sc.ctx[longest] == 262144
    sample = [int(np.argmin(sc.ctx)), int(rng.integers(0, 512)), longest]
    ses.fill(threads=16, requests=sample)
    # the 262144-token request is checked on the first attention and SSM layer only
    # (the oracle needs about 10 s and 10 GB per attention layer at that length)
    first = inputs.ModelSpec("first_layers", spec.dtype, spec.page_tokens, spec.n_q_heads,
                             spec.n_kv_heads, spec.head_dim, spec.ssm_heads, spec.ssm_headdim,
                             spec.ssm_dstate, (inputs.ATTN, inputs.SSM), spec.scale_inputs)
    refs = {r: RequestReference(first if r == longest else spec, sc.seed, r, int(sc.ctx[r]))
            for r in sample}
    watch = np.concatenate([ses.kv[:, r, : sc.n_pages[r]].reshape(-1)[:: 11] for r in sample]
                           + [ses.ssm[:, sample].reshape(-1)])
    before = {int(h): ses.read_unit(int(h)).copy() for h in watch[:: 7]}
    inp = inputs.step_inputs(spec, sc.batch, sc.seed)
    o, y = ses.step(inp)
    _check_sample(ses, refs, inp, o, y, "cfg5")
    usable = sc.arena_bytes // 128 * 128
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
        assert st1["live"] == st0["live"] and 0 < res.units_copied <= n
        _check_handles_resolve_everywhere(ses, watch)
    for h, data in before.items():
        if (h >> 30) == 0:            # KV pages are read-only in a step; SSM blocks were updated by it
            assert np.array_equal(ses.read_unit(h), data)
    # the step after the migrations reproduces the attention rows bit for bit
    o2, y2 = ses.step(inp)
    assert np.array_equal(o2[:, sample], o[:, sample])
    assert av.avmp_migrate(ses.p, 0, 1 << 29)[0] == av.AVMP_ERR_CAPACITY     # refused, nothing changes
    assert av.avmp_stats(ses.p)["capacity"] == st1["capacity"]
    ses.close()
