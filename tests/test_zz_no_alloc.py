"""avmp_decode_step_noalloc, the decode step for callers that cannot allocate: same
kernels as avmp_decode_step with the work buffer in a static device array.  Checked
through the C ABI against avmp_decode_step on a twin session (bit-identical outputs
and states), on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

from gen import inputs

pytestmark = pytest.mark.gpu


def _sub_step(av, gh, ses, inp, n, ctx, conv=None):
    """A step over the first n requests of a session with the given context lengths
    (each at most what is resident) and a handle row just wide enough for them."""
    import torch
    spec = ses.sc.spec
    ctx = np.asarray(ctx, dtype=np.uint32)
    mp = max(1, int(-(-int(ctx.max()) // spec.page_tokens)))
    kv = gh.to_dev(np.ascontiguousarray(ses.kv[:, :n, :mp]))
    ssm = gh.to_dev(np.ascontiguousarray(ses.ssm[:, :n]))
    d = {k: gh.to_dev(np.ascontiguousarray(v if k == "A" else v[:, :n])) for k, v in inp.items()}
    cw = cb = None
    if spec.conv_kernel:
        cw, cb = gh.to_dev(conv[0]), gh.to_dev(conv[1])
    o = torch.full((spec.n_attn, n, spec.n_q_heads, spec.head_dim), float("nan"),
                   dtype=torch.float32, device=gh.DEV)
    y = torch.full((spec.n_ssm, n, spec.ssm_heads, spec.ssm_headdim), float("nan"),
                   dtype=torch.float32, device=gh.DEV)
    st, keep = av.make_step(n, spec.layer_kinds, mp, kv, gh.to_dev(ctx), d["q"], o, ssm, d["x"],
                            d["dt"], d["A"], d["B"], d["C"], y, None, None, d.get("xbc"), cw, cb)
    return st, keep, o, y


CASES = {
    "jamba_heads_bf16": (inputs.scaled_down(inputs.JAMBA_MINI, 1), [700, 16, 2049, 33, 1, 260], 0),
    "tiny_fp32": (inputs.TINY, [64, 16, 200, 17, 300], 0),
    "conv_window_bf16": (inputs.with_conv(inputs.ModelSpec(
        "small_conv", "bf16", 16, 8, 2, 64, 8, 16, 32, (inputs.SSM, inputs.ATTN, inputs.SSM), True), 4),
        [90, 500, 31, 160], 4),
}


@pytest.mark.parametrize("case", sorted(CASES))
def test_noalloc_step_matches_decode_step_twice_second_call_smaller(case):
    import torch
    from paper_2605_22416_amd import binding as av
    from tests import gpu_harness as gh
    spec, ctx, conv_k = CASES[case]
    sc = inputs.make_scenario(spec, "uniform_short", len(ctx), seed=77, ctx=ctx)
    conv = inputs.conv_weights(spec, 77) if conv_k else None
    ref, dut = gh.GpuPools(sc), gh.GpuPools(sc)
    ref.fill()
    dut.fill()
    calls = [(len(ctx), ctx, 0),
             (len(ctx) - 2, [max(1, c // 2) for c in ctx[:-2]], 1)]      # fewer, shorter requests
    for n, cx, step in calls:
        inp = inputs.step_inputs(spec, len(ctx), seed=77, step=step)
        st_r, keep_r, o_r, y_r = _sub_step(av, gh, ref, inp, n, cx, conv)
        st_d, keep_d, o_d, y_d = _sub_step(av, gh, dut, inp, n, cx, conv)
        assert av.avmp_decode_step(ref.p, st_r) == av.AVMP_OK, av.avmp_last_error()
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        assert av.avmp_decode_step_noalloc(dut.p, st_d) == av.AVMP_OK, av.avmp_last_error()
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before, "the call changed the free device memory"
        assert torch.isfinite(o_d).all() and torch.isfinite(y_d).all()
        assert torch.equal(o_r, o_d), "%s call %d: attention outputs differ" % (case, step)
        assert torch.equal(y_r, y_d), "%s call %d: SSM outputs differ" % (case, step)
        for ls in range(spec.n_ssm):
            assert np.array_equal(ref.states(ls), dut.states(ls)), "state of SSM layer %d" % ls
        if conv_k:
            for ls in range(spec.n_ssm):
                assert np.array_equal(ref.conv_windows(ls), dut.conv_windows(ls))
    assert av.avmp_workspace_info(dut.p)[1:] == (0, 0), "the static path must not touch the library's work buffer"
    assert av.avmp_device_faults(dut.p) == (av.AVMP_OK, 0)
    ref.close()
    dut.close()


def test_noalloc_step_refuses_queued_updates_and_oversized_steps():
    import torch
    from paper_2605_22416_amd import binding as av
    from tests import gpu_harness as gh
    spec = inputs.scaled_down(inputs.JAMBA_MINI, 1)
    ctx = [40, 300]
    sc = inputs.make_scenario(spec, "uniform_short", len(ctx), seed=78, ctx=ctx, headroom=2.0)
    g = gh.GpuPools(sc)
    g.fill()
    inp = inputs.step_inputs(spec, len(ctx), seed=78)
    st, keep, o, y = _sub_step(av, gh, g, inp, len(ctx), ctx)
    # something queued: the call must not push it (that takes pinned memory) and says so
    rc, extra = av.avmp_alloc(g.p, av.AVMP_POOL_KV, 1)
    assert rc == av.AVMP_OK
    assert av.avmp_decode_step_noalloc(g.p, st) == av.AVMP_ERR_INVALID_ARG
    assert "avmp_flush" in av.avmp_last_error()
    assert av.avmp_flush(g.p) == av.AVMP_OK
    assert av.avmp_decode_step_noalloc(g.p, st) == av.AVMP_OK, av.avmp_last_error()
    torch.cuda.synchronize()
    assert torch.isfinite(o).all() and torch.isfinite(y).all()
    # a handle row so wide that the slots of the step cannot fit the static array: refused
    # before anything is read (the row itself is never touched)
    st.max_pages = av.AVMP_NOALLOC_WORKSPACE_BYTES // (4 * len(ctx)) + 1
    assert av.avmp_decode_step_noalloc(g.p, st) == av.AVMP_ERR_INVALID_ARG
    assert str(av.AVMP_NOALLOC_WORKSPACE_BYTES) in av.avmp_last_error()
    g.close()
