"""GPU parity on seeded random shapes: model shape, layer pattern, batch, contexts
(zero and ragged included), placement, state storage type and convolution window
are all drawn per seed; two decode steps each, the second one with a migration in
between, against the CPU oracle.  Tolerances as in test_gpu_parity.py, with two
things the drawn shapes need: a row of y is measured against the size of the
terms that were summed into it (the oracle's sum_n |S*C|; rows of one element and
unscaled inputs cancel freely, and fp32 rounding noise goes with the terms, not
with what is left of them), and with the state stored as bf16 the second step is
held to one bf16 ulp, 2^-7: it starts from stored codes that may differ from the
oracle's by one where the exact value sat on a rounding boundary."""
import numpy as np
import pytest

from oracle import avmp_oracle as orc
from gen import inputs
from tests import helpers
from tests.test_gpu_parity import _both, _check_outputs, _check_states, _check_translation

pytestmark = pytest.mark.gpu


def _draw(seed, conv_inside=False):
    rng = np.random.default_rng([seed, 777])
    dtype = "bf16" if rng.random() < 0.6 else "f32"
    vec = 8 if dtype == "bf16" else 4
    G = int(rng.choice([1, 2, 3, 4, 8]))
    Hq = G * int(rng.choice([1, 2, 3, 4, 8, 16]))
    D = int(rng.choice([16, 32, 64, 128, 256] if dtype == "bf16" else [4, 12, 32, 64, 100]))
    state_dtype = "bf16" if rng.random() < 0.35 else "f32"
    N = int(rng.choice([8, 16, 32, 64, 128, 256] if state_dtype == "bf16" or dtype == "bf16"
                       else [4, 8, 16, 64, 128]))
    H = int(rng.integers(1, 7))
    P = int(rng.choice([1, 3, 8, 24, 32, 64, 128]))
    K = int(rng.choice([0, 0, 2, 3, 4]))
    if conv_inside:      # the shape at which the recurrence kernel runs the convolution itself
        H, P, N, K = int(rng.integers(1, 10)), 64, 128, 4
    kinds = tuple(int(k) for k in rng.integers(0, 2, size=int(rng.integers(2, 5))))
    if inputs.ATTN not in kinds:
        kinds = kinds + (inputs.ATTN,)
    if inputs.SSM not in kinds:
        kinds = (inputs.SSM,) + kinds
    spec = inputs.ModelSpec("rand%d" % seed, dtype, 16, Hq, G, D, H, P, N, kinds, bool(rng.random() < 0.7),
                            state_dtype=state_dtype, conv_kernel=K)
    batch = int(rng.integers(1, 8))
    ctx = [int(c) for c in rng.choice([0, 1, 15, 16, 17, 40, 129, 333, 600], size=batch)]
    # the convolution kernel moves 16-byte groups of channels: other shapes are refused at create
    refused = bool(K and ((H * P) % vec or N % vec))
    return spec, ctx, rng, refused


@pytest.mark.parametrize("seed", range(120))
def test_random_shape(seed):
    _run(seed, *_draw(seed), steps=2)


@pytest.mark.parametrize("seed", range(500, 524))
def test_random_shape_with_the_convolution_inside_the_recurrence_kernel(seed):
    """Headdim 64 x dstate 128 with four taps, everything else drawn; four steps, so that the
    window turns over completely."""
    _run(seed, *_draw(seed, conv_inside=True), steps=4)


def _run(seed, spec, ctx, rng, refused, steps):
    from paper_2605_22416_amd import binding as av
    what = "seed %d: %s ctx %s" % (seed, spec, ctx)
    print(what, flush=True)
    sc = inputs.make_scenario(spec, "tiny", len(ctx), seed=1000 + seed, ctx=ctx, headroom=1.6)
    if refused:
        # a shape the library does not take is an error at create, on the size call too, and
        # nothing is launched; the same model without the window is taken
        cfg, keep = av.make_config(spec.dtype, spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.ssm_heads,
                                   spec.ssm_headdim, spec.ssm_dstate, sc.kv_capacity, sc.ssm_capacity,
                                   state_dtype=spec.state_dtype, conv_kernel=spec.conv_kernel)
        assert av.avmp_geometry(cfg, sc.arena_bytes)[0] == av.AVMP_ERR_INVALID_ARG, what
        assert av.avmp_pools_create(cfg, None, sc.arena_bytes) == (av.AVMP_ERR_INVALID_ARG, None), what
        cfg.ssm_conv_kernel = 0
        assert av.avmp_geometry(cfg, sc.arena_bytes)[0] == av.AVMP_OK, what
        return
    sc.fresh[rng.random(len(ctx)) < 0.3] = True
    op, g, kv, ssm = _both(sc, poison=True)
    conv = inputs.conv_weights(spec, seed=seed) if spec.conv_kernel else None
    extra = dict(xbc=None, conv_w=None, conv_b=None)
    for step in range(steps):
        if step == 1:                      # capacity moves between the steps, live units with it
            donor = int(rng.integers(0, 2))
            n = max(1, int(av.avmp_stats(g.p)["free"][donor]) // 2)
            ores = op.migrate(donor, n)
            rc, res = av.avmp_migrate(g.p, donor, n)
            assert rc == ores.code, what
            if rc == av.AVMP_OK:
                assert (res.units_copied, res.recipient_gain, res.bytes_wasted) == \
                    (ores.units_copied, ores.recipient_gain, ores.bytes_wasted), what
            assert av.avmp_stats(g.p) == op.stats(), what
            _check_translation(g, op, list(kv.reshape(-1)) + list(ssm.reshape(-1)))
        inp = inputs.step_inputs(spec, len(ctx), seed=1000 + seed, step=step)
        if conv is not None:
            extra = dict(xbc=inp["xbc"], conv_w=conv[0], conv_b=conv[1])
        ref_o, ref_y = op.decode_step(spec.layer_kinds, kv, sc.ctx, inp["q"], ssm, inp["x"], inp["dt"],
                                      inp["A"], inp["B"], inp["C"], **extra)
        o, y = g.step(inp, conv=conv)
        y_scale = np.stack([np.stack([op.output_scale[int(h)] for h in ssm[ls]]) for ls in range(spec.n_ssm)])
        _check_outputs(spec, o, y, ref_o, ref_y, what + " step %d" % step, y_scale=y_scale,
                       y_tol=2.0 ** -7 if spec.state_dtype == "bf16" and step > 0 else None)
    if spec.state_dtype == "f32":
        _check_states(spec, g, op, ssm, what)
    if spec.conv_kernel:
        a, n = spec.ssm_state_bytes, spec.conv_window_bytes
        for ls in range(spec.n_ssm):
            got = g.conv_windows(ls)
            for r in range(len(ctx)):
                assert np.array_equal(got[r], op.unit_view(int(ssm[ls, r]))[a: a + n]), what
    g.close()
