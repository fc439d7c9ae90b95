"""Pins for the oracle's paged attention and SSM step.

Attention is pinned to a library routine (torch's scaled-dot-product attention
on dense, non-paged float64 tensors) and to special cases with known answers;
the SSM step to the closed form of the unrolled recurrence, to a brute-force
scalar loop and to special cases.  Placement invariance and NaN poisoning
check that results depend on logical content only.
"""
import math

import numpy as np
import pytest
import torch

from oracle import avmp_oracle as orc
from gen import inputs
from tests import helpers


def _spec(dtype, Hq, G, D, H=2, P=4, N=8):
    return inputs.ModelSpec("t", dtype, 16, Hq, G, D, H, P, N, (0, 1), False)


def _dense_sdpa(q, K, V, Hq, G):
    """Textbook attention through the library: q [Hq][D], K, V [ctx][G][D] float64."""
    rep = Hq // G
    k = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(rep, dim=0)      # [Hq][ctx][D]
    v = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(rep, dim=0)
    o = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q)[:, None, :], k, v)
    return o[:, 0, :].numpy()


def _paged_setup(spec, ctx, seed, permute=True):
    """Pools holding logical K, V (returned as exact float64) written token by token."""
    sc = inputs.make_scenario(spec, "tiny", len(ctx), seed, ctx=ctx, permute=permute)
    p, kv, ssm = helpers.build_oracle(sc)
    rng = np.random.default_rng(seed + 100)
    p.arena[:] = 0xFF
    logical = []
    for r, n in enumerate(ctx):
        Kb = inputs.elements(rng, (n, spec.n_kv_heads, spec.head_dim), 1.0, spec.dtype)
        Vb = inputs.elements(rng, (n, spec.n_kv_heads, spec.head_dim), 1.0, spec.dtype)
        for t in range(n):
            p.write_kv_token(int(kv[0, r, t // 16]), t % 16, Kb[t], Vb[t])
        logical.append((orc.as_f64(Kb, spec.dtype), orc.as_f64(Vb, spec.dtype)))
    q = inputs.elements(rng, (len(ctx), spec.n_q_heads, spec.head_dim), 1.0, spec.dtype)
    return sc, p, kv, q, logical


@pytest.mark.parametrize("dtype,Hq,G,D", [("f32", 4, 2, 64), ("bf16", 8, 2, 32), ("bf16", 4, 1, 128),
                                          ("f32", 3, 3, 16)])
def test_paged_attention_equals_dense_library_attention(dtype, Hq, G, D):
    spec = _spec(dtype, Hq, G, D)
    ctx = [1, 15, 16, 17, 40, 64]
    sc, p, kv, q, logical = _paged_setup(spec, ctx, seed=5)
    o = p.paged_attention(kv[0], sc.ctx, q)
    qf = orc.as_f64(q, dtype)
    for r in range(len(ctx)):
        ref = _dense_sdpa(qf[r], logical[r][0], logical[r][1], Hq, G)
        np.testing.assert_allclose(o[r], ref, rtol=1e-12, atol=1e-13)


def test_attention_special_cases():
    spec = _spec("f32", 4, 2, 64)
    sc, p, kv, q, logical = _paged_setup(spec, [1, 33], seed=8)
    o = p.paged_attention(kv[0], sc.ctx, q)
    # one token: softmax weight is exactly 1, the output is that token's V
    for j in range(4):
        assert np.array_equal(o[0, j], logical[0][1][0, j // 2])
    # all keys equal: uniform weights, output = mean of V
    sc, p, kv, q, logical = _paged_setup(spec, [20], seed=9)
    K0 = np.ascontiguousarray(logical[0][0][0]).astype(np.float32)
    Vb = logical[0][1].astype(np.float32)
    for t in range(20):
        p.write_kv_token(int(kv[0, 0, t // 16]), t % 16, K0, Vb[t])
    o = p.paged_attention(kv[0], sc.ctx, q)
    for j in range(4):
        np.testing.assert_allclose(o[0, j], logical[0][1][:, j // 2].mean(axis=0), rtol=1e-12, atol=1e-14)
    # zero tokens: defined as a zero row, nothing is resolved
    z = p.paged_attention(np.full((1, 1), 0xFFFFFFFF, dtype=np.uint32), np.array([0], dtype=np.uint32), q[:1])
    assert not z.any()


def test_attention_grouping_maps_query_head_j_to_kv_head_j_div_group():
    # make KV head 1 the only one with a non-zero V: only query heads 2,3 (group 1) see it
    spec = _spec("f32", 4, 2, 16)
    sc, p, kv, q, logical = _paged_setup(spec, [5], seed=10)
    V = np.zeros((5, 2, 16), dtype=np.float32)
    V[:, 1, :] = 1.0
    K = logical[0][0].astype(np.float32)
    for t in range(5):
        p.write_kv_token(int(kv[0, 0, 0]), t, K[t], V[t])
    o = p.paged_attention(kv[0], sc.ctx, q)
    assert not o[0, 0].any() and not o[0, 1].any()
    np.testing.assert_allclose(o[0, 2], 1.0, rtol=1e-14)
    np.testing.assert_allclose(o[0, 3], 1.0, rtol=1e-14)


def test_softmax_scale_is_one_over_sqrt_d():
    # two tokens, q.k differs by exactly D between them -> weights e^{sqrt(D)} : 1
    spec = _spec("f32", 1, 1, 16)
    sc, p, kv, _, _ = _paged_setup(spec, [2], seed=11)
    K = np.zeros((2, 1, 16), dtype=np.float32)
    K[0] = 1.0
    V = np.zeros((2, 1, 16), dtype=np.float32)
    V[0] = 1.0
    for t in range(2):
        p.write_kv_token(int(kv[0, 0, 0]), t, K[t], V[t])
    q = np.ones((1, 1, 16), dtype=np.float32)
    o = p.paged_attention(kv[0], sc.ctx, q)
    w = math.exp(4.0) / (math.exp(4.0) + 1.0)
    np.testing.assert_allclose(o[0, 0], w, rtol=1e-14)


def test_page_layout_offsets_are_a_bijection_and_match_the_decoder():
    for dtype, G, D in (("f32", 2, 64), ("bf16", 8, 128), ("bf16", 1, 16)):
        spec = _spec(dtype, G, G, D)
        sh = helpers.oracle_shape(spec)
        p = orc.Pools(sh, 2 * sh.unit_bytes(0) + sh.unit_bytes(1), 2, 1)
        offs = [p.kv_element_offset(w, g, t, d) for w in "kv" for g in range(G)
                for t in range(16) for d in range(D)]
        assert sorted(offs) == list(range(0, sh.unit_bytes(0), sh.elem_bytes))
        # a 16-byte chunk of K holds consecutive dims of one token; consecutive
        # tokens of that dim chunk are adjacent; V keeps a dim's 16 tokens adjacent
        x = 16 // sh.elem_bytes
        assert p.kv_element_offset("k", 0, 3, 1) - p.kv_element_offset("k", 0, 3, 0) == sh.elem_bytes
        assert p.kv_element_offset("k", 0, 4, 0) - p.kv_element_offset("k", 0, 3, 0) == 16
        assert p.kv_element_offset("k", 0, 0, x) - p.kv_element_offset("k", 0, 0, 0) == 16 * 16
        assert p.kv_element_offset("v", 0, 1, 0) - p.kv_element_offset("v", 0, 0, 0) == sh.elem_bytes
        assert p.kv_element_offset("v", 0, 0, 1) - p.kv_element_offset("v", 0, 0, 0) == 16 * sh.elem_bytes
        assert p.kv_element_offset("v", 0, 0, 0) == sh.unit_bytes(0) // 2


# ---- SSM step -------------------------------------------------------------------
def _ssm_setup(spec, batch, seed):
    sc = inputs.make_scenario(spec, "tiny", batch, seed, ctx=[16] * batch)
    p, kv, ssm = helpers.build_oracle(sc)
    return sc, p, ssm


def test_ssm_unrolled_recurrence_closed_form():
    spec = _spec("f32", 1, 1, 16, H=3, P=5, N=8)
    batch, T = 2, 6
    sc, p, ssm = _ssm_setup(spec, batch, seed=3)
    xs, dts, Bs, Cs = [], [], [], []
    A = None
    ys = []
    for t in range(T):
        inp = inputs.step_inputs(spec, batch, seed=40, step=t)
        A = inputs.step_inputs(spec, batch, seed=40, step=0)["A"]          # decay is a model constant
        ys.append(p.ssm_step(ssm[0], inp["x"][0], inp["dt"][0], A[0], inp["B"][0], inp["C"][0]))
        xs.append(inp["x"][0].astype(np.float64)); dts.append(inp["dt"][0].astype(np.float64))
        Bs.append(inp["B"][0].astype(np.float64)); Cs.append(inp["C"][0].astype(np.float64))
    Af = A[0].astype(np.float64)
    for r in range(batch):
        for h in range(3):
            for pp in range(5):
                want = 0.0
                for s in range(T):
                    decay = 1.0
                    for u in range(s + 1, T):
                        decay *= math.exp(dts[u][r, h] * Af[h])
                    want += decay * dts[s][r, h] * float(Cs[T - 1][r] @ Bs[s][r]) * xs[s][r, h, pp]
                # the state is rounded to fp32 between steps, hence 1e-6 rather than 1e-15
                assert abs(ys[-1][r, h, pp] - want) <= 2e-6 * max(1.0, abs(want))


def test_ssm_step_bruteforce_scalar_loops():
    spec = _spec("bf16", 1, 1, 16, H=2, P=3, N=4)
    sc, p, ssm = _ssm_setup(spec, 2, seed=4)
    rng = np.random.default_rng(0)
    S0 = []
    for r in range(2):
        blk = p.unit_view(int(ssm[0, r])).view(np.float32)
        blk[:] = rng.standard_normal(blk.size).astype(np.float32)
        S0.append(blk.copy().reshape(2, 3, 4))
    inp = inputs.step_inputs(spec, 2, seed=41)
    y = p.ssm_step(ssm[0], inp["x"][0], inp["dt"][0], inp["A"][0], inp["B"][0], inp["C"][0])
    x = inputs.bf16_bits_to_f32(inp["x"][0]).astype(np.float64)
    B = inputs.bf16_bits_to_f32(inp["B"][0]).astype(np.float64)
    C = inputs.bf16_bits_to_f32(inp["C"][0]).astype(np.float64)
    for r in range(2):
        S1 = p.unit_view(int(ssm[0, r])).view(np.float32).reshape(2, 3, 4)
        for h in range(2):
            a = math.exp(float(inp["dt"][0][r, h]) * float(inp["A"][0][h]))
            for pp in range(3):
                acc = 0.0
                size = 0.0
                for n in range(4):
                    s = a * float(S0[r][h, pp, n]) + float(inp["dt"][0][r, h]) * x[r, h, pp] * B[r, n]
                    assert S1[h, pp, n] == np.float32(s)
                    acc += s * C[r, n]
                    size += abs(s * C[r, n])
                assert abs(y[r, h, pp] - acc) < 1e-14
                # the size of the terms behind y, which GPU tests measure rounding noise against:
                # never less than |y|, and exactly the sum of the absolute products
                scale = p.output_scale[int(ssm[0, r])][h, pp]
                assert abs(scale - size) < 1e-14 and scale >= abs(y[r, h, pp]) - 1e-14


def test_ssm_special_cases():
    spec = _spec("f32", 1, 1, 16, H=2, P=3, N=4)
    sc, p, ssm = _ssm_setup(spec, 1, seed=6)
    inp = inputs.step_inputs(spec, 1, seed=42)
    x, dt, A, B, C = (inp[k][0] for k in ("x", "dt", "A", "B", "C"))
    # fresh (zeroed) block: y = dt * (C.B) * x
    assert not p.unit_view(int(ssm[0, 0])).any()
    y = p.ssm_step(ssm[0], x, dt, A, B, C)
    cb = float(C[0].astype(np.float64) @ B[0].astype(np.float64))
    np.testing.assert_allclose(y[0], dt[0][:, None].astype(np.float64) * cb * x[0], rtol=1e-13)
    # B = 0: the state only decays by a = exp(dt*A)
    S = p.unit_view(int(ssm[0, 0])).view(np.float32).reshape(2, 3, 4).copy()
    p.ssm_step(ssm[0], x, dt, A, np.zeros_like(B), C)
    S2 = p.unit_view(int(ssm[0, 0])).view(np.float32).reshape(2, 3, 4)
    a = np.exp(dt[0].astype(np.float64) * A.astype(np.float64))
    assert np.array_equal(S2, (a[:, None, None] * S).astype(np.float32))
    assert (a < 1).all() and (a > 0).all()
    # A = 0: no decay, the state is a running sum of dt*x*B
    S = S2.copy()
    p.ssm_step(ssm[0], x, dt, np.zeros_like(A), B, C)
    S3 = p.unit_view(int(ssm[0, 0])).view(np.float32).reshape(2, 3, 4)
    want = S.astype(np.float64) + (dt[0][:, None] * x[0].astype(np.float64))[:, :, None] * B[0][None, None, :]
    assert np.array_equal(S3, want.astype(np.float32))


# ---- P5 / P9: placement invariance and masking ------------------------------------
def _run_tiny(placement_seed, poison, permute=True):
    spec = inputs.TINY
    sc = inputs.make_scenario(spec, "tiny", 4, seed=1001, placement_seed=placement_seed, permute=permute)
    p, kv, ssm = helpers.build_oracle(sc)
    helpers.fill_oracle(p, sc, kv, ssm, poison=poison)
    inp = inputs.step_inputs(spec, 4, seed=1001)
    o, y = p.decode_step(spec.layer_kinds, kv, sc.ctx, inp["q"], ssm, inp["x"], inp["dt"], inp["A"],
                         inp["B"], inp["C"])
    state = np.stack([p.unit_view(int(h)).view(np.float32).copy() for h in ssm[0]])
    slots = [p.resolve(int(h))[1] for h in kv[0, 0, : sc.n_pages[0]]]
    return o, y, state, slots, (kv, ssm)


def test_results_do_not_depend_on_physical_placement_or_poison():
    base = _run_tiny(None, poison=False, permute=False)
    assert base[3] == sorted(base[3])                       # identity rank: ascending slots
    seen = {tuple(base[3])}
    for ps, poison in ((11, False), (12, True), (13, True)):
        o, y, state, slots, hs = _run_tiny(ps, poison)
        assert np.array_equal(o, base[0]) and np.array_equal(y, base[1])
        assert np.array_equal(state, base[2])
        assert np.isfinite(o).all() and np.isfinite(y).all()
        assert np.array_equal(hs[0], base[4][0]) and np.array_equal(hs[1], base[4][1])
        seen.add(tuple(slots))
    assert len(seen) == 4                                   # the placements really differed


def test_tiny_step_is_identical_after_migrating_four_free_pages():
    spec = inputs.TINY
    sc = inputs.make_scenario(spec, "tiny", 4, seed=1001)
    inp = inputs.step_inputs(spec, 4, seed=1001)
    outs = []
    for migrate in (False, True):
        unit_kv, unit_ssm = spec.kv_page_bytes, spec.ssm_block_bytes
        sc.kv_capacity, sc.ssm_capacity = 64, 8
        sc.arena_bytes = 64 * unit_kv + 8 * unit_ssm
        prng = np.random.default_rng(2)
        sc.slot_rank = [prng.permutation(sc.arena_bytes // unit_kv), prng.permutation(sc.arena_bytes // unit_ssm)]
        p, kv, ssm = helpers.build_oracle(sc)
        helpers.fill_oracle(p, sc, kv, ssm)
        if migrate:
            r = p.migrate(orc.POOL_KV, 4)
            assert r.code == orc.OK and r.recipient_gain == 8
            assert p.stats()["capacity"] == (60, 16)
        outs.append(p.decode_step(spec.layer_kinds, kv, sc.ctx, inp["q"], ssm, inp["x"], inp["dt"],
                                  inp["A"], inp["B"], inp["C"]))
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])


def test_single_request_reference_equals_the_whole_batch_oracle():
    """A request's outputs depend on its own units only: rebuilding it alone in
    small pools gives the very same numbers as the oracle run on the whole batch."""
    from oracle.sampled import RequestReference
    spec = inputs.TINY
    sc = inputs.make_scenario(spec, "tiny", 4, seed=1001)
    p, kv, ssm = helpers.build_oracle(sc)
    helpers.fill_oracle(p, sc, kv, ssm)
    refs = [RequestReference(spec, 1001, r, int(sc.ctx[r])) for r in range(4)]
    for step in range(2):
        inp = inputs.step_inputs(spec, 4, seed=1001, step=step)
        o, y = p.decode_step(spec.layer_kinds, kv, sc.ctx, inp["q"], ssm, inp["x"], inp["dt"],
                             inp["A"], inp["B"], inp["C"])
        for r in range(4):
            o1, y1 = refs[r].step(inp)
            assert np.array_equal(o1, o[:, r]) and np.array_equal(y1, y[:, r])
            assert np.array_equal(refs[r].state(0), p.unit_view(int(ssm[0, r])).view(np.float32).reshape(4, 32, 16))


def test_append_then_attend_equals_dense_attention_over_the_longer_sequence():
    """The append path against the library routine: writing token ctx into its page
    and attending over ctx + 1 tokens is dense attention over the concatenation."""
    spec = _spec("bf16", 8, 2, 32)
    ctx = [1, 15, 16, 31, 47]               # 16 and 32 land on a page boundary: new page needed
    sc, p, kv, q, logical = _paged_setup(spec, [c + 1 for c in ctx], seed=21)   # pages for ctx+1 exist
    rng = np.random.default_rng(5)
    k_new = inputs.elements(rng, (1, len(ctx), 2, 32), 1.0, "bf16")
    v_new = inputs.elements(rng, (1, len(ctx), 2, 32), 1.0, "bf16")
    ssm = np.zeros((0, len(ctx)), dtype=np.uint32)
    z = np.zeros((0,))
    o, _ = p.decode_step((0,), kv, np.array(ctx, dtype=np.uint32), q[None], ssm, z, z, z, z, z,
                         k_new=k_new, v_new=v_new)
    qf = orc.as_f64(q, "bf16")
    for r, n in enumerate(ctx):
        K = np.concatenate([logical[r][0][:n], orc.as_f64(k_new[0, r], "bf16")[None]])
        V = np.concatenate([logical[r][1][:n], orc.as_f64(v_new[0, r], "bf16")[None]])
        np.testing.assert_allclose(o[0, r], _dense_sdpa(qf[r], K, V, 8, 2), rtol=1e-12, atol=1e-13)


def test_bf16_rounding_equals_the_library_conversion():
    """round_to_bf16_bits against torch's float -> bfloat16 (round to nearest even),
    on random values, exact ties and values one float32 ulp either side of a tie."""
    rng = np.random.default_rng(2)
    v = np.concatenate([rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000)),
                        [0.0, -0.0, 1.0, -1.0, 3.0e-30, 6.5e30]]).astype(np.float32)
    base = (v.view(np.uint32) & np.uint32(0xFFFF0000))
    ties = (base | np.uint32(0x8000)).view(np.float32)            # exactly halfway between two bf16 values
    near = np.concatenate([(base | np.uint32(0x8001)).view(np.float32), (base | np.uint32(0x7FFF)).view(np.float32)])
    allv = np.concatenate([v, ties, near])
    want = torch.from_numpy(allv).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = orc.round_to_bf16_bits(allv.astype(np.float64))
    assert np.array_equal(got, want)


def test_ssm_step_with_bf16_state_storage():
    """State stored as bf16: y still comes from the un-rounded updated state, the
    block holds its nearest bf16 (B = 0: exactly bf16(a * s), checked through torch)."""
    spec = inputs.with_state_dtype(_spec("bf16", 1, 1, 16, H=2, P=3, N=8), "bf16")
    assert spec.ssm_block_bytes == 2 * 3 * 8 * 2
    sc, p, ssm = _ssm_setup(spec, 1, seed=13)
    h = int(ssm[0, 0])
    assert p.unit[1] == spec.ssm_block_bytes
    p.unit_view(h)[:] = inputs.unit_content(spec, 13, 1, 0, 0, 0)
    S0 = p.state_values(h).copy()
    inp = inputs.step_inputs(spec, 1, seed=43)
    x, dt, A, B, C = (inp[k][0] for k in ("x", "dt", "A", "B", "C"))
    y = p.ssm_step(ssm[0], x, dt, A, np.zeros_like(B), C)
    a = np.exp(dt[0].astype(np.float64) * A.astype(np.float64))
    exact = a[:, None, None] * S0
    want = torch.from_numpy(exact).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(p.state_values(h), want)
    Cf = orc.as_f64(C, "bf16")
    np.testing.assert_allclose(y[0], (exact * Cf[0][None, None, :]).sum(axis=2), rtol=1e-13)
    # with B != 0 the stored value is within half a bf16 ulp of the exact update
    S1 = p.state_values(h).copy()
    p.ssm_step(ssm[0], x, dt, A, B, C)
    xf, Bf = orc.as_f64(x, "bf16"), orc.as_f64(B, "bf16")
    exact = a[:, None, None] * S1 + (dt[0].astype(np.float64)[:, None] * xf[0])[:, :, None] * Bf[0][None, None, :]
    assert (np.abs(p.state_values(h) - exact) <= np.abs(exact) * 2.0 ** -8).all()


# ---------------------------------------------------------------------------
# the short convolution in front of the recurrence (blocks with a window)
# ---------------------------------------------------------------------------
def _library_causal_conv_silu(u_seq, w, b):
    """u_seq [T][C], w [K][C], b [C] float64 -> SiLU(causal depthwise convolution) [T][C],
    through torch's conv1d over the whole sequence (zeros before the first token)."""
    K = w.shape[0]
    x = torch.from_numpy(np.ascontiguousarray(u_seq.T))[None]                  # [1][C][T]
    wt = torch.from_numpy(np.ascontiguousarray(w.T))[:, None, :]               # [C][1][K]
    out = torch.nn.functional.conv1d(x, wt, bias=torch.from_numpy(b), padding=K - 1,
                                     groups=w.shape[1])[0, :, : u_seq.shape[0]]
    return torch.nn.functional.silu(out).numpy().T


@pytest.mark.parametrize("dtype,K", [("f32", 4), ("bf16", 3), ("bf16", 2)])
def test_conv_step_token_by_token_equals_library_convolution_over_the_sequence(dtype, K):
    spec = inputs.with_conv(_spec(dtype, 1, 1, 16, H=2, P=4, N=8), K)
    assert spec.conv_dim == 2 * 4 + 16
    batch, T = 3, 9
    sc, p, ssm = _ssm_setup(spec, batch, seed=8)
    p.arena[:] = 0xFF
    for r in range(batch):
        p.unit_view(int(ssm[0, r]))[:] = 0                    # fresh blocks
    w, b = inputs.conv_weights(spec, seed=8)
    us, outs = [], []
    for t in range(T):
        u = inputs.step_inputs(spec, batch, seed=8, step=t)["xbc"][0]
        us.append(u)
        x, B, C = p.conv_step(ssm[0], u, w[0], b[0])
        assert x.shape == (batch, 2, 4) and B.shape == C.shape == (batch, 8)
        outs.append(np.concatenate([x.reshape(batch, -1), B, C], axis=1))
    wf, bf = orc.as_f64(w[0], dtype), orc.as_f64(b[0], dtype)
    for r in range(batch):
        seq = np.stack([orc.as_f64(u[r], dtype) for u in us])
        ref = _library_causal_conv_silu(seq, wf, bf)
        np.testing.assert_allclose(np.stack([o[r] for o in outs]), ref, rtol=1e-12, atol=1e-14)
        # the window is the last K-1 inputs, oldest first, stored as they came
        assert np.array_equal(p.conv_window(int(ssm[0, r])), seq[T - (K - 1):])
        # the recurrent state in front of the window was not touched
        assert not p.unit_view(int(ssm[0, r]))[: spec.ssm_state_bytes].any()


def test_conv_step_continues_from_a_stored_window():
    """A block whose window holds inputs a, b, c continues the sequence a, b, c, u0, u1, ..."""
    spec = inputs.with_conv(_spec("f32", 1, 1, 16, H=1, P=8, N=4), 4)
    sc, p, ssm = _ssm_setup(spec, 1, seed=9)
    rng = np.random.default_rng(9)
    h = int(ssm[0, 0])
    past = rng.standard_normal((3, spec.conv_dim)).astype(np.float32)
    blk = p.unit_view(h)
    blk[spec.ssm_state_bytes: spec.ssm_state_bytes + past.nbytes] = past.view(np.uint8).reshape(-1)
    assert np.array_equal(p.conv_window(h), past.astype(np.float64))
    w, b = inputs.conv_weights(spec, seed=9)
    new = rng.standard_normal((2, 1, spec.conv_dim)).astype(np.float32)
    got = []
    for t in range(2):
        x, B, C = p.conv_step(ssm[0], new[t], w[0], b[0])
        got.append(np.concatenate([x.reshape(-1), B[0], C[0]]))
    seq = np.concatenate([past, new[:, 0]]).astype(np.float64)
    ref = _library_causal_conv_silu(seq, w[0].astype(np.float64), b[0].astype(np.float64))
    np.testing.assert_allclose(np.stack(got), ref[3:], rtol=1e-12, atol=1e-14)


def test_conv_special_cases():
    spec = inputs.with_conv(_spec("f32", 1, 1, 16, H=1, P=4, N=4), 4)
    sc, p, ssm = _ssm_setup(spec, 1, seed=10)
    Cd = spec.conv_dim
    u = np.linspace(-2.0, 2.0, Cd, dtype=np.float32)[None]
    zero_w, zero_b = np.zeros((4, Cd), np.float32), np.zeros(Cd, np.float32)
    # no taps, bias only: SiLU(b), and SiLU(0) = 0
    bias = np.linspace(-3.0, 3.0, Cd, dtype=np.float32)
    x, B, C = p.conv_step(ssm[0], u, zero_w, bias)
    out = np.concatenate([x.reshape(-1), B[0], C[0]])
    np.testing.assert_allclose(out, bias / (1.0 + np.exp(-bias.astype(np.float64))), rtol=1e-15)
    # only the newest tap set to one: SiLU of the token itself, whatever the window holds
    w = zero_w.copy(); w[3] = 1.0
    x, B, C = p.conv_step(ssm[0], 2 * u, w, zero_b)
    out = np.concatenate([x.reshape(-1), B[0], C[0]])
    uf = 2 * u[0].astype(np.float64)
    np.testing.assert_allclose(out, uf / (1.0 + np.exp(-uf)), rtol=1e-15)
    # only the oldest tap: the token from three steps ago (u went in first, then 2u, now 3u, 4u)
    w = zero_w.copy(); w[0] = 1.0
    p.conv_step(ssm[0], 3 * u, w, zero_b)
    x, B, C = p.conv_step(ssm[0], 4 * u, w, zero_b)
    out = np.concatenate([x.reshape(-1), B[0], C[0]])
    uf = u[0].astype(np.float64)
    np.testing.assert_allclose(out, uf / (1.0 + np.exp(-uf)), rtol=1e-15)
    # channel order of the outputs: x [H][P] first, then B, then C
    assert np.array_equal(x.reshape(-1), out[:4]) and np.array_equal(B[0], out[4:8]) and np.array_equal(C[0], out[8:])


def test_decode_step_with_convolution_feeds_unrounded_outputs_to_the_recurrence():
    """The composed step equals: library convolution of the token, then the (separately
    pinned) recurrence on those values as they are; inputs x, B, C are ignored."""
    spec = inputs.with_conv(_spec("bf16", 1, 1, 16, H=2, P=4, N=8), 4)
    batch = 2
    sc, pa, ssm = _ssm_setup(spec, batch, seed=11)
    _, pb, ssm_b = _ssm_setup(spec, batch, seed=11)
    assert np.array_equal(ssm, ssm_b)
    for r in range(batch):
        content = inputs.unit_content(spec, 11, inputs.POOL_SSM, 0, r)
        pa.unit_view(int(ssm[0, r]))[:] = content
        pb.unit_view(int(ssm[0, r]))[:] = content
    w, b = inputs.conv_weights(spec, seed=11)
    kv = np.full((0, batch, 1), orc.INVALID_HANDLE, dtype=np.uint32)
    for t in range(3):
        inp = inputs.step_inputs(spec, batch, seed=11, step=t)
        windows = [pb.conv_window(int(ssm[0, r])) for r in range(batch)]
        _, y = pa.decode_step((1,), kv, sc.ctx, inp["q"], ssm, None, inp["dt"], inp["A"], None, None,
                              xbc=inp["xbc"], conv_w=w, conv_b=b)
        conv = []
        for r in range(batch):
            seq = np.concatenate([windows[r], orc.as_f64(inp["xbc"][0][r], "bf16")[None]])
            conv.append(_library_causal_conv_silu(seq, orc.as_f64(w[0], "bf16"), orc.as_f64(b[0], "bf16"))[-1])
        conv = np.stack(conv)
        yb = pb.ssm_step(ssm[0], conv[:, :8].reshape(batch, 2, 4), inp["dt"][0], inp["A"][0],
                         conv[:, 8:16], conv[:, 16:], exact_inputs=True)
        pb.conv_step(ssm[0], inp["xbc"][0], w[0], b[0])          # only to move pb's window on
        np.testing.assert_allclose(y[0], yb, rtol=1e-11, atol=1e-13)
        for r in range(batch):
            assert np.array_equal(pa.unit_view(int(ssm[0, r])), pb.unit_view(int(ssm[0, r])))


def test_exact_inputs_equal_encoded_inputs_when_the_values_are_representable():
    spec = _spec("bf16", 1, 1, 16, H=2, P=3, N=8)
    sc, pa, ssm = _ssm_setup(spec, 2, seed=12)
    _, pb, _ = _ssm_setup(spec, 2, seed=12)
    inp = inputs.step_inputs(spec, 2, seed=12)
    ya = pa.ssm_step(ssm[0], inp["x"][0], inp["dt"][0], inp["A"][0], inp["B"][0], inp["C"][0])
    yb = pb.ssm_step(ssm[0], orc.as_f64(inp["x"][0], "bf16"), inp["dt"][0], inp["A"][0],
                     orc.as_f64(inp["B"][0], "bf16"), orc.as_f64(inp["C"][0], "bf16"), exact_inputs=True)
    assert np.array_equal(ya, yb) and np.array_equal(pa.arena, pb.arena)


def test_block_size_with_a_convolution_window():
    spec = inputs.with_conv(inputs.JAMBA_MINI, 4)
    assert spec.conv_dim == 128 * 64 + 2 * 128
    assert spec.ssm_block_bytes == 4 * 128 * 64 * 128 + 3 * 8448 * 2
    assert helpers.oracle_shape(spec).unit_bytes(orc.POOL_SSM) == spec.ssm_block_bytes
    odd = inputs.with_conv(_spec("bf16", 1, 1, 16, H=1, P=3, N=8), 2)      # 19 channels
    assert odd.ssm_block_bytes == (1 * 3 * 8 * 4 + 19 * 2 + 15) // 16 * 16
    assert helpers.oracle_shape(odd).unit_bytes(orc.POOL_SSM) == odd.ssm_block_bytes
