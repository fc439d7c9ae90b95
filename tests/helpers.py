"""Shared test plumbing: build the oracle's pools from a Scenario, fill units."""
import numpy as np

from oracle import avmp_oracle as orc
from gen import inputs


def oracle_shape(spec):
    return orc.Shape(spec.dtype, spec.page_tokens, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                     spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate, spec.state_dtype,
                     spec.conv_kernel, spec.pad_ssm_to_kv_page)


def alloc_order(sc):
    """The allocation calls both sides replay: per request, its pages for each
    attention layer, then its blocks for all SSM layers."""
    calls = []
    for r in range(sc.batch):
        for la in range(sc.spec.n_attn):
            if sc.n_pages[r] > 0:
                calls.append((inputs.POOL_KV, int(sc.n_pages[r]), ("kv", la, r)))
        if sc.spec.n_ssm:
            calls.append((inputs.POOL_SSM, sc.spec.n_ssm, ("ssm", r)))
    return calls


def empty_handle_tables(sc):
    kv = np.full((sc.spec.n_attn, sc.batch, sc.max_pages), 0xFFFFFFFF, dtype=np.uint32)
    ssm = np.full((sc.spec.n_ssm, sc.batch), 0xFFFFFFFF, dtype=np.uint32)
    return kv, ssm


def place_handles(kv, ssm, tag, hs):
    if tag[0] == "kv":
        kv[tag[1], tag[2], : len(hs)] = hs
    else:
        ssm[:, tag[1]] = hs


def build_oracle(sc, with_data=True):
    p = orc.Pools(oracle_shape(sc.spec), sc.arena_bytes, sc.kv_capacity, sc.ssm_capacity,
                  slot_rank=sc.slot_rank, with_data=with_data)
    kv, ssm = empty_handle_tables(sc)
    for pool, n, tag in alloc_order(sc):
        code, hs = p.alloc(pool, n)
        assert code == orc.OK
        place_handles(kv, ssm, tag, hs)
    return p, kv, ssm


def unit_jobs(sc):
    """(pool, layer, request, index) of every live unit, with its handle-table position."""
    jobs = []
    for la in range(sc.spec.n_attn):
        for r in range(sc.batch):
            for i in range(int(sc.n_pages[r])):
                jobs.append((inputs.POOL_KV, la, r, i))
    for ls in range(sc.spec.n_ssm):
        for r in range(sc.batch):
            if not sc.fresh[r]:
                jobs.append((inputs.POOL_SSM, ls, r, 0))
    return jobs


def job_handle(job, kv, ssm):
    pool, layer, r, i = job
    return int(kv[layer, r, i]) if pool == inputs.POOL_KV else int(ssm[layer, r])


def poison_tail(spec, page, n_valid, opools):
    """NaN in every K and V element of token slots >= n_valid of one page."""
    nan = np.array([np.nan], dtype=np.float32)
    pat = nan.view(np.uint8) if spec.dtype == "f32" else inputs.f32_to_bf16_bits(nan).view(np.uint8)
    for t in range(n_valid, spec.page_tokens):
        for g in range(spec.n_kv_heads):
            for d in range(spec.head_dim):
                for which in ("k", "v"):
                    o = opools.kv_element_offset(which, g, t, d)
                    page[o: o + spec.elem_bytes] = pat


def fill_oracle(p, sc, kv, ssm, poison=False, scale_inputs=None):
    spec = sc.spec
    if poison:
        p.arena[:] = 0xFF                  # all-ones bytes are NaN in fp32 and in bf16
        for ls in range(spec.n_ssm):       # fresh blocks stay zero (the allocator zeroed them)
            for r in range(sc.batch):
                if sc.fresh[r]:
                    p.unit_view(int(ssm[ls, r]))[:] = 0
    for job in unit_jobs(sc):
        data = inputs.unit_content(spec, sc.seed, *job, scale_inputs=scale_inputs).copy()
        pool, layer, r, i = job
        if poison and pool == inputs.POOL_KV and i == sc.n_pages[r] - 1:
            poison_tail(spec, data, int(sc.ctx[r]) - i * spec.page_tokens, p)
        p.unit_view(job_handle(job, kv, ssm))[:] = data


def rel_err_rows(got, ref, axis=-1):
    """Per-row max-norm relative error: |got-ref|_inf / max(|ref|_inf, tiny)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    num = np.abs(got - ref).max(axis=axis)
    den = np.maximum(np.abs(ref).max(axis=axis), 1e-30)
    return num / den
