"""Oracle results for single requests of a large batch (TEST INFRASTRUCTURE ONLY).

At full workload sizes the oracle cannot hold or walk the whole arena, but a
request's outputs depend on that request's own pages and blocks only, and every
unit's contents are a pure function of (seed, pool, layer, request, index).
This module rebuilds one request in a small pool of its own and runs the
oracle's decode step on it, step after step.  It adds no arithmetic of its own.
"""
from __future__ import annotations

import numpy as np

from oracle import avmp_oracle as orc
from gen import inputs


def oracle_shape(spec) -> orc.Shape:
    return orc.Shape(spec.dtype, spec.page_tokens, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                     spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate, spec.state_dtype,
                     spec.conv_kernel, spec.pad_ssm_to_kv_page)


class RequestReference:
    """One request of a scenario, rebuilt in its own small pools."""

    def __init__(self, spec, seed: int, r: int, ctx: int, fresh: bool = False, scale_inputs=None,
                 attn_ordinals=None, ssm_ordinals=None):
        """spec may hold fewer layers than the scenario's model: attn_ordinals / ssm_ordinals
        then say which of the model's attention / SSM layers (by ordinal among their kind)
        the reference's layers stand for, i.e. whose unit contents they are filled with
        (default: the first ones).  step() must be given inputs cut to the same layers."""
        self.spec, self.r = spec, r
        ao = list(range(spec.n_attn)) if attn_ordinals is None else list(attn_ordinals)
        so = list(range(spec.n_ssm)) if ssm_ordinals is None else list(ssm_ordinals)
        assert len(ao) == spec.n_attn and len(so) == spec.n_ssm
        n_pages = -(-int(ctx) // spec.page_tokens)
        kv_cap = max(1, n_pages * spec.n_attn)
        ssm_cap = max(1, spec.n_ssm)
        arena = kv_cap * spec.kv_page_bytes + ssm_cap * spec.ssm_block_bytes
        self.pools = orc.Pools(oracle_shape(spec), arena, kv_cap, ssm_cap)
        self.ctx = np.array([ctx], dtype=np.uint32)
        self.kv = np.full((spec.n_attn, 1, max(n_pages, 1)), orc.INVALID_HANDLE, dtype=np.uint32)
        for la in range(spec.n_attn):
            if n_pages:
                self.kv[la, 0, :n_pages] = self.pools.alloc(orc.POOL_KV, n_pages)[1]
        self.ssm = np.zeros((spec.n_ssm, 1), dtype=np.uint32)
        if spec.n_ssm:
            self.ssm[:, 0] = self.pools.alloc(orc.POOL_SSM, spec.n_ssm)[1]
        for la in range(spec.n_attn):
            for i in range(n_pages):
                self.pools.unit_view(int(self.kv[la, 0, i]))[:] = inputs.unit_content(
                    spec, seed, inputs.POOL_KV, ao[la], r, i, scale_inputs=scale_inputs)
        if not fresh:
            for ls in range(spec.n_ssm):
                self.pools.unit_view(int(self.ssm[ls, 0]))[:] = inputs.unit_content(
                    spec, seed, inputs.POOL_SSM, so[ls], r, 0, scale_inputs=scale_inputs)

    def step(self, inp, conv=None):
        """inp: the whole batch's step inputs; conv: (taps, bias) of the short convolution
        for models that have one.  Returns (o [n_attn][Hq][D], y [n_ssm][H][P]) float64."""
        r = self.r
        one = {k: (v if k == "A" else v[:, r: r + 1]) for k, v in inp.items()}
        extra = {}
        if self.spec.conv_kernel:
            extra = dict(xbc=one["xbc"], conv_w=conv[0], conv_b=conv[1])
        o, y = self.pools.decode_step(self.spec.layer_kinds, self.kv, self.ctx, one["q"], self.ssm,
                                      one["x"], one["dt"], one["A"], one["B"], one["C"], **extra)
        return o[:, 0], y[:, 0]

    def state(self, layer: int) -> np.ndarray:
        return self.pools.state_values(int(self.ssm[layer, 0]))

    def load_block(self, layer: int, raw: np.ndarray) -> None:
        """Replace the bytes of this request's block of one SSM layer (e.g. by what the
        other side has stored, so that the next step starts from the same state)."""
        self.pools.unit_view(int(self.ssm[layer, 0]))[:] = np.asarray(raw, dtype=np.uint8)
