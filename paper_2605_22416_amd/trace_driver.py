"""Allocator-level serving traces on metadata-only pools (no device): how many
capacity errors the same request stream causes on a static split and with the
rebalancing policy switched on (Method, "Dynamic Pool Rebalancing"; the three
workload shapes of "Experimental Setup").  Host logic of the library only; the
paper's own harness, traces and counts are not reproduced, the comparison is a
direction, not a number.

A tick admits the requests that arrive (all KV pages of the prompt for every
attention layer plus one SSM block per SSM layer, all or nothing), then every
live request decodes one token (a new page per attention layer on each 16-token
boundary) and leaves after its output length.  A refused allocation counts as
one capacity error and the request is dropped with everything it held.

    python -m paper_2605_22416_amd.trace_driver
"""
from __future__ import annotations

import argparse
import json
import math
from typing import Dict, List

import numpy as np

from . import binding as av
from gen import inputs


def _prompt_lengths(workload: str, rng: np.random.Generator, n: int) -> np.ndarray:
    if workload == "uniform_short":
        return rng.integers(128, 1025, size=n)
    if workload == "mixed_long":
        return np.clip(np.rint(np.exp(math.log(4096.0) + rng.standard_normal(n))), 256, 65536).astype(np.int64)
    if workload == "agentic_burst":
        return rng.integers(64, 1025, size=n)
    raise ValueError(workload)


def _arrivals(workload: str, rng: np.random.Generator, tick: int, rate: float) -> int:
    if workload == "agentic_burst":              # quiet stretches, then many requests at once
        return int(rng.poisson(rate * 12)) if tick % 12 == 0 else 0
    return int(rng.poisson(rate))


def run_trace(workload: str, seed: int, dynamic: bool, ssm_share: float = 0.5,
              budget_bytes: int = 4 << 30, ticks: int = 3000, spec: inputs.ModelSpec = inputs.JAMBA_MINI,
              policy: Dict = None) -> Dict:
    """One trace.  ssm_share: fraction of the budget the SSM pool starts with (a static
    split keeps it).  Returns counters."""
    kv_cap = int(budget_bytes * (1.0 - ssm_share)) // spec.kv_page_bytes
    ssm_cap = int(budget_bytes * ssm_share) // spec.ssm_block_bytes
    arena = kv_cap * spec.kv_page_bytes + ssm_cap * spec.ssm_block_bytes
    cfg, _keep = av.make_config(spec.dtype, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                                spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate, kv_cap, ssm_cap,
                                state_dtype=spec.state_dtype)
    rc, p = av.avmp_pools_create(cfg, None, arena)
    if rc != av.AVMP_OK:
        raise RuntimeError(av.avmp_last_error())
    if policy:
        assert av.avmp_policy_set(p, **policy) == av.AVMP_OK

    def alloc(pool: int, n: int):
        if dynamic:
            rc_, hs, _ = av.avmp_alloc_auto(p, pool, n)
        else:
            rc_, hs = av.avmp_alloc(p, pool, n)
        return rc_, hs

    rng = np.random.default_rng([seed, 11])
    # offered load: requests whose steady-state footprint is about the whole budget
    mean_len = {"uniform_short": 576 + 64, "mixed_long": 6700 + 64, "agentic_burst": 544 + 64}[workload]
    per_req = spec.n_ssm * spec.ssm_block_bytes + spec.n_attn * math.ceil(mean_len / 16) * spec.kv_page_bytes
    mean_out = 72
    rate = 1.05 * budget_bytes / per_req / mean_out          # arrivals per tick, 5 % over capacity
    live: List[Dict] = []
    errors = admitted = finished = 0
    for tick in range(ticks):
        n_new = _arrivals(workload, rng, tick, rate)
        for length in _prompt_lengths(workload, rng, n_new):
            pages = spec.n_attn * math.ceil(int(length) / 16)
            rc1, kvh = alloc(0, pages)
            if rc1 != av.AVMP_OK:
                errors += 1
                continue
            rc2, sh = alloc(1, spec.n_ssm)
            if rc2 != av.AVMP_OK:
                errors += 1
                av.avmp_free(p, kvh)
                continue
            admitted += 1
            live.append({"len": int(length), "left": int(rng.integers(16, 129)),
                         "handles": list(kvh) + list(sh)})
        survivors = []
        for rq in live:
            if rq["len"] % 16 == 0:                           # the new token opens a page per layer
                rc1, kvh = alloc(0, spec.n_attn)
                if rc1 != av.AVMP_OK:
                    errors += 1
                    av.avmp_free(p, rq["handles"])
                    continue
                rq["handles"].extend(kvh)
            rq["len"] += 1
            rq["left"] -= 1
            if rq["left"] == 0:
                av.avmp_free(p, rq["handles"])
                finished += 1
            else:
                survivors.append(rq)
        live = survivors
    st = av.avmp_stats(p)
    out = {"workload": workload, "seed": seed, "dynamic": dynamic, "ssm_share": ssm_share,
           "capacity_errors": errors, "admitted": admitted, "finished": finished,
           "migrations": int(st["migrations"]), "final_capacity": tuple(st["capacity"])}
    av.avmp_pools_destroy(p)
    return out


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--seeds", type=int, default=3)
    ap.add_argument("--ticks", type=int, default=3000)
    args = ap.parse_args()
    rows = []
    for workload in ("uniform_short", "mixed_long", "agentic_burst"):
        for name, dynamic, share in (("static 0.5", False, 0.5), ("static 0.9", False, 0.9),
                                     ("dynamic from 0.5", True, 0.5)):
            res = [run_trace(workload, s, dynamic, share, ticks=args.ticks) for s in range(args.seeds)]
            rows.append({"workload": workload, "variant": name,
                         "capacity_errors": [r["capacity_errors"] for r in res],
                         "finished": [r["finished"] for r in res],
                         "migrations": [r["migrations"] for r in res]})
            print(json.dumps(rows[-1]), flush=True)


if __name__ == "__main__":
    main()
