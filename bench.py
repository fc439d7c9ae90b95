#!/usr/bin/env python3
"""Benchmark of the hybrid decode path on one MI355X.

Workload: the Jamba-mini-like decode step (4 attention + 28 SSM layers, bf16 in
/ fp32 accumulate, 32 query / 8 KV heads x 128, 16-token pages, SSM 128 heads x
64 x 128, batch 64, contexts uniform in [128, 2048], pools sized to 1.2x demand
with seeded random placement).  One timed step is one pass of the whole path:
  churn      one request's worth of handles is freed and re-allocated
             (4 x 68 KV pages + 28 SSM blocks), table updates flushed on-stream
  decode     translation + paged GQA attention + SSM update for all 32 layers
  migration  128 KV pages of capacity (the paper's default batch) move to the
             SSM pool and back, with live pages copied and the table rewritten
Inputs are resident in HBM before the timed region.  The value reported is the
algorithmic bytes of a step divided by the time of a step.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
PREWARM_STEPS = 10

# Counter-measured HBM traffic per launch, written by `bench.py --write-traffic` from two
# `rocprofv3 --pmc` runs of the default bench (FETCH_SIZE, then WRITE_SIZE) and read back here.
# A figure is reported only for the workload it was measured on and only while the kernel
# source still has the digest it was measured with; otherwise `traffic` is null.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")
KERNEL_SOURCES = {
    # the fp32-state kernel and the access helpers it streams its tile with: from the helpers'
    # comment to the start of the bf16-state section
    "ssm": ("ssm_update.hip", "// The state tile goes through buffer accesses",
            "// Same update with the state stored as bf16"),
    "attention": ("attn_mfma.hip", None, None),          # attention + merge + preparation kernels
}
KERNEL_MATCH = {"ssm": ("ssm_update_kernel", "ssm_update_mamba2_kernel"), "attention": ("attn_mfma_kernel", "attn_merge_runs_kernel")}


def source_digest(kind):
    """Digest of a kernel's source as the compiler sees it: comments and white space do not
    count, so rewording a comment does not retire a measurement."""
    import hashlib
    import re
    name, start, stop = KERNEL_SOURCES[kind]
    try:
        text = open(os.path.join(ROOT, "paper_2605_22416_amd", "csrc", name)).read()
        if start is not None:
            text = text[text.index(start):text.index(stop)]
    except (OSError, ValueError):
        return None
    text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
    text = re.sub(r"//[^\n]*", " ", text)          # the sources hold no "//" inside string literals
    return hashlib.sha256(" ".join(text.split()).encode()).hexdigest()[:16]


def measured_traffic(kind, batch, workload, seed):
    """HBM bytes per layer of one kernel kind from profiles/traffic.json, or None."""
    try:
        rec = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        return None
    k = rec.get("kernels", {}).get(kind)
    if (k is None or k.get("source_sha256_16") != source_digest(kind) or rec.get("batch") != batch
            or rec.get("workload") != workload or rec.get("seed") != seed):
        return None
    return k["bytes_per_layer"]


def write_traffic(fetch_csv, write_csv, batch, workload, seed):
    """Turns the counter_collection.csv files of two rocprofv3 --pmc runs of this bench
    (FETCH_SIZE and WRITE_SIZE, KiB per dispatch) into profiles/traffic.json.  Each counter is
    scaled by what it reads for the migration copy kernel, whose dispatches move a known number
    of bytes each way: grid size / 1024 work-items per 64 KiB page."""
    import csv
    page = 65536
    out = {"batch": batch, "workload": workload, "seed": seed, "kernels": {}, "scale": {},
           "unit": "HBM bytes per layer (fetch + write), averaged over the run's launches"}
    per_kind = {}
    for counter, path in (("FETCH_SIZE", fetch_csv), ("WRITE_SIZE", write_csv)):
        known = seen = 0.0
        sums = {k: [0.0, 0] for k in KERNEL_MATCH}
        parts = {k: {m: [0.0, 0] for m in KERNEL_MATCH[k]} for k in KERNEL_MATCH}
        for row in csv.DictReader(open(path)):
            if row["Counter_Name"] != counter:
                continue
            name, val = row["Kernel_Name"], float(row["Counter_Value"]) * 1024.0
            if "migrate_copy_kernel" in name:
                known += int(row["Grid_Size"]) // 1024 * page
                seen += val
            for kind, matches in KERNEL_MATCH.items():
                for m in matches:
                    if m in name:
                        parts[kind][m][0] += val
                        parts[kind][m][1] += 1
        if seen <= 0:
            raise SystemExit("no migrate_copy_kernel dispatch in %s: cannot scale %s" % (path, counter))
        scale = known / seen
        out["scale"][counter] = {"factor": scale, "copy_bytes_known": known, "copy_bytes_read": seen}
        for kind in KERNEL_MATCH:
            total = sum(v[0] / v[1] for v in parts[kind].values() if v[1])     # per launch, kernels of a layer added
            per_kind.setdefault(kind, {})[counter] = total * scale
    for kind, c in per_kind.items():
        out["kernels"][kind] = {"bytes_per_layer": int(round(c["FETCH_SIZE"] + c["WRITE_SIZE"])),
                                "fetch_bytes": int(round(c["FETCH_SIZE"])), "write_bytes": int(round(c["WRITE_SIZE"])),
                                "kernels": list(KERNEL_MATCH[kind]), "source_sha256_16": source_digest(kind)}
    out["command"] = ("rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir> -o f -- python3 bench.py "
                      "--no-cpu-baseline --no-capacity-sweep --no-kernel-events --steps 4 --warmup 1   (and the same with "
                      "WRITE_SIZE); then python3 bench.py --write-traffic <f_counter_collection.csv> "
                      "<w_counter_collection.csv>")
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print(json.dumps(out))


def attention_bytes(spec, ctx):
    """Algorithmic bytes of one attention layer for one request: valid K/V tokens,
    q in, o out, one handle + one table entry per page."""
    e = spec.elem_bytes
    pages = (int(ctx) + spec.page_tokens - 1) // spec.page_tokens
    return (int(ctx) * 2 * spec.n_kv_heads * spec.head_dim * e + spec.n_q_heads * spec.head_dim * e
            + spec.n_q_heads * spec.head_dim * 4 + pages * 8)


def ssm_bytes(spec):
    """Algorithmic bytes of one SSM layer for one request: state read + write,
    x in, y out, B, C, dt and the handle + table entry."""
    e = spec.elem_bytes
    H, P, N = spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate
    if spec.conv_kernel:
        # the token's x, B, C channels enter once, before the convolution; its window is read
        # and written; the fp32 values between convolution and recurrence are not counted
        return (2 * H * P * N * spec.state_bytes + 2 * spec.conv_window_bytes + spec.conv_dim * e
                + H * P * 4 + H * 4 + 8)
    return 2 * H * P * N * spec.state_bytes + H * P * e + H * P * 4 + 2 * N * e + H * 4 + 8


# ---- the CPU oracle, timed on the host cores (runs before anything touches the GPU, so that
# ---- worker processes can be forked) ---------------------------------------------------------
_ORACLE_JOB = {}


def _oracle_request(r):
    """One request through all layers of the oracle; worker-side.  Returns float32 outputs."""
    import numpy as np
    from oracle.sampled import RequestReference
    j = _ORACLE_JOB
    ref = RequestReference(j["spec"], j["seed"], r, int(j["ctx"][r]), bool(j["fresh"][r]))
    t0 = time.perf_counter()
    o, y = ref.step(j["inp"], j["conv"])
    return r, time.perf_counter() - t0, o.astype(np.float32), y.astype(np.float32)


def _worker_init():
    try:                                  # one numeric thread per worker process
        from threadpoolctl import threadpool_limits
        threadpool_limits(1)
    except Exception:
        pass


def host_workers():
    """Worker processes for the all-cores leg: the cores this process may run on, at most 16
    (a host's share of cores per GPU on an eight-GPU node)."""
    try:
        n = len(os.sched_getaffinity(0))
    except (AttributeError, OSError):
        n = os.cpu_count() or 1
    return max(1, min(16, n))


def oracle_pool_run(spec, seed, ctx, fresh, inp, conv, workers, keep_outputs):
    """Every request of a batch through the oracle, one request per task, longest first, on
    `workers` forked processes.  Returns (wall seconds, summed worker seconds, outputs)."""
    import multiprocessing as mp
    import numpy as np
    _ORACLE_JOB.update(spec=spec, seed=seed, ctx=ctx, fresh=fresh, inp=inp, conv=conv)
    order = [int(r) for r in np.argsort(-np.asarray(ctx, dtype=np.int64), kind="stable")]
    outs, busy = {}, 0.0
    with mp.get_context("fork").Pool(workers, initializer=_worker_init) as pool:
        pool.map(abs, range(workers))     # processes are up before the clock starts
        t0 = time.perf_counter()
        for r, dt, o, y in pool.imap_unordered(_oracle_request, order, chunksize=1):
            busy += dt
            if keep_outputs:
                outs[r] = (o, y)
        wall = time.perf_counter() - t0
    _ORACLE_JOB.clear()
    return wall, busy, outs


def batch_bytes(spec, ctx):
    return sum(spec.n_attn * attention_bytes(spec, c) + spec.n_ssm * ssm_bytes(spec) for c in ctx)


def cpu_baseline(spec, sc, inp, seed, conv=None, single_budget_s=6.0, others=True):
    """The oracle as it stands, on the host: every request of the batch once over all host
    cores (forked workers, a request per task), a single-thread leg on the first requests,
    and the other workload shapes (mixed_long at full size; agentic_burst and capacity cut to
    an eighth, as stated in their entries).  Returns (record, {request: (o, y)})."""
    from gen import inputs
    from oracle.sampled import RequestReference
    workers = host_workers()
    wall, busy, outs = oracle_pool_run(spec, seed, sc.ctx, sc.fresh, inp, conv, workers, True)
    nbytes = batch_bytes(spec, sc.ctx)
    rec = {"value": nbytes / wall / 1e9, "unit": "GB/s", "cores": workers,
           "cores_available": os.cpu_count(), "kind": "oracle",
           "sample": "all %d requests of the batch (all %d layers each), one request per task on %d "
                     "forked worker processes: %.1f s of wall time, %.1f s of worker time, same "
                     "algorithmic-byte numerator" % (sc.batch, len(spec.layer_kinds), workers, wall, busy),
           "us_per_step": wall * 1e6}
    # single thread, in this process
    done, elapsed = 0, 0.0
    for r in range(sc.batch):
        ref = RequestReference(spec, seed, r, int(sc.ctx[r]), bool(sc.fresh[r]))
        t0 = time.perf_counter()
        ref.step(inp, conv)
        elapsed += time.perf_counter() - t0
        done += 1
        if elapsed >= single_budget_s and done >= 2:
            break
    rec["single_thread"] = {"value": batch_bytes(spec, sc.ctx[:done]) / elapsed / 1e9, "unit": "GB/s",
                            "cores": 1, "sample": "requests 0..%d, %.1f s" % (done - 1, elapsed),
                            "us_per_step_extrapolated": elapsed / done * sc.batch * 1e6}
    if others and not spec.conv_kernel and spec.state_dtype == "f32":
        import numpy as np
        rec["other_configs"] = {}
        plans = [("mixed_long", 32, 1003, None, "full size: batch 32"),
                 ("agentic_burst", 32, 1004, None, "an eighth: batch 32 of 256"),
                 ("capacity", 64, 1005, 32768,
                  "an eighth: 64 of the 512 requests U[1024,8192] and one long request of 32768 tokens "
                  "(the workload has four of 262144)")]
        for name, batch, wseed, long_ctx, what in plans:
            wsc = inputs.make_scenario(spec, name, batch, wseed)
            ctx, fresh = wsc.ctx, wsc.fresh
            if long_ctx is not None:
                ctx = np.concatenate([ctx[:batch], np.array([long_ctx], dtype=np.uint32)])
                fresh = np.zeros(len(ctx), dtype=bool)
            winp = inputs.step_inputs(spec, len(ctx), wseed)
            w, bsy, _ = oracle_pool_run(spec, wseed, ctx, fresh, winp, None, workers, False)
            rec["other_configs"][name] = {"value": batch_bytes(spec, ctx) / w / 1e9, "unit": "GB/s",
                                          "cores": workers, "sample": what, "us_per_step": w * 1e6,
                                          "worker_seconds": bsy, "tokens": int(np.asarray(ctx, dtype=np.int64).sum())}
    return rec, outs


# The default workload is the one the headline metric is quoted on; the others are the
# remaining workload shapes, runnable for their own numbers (contents zero-filled where a
# full fill would take minutes: timing does not depend on the values).
WORKLOADS = {
    "uniform_short": dict(batch=64, seed=1002, scenario=dict(headroom=1.2), fill=True,
                          churn=(272, 28), mig_pages=128, sweep=(64, 1024, 3072),
                          text="uniform_short contexts U[128,2048], pools 1.2x demand"),
    "mixed_long": dict(batch=32, seed=1003, scenario=dict(occupancy=0.95), fill=True,
                       churn=(64, 28), mig_pages=1024, sweep=(64, 1024),
                       text="mixed_long contexts lognormal(median 4096, sigma 1) in [256,65536], "
                            "KV pool 95 % occupied"),
    "agentic_burst": dict(batch=256, seed=1004, scenario=dict(headroom=1.2), fill=False,
                          churn=(224, 32), mig_pages=512, sweep=(64, 1024),
                          text="agentic_burst: half U[64,1024], half newly admitted with 1-4 pages"),
    "capacity": dict(batch=512, seed=1005, scenario=dict(headroom=1.7), fill=False,
                     churn=(272, 28), mig_pages=128, sweep=(64, 1024, 16384),
                     text="capacity: U[1024,8192] + 4 x 262144 tokens, pools filling about 200 GB"),
}


def capacity_migration_sweep(spec, stream, batches=((64, 6), (1024, 6), (16384, 4))):
    """Migration batches of 64, 1024 and 16384 pages on pools that fill about 200 GB of HBM
    (the capacity-scale workload's pools: 512 requests of U[1024,8192] tokens plus four of
    262144), worst case: the KV pool's slots are ranked from the top down, so the live pages
    occupy its highest slots and EVERY slot a migration vacates holds a live page that has to
    be copied.  Contents are whatever the fresh arena holds (a copy does not care).  Capacity
    is not given back between batches: each one vacates the next stretch of live pages.
    Wall time of the avmp_migrate call up to the end of its copies, device idle before."""
    import numpy as np
    import torch
    from gen import inputs
    from paper_2605_22416_amd import binding as av
    sc = inputs.make_scenario(spec, "capacity", 512, 1005, headroom=1.7, permute=False)
    need = sc.arena_bytes + (2 << 30)
    free = torch.cuda.mem_get_info()[0]
    if free < need:
        return {"skipped": "needs %.0f GB of free HBM, %.0f GB are free" % (need / 1e9, free / 1e9)}
    n_slots = sc.arena_bytes // spec.kv_page_bytes
    top_down = np.arange(n_slots - 1, -1, -1, dtype=np.uint32)       # rank of slot s: highest slot first
    arena = torch.empty(sc.arena_bytes, dtype=torch.uint8, device="cuda:0")
    cfg, keep = av.make_config(spec.dtype, spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.ssm_heads,
                               spec.ssm_headdim, spec.ssm_dstate, sc.kv_capacity, sc.ssm_capacity,
                               slot_rank=[top_down, None])
    rc, p = av.avmp_pools_create(cfg, arena, sc.arena_bytes)
    assert rc == av.AVMP_OK, av.avmp_last_error()
    live = int(sc.n_pages.sum()) * spec.n_attn
    left = live
    while left:
        n = min(left, 1 << 18)
        rc, _ = av.avmp_alloc(p, 0, n)
        assert rc == av.AVMP_OK, av.avmp_last_error()
        left -= n
    assert av.avmp_flush(p, stream) == av.AVMP_OK
    torch.cuda.synchronize()
    rows = []
    av.avmp_profile_enable(p, True)
    for n, reps in batches:
        walls, kernels = [], []
        for _ in range(reps):
            av.avmp_profile_read(p, stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            rc, res = av.avmp_migrate(p, 0, n, stream)
            t1 = time.perf_counter()
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            assert rc == av.AVMP_OK and res.units_copied == n, (rc, res.units_copied, av.avmp_last_error())
            rc, pr = av.avmp_profile_read(p, stream)
            walls.append((t2 - t0, t1 - t0))
            kernels.append(pr["migrate_copy"][0] * 1e-3)
        wall = sorted(w for w, _ in walls)[len(walls) // 2]
        host = sorted(h for _, h in walls)[len(walls) // 2]
        kern = sorted(kernels)[len(kernels) // 2]
        moved = 2.0 * n * spec.kv_page_bytes
        rows.append({"pages": n, "pages_copied": n, "repeats": reps, "us_wall_median": wall * 1e6,
                     "us_host_call_median": host * 1e6, "us_copy_kernels_median": kern * 1e6,
                     "pages_per_s_wall": n / wall, "GBps_wall": moved / wall / 1e9,
                     "GBps_copy_kernels": moved / kern / 1e9 if kern > 0 else None,
                     "pages_per_s_best": n / min(w for w, _ in walls)})
    av.avmp_profile_enable(p, False)
    st = av.avmp_stats(p)
    torch.cuda.synchronize()
    av.avmp_pools_destroy(p)
    del arena
    torch.cuda.empty_cache()
    return {"arena_GB": sc.arena_bytes / 1e9, "kv_pages_live": live, "kv_capacity_pages_at_start": sc.kv_capacity,
            "placement": "live pages in the pool's highest slots: every vacated slot is live (worst case)",
            "bound_pages_per_s": HBM_PEAK_GBPS * 1e9 / (2 * spec.kv_page_bytes),
            "rows": rows, "migrations": st["migrations"], "units_copied": st["units_copied"]}


def migration_compare(args, spec, sc, chunk):
    """The same migrations on two fresh copies of the same pools (all units live where the
    scenario puts them, contents zero): once moving live units with the copy kernel, once by
    exchanging the physical chunks behind source and destination slot.  Wall time per call,
    device idle before and after."""
    import torch
    from paper_2605_22416_amd import binding as av
    from paper_2605_22416_amd.session import DeviceSession
    ratio = spec.ssm_block_bytes // spec.kv_page_bytes
    plan = [(0, n) for n in (64, 1024, 16384)] + [(1, n) for n in (1, 16, 256)]
    rows = []
    setup = {}
    for mode in ("copy", "remap"):
        t0 = time.perf_counter()
        ses = DeviceSession(sc, fill_byte=None, vmm_chunk=chunk, remap=(mode == "remap"))
        torch.cuda.synchronize()
        setup[mode] = time.perf_counter() - t0
        for donor, n in plan:
            st = av.avmp_stats(ses.p)
            if n > st["free"][donor]:
                continue
            unit = spec.kv_page_bytes if donor == 0 else spec.ssm_block_bytes
            if mode == "remap" and unit % chunk != 0:
                continue                     # such a donor copies in either mode
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            rc, res = av.avmp_migrate(ses.p, donor, n)
            assert rc == av.AVMP_OK, av.avmp_last_error()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t1
            rows.append({"mode": mode, "donor": "kv" if donor == 0 else "ssm", "units": n,
                         "live_units_moved": int(res.units_copied), "seconds": dt,
                         "capacity_units_per_s": n / dt,
                         "moved_GBps": res.units_copied * unit / dt / 1e9,
                         "us_per_moved_unit": dt / res.units_copied * 1e6 if res.units_copied
                         else None})
            # give the capacity back so that the next entry starts from the same split
            back = n * spec.kv_page_bytes // spec.ssm_block_bytes if donor == 0 else n * ratio
            rc, _ = av.avmp_migrate(ses.p, 1 - donor, back)
            assert rc == av.AVMP_OK, av.avmp_last_error()
        torch.cuda.synchronize()
        ses.close()
    return {"metric": "migration_copy_vs_physical_remap", "unit": "capacity units/s",
            "config": {"workload": "%s, batch %d, seed %d" % (args.workload, sc.batch, args.seed),
                       "arena_GB": sc.arena_bytes / 1e9, "vmm_chunk_KiB": chunk // 1024,
                       "kv_page_bytes": spec.kv_page_bytes, "ssm_block_bytes": spec.ssm_block_bytes},
            "arena_setup_s": setup, "rows": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="uniform_short")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--state-dtype", choices=("f32", "bf16"), default="f32",
                    help="storage type of the SSM state blocks (f32 is the headline configuration)")
    ap.add_argument("--conv-kernel", type=int, default=0, choices=(0, 2, 3, 4),
                    help="taps of the short convolution in front of the recurrence; the SSM blocks "
                         "then also hold its window (0, the headline configuration: none)")
    ap.add_argument("--pad-ssm-to-kv-page", action="store_true",
                    help="pad every SSM block to a whole number of KV pages (the unified-pool sizing); "
                         "with a convolution window the state tiles then keep their 64 KiB alignment")
    ap.add_argument("--graph", action="store_true",
                    help="replay the decode part of the step from a HIP graph captured once (churn "
                         "and migration stay eager; their table updates are flushed before each replay)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-capacity-sweep", action="store_true",
                    help="skip the migration sweep on pools filling about 200 GB of HBM")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="skip the second pass that brackets every kernel with HIP events")
    ap.add_argument("--fill-threads", type=int, default=16)
    ap.add_argument("--backing", choices=("plain", "vmm"), default="plain",
                    help="plain (default): the arena is a torch tensor; vmm: it comes from the library's "
                         "own allocator, attached through the HIP virtual-memory API in chunks (same "
                         "speed with large chunks).  The timed step migrates by copy either way")
    ap.add_argument("--vmm-chunk-kib", type=int, default=None,
                    help="chunk size of the vmm arena (default 1 GiB; 2 MiB for --migration-compare, "
                         "where units must be whole chunks)")
    ap.add_argument("--write-traffic", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="instead of the benchmark: write profiles/traffic.json from the "
                         "counter_collection.csv files of two rocprofv3 --pmc runs of this bench "
                         "(FETCH_SIZE, WRITE_SIZE)")
    ap.add_argument("--migration-compare", action="store_true",
                    help="instead of the decode benchmark: time migrations of the same pools done "
                         "by copy and by exchanging physical chunks, on a vmm arena")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on ONE GPU (pools, table and kernels are device-local; "
              "no collectives exist to measure); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.write_traffic:
        wl = WORKLOADS[args.workload]
        write_traffic(args.write_traffic[0], args.write_traffic[1],
                      wl["batch"] if args.batch is None else args.batch, args.workload,
                      wl["seed"] if args.seed is None else args.seed)
        return

    import numpy as np
    from gen import inputs

    spec = inputs.JAMBA_MINI
    if args.state_dtype != "f32":
        spec = inputs.with_state_dtype(spec, args.state_dtype)
    if args.conv_kernel:
        spec = inputs.with_conv(spec, args.conv_kernel)
    if args.pad_ssm_to_kv_page:
        spec = inputs.with_padded_blocks(spec)
    wl = WORKLOADS[args.workload]
    args.batch = wl["batch"] if args.batch is None else args.batch
    args.seed = wl["seed"] if args.seed is None else args.seed
    sc = inputs.make_scenario(spec, args.workload, args.batch, args.seed, **wl["scenario"])
    inp = inputs.step_inputs(spec, sc.batch, args.seed)
    conv = inputs.conv_weights(spec, args.seed) if spec.conv_kernel else None
    if not wl["fill"]:
        args.no_cpu_baseline = True          # nothing to compare: the arena will hold zeros
    # The oracle legs fork worker processes, so they run before this process touches the GPU.
    base, ref_out = None, {}
    if not args.no_cpu_baseline and not args.migration_compare:
        base, ref_out = cpu_baseline(spec, sc, inp, args.seed, conv=conv,
                                     others=args.workload == "uniform_short")

    import torch
    from paper_2605_22416_amd import binding as av
    from paper_2605_22416_amd.session import DeviceSession

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback", file=sys.stderr)
        sys.exit(1)
    # SSM blocks count down from the top of the arena.  4 MiB blocks on 4 MiB boundaries measured
    # 87.1 us per SSM layer against 88.5 us at a 64 KiB-granular offset and 91.5 us at an odd
    # multiple of 2 MiB, so the arena's size is made a multiple of 4 MiB for them; 2 MiB blocks
    # (bf16 state) measured 1 % better where the pool sizes happen to put them, and stay there
    block_pow2 = spec.ssm_block_bytes & -spec.ssm_block_bytes
    slack = -sc.arena_bytes % block_pow2 if block_pow2 >= (4 << 20) else 0
    if slack:
        sc = inputs.make_scenario(spec, args.workload, args.batch, args.seed, slack_bytes=slack,
                                  **wl["scenario"])
    vmm_chunk = None
    if args.backing == "vmm" and not args.migration_compare and av.avmp_vmm_min_chunk() == 0:
        print("bench.py: this device has no virtual-memory support; using --backing plain", file=sys.stderr)
        args.backing = "plain"
    if args.backing == "vmm" or args.migration_compare:
        if args.vmm_chunk_kib is None:
            args.vmm_chunk_kib = 2048 if args.migration_compare else 1 << 20
        vmm_chunk = args.vmm_chunk_kib * 1024
        slack += -sc.arena_bytes % vmm_chunk       # the arena must be whole chunks
        sc = inputs.make_scenario(spec, args.workload, args.batch, args.seed, slack_bytes=slack,
                                  **wl["scenario"])
        assert sc.arena_bytes % vmm_chunk == 0
    if args.migration_compare:
        print(json.dumps(migration_compare(args, spec, sc, vmm_chunk)))
        return
    t0 = time.perf_counter()
    ses = DeviceSession(sc, fill_byte=None if wl["fill"] else 0, vmm_chunk=vmm_chunk, remap=False)
    if wl["fill"]:
        ses.fill(threads=args.fill_threads)
    setup_s = time.perf_counter() - t0
    stream = torch.cuda.current_stream()
    st, keep, o, y = ses.prepare_step(inp, conv=conv)

    # ---- correctness of the very first step against the oracle, every request ----------
    parity = None
    ses.launch(st, stream)
    torch.cuda.synchronize()
    if ref_out:
        o_h, y_h = o.cpu().numpy(), y.cpu().numpy()
        eo = ey = 0.0
        for r, (ref_o, ref_y) in ref_out.items():
            eo = max(eo, float((np.abs(o_h[:, r] - ref_o).max(axis=-1)
                                / np.maximum(np.abs(ref_o).max(axis=-1), 1e-30)).max()))
            ey = max(ey, float((np.abs(y_h[:, r] - ref_y).max(axis=-1)
                                / np.maximum(np.abs(ref_y).max(axis=-1), 1e-30)).max()))
        parity = {"requests": len(ref_out), "attention_max_rel_err": eo, "ssm_max_rel_err": ey,
                  "tolerance": 2e-3}
        ref_out = None
        if eo > 2e-3 or ey > 2e-3:
            print("bench.py: GPU step disagrees with the oracle: %r" % parity, file=sys.stderr)
            sys.exit(1)

    # ---- the timed step ----------------------------------------------------------------
    churn_kv, churn_ssm = wl["churn"]
    free0 = av.avmp_stats(ses.p)["free"]
    # small batches leave less room than the preset asks for
    churn_kv, churn_ssm = max(1, min(churn_kv, free0[0] // 2)), max(1, min(churn_ssm, free0[1]))
    rc, ghost_kv = av.avmp_alloc(ses.p, 0, churn_kv)
    assert rc == av.AVMP_OK, av.avmp_last_error()
    rc, ghost_ssm = av.avmp_alloc(ses.p, 1, churn_ssm)
    assert rc == av.AVMP_OK, av.avmp_last_error()
    mig_pages = min(wl["mig_pages"], (free0[0] - churn_kv) // 64 * 64)
    mig_blocks_back = mig_pages * spec.kv_page_bytes // spec.ssm_block_bytes
    copies = [0]

    graph = None
    if args.graph:
        # everything from here on runs on one side stream, which is also the capture stream
        stream = torch.cuda.Stream()
        torch.cuda.set_stream(stream)
        assert av.avmp_flush(ses.p, stream) == av.AVMP_OK
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        graph.capture_begin()
        rc = av.avmp_decode_step(ses.p, st, stream)
        graph.capture_end()
        assert rc == av.AVMP_OK, av.avmp_last_error()
        torch.cuda.synchronize()
    replay = [graph is not None]

    def one_step():
        nonlocal ghost_kv, ghost_ssm
        assert av.avmp_free(ses.p, np.concatenate([ghost_kv, ghost_ssm])) == av.AVMP_OK
        rc1, ghost_kv = av.avmp_alloc(ses.p, 0, churn_kv)
        rc2, ghost_ssm = av.avmp_alloc(ses.p, 1, churn_ssm)
        assert rc1 == av.AVMP_OK and rc2 == av.AVMP_OK
        if replay[0]:
            assert av.avmp_flush(ses.p, stream) == av.AVMP_OK     # the graph holds no queued updates
            graph.replay()
        else:
            ses.launch(st, stream)
        if mig_pages == 0 or mig_blocks_back == 0:      # no room for a round trip at this size
            return
        rc1, res = av.avmp_migrate(ses.p, 0, mig_pages, stream)
        assert rc1 == av.AVMP_OK, av.avmp_last_error()
        copies[0] += res.units_copied
        rc2, res = av.avmp_migrate(ses.p, 1, mig_blocks_back, stream)
        assert rc2 == av.AVMP_OK, av.avmp_last_error()
        copies[0] += res.units_copied * (spec.ssm_block_bytes // spec.kv_page_bytes)

    # a fixed number of untimed steps first (clocks and caches of a fresh process settle), then the
    # requested warm-up: the figure is a steady-state one whatever --warmup says
    for _ in range(PREWARM_STEPS + args.warmup):
        one_step()
    torch.cuda.synchronize()
    # timed region: exactly `steps` steps, nothing but the path on the stream
    copies[0] = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    copies_timed = copies[0]
    # the same steps again with one event per step on the stream: the spread of step times
    # (an event record takes a few us of stream time, so it stays out of the region above)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    marks[0].record(stream)
    for i in range(args.steps):
        one_step()
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    per_step_us = np.array([marks[i].elapsed_time(marks[i + 1]) * 1e3 for i in range(args.steps)])
    step_us = {"median": float(np.median(per_step_us)), "p10": float(np.percentile(per_step_us, 10)),
               "p90": float(np.percentile(per_step_us, 90)), "min": float(per_step_us.min()),
               "max": float(per_step_us.max())}
    # the same `steps` steps again with a HIP event pair around every kernel launch (on the
    # launch stream): per-kernel durations for the roofline.  The event pairs cost a few us
    # per launch, which is why the headline region above runs without them.
    events = not args.no_kernel_events
    wall_ev, prof, empty_pair_us = None, {}, None
    if events:
        replay[0] = False                 # per-kernel events need eager launches
        av.avmp_profile_enable(ses.p, True)
        av.avmp_profile_read(ses.p, stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one_step()
        torch.cuda.synchronize()
        wall_ev = time.perf_counter() - t0
        rc, prof = av.avmp_profile_read(ses.p, stream)
        av.avmp_profile_enable(ses.p, False)
        # what such a pair reads with nothing between its two records: the share of every
        # per-kernel figure below that is the measurement, not the kernel
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                 for _ in range(64)]
        for ea, eb in pairs:
            ea.record(stream)
            eb.record(stream)
        torch.cuda.synchronize()
        empty_pair_us = float(np.median([ea.elapsed_time(eb) * 1e3 for ea, eb in pairs]))
    copies[0] = copies_timed
    rc, faults = av.avmp_device_faults(ses.p)
    assert rc == av.AVMP_OK and faults == 0, "untranslatable handles: %d" % faults
    assert np.isfinite(o.cpu().numpy()).all() and np.isfinite(y.cpu().numpy()).all()

    attn_layer_bytes = sum(attention_bytes(spec, c) for c in sc.ctx)
    ssm_layer_bytes = sc.batch * ssm_bytes(spec)
    copy_bytes_step = copies[0] / args.steps * 2 * spec.kv_page_bytes
    step_bytes = spec.n_attn * attn_layer_bytes + spec.n_ssm * ssm_layer_bytes + copy_bytes_step
    ms_per_step = wall / args.steps * 1e3
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    kernels = {}
    per_launch = {"attention": attn_layer_bytes, "ssm": ssm_layer_bytes}
    if spec.conv_kernel:
        # per kernel, the fp32 x, B, C between the two count: written by one, read by the other
        H, P, N, e = spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate, spec.elem_bytes
        per_launch["ssm"] = sc.batch * (2 * spec.ssm_state_bytes + 2 * H * P * 4 + 2 * N * 4 + H * 4 + 8)
        per_launch["conv"] = (sc.batch * (2 * spec.conv_window_bytes + spec.conv_dim * (e + 4) + 8)
                              + (spec.conv_kernel + 1) * spec.conv_dim * e)
    for name, (ms, n) in prof.items():
        if n:
            k = {"launches": int(n), "avg_us": ms / n * 1e3}
            if name in per_launch:
                k["GBps"] = per_launch[name] / (ms / n * 1e-3) / 1e9
            kernels[name] = k
    roofline = None
    if "ssm" in kernels:
        a = kernels["ssm"]["GBps"]
        if args.state_dtype != "f32":
            ssm_kernel = "ssm_update_bf16state_kernel"
        elif spec.ssm_dstate == 128 and spec.ssm_headdim == 64:
            ssm_kernel = "ssm_update_mamba2_kernel"
        else:
            ssm_kernel = "ssm_update_kernel"
        roofline = {"kernel": ssm_kernel, "bound": "hbm", "achieved": a,
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": a / HBM_PEAK_GBPS,
                    "traffic": measured_traffic("ssm", sc.batch, args.workload, args.seed)
                    if args.state_dtype == "f32" and not spec.conv_kernel else None,
                    "bytes_per_launch": per_launch["ssm"],
                    "avg_launch_us": kernels["ssm"]["avg_us"]}
    roofline_attention = None
    if "attention" in kernels:
        # everything an attention layer launches: the attention kernel, the merge of its partial
        # results, and the layer's share of the once-per-step preparation (run plan + translation
        # of all KV handles)
        parts = {"attention": kernels["attention"]["avg_us"]}
        if "attention_merge" in kernels:
            parts["attention_merge"] = kernels["attention_merge"]["avg_us"]
        if "attention_prepare" in kernels:
            parts["attention_prepare_share"] = (kernels["attention_prepare"]["avg_us"]
                                                * kernels["attention_prepare"]["launches"]
                                                / kernels["attention"]["launches"])
        layer_us = sum(parts.values())
        a = attn_layer_bytes / (layer_us * 1e-6) / 1e9
        roofline_attention = {"kernel": "attention kernel + merge kernel + attn_prepare_kernel / attention layers",
                              "bound": "hbm", "achieved": a,
                              "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": a / HBM_PEAK_GBPS,
                              "traffic": measured_traffic("attention", sc.batch, args.workload, args.seed),
                              "bytes_per_launch": attn_layer_bytes,
                              "avg_layer_us": layer_us, "avg_us_by_kernel": parts}

    # ---- alloc / free churn alone (outside the timed region): host logic + table scatter --
    n_rounds = 200
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(n_rounds):
        assert av.avmp_free(ses.p, np.concatenate([ghost_kv, ghost_ssm])) == av.AVMP_OK
        rc1, ghost_kv = av.avmp_alloc(ses.p, 0, churn_kv)
        rc2, ghost_ssm = av.avmp_alloc(ses.p, 1, churn_ssm)
        assert rc1 == av.AVMP_OK and rc2 == av.AVMP_OK
        assert av.avmp_flush(ses.p, stream) == av.AVMP_OK      # table entries + zero fills of the blocks
    torch.cuda.synchronize()
    dt_churn = time.perf_counter() - t1
    churn = {"handles_per_round": int(churn_kv + churn_ssm), "rounds": n_rounds,
             "us_per_round": dt_churn / n_rounds * 1e6,
             "handles_freed_and_allocated_per_s": 2 * (churn_kv + churn_ssm) * n_rounds / dt_churn}

    # ---- migration sweep (outside the timed region): pages/s of capacity moved ----------
    sweep = []
    av.avmp_profile_enable(ses.p, True)
    for n in wl["sweep"]:
        if n > av.avmp_stats(ses.p)["free"][0]:
            continue
        walls, kernel_ms, copied = [], [], 0
        for _ in range(5):               # median of five: the same capacity goes out and comes back
            av.avmp_profile_read(ses.p, stream)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            rc, res = av.avmp_migrate(ses.p, 0, n, stream)
            assert rc == av.AVMP_OK
            torch.cuda.synchronize()
            walls.append(time.perf_counter() - t1)
            rc, pr = av.avmp_profile_read(ses.p, stream)
            kernel_ms.append(pr["migrate_copy"][0])
            copied = max(copied, int(res.units_copied))     # the first pass moves the live pages down
            if res.recipient_gain:       # give it back (what did not make a whole block waits in the gap)
                rc2, _ = av.avmp_migrate(ses.p, 1, res.recipient_gain, stream)
                assert rc2 == av.AVMP_OK
        # later passes find the vacated range empty: the first pass is the one that copies
        dt_wall, kms = walls[0], kernel_ms[0]
        sweep.append({"pages": n, "copied": copied,
                      "pages_per_s_wall": n / dt_wall,
                      "pages_per_s_wall_nothing_to_copy": n / sorted(walls[1:])[len(walls[1:]) // 2],
                      "copy_GBps_kernel": (copied * 2 * spec.kv_page_bytes / (kms * 1e-3) / 1e9)
                      if kms > 0 else None})
    av.avmp_profile_enable(ses.p, False)
    torch.cuda.synchronize()
    ses.close()
    # ---- the capacity-scale migration sweep (pools filling about 200 GB), once the arena of
    # ---- the decode benchmark is released ----------------------------------------------------
    sweep_capacity = None
    if args.workload == "uniform_short" and not args.no_capacity_sweep and args.backing == "plain":
        torch.cuda.empty_cache()
        try:
            sweep_capacity = capacity_migration_sweep(inputs.JAMBA_MINI, stream)
        except (AssertionError, RuntimeError, MemoryError) as e:
            # an extra leg: the headline line is printed whatever happens to it
            sweep_capacity = {"failed": "%s: %s" % (type(e).__name__, e)}

    out = {
        "metric": "hybrid_decode_step_achieved_hbm_GBps_batch%d" % sc.batch,
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "us_per_step": ms_per_step * 1e3, "step_us": step_us,
        "untimed_steps_before_warmup": PREWARM_STEPS,
        "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBPS,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "jamba_mini_like decode step, %s, batch %d, 4 attention + 28 SSM "
                               "layers, seeded random placement; step = churn (%d pages + %d blocks "
                               "freed and re-allocated) + decode + %d-page migration round trip"
                               % (wl["text"], sc.batch, churn_kv, churn_ssm, mig_pages),
                   "name": args.workload, "batch": sc.batch, "seed": args.seed,
                   "ssm_state_dtype": args.state_dtype, "ssm_conv_kernel": args.conv_kernel,
                   "ssm_pad_to_kv_page": bool(args.pad_ssm_to_kv_page),
                   "decode_from_hip_graph": bool(args.graph),
                   "arena_backing": args.backing if vmm_chunk is None
                   else "vmm, %d KiB chunks" % args.vmm_chunk_kib,
                   "arena_GB": sc.arena_bytes / 1e9},
        "ms_per_step_with_kernel_events": (wall_ev / args.steps * 1e3) if wall_ev else None,
        "empty_event_pair_us": empty_pair_us,
        "algorithmic_bytes_per_step": step_bytes,
        "migrated_pages_per_s": 2 * mig_pages * args.steps / wall,
        "kernels": kernels, "migration_sweep": sweep, "migration_sweep_capacity": sweep_capacity,
        "churn": churn, "setup_s": setup_s,
        "roofline": roofline, "roofline_attention": roofline_attention, "cpu_baseline": base,
        "parity_sample": parity,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
