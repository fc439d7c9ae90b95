"""ctypes binding of libavmp.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/avmp.h).
Device buffers are passed as torch tensors (their data_ptr is taken) or as
integer addresses; streams as torch streams or integer hipStream_t values.
There is no fallback: if the native library is missing, importing this module
raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libavmp.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "native library %s is missing: build it with `python -m paper_2605_22416_amd.build` "
        "(there is no CPU fallback)" % LIB_PATH)


def _load():
    """Load libavmp.so against the HIP runtime that torch has already loaded.

    The caller's device memory and streams come from torch, so the library must
    talk to the same runtime instance.  torch ships its own libamdhip64 (same
    soname as the system one); importing torch first makes the loader resolve
    libavmp's dependency to that instance.  Two runtimes in one process cannot
    share pointers, so that case is refused."""
    import torch  # noqa: F401
    tlib = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    global hip_runtime
    hip_runtime = C.CDLL(tlib if os.path.exists(tlib) else "libamdhip64.so", mode=C.RTLD_GLOBAL)
    handle = C.CDLL(LIB_PATH)
    runtimes = set()
    with open("/proc/self/maps") as f:
        for line in f:
            path = line.split()[-1]
            if "libamdhip64" in os.path.basename(path):
                runtimes.add(os.path.realpath(path))
    if len(runtimes) > 1:
        raise ImportError("two HIP runtimes are loaded in this process (%s): import "
                          "paper_2605_22416_amd.binding before anything else loads libamdhip64"
                          % ", ".join(sorted(runtimes)))
    return handle


hip_runtime = None      # the HIP runtime both torch and the library use (set by _load)
lib = _load()

AVMP_OK, AVMP_ERR_CAPACITY, AVMP_ERR_INVALID_HANDLE, AVMP_ERR_INVALID_ARG, AVMP_ERR_DEVICE = range(5)
AVMP_POOL_KV, AVMP_POOL_SSM = 0, 1
AVMP_F32, AVMP_BF16 = 0, 1
AVMP_LAYER_ATTENTION, AVMP_LAYER_SSM = 0, 1
AVMP_INVALID_HANDLE = 0xFFFFFFFF


class avmp_config_t(C.Structure):
    _fields_ = [("dtype", C.c_uint32), ("attention_page_tokens", C.c_uint32),
                ("n_q_heads", C.c_uint32), ("n_kv_heads", C.c_uint32), ("head_dim", C.c_uint32),
                ("ssm_heads", C.c_uint32), ("ssm_headdim", C.c_uint32), ("ssm_dstate", C.c_uint32),
                ("ssm_state_dtype", C.c_uint32), ("ssm_conv_kernel", C.c_uint32),
                ("ssm_pad_to_kv_page", C.c_uint32), ("kv_capacity", C.c_uint32), ("ssm_capacity", C.c_uint32),
                ("max_vid", C.c_uint32 * 2), ("slot_rank", C.POINTER(C.c_uint32) * 2)]


class avmp_geometry_t(C.Structure):
    _fields_ = [("unit_bytes", C.c_uint64 * 2), ("ssm_native_bytes", C.c_uint64),
                ("usable_bytes", C.c_uint64),
                ("max_slots", C.c_uint32 * 2)]


class avmp_migrate_result_t(C.Structure):
    _fields_ = [("units_copied", C.c_uint32), ("recipient_gain", C.c_uint32),
                ("bytes_wasted", C.c_uint64)]


class avmp_stats_t(C.Structure):
    _fields_ = [("capacity", C.c_uint32 * 2), ("live", C.c_uint32 * 2), ("free_units", C.c_uint32 * 2),
                ("gap_bytes", C.c_uint64), ("ops", C.c_uint64), ("capacity_errors", C.c_uint64),
                ("migrations", C.c_uint64), ("units_copied", C.c_uint64),
                ("bytes_migrated", C.c_uint64), ("bytes_wasted", C.c_uint64)]


class avmp_step_t(C.Structure):
    _fields_ = [("batch", C.c_uint32), ("n_layers", C.c_uint32), ("layer_kind", C.c_void_p),
                ("max_pages", C.c_uint32), ("kv_handles", C.c_void_p), ("ctx", C.c_void_p),
                ("q", C.c_void_p), ("o", C.c_void_p), ("ssm_handles", C.c_void_p),
                ("x", C.c_void_p), ("dt", C.c_void_p), ("A", C.c_void_p), ("B", C.c_void_p),
                ("C", C.c_void_p), ("y", C.c_void_p), ("k_new", C.c_void_p), ("v_new", C.c_void_p),
                ("xbc", C.c_void_p), ("conv_taps", C.c_void_p), ("conv_bias", C.c_void_p)]


(AVMP_K_ATTENTION, AVMP_K_ATTENTION_MERGE, AVMP_K_SSM, AVMP_K_MIGRATE_COPY, AVMP_K_TABLE,
 AVMP_K_CONV, AVMP_K_ATTENTION_PREPARE) = range(7)
AVMP_K_COUNT = 7
KERNEL_NAMES = ("attention", "attention_merge", "ssm", "migrate_copy", "table", "conv",
                "attention_prepare")


class avmp_profile_t(C.Structure):
    _fields_ = [("ms", C.c_double * AVMP_K_COUNT), ("launches", C.c_uint64 * AVMP_K_COUNT)]


class avmp_policy_t(C.Structure):
    _fields_ = [("threshold_low", C.c_double), ("threshold_high", C.c_double),
                ("migration_batch_size", C.c_uint32), ("reserved", C.c_uint32),
                ("min_rebalance_interval_ops", C.c_uint64)]


class avmp_policy_state_t(C.Structure):
    _fields_ = [("state", C.c_uint32), ("has_rebalanced", C.c_uint32),
                ("last_rebalance_op", C.c_uint64), ("rebalance_count", C.c_uint64),
                ("oom_events", C.c_uint64)]


AVMP_BALANCED, AVMP_KV_PRESSURED, AVMP_SSM_PRESSURED, AVMP_REBALANCING = range(4)

_P = C.c_void_p
lib.avmp_last_error.restype = C.c_char_p
lib.avmp_last_error.argtypes = []
lib.avmp_geometry.argtypes = [C.POINTER(avmp_config_t), C.c_size_t, C.POINTER(avmp_geometry_t)]
lib.avmp_pools_create.argtypes = [C.POINTER(avmp_config_t), _P, C.c_size_t, C.POINTER(_P)]
lib.avmp_pools_destroy.argtypes = [_P]
lib.avmp_alloc.argtypes = [_P, C.c_int, C.c_uint32, _P]
lib.avmp_free.argtypes = [_P, _P, C.c_uint32]
lib.avmp_migrate.argtypes = [_P, C.c_int, C.c_uint32, _P, C.POINTER(avmp_migrate_result_t)]
lib.avmp_decode_step.argtypes = [_P, C.POINTER(avmp_step_t), _P]
lib.avmp_absorb_gap.argtypes = [_P, C.c_int, C.POINTER(avmp_migrate_result_t)]
lib.avmp_decode_step_noalloc.argtypes = [_P, C.POINTER(avmp_step_t), _P]
lib.avmp_flush.argtypes = [_P, _P]
lib.avmp_workspace_reserve.argtypes = [_P, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32]
lib.avmp_workspace_info.argtypes = [_P, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
lib.avmp_translate.argtypes = [_P, _P, C.c_uint32, _P, _P]
lib.avmp_resolve.argtypes = [_P, C.c_uint32, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32),
                             C.POINTER(C.c_uint64)]
lib.avmp_stats.argtypes = [_P, C.POINTER(avmp_stats_t)]
lib.avmp_device_faults.argtypes = [_P, _P, C.POINTER(C.c_uint64)]
lib.avmp_policy_set.argtypes = [_P, C.POINTER(avmp_policy_t)]
lib.avmp_policy_state.argtypes = [_P, C.POINTER(avmp_policy_state_t)]
lib.avmp_alloc_auto.argtypes = [_P, C.c_int, C.c_uint32, _P, _P, C.POINTER(C.c_uint32)]
lib.avmp_profile_enable.argtypes = [_P, C.c_int]
lib.avmp_profile_read.argtypes = [_P, _P, C.POINTER(avmp_profile_t)]
lib.avmp_vmm_min_chunk.argtypes = []
lib.avmp_vmm_min_chunk.restype = C.c_uint64
lib.avmp_vmm_arena_create.argtypes = [C.c_uint64, C.c_uint64, C.POINTER(_P)]
lib.avmp_vmm_arena_base.argtypes = [_P]
lib.avmp_vmm_arena_base.restype = C.c_void_p
lib.avmp_vmm_arena_destroy.argtypes = [_P]
lib.avmp_migrate_by_remap.argtypes = [_P, _P]
for _f in ("avmp_vmm_arena_create", "avmp_vmm_arena_destroy", "avmp_migrate_by_remap"):
    getattr(lib, _f).restype = C.c_int
for _f in ("avmp_geometry", "avmp_pools_create", "avmp_pools_destroy", "avmp_alloc", "avmp_free",
           "avmp_migrate", "avmp_decode_step", "avmp_flush", "avmp_translate", "avmp_resolve",
           "avmp_stats", "avmp_device_faults", "avmp_profile_enable", "avmp_profile_read",
           "avmp_policy_set", "avmp_policy_state", "avmp_alloc_auto", "avmp_workspace_reserve",
           "avmp_workspace_info", "avmp_decode_step_noalloc", "avmp_absorb_gap"):
    getattr(lib, _f).restype = C.c_int


def avmp_last_error() -> str:
    return lib.avmp_last_error().decode()


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return int(t)


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    if hasattr(s, "cuda_stream"):
        return s.cuda_stream
    return int(s)


def make_config(dtype: str, n_q_heads: int, n_kv_heads: int, head_dim: int, ssm_heads: int,
                ssm_headdim: int, ssm_dstate: int, kv_capacity: int, ssm_capacity: int,
                slot_rank: Optional[Sequence[Optional[np.ndarray]]] = None,
                max_vid: Sequence[int] = (0, 0), page_tokens: int = 16, state_dtype: str = "f32",
                conv_kernel: int = 0, pad_ssm_to_kv_page: bool = False):
    """Returns (avmp_config_t, keepalive): keepalive holds the rank arrays the struct points to."""
    cfg = avmp_config_t()
    cfg.dtype = AVMP_F32 if dtype == "f32" else AVMP_BF16
    cfg.attention_page_tokens = page_tokens
    cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim = n_q_heads, n_kv_heads, head_dim
    cfg.ssm_heads, cfg.ssm_headdim, cfg.ssm_dstate = ssm_heads, ssm_headdim, ssm_dstate
    cfg.ssm_state_dtype = AVMP_F32 if state_dtype == "f32" else AVMP_BF16
    cfg.ssm_conv_kernel = conv_kernel
    cfg.ssm_pad_to_kv_page = 1 if pad_ssm_to_kv_page else 0
    cfg.kv_capacity, cfg.ssm_capacity = kv_capacity, ssm_capacity
    cfg.max_vid[0], cfg.max_vid[1] = max_vid
    keep = []
    for p in range(2):
        r = None if slot_rank is None else slot_rank[p]
        if r is None:
            cfg.slot_rank[p] = C.POINTER(C.c_uint32)()
        else:
            a = np.ascontiguousarray(r, dtype=np.uint32)
            keep.append(a)
            cfg.slot_rank[p] = a.ctypes.data_as(C.POINTER(C.c_uint32))
    return cfg, keep


def avmp_geometry(cfg: avmp_config_t, arena_bytes: int):
    g = avmp_geometry_t()
    rc = lib.avmp_geometry(C.byref(cfg), arena_bytes, C.byref(g))
    return rc, g


def avmp_pools_create(cfg: avmp_config_t, arena, arena_bytes: int):
    """arena: torch uint8 tensor on the device, an integer address, or None (metadata only)."""
    out = _P()
    rc = lib.avmp_pools_create(C.byref(cfg), _ptr(arena), arena_bytes, C.byref(out))
    return rc, (out.value if rc == AVMP_OK else None)


def avmp_pools_destroy(pools) -> int:
    return lib.avmp_pools_destroy(pools)


def avmp_alloc(pools, pool: int, n: int):
    out = np.empty(max(n, 1), dtype=np.uint32)
    rc = lib.avmp_alloc(pools, pool, n, out.ctypes.data)
    return rc, (out[:n] if rc == AVMP_OK else None)


def avmp_free(pools, handles) -> int:
    h = np.ascontiguousarray(handles, dtype=np.uint32)
    return lib.avmp_free(pools, h.ctypes.data, h.size)


def avmp_migrate(pools, donor_pool: int, n_donor_units: int, stream=None):
    res = avmp_migrate_result_t()
    rc = lib.avmp_migrate(pools, donor_pool, n_donor_units, _stream(stream), C.byref(res))
    return rc, res


def avmp_absorb_gap(pools, pool: int):
    res = avmp_migrate_result_t()
    rc = lib.avmp_absorb_gap(pools, pool, C.byref(res))
    return rc, res


def make_step(batch: int, layer_kinds: Sequence[int], max_pages: int, kv_handles, ctx, q, o,
              ssm_handles, x, dt, A, B, Cm, y, k_new=None, v_new=None, xbc=None, conv_taps=None,
              conv_bias=None):
    """Returns (avmp_step_t, keepalive).  Tensors must stay alive until the step has run."""
    st = avmp_step_t()
    kinds = np.ascontiguousarray(layer_kinds, dtype=np.uint8)
    st.batch, st.n_layers, st.max_pages = batch, len(kinds), max_pages
    st.layer_kind = kinds.ctypes.data
    st.kv_handles, st.ctx, st.q, st.o = _ptr(kv_handles), _ptr(ctx), _ptr(q), _ptr(o)
    st.ssm_handles, st.x, st.dt, st.A = _ptr(ssm_handles), _ptr(x), _ptr(dt), _ptr(A)
    st.B, st.C, st.y = _ptr(B), _ptr(Cm), _ptr(y)
    st.k_new, st.v_new = _ptr(k_new), _ptr(v_new)
    st.xbc, st.conv_taps, st.conv_bias = _ptr(xbc), _ptr(conv_taps), _ptr(conv_bias)
    return st, (kinds, kv_handles, ctx, q, o, ssm_handles, x, dt, A, B, Cm, y, k_new, v_new,
                xbc, conv_taps, conv_bias)


def avmp_decode_step(pools, step: avmp_step_t, stream=None) -> int:
    return lib.avmp_decode_step(pools, C.byref(step), _stream(stream))


AVMP_NOALLOC_WORKSPACE_BYTES = 32 << 20


def avmp_decode_step_noalloc(pools, step: avmp_step_t, stream=None) -> int:
    return lib.avmp_decode_step_noalloc(pools, C.byref(step), _stream(stream))


def avmp_workspace_reserve(pools, n_attention_layers: int, n_ssm_layers: int, batch: int,
                           max_pages: int) -> int:
    return lib.avmp_workspace_reserve(pools, n_attention_layers, n_ssm_layers, batch, max_pages)


def avmp_workspace_info(pools):
    """Returns (rc, bytes, allocations so far)."""
    nbytes, allocs = C.c_uint64(), C.c_uint64()
    rc = lib.avmp_workspace_info(pools, C.byref(nbytes), C.byref(allocs))
    return rc, nbytes.value, allocs.value


def avmp_flush(pools, stream=None) -> int:
    return lib.avmp_flush(pools, _stream(stream))


def avmp_translate(pools, handles_dev, n: int, offsets_dev, stream=None) -> int:
    return lib.avmp_translate(pools, _ptr(handles_dev), n, _ptr(offsets_dev), _stream(stream))


def avmp_resolve(pools, handle: int):
    pool, slot, off = C.c_uint32(), C.c_uint32(), C.c_uint64()
    rc = lib.avmp_resolve(pools, int(handle), C.byref(pool), C.byref(slot), C.byref(off))
    return rc, pool.value, slot.value, off.value


def avmp_stats(pools) -> dict:
    st = avmp_stats_t()
    rc = lib.avmp_stats(pools, C.byref(st))
    if rc != AVMP_OK:
        raise RuntimeError(avmp_last_error())
    return {"capacity": tuple(st.capacity), "live": tuple(st.live), "free": tuple(st.free_units),
            "gap_bytes": st.gap_bytes, "ops": st.ops, "capacity_errors": st.capacity_errors,
            "migrations": st.migrations, "units_copied": st.units_copied,
            "bytes_migrated": st.bytes_migrated, "bytes_wasted": st.bytes_wasted}


def avmp_device_faults(pools, stream=None):
    out = C.c_uint64()
    rc = lib.avmp_device_faults(pools, _stream(stream), C.byref(out))
    return rc, out.value


def avmp_profile_enable(pools, on: bool) -> int:
    return lib.avmp_profile_enable(pools, 1 if on else 0)


def avmp_profile_read(pools, stream=None):
    """Returns (rc, {kernel name: (total ms, launches)})."""
    out = avmp_profile_t()
    rc = lib.avmp_profile_read(pools, _stream(stream), C.byref(out))
    return rc, {KERNEL_NAMES[k]: (out.ms[k], out.launches[k]) for k in range(AVMP_K_COUNT)}


def avmp_policy_set(pools, threshold_low=0.05, threshold_high=0.30, migration_batch_size=128,
                    min_rebalance_interval_ops=1000) -> int:
    pol = avmp_policy_t(threshold_low, threshold_high, migration_batch_size, 0,
                        min_rebalance_interval_ops)
    return lib.avmp_policy_set(pools, C.byref(pol))


def avmp_policy_state(pools) -> dict:
    st = avmp_policy_state_t()
    rc = lib.avmp_policy_state(pools, C.byref(st))
    if rc != AVMP_OK:
        raise RuntimeError(avmp_last_error())
    return {"state": st.state, "has_rebalanced": bool(st.has_rebalanced),
            "last_rebalance_op": st.last_rebalance_op, "rebalance_count": st.rebalance_count,
            "oom_events": st.oom_events}


def avmp_alloc_auto(pools, pool: int, n: int, stream=None):
    """Returns (rc, handles or None, donor units migrated by this call)."""
    out = np.empty(max(n, 1), dtype=np.uint32)
    moved = C.c_uint32()
    rc = lib.avmp_alloc_auto(pools, pool, n, out.ctypes.data, _stream(stream), C.byref(moved))
    return rc, (out[:n] if rc == AVMP_OK else None), moved.value


def avmp_vmm_min_chunk() -> int:
    return int(lib.avmp_vmm_min_chunk())


def avmp_vmm_arena_create(nbytes: int, chunk_bytes: int):
    out = _P()
    rc = lib.avmp_vmm_arena_create(nbytes, chunk_bytes, C.byref(out))
    return rc, (out.value if rc == AVMP_OK else None)


def avmp_vmm_arena_base(arena) -> int:
    return int(lib.avmp_vmm_arena_base(arena) or 0)


def avmp_vmm_arena_destroy(arena) -> int:
    return lib.avmp_vmm_arena_destroy(arena)


def avmp_migrate_by_remap(pools, arena) -> int:
    return lib.avmp_migrate_by_remap(pools, arena)
