"""Device-side session: builds the library's pools from a Scenario, fills the
device arena from the seeded generators and runs decode steps through the C
ABI.  torch supplies device memory and streams only; every step of the path
runs in the library's kernels."""
from __future__ import annotations

import ctypes
from typing import Callable, Dict, Optional

import numpy as np
import torch

from . import binding as av
from gen import inputs

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    """numpy -> device tensor with the same bytes (unsigned types go through a signed view)."""
    a = np.ascontiguousarray(a)
    view = {np.dtype(np.uint32): np.int32, np.dtype(np.uint16): np.int16,
            np.dtype(np.uint64): np.int64}.get(a.dtype)
    if view is not None:
        a = a.view(view)
    return torch.from_numpy(a).to(DEV)


def alloc_order(sc: inputs.Scenario):
    """Allocation calls of a scenario: per request, its pages for each attention
    layer, then its blocks for all SSM layers."""
    calls = []
    for r in range(sc.batch):
        for la in range(sc.spec.n_attn):
            if sc.n_pages[r] > 0:
                calls.append((inputs.POOL_KV, int(sc.n_pages[r]), ("kv", la, r)))
        if sc.spec.n_ssm:
            calls.append((inputs.POOL_SSM, sc.spec.n_ssm, ("ssm", r)))
    return calls


def unit_jobs(sc: inputs.Scenario, requests=None):
    """(pool, layer, request, index) of every unit that starts with generated contents
    (of the given requests only, if a list is given)."""
    rs = range(sc.batch) if requests is None else list(requests)
    jobs = []
    for la in range(sc.spec.n_attn):
        for r in rs:
            for i in range(int(sc.n_pages[r])):
                jobs.append((inputs.POOL_KV, la, r, i))
    for ls in range(sc.spec.n_ssm):
        for r in rs:
            if not sc.fresh[r]:
                jobs.append((inputs.POOL_SSM, ls, r, 0))
    return jobs


def _hip(name: str, *args):
    """Call the shared HIP runtime directly (for memory torch cannot wrap)."""
    fn = getattr(av.hip_runtime, name)
    fn.restype = ctypes.c_int
    rc = fn(*args)
    if rc != 0:
        raise RuntimeError("%s failed with HIP error %d" % (name, rc))


class DeviceSession:
    """vmm_chunk: None puts the arena in a torch tensor; a chunk size in bytes puts it
    in an arena of the library's own, attached chunk by chunk through the HIP
    virtual-memory API, and switches migration to exchanging chunks."""

    def __init__(self, sc: inputs.Scenario, fill_byte: Optional[int] = 0,
                 vmm_chunk: Optional[int] = None, remap: bool = True):
        spec = sc.spec
        self.sc = sc
        self.vmm = None
        self.p = None
        if vmm_chunk is None:
            self.arena = torch.empty(sc.arena_bytes, dtype=torch.uint8, device=DEV)
            self.base = self.arena.data_ptr()
            if fill_byte is not None:
                self.arena.fill_(fill_byte)
        else:
            torch.cuda.init()
            self.arena = None
            rc, self.vmm = av.avmp_vmm_arena_create(sc.arena_bytes, vmm_chunk)
            if rc != av.AVMP_OK:
                raise RuntimeError("avmp_vmm_arena_create: " + av.avmp_last_error())
            self.base = av.avmp_vmm_arena_base(self.vmm)
            if fill_byte is not None:
                _hip("hipMemset", ctypes.c_void_p(self.base), ctypes.c_int(fill_byte),
                     ctypes.c_size_t(sc.arena_bytes))
        cfg, self._keep = av.make_config(spec.dtype, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                                         spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate,
                                         sc.kv_capacity, sc.ssm_capacity, slot_rank=sc.slot_rank,
                                         state_dtype=spec.state_dtype, conv_kernel=spec.conv_kernel,
                                         pad_ssm_to_kv_page=spec.pad_ssm_to_kv_page)
        rc, self.p = av.avmp_pools_create(cfg, self.base, sc.arena_bytes)
        if rc != av.AVMP_OK:
            raise RuntimeError("avmp_pools_create: " + av.avmp_last_error())
        if self.vmm is not None and remap:
            self._ok(av.avmp_migrate_by_remap(self.p, self.vmm))
        self.kv = np.full((spec.n_attn, sc.batch, sc.max_pages), 0xFFFFFFFF, dtype=np.uint32)
        self.ssm = np.full((spec.n_ssm, sc.batch), 0xFFFFFFFF, dtype=np.uint32)
        for pool, n, tag in alloc_order(sc):
            rc, hs = av.avmp_alloc(self.p, pool, n)
            if rc != av.AVMP_OK:
                raise RuntimeError("avmp_alloc: " + av.avmp_last_error())
            if tag[0] == "kv":
                self.kv[tag[1], tag[2], : len(hs)] = hs
            else:
                self.ssm[:, tag[1]] = hs
        self.sync_handles()
        # new SSM blocks are zeroed by a queued fill; it must run before data is written
        self._ok(av.avmp_flush(self.p))
        torch.cuda.synchronize()
        self._step_keep = None

    def _ok(self, rc):
        if rc != av.AVMP_OK:
            raise RuntimeError(av.avmp_last_error())

    def sync_handles(self):
        self.kv_dev, self.ssm_dev = to_dev(self.kv), to_dev(self.ssm)
        self.ctx_dev = to_dev(self.sc.ctx)

    def close(self):
        if self.p is not None:
            torch.cuda.synchronize()
            av.avmp_pools_destroy(self.p)
            self.p = None
        if self.vmm is not None:
            av.avmp_vmm_arena_destroy(self.vmm)
            self.vmm = None
        self.arena = None                      # the device memory goes back to torch

    # ---- unit access by handle (host resolve + a slice of the arena tensor) ----
    def unit_range(self, h: int):
        rc, pool, slot, off = av.avmp_resolve(self.p, int(h))
        self._ok(rc)
        return off, self.sc.spec.kv_page_bytes if pool == 0 else self.sc.spec.ssm_block_bytes

    def write_unit(self, h: int, data: np.ndarray):
        off, n = self.unit_range(h)
        data = np.ascontiguousarray(data)
        assert data.nbytes == n
        if self.arena is not None:
            self.arena[off: off + n].copy_(torch.from_numpy(data.view(np.uint8).reshape(-1)))
        else:
            _hip("hipMemcpy", ctypes.c_void_p(self.base + off), ctypes.c_void_p(data.ctypes.data),
                 ctypes.c_size_t(n), ctypes.c_int(1))      # host to device

    def read_unit(self, h: int) -> np.ndarray:
        off, n = self.unit_range(h)
        if self.arena is not None:
            return self.arena[off: off + n].cpu().numpy()
        out = np.empty(n, dtype=np.uint8)
        _hip("hipMemcpy", ctypes.c_void_p(out.ctypes.data), ctypes.c_void_p(self.base + off),
             ctypes.c_size_t(n), ctypes.c_int(2))          # device to host
        return out

    def job_handle(self, job) -> int:
        pool, layer, r, i = job
        return int(self.kv[layer, r, i]) if pool == inputs.POOL_KV else int(self.ssm[layer, r])

    def fill(self, transform: Optional[Callable] = None, scale_inputs=None, threads: int = 8,
             requests=None):
        """Write the generated contents of every live unit (or of the given requests'
        units only).  transform(job, bytes) may edit a unit's bytes before they are stored."""
        sc = self.sc
        jobs = unit_jobs(sc, requests)

        def sink(i, data):
            if transform is not None:
                data = transform(jobs[i], data)
            self.write_unit(self.job_handle(jobs[i]), data)

        inputs.fill_units(sc.spec, sc.seed, jobs, sink, threads=threads, scale_inputs=scale_inputs)
        torch.cuda.synchronize()

    # ---- decode steps ------------------------------------------------------------
    def prepare_step(self, inp: Dict[str, np.ndarray], k_new=None, v_new=None, conv=None):
        """Upload one step's activations (and the appended token's K, V rows, if
        given; and the (taps, bias) of the short convolution for models that have
        one), allocate outputs, build the descriptor."""
        sc, spec = self.sc, self.sc.spec
        d = {k: to_dev(v) for k, v in inp.items()}
        cw = cb = None
        if spec.conv_kernel:
            cw, cb = to_dev(conv[0]), to_dev(conv[1])
        kn = to_dev(k_new) if k_new is not None else None
        vn = to_dev(v_new) if v_new is not None else None
        o = torch.full((spec.n_attn, sc.batch, spec.n_q_heads, spec.head_dim), float("nan"),
                       dtype=torch.float32, device=DEV)
        y = torch.full((spec.n_ssm, sc.batch, spec.ssm_heads, spec.ssm_headdim), float("nan"),
                       dtype=torch.float32, device=DEV)
        st, keep = av.make_step(sc.batch, spec.layer_kinds, self.kv.shape[2], self.kv_dev,
                                self.ctx_dev, d["q"], o, self.ssm_dev, d["x"], d["dt"], d["A"],
                                d["B"], d["C"], y, kn, vn, d.get("xbc"), cw, cb)
        return st, keep, o, y

    def launch(self, st, stream=None):
        self._ok(av.avmp_decode_step(self.p, st, stream))

    def step(self, inp: Dict[str, np.ndarray], stream=None, k_new=None, v_new=None, conv=None):
        """One decode step; returns (o, y) as numpy float32 and checks the fault counter."""
        st, keep, o, y = self.prepare_step(inp, k_new, v_new, conv)
        self.launch(st, stream)
        torch.cuda.synchronize()
        rc, faults = av.avmp_device_faults(self.p)
        self._ok(rc)
        if faults:
            raise RuntimeError("kernels met %d untranslatable handles" % faults)
        return o.cpu().numpy(), y.cpu().numpy()

    def states(self, layer: int, requests=None) -> np.ndarray:
        """SSM blocks of one SSM layer read back by handle: [len(requests)][H][P][N] as
        float32 (bf16 storage is widened; every bf16 value is a float32)."""
        spec = self.sc.spec
        rs = range(self.sc.batch) if requests is None else requests
        out = []
        for r in rs:
            raw = self.read_unit(int(self.ssm[layer, r]))[: spec.ssm_state_bytes]
            vals = raw.view(np.float32) if spec.state_dtype == "f32" else inputs.bf16_bits_to_f32(raw.view(np.uint16))
            out.append(vals.reshape(spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate))
        return np.stack(out)

    def conv_windows(self, layer: int) -> np.ndarray:
        """The convolution windows of one SSM layer as raw bytes [batch][window bytes]."""
        spec = self.sc.spec
        a, n = spec.ssm_state_bytes, spec.conv_window_bytes
        return np.stack([self.read_unit(int(self.ssm[layer, r]))[a: a + n]
                         for r in range(self.sc.batch)])

    def translate(self, handles: np.ndarray) -> np.ndarray:
        h = to_dev(np.ascontiguousarray(handles, dtype=np.uint32).reshape(-1))
        out = torch.empty(h.numel(), dtype=torch.int64, device=DEV)
        self._ok(av.avmp_translate(self.p, h, h.numel(), out))
        torch.cuda.synchronize()
        return out.cpu().numpy().view(np.uint64)
