"""GPU-side test plumbing: build the library's pools from a Scenario, fill the
device arena with the same bytes the oracle gets, run decode steps through the
C ABI.  torch is used for device memory only."""
import numpy as np
import torch

from paper_2605_22416_amd import binding as av
from paper_2605_22416_amd import inputs
from tests import helpers

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    """numpy -> device tensor with the same bytes (unsigned types go through a signed view)."""
    a = np.ascontiguousarray(a)
    view = {np.dtype(np.uint32): np.int32, np.dtype(np.uint16): np.int16,
            np.dtype(np.uint64): np.int64}.get(a.dtype)
    if view is not None:
        a = a.view(view)
    return torch.from_numpy(a).to(DEV)


class GpuPools:
    def __init__(self, sc: inputs.Scenario, fill_byte: int = 0):
        spec = sc.spec
        self.sc = sc
        self.arena = torch.empty(sc.arena_bytes, dtype=torch.uint8, device=DEV)
        self.arena.fill_(fill_byte)
        cfg, self._keep = av.make_config(spec.dtype, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                                         spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate,
                                         sc.kv_capacity, sc.ssm_capacity, slot_rank=sc.slot_rank)
        rc, self.p = av.avmp_pools_create(cfg, self.arena, sc.arena_bytes)
        assert rc == av.AVMP_OK, av.avmp_last_error()
        self.kv, self.ssm = helpers.empty_handle_tables(sc)
        for pool, n, tag in helpers.alloc_order(sc):
            rc, hs = av.avmp_alloc(self.p, pool, n)
            assert rc == av.AVMP_OK, av.avmp_last_error()
            helpers.place_handles(self.kv, self.ssm, tag, hs)
        self.sync_handles()
        # fresh SSM blocks are zeroed by the queued fill; it must run before data is written
        assert av.avmp_flush(self.p) == av.AVMP_OK, av.avmp_last_error()
        torch.cuda.synchronize()

    def sync_handles(self):
        self.kv_dev, self.ssm_dev = to_dev(self.kv), to_dev(self.ssm)
        self.ctx_dev = to_dev(self.sc.ctx)

    def close(self):
        if self.p is not None:
            torch.cuda.synchronize()
            av.avmp_pools_destroy(self.p)
            self.p = None

    def unit(self, h: int) -> torch.Tensor:
        rc, pool, slot, off = av.avmp_resolve(self.p, int(h))
        assert rc == av.AVMP_OK
        n = self.sc.spec.kv_page_bytes if pool == 0 else self.sc.spec.ssm_block_bytes
        return self.arena[off: off + n]

    def write_unit(self, h: int, data: np.ndarray):
        self.unit(h).copy_(torch.from_numpy(np.ascontiguousarray(data)))

    def read_unit(self, h: int) -> np.ndarray:
        return self.unit(h).cpu().numpy()

    def fill(self, opools=None, poison=False, scale_inputs=None, threads=8):
        """Same bytes as helpers.fill_oracle.  opools (an oracle Pools) is only asked
        where the tail token slots of a page are, to plant NaN there."""
        sc, spec = self.sc, self.sc.spec
        jobs = helpers.unit_jobs(sc)

        def sink(i, data):
            pool, layer, r, idx = jobs[i]
            if poison and pool == inputs.POOL_KV and idx == sc.n_pages[r] - 1:
                data = data.copy()
                helpers.poison_tail(spec, data, int(sc.ctx[r]) - idx * spec.page_tokens, opools)
            self.write_unit(helpers.job_handle(jobs[i], self.kv, self.ssm), data)

        inputs.fill_units(spec, sc.seed, jobs, sink, threads=threads, scale_inputs=scale_inputs)
        torch.cuda.synchronize()

    def step(self, inp, stream=None):
        """One decode step through the C ABI; returns (o, y) as numpy float32."""
        sc, spec = self.sc, self.sc.spec
        d = {k: to_dev(v) for k, v in inp.items()}
        o = torch.full((spec.n_attn, sc.batch, spec.n_q_heads, spec.head_dim), float("nan"),
                       dtype=torch.float32, device=DEV)
        y = torch.full((spec.n_ssm, sc.batch, spec.ssm_heads, spec.ssm_headdim), float("nan"),
                       dtype=torch.float32, device=DEV)
        st, keep = av.make_step(sc.batch, spec.layer_kinds, self.kv.shape[2], self.kv_dev, self.ctx_dev,
                                d["q"], o, self.ssm_dev, d["x"], d["dt"], d["A"], d["B"], d["C"], y)
        rc = av.avmp_decode_step(self.p, st, stream)
        assert rc == av.AVMP_OK, av.avmp_last_error()
        torch.cuda.synchronize()
        rc, faults = av.avmp_device_faults(self.p)
        assert rc == av.AVMP_OK and faults == 0, "kernels met %d untranslatable handles" % faults
        return o.cpu().numpy(), y.cpu().numpy()

    def states(self, layer: int) -> np.ndarray:
        """SSM blocks of one SSM layer, read back by handle: [batch][H][P][N] fp32."""
        spec = self.sc.spec
        return np.stack([self.read_unit(int(h)).view(np.float32).reshape(
            spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate) for h in self.ssm[layer]])

    def translate(self, handles: np.ndarray) -> np.ndarray:
        h = to_dev(np.ascontiguousarray(handles, dtype=np.uint32).reshape(-1))
        out = torch.empty(h.numel(), dtype=torch.int64, device=DEV)
        rc = av.avmp_translate(self.p, h, h.numel(), out)
        assert rc == av.AVMP_OK, av.avmp_last_error()
        torch.cuda.synchronize()
        return out.cpu().numpy().view(np.uint64)


def oracle_states(op, ssm_handles, spec) -> np.ndarray:
    return np.stack([op.unit_view(int(h)).view(np.float32).reshape(
        spec.ssm_heads, spec.ssm_headdim, spec.ssm_dstate).copy() for h in ssm_handles])
