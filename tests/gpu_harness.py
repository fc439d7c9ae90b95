"""GPU-side test plumbing: the package's DeviceSession plus helpers that feed
it the same bytes the oracle gets."""
import numpy as np

from gen import inputs
from paper_2605_22416_amd.session import DEV, DeviceSession, to_dev  # noqa: F401
from tests import helpers


class GpuPools(DeviceSession):
    def fill(self, opools=None, poison=False, scale_inputs=None, threads=8):
        """Same bytes as helpers.fill_oracle.  opools (an oracle Pools) is only asked
        where the tail token slots of a page are, to plant NaN there."""
        sc, spec = self.sc, self.sc.spec

        def transform(job, data):
            pool, layer, r, idx = job
            if poison and pool == inputs.POOL_KV and idx == sc.n_pages[r] - 1:
                data = data.copy()
                helpers.poison_tail(spec, data, int(sc.ctx[r]) - idx * spec.page_tokens, opools)
            return data

        super().fill(transform=transform if poison else None, scale_inputs=scale_inputs,
                     threads=threads)


def oracle_states(op, ssm_handles, spec) -> np.ndarray:
    return np.stack([op.state_values(int(h)) for h in ssm_handles])
