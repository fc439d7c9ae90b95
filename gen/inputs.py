"""Seeded synthetic inputs for the hybrid decode path.

Only shapes, sizes and random values live here: model shapes, context-length
mixes in the shapes of the paper's three synthetic workloads (Evaluation,
"Experimental Setup": uniform_short, mixed_long, agentic_burst) plus a tiny and
a capacity-scale case, physical placement permutations, per-step activations
and the contents of KV pages and SSM blocks.  None of the method's arithmetic
is here, so the GPU library's tests and the CPU checker can both be fed from
this module without sharing any of their own code.

All values are numpy arrays.  bf16 data is carried as uint16 bit patterns.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

ATTN, SSM = 0, 1          # layer kinds
POOL_KV, POOL_SSM = 0, 1


@dataclass(frozen=True)
class ModelSpec:
    name: str
    dtype: str                      # "f32" or "bf16": K, V, q, x, B, C element type
    page_tokens: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ssm_heads: int
    ssm_headdim: int
    ssm_dstate: int
    layer_kinds: Tuple[int, ...]    # model order; 0 = attention, 1 = SSM
    scale_inputs: bool              # q, K, V, x drawn N(0,1) then scaled by 1/sqrt(head dim)
    state_dtype: str = "f32"        # storage type of the SSM state in its block: "f32" or "bf16"
    conv_kernel: int = 0            # taps of the short convolution in front of the recurrence;
                                    # 0 = the block holds the recurrent state alone
    pad_ssm_to_kv_page: bool = False  # unified-pool sizing: the block padded to whole KV pages

    @property
    def state_bytes(self) -> int:
        return 4 if self.state_dtype == "f32" else 2

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def n_attn(self) -> int:
        return sum(1 for k in self.layer_kinds if k == ATTN)

    @property
    def n_ssm(self) -> int:
        return sum(1 for k in self.layer_kinds if k == SSM)

    @property
    def kv_page_bytes(self) -> int:
        return self.page_tokens * 2 * self.n_kv_heads * self.head_dim * self.elem_bytes

    @property
    def conv_dim(self) -> int:
        """Channels that pass through the short convolution: x [H][P], then B [N], then C [N]."""
        return self.ssm_heads * self.ssm_headdim + 2 * self.ssm_dstate

    @property
    def ssm_state_bytes(self) -> int:
        return self.ssm_heads * self.ssm_headdim * self.ssm_dstate * self.state_bytes

    @property
    def conv_window_bytes(self) -> int:
        return (self.conv_kernel - 1) * self.conv_dim * self.elem_bytes if self.conv_kernel else 0

    @property
    def ssm_native_bytes(self) -> int:
        return (self.ssm_state_bytes + self.conv_window_bytes + 15) // 16 * 16

    @property
    def ssm_block_bytes(self) -> int:
        n = self.ssm_native_bytes
        if self.pad_ssm_to_kv_page:
            n = -(-n // self.kv_page_bytes) * self.kv_page_bytes
        return n


# one attention + one SSM layer, fp32, 4 query / 2 KV heads x 64, SSM 4 x 32 x 16
TINY = ModelSpec("tiny_fp32", "f32", 16, 4, 2, 64, 4, 32, 16, (ATTN, SSM), False)

# Jamba-mini-like: 32 layers, attention : SSM = 1 : 7 (Background, "Hybrid
# Mamba-Transformer Architectures"); the attention layer sits mid-block.
JAMBA_MINI = ModelSpec("jamba_mini_like", "bf16", 16, 32, 8, 128, 128, 64, 128,
                       tuple(ATTN if i % 8 == 4 else SSM for i in range(32)), True)


def scaled_down(spec: ModelSpec, n_blocks: int = 1, name: Optional[str] = None) -> ModelSpec:
    """Same head shapes, fewer layers (n_blocks repeats of 1 attention + 7 SSM)."""
    kinds = tuple(ATTN if i % 8 == 4 else SSM for i in range(8 * n_blocks))
    return replace(spec, name=name or spec.name + "_%dblk" % n_blocks, layer_kinds=kinds)


def with_conv(spec: ModelSpec, conv_kernel: int = 4) -> ModelSpec:
    """Same model whose SSM blocks also hold the last conv_kernel-1 inputs of the short convolution."""
    return replace(spec, name=spec.name + "_conv%d" % conv_kernel, conv_kernel=conv_kernel)


def with_padded_blocks(spec: ModelSpec) -> ModelSpec:
    """Same model with every SSM block padded up to a whole number of KV pages."""
    return replace(spec, name=spec.name + "_padded", pad_ssm_to_kv_page=True)


def with_state_dtype(spec: ModelSpec, state_dtype: str) -> ModelSpec:
    """Same model with the SSM state stored as "f32" or "bf16" in its block."""
    return replace(spec, name=spec.name + "_state_" + state_dtype, state_dtype=state_dtype)


# ----------------------------------------------------------------------------
# element helpers
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def elements(rng: np.random.Generator, shape, scale: float, dtype: str) -> np.ndarray:
    """N(0, scale^2) values in the element type (float32, or bf16 bit patterns)."""
    a = rng.standard_normal(shape, dtype=np.float32)
    if scale != 1.0:
        a *= np.float32(scale)
    return a if dtype == "f32" else f32_to_bf16_bits(a)


# ----------------------------------------------------------------------------
# context-length mixes
# ----------------------------------------------------------------------------
def ctx_lengths(workload: str, batch: int, rng: np.random.Generator) -> np.ndarray:
    if workload == "tiny":
        c = rng.integers(16, 65, size=batch)
    elif workload == "uniform_short":
        c = rng.integers(128, 2049, size=batch)
    elif workload == "mixed_long":
        c = np.rint(np.exp(math.log(4096.0) + rng.standard_normal(batch)))
        c = np.clip(c, 256, 65536)
    elif workload == "agentic_burst":
        # half resident requests, half newly admitted ones holding 1..4 pages
        n_new = batch // 2
        old = rng.integers(64, 1025, size=batch - n_new)
        pages = rng.integers(1, 5, size=n_new)
        new = 16 * pages - rng.integers(0, 16, size=n_new)
        c = np.concatenate([old, new])
    elif workload == "capacity":
        c = np.concatenate([rng.integers(1024, 8193, size=batch), np.full(4, 262144)])
    else:
        raise ValueError("unknown workload " + workload)
    return c.astype(np.uint32)


@dataclass
class Scenario:
    """A logical batch plus the physical set-up both sides are built from."""
    spec: ModelSpec
    workload: str
    seed: int
    ctx: np.ndarray                         # [batch] uint32
    n_pages: np.ndarray                     # [batch] pages per request per attention layer
    fresh: np.ndarray                       # [batch] bool: SSM blocks start zeroed
    kv_capacity: int
    ssm_capacity: int
    arena_bytes: int
    slot_rank: List[np.ndarray]             # per pool: permutation of all possible slots

    @property
    def batch(self) -> int:
        return len(self.ctx)

    @property
    def max_pages(self) -> int:
        return max(1, int(self.n_pages.max())) if len(self.n_pages) else 1


def make_scenario(spec: ModelSpec, workload: str, batch: int, seed: int,
                  headroom: float = 1.2, occupancy: Optional[float] = None,
                  ctx: Optional[Sequence[int]] = None, permute: bool = True,
                  placement_seed: Optional[int] = None, slack_bytes: int = 0) -> Scenario:
    """Pools sized to headroom x demand (or demand / occupancy for the KV pool),
    physical slots ranked by a seeded permutation."""
    rng = np.random.default_rng([seed, 0])
    c = np.asarray(ctx, dtype=np.uint32) if ctx is not None else ctx_lengths(workload, batch, rng)
    n_pages = (c.astype(np.int64) + spec.page_tokens - 1) // spec.page_tokens
    fresh = np.zeros(len(c), dtype=bool)
    if workload == "agentic_burst" and ctx is None:
        fresh[len(c) - len(c) // 2:] = True
    live_pages = int(n_pages.sum()) * spec.n_attn
    live_blocks = len(c) * spec.n_ssm
    if occupancy is not None:
        kv_cap = int(math.ceil(live_pages / occupancy))
    else:
        kv_cap = int(math.ceil(live_pages * headroom))
    ssm_cap = int(math.ceil(live_blocks * headroom))
    kv_cap, ssm_cap = max(kv_cap, 1), max(ssm_cap, 1)
    arena = kv_cap * spec.kv_page_bytes + ssm_cap * spec.ssm_block_bytes + slack_bytes
    arena = (arena + 127) // 128 * 128
    prng = np.random.default_rng([seed if placement_seed is None else placement_seed, 1])
    ranks = []
    for unit in (spec.kv_page_bytes, spec.ssm_block_bytes):
        n = arena // unit
        ranks.append(prng.permutation(n).astype(np.uint32) if permute
                     else np.arange(n, dtype=np.uint32))
    return Scenario(spec, workload, seed, c, n_pages, fresh, kv_cap, ssm_cap, arena, ranks)


# ----------------------------------------------------------------------------
# per-step activations
# ----------------------------------------------------------------------------
def step_inputs(spec: ModelSpec, batch: int, seed: int, step: int = 0,
                scale_inputs: Optional[bool] = None) -> Dict[str, np.ndarray]:
    """q [n_attn][batch][Hq][D], x [n_ssm][batch][H][P], dt [n_ssm][batch][H] (softplus of
    N(0,1), so positive), A [n_ssm][H] = -exp(U[-2,0]), B and C [n_ssm][batch][N] ~ N(0, 1/16)."""
    rng = np.random.default_rng([seed, 2, step])
    sc = spec.scale_inputs if scale_inputs is None else scale_inputs
    qs = 1.0 / math.sqrt(spec.head_dim) if sc else 1.0
    xs = 1.0 / math.sqrt(spec.ssm_headdim) if sc else 1.0
    q = elements(rng, (spec.n_attn, batch, spec.n_q_heads, spec.head_dim), qs, spec.dtype)
    x = elements(rng, (spec.n_ssm, batch, spec.ssm_heads, spec.ssm_headdim), xs, spec.dtype)
    z = rng.standard_normal((spec.n_ssm, batch, spec.ssm_heads))
    dt = np.logaddexp(0.0, z).astype(np.float32)
    A = (-np.exp(rng.uniform(-2.0, 0.0, size=(spec.n_ssm, spec.ssm_heads)))).astype(np.float32)
    B = elements(rng, (spec.n_ssm, batch, spec.ssm_dstate), 0.25, spec.dtype)
    C = elements(rng, (spec.n_ssm, batch, spec.ssm_dstate), 0.25, spec.dtype)
    out = {"q": q, "x": x, "dt": dt, "A": A, "B": B, "C": C}
    if spec.conv_kernel:
        # what enters the short convolution for this token: x, B and C channels side by side
        crng = np.random.default_rng([seed, 5, step])
        out["xbc"] = elements(crng, (spec.n_ssm, batch, spec.conv_dim), xs, spec.dtype)
    return out


def conv_weights(spec: ModelSpec, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Taps [n_ssm][K][conv_dim] ~ N(0, 1/K) (tap K-1 meets the newest token) and
    bias [n_ssm][conv_dim] ~ N(0, 1/16), both in the element dtype."""
    rng = np.random.default_rng([seed, 6])
    K = spec.conv_kernel
    w = elements(rng, (spec.n_ssm, K, spec.conv_dim), 1.0 / math.sqrt(K), spec.dtype)
    b = elements(rng, (spec.n_ssm, spec.conv_dim), 0.25, spec.dtype)
    return w, b


def new_token_kv(spec: ModelSpec, batch: int, seed: int, step: int = 0,
                 scale_inputs: Optional[bool] = None) -> Tuple[np.ndarray, np.ndarray]:
    """K and V rows of the token a step appends: [n_attn][batch][Hkv][D] each."""
    rng = np.random.default_rng([seed, 4, step])
    sc = spec.scale_inputs if scale_inputs is None else scale_inputs
    s = 1.0 / math.sqrt(spec.head_dim) if sc else 1.0
    shape = (spec.n_attn, batch, spec.n_kv_heads, spec.head_dim)
    return elements(rng, shape, s, spec.dtype), elements(rng, shape, s, spec.dtype)


# ----------------------------------------------------------------------------
# unit contents: a pure function of (seed, pool, layer ordinal, request, index)
# so that any single page or block can be regenerated without the whole arena
# ----------------------------------------------------------------------------
def unit_content(spec: ModelSpec, seed: int, pool: int, layer: int, request: int,
                 index: int = 0, scale_inputs: Optional[bool] = None) -> np.ndarray:
    """Bytes of one KV page (K and V values for page `index` of `request` in
    attention layer ordinal `layer`) or of one SSM state block (N(0,1) in the state dtype)."""
    rng = np.random.default_rng([seed, 3, pool, layer, request, index])
    if pool == POOL_KV:
        sc = spec.scale_inputs if scale_inputs is None else scale_inputs
        s = 1.0 / math.sqrt(spec.head_dim) if sc else 1.0
        n = spec.kv_page_bytes // spec.elem_bytes
        return elements(rng, n, s, spec.dtype).view(np.uint8)
    if not spec.conv_kernel and not spec.pad_ssm_to_kv_page:
        n = spec.ssm_block_bytes // spec.state_bytes
        return elements(rng, n, 1.0, spec.state_dtype).view(np.uint8)
    # recurrent state, then the window of the last K-1 convolution inputs [K-1][conv_dim]
    sc = spec.scale_inputs if scale_inputs is None else scale_inputs
    s = 1.0 / math.sqrt(spec.ssm_headdim) if sc else 1.0
    out = np.zeros(spec.ssm_block_bytes, dtype=np.uint8)
    n = spec.ssm_state_bytes // spec.state_bytes
    out[: spec.ssm_state_bytes] = elements(rng, n, 1.0, spec.state_dtype).view(np.uint8)
    if spec.conv_kernel:
        m = (spec.conv_kernel - 1) * spec.conv_dim
        out[spec.ssm_state_bytes: spec.ssm_state_bytes + spec.conv_window_bytes] = \
            elements(rng, m, s, spec.dtype).view(np.uint8)
    return out


def fill_units(spec: ModelSpec, seed: int, jobs: Sequence[Tuple[int, int, int, int]],
               sink, threads: int = 8, scale_inputs: Optional[bool] = None) -> None:
    """Generate unit_content for each job (pool, layer, request, index) on a
    thread pool and hand (job_number, bytes) to sink() in the calling thread."""
    def work(j):
        return unit_content(spec, seed, *j, scale_inputs=scale_inputs)
    if threads <= 1:
        for i, j in enumerate(jobs):
            sink(i, work(j))
        return
    with ThreadPoolExecutor(max_workers=threads) as ex:
        window = 4 * threads
        pending = []
        it = iter(enumerate(jobs))
        done = False
        while pending or not done:
            while not done and len(pending) < window:
                try:
                    i, j = next(it)
                except StopIteration:
                    done = True
                    break
                pending.append((i, ex.submit(work, j)))
            if pending:
                i, f = pending.pop(0)
                sink(i, f.result())
