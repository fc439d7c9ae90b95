"""CPU oracle for the asymmetric-pool hybrid decode path (TEST INFRASTRUCTURE ONLY).

This module is a plain, slow, float64 restatement of what the path computes:
the 32-bit virtual handle and the virtual page table (Method, "Asymmetric
Virtual Page Table" and Fig. 1), allocate/free with the capacity error and the
capacity migration between the two pools (Method, "Dynamic Pool Rebalancing"),
paged grouped-query decode attention over the KV-page pool and the Mamba-2
style single-token state update in the SSM-block pool (Background, "KV Cache
and SSM State Management": scatter-gather page lookups for KV, contiguous
in-place read/write for SSM state).

It exists so that tests, the smoke check and the benchmark's CPU-baseline leg
can compare the GPU library with it.  Nothing in the product imports it, and
it imports nothing from the product: it has its own handle codec, its own
geometry arithmetic and its own page-layout index formulas.

Parity pins: every function here is pinned by tests in tests/test_oracle_*.py
(worked example of Fig. 1, closed-form unit sizes, dense attention through a
library routine - also for the append path -, unrolled recurrence closed form,
two-counter capacity model, migration conservation laws, the paper's default
policy parameters and each edge of Fig. 2).  Not pinned, because the paper's harness and
traces are not available: the paper's OOM counts, goodput and bootstrap CIs
("parity unpinned"; not attempted).

Readings taken where the paper is silent are listed in the design notes and
repeated next to the code that depends on them.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

# ----------------------------------------------------------------------------
# Handle codec (Method, "Asymmetric Virtual Page Table"; Fig. 1: a 32-bit
# handle = pool_id tag + page_id).  The paper does not give the bit split;
# reading: 2-bit tag in the top bits (room for the third pool named under
# Future Work), 30-bit page id.  All-ones is the invalid handle.
# ----------------------------------------------------------------------------
POOL_KV = 0
POOL_SSM = 1
N_POOLS = 2
PAGE_ID_BITS = 30
PAGE_ID_MASK = (1 << PAGE_ID_BITS) - 1
INVALID_HANDLE = 0xFFFFFFFF
UNMAPPED = 0xFFFFFFFF

OK = 0
ERR_CAPACITY = 1          # the paper's CapacityError
ERR_INVALID_HANDLE = 2
ERR_INVALID_ARG = 3


def encode_handle(pool_id: int, page_id: int) -> int:
    if not (0 <= pool_id < 4) or not (0 <= page_id <= PAGE_ID_MASK):
        raise ValueError("handle field out of range")
    return (pool_id << PAGE_ID_BITS) | page_id


def decode_handle(h: int) -> Tuple[int, int]:
    h = int(h) & 0xFFFFFFFF
    return h >> PAGE_ID_BITS, h & PAGE_ID_MASK


def round_up(v: int, m: int) -> int:
    return (v + m - 1) // m * m


# ----------------------------------------------------------------------------
# Shapes and unit sizes (Method, "Asymmetric Virtual Page Table": a KV page is
# attention_page_tokens x per_token_bytes, an SSM block is state_dim x
# bytes_per_element; 128-byte slab alignment, 16-byte page alignment).
# Reading: one KV page holds K and V of ONE attention layer for all KV heads,
# mirroring the per-layer SSM block of Fig. 1's caption.
# ----------------------------------------------------------------------------
ELEM_BYTES = {"f32": 4, "bf16": 2}
SLAB_ALIGN = 128
PAGE_ALIGN = 16


@dataclass(frozen=True)
class Shape:
    dtype: str            # element type of K, V, q, x, B, C: "f32" or "bf16"
    page_tokens: int      # attention_page_tokens (paper default 16)
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ssm_heads: int        # H
    ssm_headdim: int      # P
    ssm_dstate: int       # N
    state_dtype: str = "f32"   # storage type of the SSM state (bytes_per_element of the block)
    conv_kernel: int = 0       # K taps of the short causal convolution in front of the
                               # recurrence; 0 = the block is the recurrent state alone
    pad_ssm_to_kv_page: bool = False   # sizing of a unified pool (Background, "Existing Cache
                               # Management"; Evaluation, the padded_unified baseline): the SSM
                               # block is padded up to a whole number of attention pages

    @property
    def conv_dim(self) -> int:
        """Channels of the convolution: x [H][P], then B [N], then C [N]."""
        return self.ssm_heads * self.ssm_headdim + 2 * self.ssm_dstate

    @property
    def elem_bytes(self) -> int:
        return ELEM_BYTES[self.dtype]

    @property
    def state_bytes(self) -> int:
        return ELEM_BYTES[self.state_dtype]

    @property
    def per_token_bytes(self) -> int:
        return 2 * self.n_kv_heads * self.head_dim * self.elem_bytes

    @property
    def state_dim(self) -> int:
        return self.ssm_heads * self.ssm_headdim * self.ssm_dstate

    def unit_bytes(self, pool: int) -> int:
        if pool == POOL_KV:
            raw = self.page_tokens * self.per_token_bytes
        else:
            raw = self.state_dim * self.state_bytes    # state_dim x bytes_per_element
            if self.conv_kernel:                       # + the last K-1 convolution inputs
                raw += (self.conv_kernel - 1) * self.conv_dim * self.elem_bytes
        unit = round_up(raw, PAGE_ALIGN)
        if pool == POOL_SSM and self.pad_ssm_to_kv_page:
            unit = round_up(unit, self.unit_bytes(POOL_KV))
        return unit

    def native_ssm_bytes(self) -> int:
        """What the block holds without the unified-pool padding."""
        return Shape(self.dtype, self.page_tokens, self.n_q_heads, self.n_kv_heads, self.head_dim,
                     self.ssm_heads, self.ssm_headdim, self.ssm_dstate, self.state_dtype,
                     self.conv_kernel).unit_bytes(POOL_SSM)


def decode_elements(raw: np.ndarray, dtype: str) -> np.ndarray:
    """Bytes -> float64 values.  bf16 is the top half of an IEEE fp32."""
    if dtype == "f32":
        return raw.view(np.float32).astype(np.float64)
    u = raw.view(np.uint16).astype(np.uint32) << 16
    return u.view(np.float32).astype(np.float64)


def round_to_bf16_bits(v: np.ndarray) -> np.ndarray:
    """float64 -> nearest bf16 (8 significant bits, ties to even), as uint16 bit patterns.
    Written from the format's definition: v = m * 2^e with 0.5 <= |m| < 1 is kept to
    a multiple of 2^(e-8) (8 significant bits), and never finer than 2^-133, the
    smallest subnormal."""
    v = np.asarray(v, dtype=np.float64)
    m, e = np.frexp(v)
    qe = np.maximum(e - 8, -133)
    q = np.ldexp(np.rint(np.ldexp(v, -qe)), qe)           # np.rint rounds halves to even
    return (q.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)   # exact: q is representable


def as_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Input array (float32, or uint16 bit patterns for bf16) -> float64."""
    a = np.ascontiguousarray(a)
    if dtype == "bf16":
        if a.dtype != np.uint16:
            raise TypeError("bf16 inputs are passed as uint16 bit patterns")
        return decode_elements(a.reshape(-1).view(np.uint8), "bf16").reshape(a.shape)
    return a.astype(np.float64)


@dataclass
class MigrateResult:
    code: int
    units_copied: int = 0
    recipient_gain: int = 0
    bytes_wasted: int = 0
    moves: List[Tuple[int, int, int]] = field(default_factory=list)  # (src, dst, vid)


class Pools:
    """Two pools in one arena behind one virtual page table.

    Geometry (reading of "shrinking it at the high end of its address space
    ... and the recipient pool grows", Method, "Dynamic Pool Rebalancing"):
    KV slot s lives at byte s*unit_kv counted up from the arena base; SSM slot
    i lives at usable - (i+1)*unit_ssm counted down from the arena top.  The
    high ends of both pools face one shared gap in the middle.
    """

    def __init__(self, shape: Shape, arena_bytes: int, kv_capacity: int,
                 ssm_capacity: int,
                 slot_rank: Optional[Sequence[Optional[np.ndarray]]] = None,
                 max_vid: Optional[Sequence[int]] = None,
                 with_data: bool = True):
        self.shape = shape
        self.unit = [shape.unit_bytes(POOL_KV), shape.unit_bytes(POOL_SSM)]
        self.usable = arena_bytes // SLAB_ALIGN * SLAB_ALIGN
        self.max_slots = [self.usable // u for u in self.unit]
        need = kv_capacity * self.unit[0] + ssm_capacity * self.unit[1]
        if need > self.usable:
            raise ValueError("initial capacities do not fit the arena")
        self.capacity = [int(kv_capacity), int(ssm_capacity)]
        self.gap = self.usable - need
        self.max_vid = list(max_vid) if max_vid is not None else list(self.max_slots)
        self.rank = []
        for p in range(N_POOLS):
            r = None if slot_rank is None else slot_rank[p]
            if r is None:
                r = np.arange(self.max_slots[p], dtype=np.int64)
            r = np.asarray(r, dtype=np.int64)
            if r.shape != (self.max_slots[p],) or \
                    not np.array_equal(np.sort(r), np.arange(self.max_slots[p])):
                raise ValueError("slot_rank must be a permutation of all possible slots")
            self.rank.append(r)
        # the virtual page table and its reverse map
        self.slot_of = [np.full(self.max_vid[p], UNMAPPED, dtype=np.int64) for p in range(N_POOLS)]
        self.vid_of = [np.full(self.max_slots[p], UNMAPPED, dtype=np.int64) for p in range(N_POOLS)]
        self.arena = np.zeros(self.usable, dtype=np.uint8) if with_data else None
        self.unrounded_state = {}      # handle -> float64 state of its last update, before storage
        self.update_scale = {}         # handle -> |a*S| + |dt*x*B| of that update (rounding-noise scale)
        self.output_scale = {}         # handle -> sum_n |S*C| behind each y of the last step (same use)
        # counters (the 64-bit logical operation counter of the paper + outcome counters)
        self.ops = 0
        self.capacity_errors = 0
        self.migrations = 0
        self.units_copied = 0
        self.bytes_migrated = 0
        self.bytes_wasted = 0

    # ---- geometry -----------------------------------------------------------
    def byte_offset(self, pool: int, slot: int) -> int:
        if pool == POOL_KV:
            return slot * self.unit[POOL_KV]
        return self.usable - (slot + 1) * self.unit[POOL_SSM]

    # ---- table ---------------------------------------------------------------
    def resolve(self, h: int) -> Optional[Tuple[int, int, int]]:
        """handle -> (pool, slot, byte offset), or None if not a live handle."""
        pool, vid = decode_handle(h)
        if pool >= N_POOLS or vid >= self.max_vid[pool]:
            return None
        slot = int(self.slot_of[pool][vid])
        if slot == UNMAPPED:
            return None
        return pool, slot, self.byte_offset(pool, slot)

    def live_count(self, pool: int) -> int:
        return int(np.count_nonzero(self.vid_of[pool][: self.capacity[pool]] != UNMAPPED))

    def free_count(self, pool: int) -> int:
        return self.capacity[pool] - self.live_count(pool)

    def _best_free_slot(self, pool: int, below: int) -> int:
        """Free slot of lowest rank among slots < below (reading: placement is a
        caller-given rank order, so that physical placement can be permuted)."""
        free = np.flatnonzero(self.vid_of[pool][:below] == UNMAPPED)
        return int(free[np.argmin(self.rank[pool][free])])

    def _lowest_free_vid(self, pool: int) -> Optional[int]:
        free = np.flatnonzero(self.slot_of[pool] == UNMAPPED)
        return int(free[0]) if free.size else None

    # ---- allocate / free (Method, "Dynamic Pool Rebalancing": allocate()
    #      raises CapacityError when the tagged pool cannot serve the request) --
    def alloc(self, pool: int, n: int) -> Tuple[int, List[int]]:
        if pool not in (POOL_KV, POOL_SSM) or n <= 0:
            return ERR_INVALID_ARG, []
        self.ops += 1
        free_vids = int(np.count_nonzero(self.slot_of[pool] == UNMAPPED))
        if self.free_count(pool) < n or free_vids < n:
            self.capacity_errors += 1
            return ERR_CAPACITY, []
        out = []
        for _ in range(n):
            vid = self._lowest_free_vid(pool)
            slot = self._best_free_slot(pool, self.capacity[pool])
            self.slot_of[pool][vid] = slot
            self.vid_of[pool][slot] = vid
            if pool == POOL_SSM and self.arena is not None:
                # a new sequence starts from the zero state
                off = self.byte_offset(pool, slot)
                self.arena[off: off + self.unit[pool]] = 0
            out.append(encode_handle(pool, vid))
        return OK, out

    def free(self, handles: Sequence[int]) -> int:
        if len(handles) == 0:
            return ERR_INVALID_ARG
        self.ops += 1
        seen = set()
        for h in handles:
            if self.resolve(h) is None or int(h) in seen:
                return ERR_INVALID_HANDLE
            seen.add(int(h))
        for h in handles:
            pool, vid = decode_handle(h)
            slot = int(self.slot_of[pool][vid])
            self.slot_of[pool][vid] = UNMAPPED
            self.vid_of[pool][slot] = UNMAPPED
        return OK

    # ---- capacity migration (Method, "Dynamic Pool Rebalancing") -------------
    def migrate(self, donor: int, n: int) -> MigrateResult:
        """Move the capacity of n donor units to the other pool.

        The donor shrinks at the high end of its slot range; live units found
        there are first copied to free slots below the new capacity (the
        paper's prototype needs no copy because its tensors are oversized; a
        single arena does).  Freed bytes plus the gap left by earlier
        migrations become floor(bytes / recipient unit) new recipient slots;
        the remainder is the paper's wasted bytes ("donor bytes freed modulo
        the recipient page size") and stays in the gap.  All-or-nothing: a
        request the donor cannot satisfy changes nothing (rollback clause).
        """
        if donor not in (POOL_KV, POOL_SSM) or n <= 0:
            return MigrateResult(ERR_INVALID_ARG)
        self.ops += 1
        if n > self.capacity[donor] or self.free_count(donor) < n:
            return MigrateResult(ERR_CAPACITY)
        recip = 1 - donor
        newcap = self.capacity[donor] - n
        res = MigrateResult(OK)
        for s in range(newcap, self.capacity[donor]):
            vid = int(self.vid_of[donor][s])
            if vid == UNMAPPED:
                continue
            dst = self._best_free_slot(donor, newcap)
            if self.arena is not None:
                so, do = self.byte_offset(donor, s), self.byte_offset(donor, dst)
                u = self.unit[donor]
                self.arena[do: do + u] = self.arena[so: so + u]
            self.vid_of[donor][dst] = vid
            self.vid_of[donor][s] = UNMAPPED
            self.slot_of[donor][vid] = dst
            res.moves.append((s, dst, vid))
        self.capacity[donor] = newcap
        avail = self.gap + n * self.unit[donor]
        gain = avail // self.unit[recip]
        self.gap = avail % self.unit[recip]
        self.capacity[recip] += gain
        res.units_copied = len(res.moves)
        res.recipient_gain = gain
        res.bytes_wasted = self.gap
        self.migrations += 1
        self.units_copied += res.units_copied
        self.bytes_migrated += n * self.unit[donor]
        self.bytes_wasted += res.bytes_wasted
        return res

    def absorb_gap(self, pool: int) -> MigrateResult:
        """Give `pool` the whole units that fit into the gap between the pools.

        The gap holds what earlier migrations left over ("donor bytes freed modulo
        the recipient page size") and whatever the arena had beyond the initial
        capacities; nobody owns those bytes, so no donor shrinks and nothing is
        copied.  The new slots are the ones just above the pool's capacity; the
        remainder stays in the gap and is counted as this step's wasted bytes.
        A gap smaller than one unit changes nothing (ERR_CAPACITY).
        """
        if pool not in (POOL_KV, POOL_SSM):
            return MigrateResult(ERR_INVALID_ARG)
        self.ops += 1
        gain = self.gap // self.unit[pool]
        if gain == 0:
            return MigrateResult(ERR_CAPACITY)
        self.capacity[pool] += gain
        self.gap -= gain * self.unit[pool]
        res = MigrateResult(OK)
        res.recipient_gain = gain
        res.bytes_wasted = self.gap
        self.migrations += 1
        self.bytes_wasted += res.bytes_wasted
        return res

    def stats(self) -> dict:
        return {
            "capacity": tuple(self.capacity),
            "live": (self.live_count(0), self.live_count(1)),
            "free": (self.free_count(0), self.free_count(1)),
            "gap_bytes": self.gap,
            "ops": self.ops,
            "capacity_errors": self.capacity_errors,
            "migrations": self.migrations,
            "units_copied": self.units_copied,
            "bytes_migrated": self.bytes_migrated,
            "bytes_wasted": self.bytes_wasted,
        }

    def state_values(self, h: int) -> np.ndarray:
        """The SSM block behind handle h as float64 [H][P][N]."""
        sh = self.shape
        n = sh.state_dim * sh.state_bytes
        return decode_elements(self.unit_view(h)[:n], sh.state_dtype).reshape(
            sh.ssm_heads, sh.ssm_headdim, sh.ssm_dstate)

    # ---- raw unit access by handle ------------------------------------------
    def unit_view(self, h: int) -> np.ndarray:
        r = self.resolve(h)
        if r is None:
            raise KeyError("not a live handle: 0x%08x" % int(h))
        pool, _, off = r
        return self.arena[off: off + self.unit[pool]]

    # ---- in-page layout -------------------------------------------------------
    # The paper does not fix the layout inside a KV page.  Layout used here
    # (x = 16 bytes / element size, T = page_tokens):
    #   K element (kv head g, token t, dim d) at element index
    #       ((g*(D/x) + d//x)*T + t)*x + d%x
    #   V element (g, t, d) at element index  Hkv*T*D + (g*D + d)*T + t
    def _page_to_kv(self, raw: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
        sh = self.shape
        T, G, D = sh.page_tokens, sh.n_kv_heads, sh.head_dim
        x = 16 // sh.elem_bytes
        e = decode_elements(raw[: 2 * T * G * D * sh.elem_bytes], sh.dtype)
        k = e[: G * T * D].reshape(G, D // x, T, x).transpose(2, 0, 1, 3).reshape(T, G, D)
        v = e[G * T * D:].reshape(G, D, T).transpose(2, 0, 1)
        return k, v          # both [T][G][D]

    def kv_element_offset(self, which: str, g: int, t: int, d: int) -> int:
        """Byte offset inside a page of one K or V element (layout above)."""
        sh = self.shape
        T, G, D = sh.page_tokens, sh.n_kv_heads, sh.head_dim
        x = 16 // sh.elem_bytes
        if which == "k":
            idx = ((g * (D // x) + d // x) * T + t) * x + d % x
        else:
            idx = G * T * D + (g * D + d) * T + t
        return idx * sh.elem_bytes

    def write_kv_token(self, h: int, t: int, k_row: np.ndarray, v_row: np.ndarray) -> None:
        """Store one token's K and V ([Hkv][D], raw element bit patterns:
        float32 or uint16) into token slot t of the page behind handle h."""
        sh = self.shape
        page = self.unit_view(h)
        kb = np.ascontiguousarray(k_row).view(np.uint8).reshape(sh.n_kv_heads, sh.head_dim, sh.elem_bytes)
        vb = np.ascontiguousarray(v_row).view(np.uint8).reshape(sh.n_kv_heads, sh.head_dim, sh.elem_bytes)
        for g in range(sh.n_kv_heads):
            for d in range(sh.head_dim):
                o = self.kv_element_offset("k", g, t, d)
                page[o: o + sh.elem_bytes] = kb[g, d]
                o = self.kv_element_offset("v", g, t, d)
                page[o: o + sh.elem_bytes] = vb[g, d]

    # ---- paged grouped-query decode attention ---------------------------------
    def paged_attention(self, handles: np.ndarray, ctx: np.ndarray, q: np.ndarray) -> np.ndarray:
        """o[r, j] = softmax_t(q[r, j] . K_t[g] / sqrt(D)) . V[:, g],  g = j // (Hq/Hkv),
        over the ctx[r] tokens held in pages handles[r, 0 .. ceil(ctx/T)-1].
        Token slots at or beyond ctx[r] in the last page are never read into
        the result.  q: [batch][Hq][D] in the element dtype.  Returns float64."""
        sh = self.shape
        T, Hq, G, D = sh.page_tokens, sh.n_q_heads, sh.n_kv_heads, sh.head_dim
        qf = as_f64(q, sh.dtype)
        batch = len(ctx)
        o = np.zeros((batch, Hq, D), dtype=np.float64)
        for r in range(batch):
            n_tok = int(ctx[r])
            if n_tok == 0:
                continue                      # no tokens: output row defined as zero
            n_pages = -(-n_tok // T)
            K = np.empty((n_pages * T, G, D))
            V = np.empty((n_pages * T, G, D))
            for i in range(n_pages):
                res = self.resolve(int(handles[r, i]))
                if res is None or res[0] != POOL_KV:
                    raise KeyError("request %d page %d: not a live KV handle" % (r, i))
                k, v = self._page_to_kv(self.arena[res[2]: res[2] + self.unit[POOL_KV]])
                K[i * T: (i + 1) * T] = k
                V[i * T: (i + 1) * T] = v
            K, V = K[:n_tok], V[:n_tok]
            for j in range(Hq):
                g = j // (Hq // G)
                s = (K[:, g, :] * qf[r, j][None, :]).sum(axis=1) / math.sqrt(D)
                p = np.exp(s - s.max())
                p /= p.sum()
                o[r, j] = (p[:, None] * V[:, g, :]).sum(axis=0)
        return o

    # ---- single-token SSM state update ----------------------------------------
    def ssm_step(self, handles: np.ndarray, x: np.ndarray, dt: np.ndarray, A: np.ndarray,
                 B: np.ndarray, C: np.ndarray, exact_inputs: bool = False) -> np.ndarray:
        """For request r, head h, channel p, state index n (state block [H][P][N], fp32):
             a = exp(dt[r,h] * A[h])
             S[h,p,n] <- a * S[h,p,n] + dt[r,h] * x[r,h,p] * B[r,n]
             y[r,h,p] = sum_n S[h,p,n] * C[r,n]          (with the updated S)
        The block is updated in place (stored rounded once to the state dtype);
        y uses the updated value before that rounding.  x: [batch][H][P], B, C: [batch][N]
        in the element dtype (float64 as they are if exact_inputs: the outputs of
        conv_step, which are not rounded on the way); dt: [batch][H] fp32; A: [H] fp32.
        Returns float64."""
        sh = self.shape
        H, P, N = sh.ssm_heads, sh.ssm_headdim, sh.ssm_dstate
        if exact_inputs:
            xf, Bf, Cf = (np.asarray(t, dtype=np.float64) for t in (x, B, C))
        else:
            xf, Bf, Cf = as_f64(x, sh.dtype), as_f64(B, sh.dtype), as_f64(C, sh.dtype)
        dtf, Af = np.asarray(dt, dtype=np.float64), np.asarray(A, dtype=np.float64)
        batch = len(handles)
        y = np.zeros((batch, H, P), dtype=np.float64)
        for r in range(batch):
            res = self.resolve(int(handles[r]))
            if res is None or res[0] != POOL_SSM:
                raise KeyError("request %d: not a live SSM handle" % r)
            raw = self.arena[res[2]: res[2] + H * P * N * sh.state_bytes]
            S = decode_elements(raw, sh.state_dtype).reshape(H, P, N)
            a = np.exp(dtf[r] * Af)                                   # [H]
            decayed = a[:, None, None] * S
            driven = (dtf[r][:, None] * xf[r])[:, :, None] * Bf[r][None, None, :]
            self.update_scale[int(handles[r])] = np.abs(decayed) + np.abs(driven)
            S = decayed + driven
            y[r] = (S * Cf[r][None, None, :]).sum(axis=2)
            self.output_scale[int(handles[r])] = (np.abs(S) * np.abs(Cf[r])[None, None, :]).sum(axis=2)
            self.unrounded_state[int(handles[r])] = S      # for tests of the storage rounding
            if sh.state_dtype == "f32":
                raw.view(np.float32)[:] = S.astype(np.float32).reshape(-1)
            else:
                raw.view(np.uint16)[:] = round_to_bf16_bits(S).reshape(-1)
        return y

    def conv_window(self, h: int) -> np.ndarray:
        """The last K-1 convolution inputs kept behind the state in block h, as
        float64 [K-1][conv_dim], oldest token first."""
        sh = self.shape
        off = sh.state_dim * sh.state_bytes
        n = (sh.conv_kernel - 1) * sh.conv_dim * sh.elem_bytes
        return decode_elements(self.unit_view(h)[off: off + n], sh.dtype).reshape(
            sh.conv_kernel - 1, sh.conv_dim)

    def conv_step(self, handles: np.ndarray, u: np.ndarray, w: np.ndarray,
                  b: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """The short causal depthwise convolution that a Mamba-2 layer (the SSM layer
        of Background, "Hybrid Mamba-Transformer Architectures") applies to x, B and C
        before the recurrence, taken one token at a time: with u_t[c] the token's input
        on channel c and the inputs of the K-1 tokens before it kept in the block,
             v[c]   = b[c] + sum_{k=0..K-1} w[k][c] * u_{t-(K-1)+k}[c]
             out[c] = v[c] / (1 + exp(-v[c]))                       (SiLU)
        after which the kept window moves on by one token (inputs are stored as they
        came, in the element dtype: no rounding).  A fresh block holds zeros, i.e. the
        sequence starts after K-1 zero inputs.  u: [batch][conv_dim], w: [K][conv_dim],
        b: [conv_dim] in the element dtype.  Returns float64 x [batch][H][P],
        B [batch][N], C [batch][N]."""
        sh = self.shape
        K, Cd = sh.conv_kernel, sh.conv_dim
        H, P, N = sh.ssm_heads, sh.ssm_headdim, sh.ssm_dstate
        uf, wf, bf = as_f64(u, sh.dtype), as_f64(w, sh.dtype), as_f64(b, sh.dtype)
        off = sh.state_dim * sh.state_bytes
        nbytes = (K - 1) * Cd * sh.elem_bytes
        out = np.zeros((len(handles), Cd), dtype=np.float64)
        u_raw = np.ascontiguousarray(u)
        for r in range(len(handles)):
            res = self.resolve(int(handles[r]))
            if res is None or res[0] != POOL_SSM:
                raise KeyError("request %d: not a live SSM handle" % r)
            raw = self.arena[res[2] + off: res[2] + off + nbytes]
            past = decode_elements(raw, sh.dtype).reshape(K - 1, Cd)
            v = bf.copy()
            for k in range(K - 1):
                v += wf[k] * past[k]
            v += wf[K - 1] * uf[r]
            out[r] = v / (1.0 + np.exp(-v))
            rows = raw.reshape(K - 1, Cd * sh.elem_bytes)
            rows[:-1] = rows[1:].copy()
            rows[-1] = u_raw[r].view(np.uint8)
        x = out[:, : H * P].reshape(len(handles), H, P)
        return x, out[:, H * P: H * P + N], out[:, H * P + N:]

    # ---- one hybrid decode step ------------------------------------------------
    def append_token(self, handles: np.ndarray, ctx: np.ndarray, k_new: np.ndarray,
                     v_new: np.ndarray) -> None:
        """Append-only KV behaviour (Background, "KV Cache and SSM State Management"):
        request r's new token goes to token slot ctx[r] % T of its page ctx[r] // T,
        whose handle the caller has already placed in handles[r].  k_new, v_new:
        [batch][Hkv][D] in the element dtype."""
        T = self.shape.page_tokens
        for r in range(len(ctx)):
            t = int(ctx[r])
            self.write_kv_token(int(handles[r, t // T]), t % T, k_new[r], v_new[r])

    def decode_step(self, layer_kinds: Sequence[int], kv_handles: np.ndarray, ctx: np.ndarray,
                    q: np.ndarray, ssm_handles: np.ndarray, x: np.ndarray, dt: np.ndarray,
                    A: np.ndarray, B: np.ndarray, C: np.ndarray,
                    k_new: Optional[np.ndarray] = None,
                    v_new: Optional[np.ndarray] = None,
                    xbc: Optional[np.ndarray] = None, conv_w: Optional[np.ndarray] = None,
                    conv_b: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
        """Layers in model order (0 = attention, 1 = SSM).  Per-kind arrays are
        indexed by the layer's ordinal among layers of its kind:
        kv_handles [n_attn][batch][max_pages], q [n_attn][batch][Hq][D],
        ssm_handles [n_ssm][batch], x [n_ssm][batch][H][P], dt [n_ssm][batch][H],
        A [n_ssm][H], B, C [n_ssm][batch][N].  ctx counts tokens already resident.
        If k_new, v_new ([n_attn][batch][Hkv][D]) are given, each attention layer
        first appends the new token and then attends over ctx + 1 tokens.
        With a convolution window in the blocks (conv_kernel > 0), x, B and C are
        ignored: each SSM layer first runs conv_step on xbc [n_ssm][batch][conv_dim]
        with conv_w [n_ssm][K][conv_dim], conv_b [n_ssm][conv_dim] and feeds its
        unrounded outputs to the recurrence.
        Returns (o [n_attn]..., y [n_ssm]...)."""
        o, y = [], []
        ia = iss = 0
        ctx = np.asarray(ctx)
        for kind in layer_kinds:
            if kind == 0:
                if k_new is not None:
                    self.append_token(kv_handles[ia], ctx, k_new[ia], v_new[ia])
                    o.append(self.paged_attention(kv_handles[ia], ctx + 1, q[ia]))
                else:
                    o.append(self.paged_attention(kv_handles[ia], ctx, q[ia]))
                ia += 1
            elif self.shape.conv_kernel:
                xc, Bc, Cc = self.conv_step(ssm_handles[iss], xbc[iss], conv_w[iss], conv_b[iss])
                y.append(self.ssm_step(ssm_handles[iss], xc, dt[iss], A[iss], Bc, Cc,
                                       exact_inputs=True))
                iss += 1
            else:
                y.append(self.ssm_step(ssm_handles[iss], x[iss], dt[iss], A[iss], B[iss], C[iss]))
                iss += 1
        sh = self.shape
        o = np.stack(o) if o else np.zeros((0, len(ctx), sh.n_q_heads, sh.head_dim))
        y = np.stack(y) if y else np.zeros((0, len(ctx), sh.ssm_heads, sh.ssm_headdim))
        return o, y


# ----------------------------------------------------------------------------
# Rebalancing policy (Method, "Dynamic Pool Rebalancing", Fig. 2, and the
# failure modes listed under Limitations).  A four-state machine whose
# transitions are evaluated ONLY inside the CapacityError handler of
# allocate(): BALANCED -> X_PRESSURED when x_free < threshold_low;
# X_PRESSURED -> REBALANCING when the other pool's free fraction exceeds
# threshold_high; REBALANCING -> BALANCED when the migration completes;
# X_PRESSURED -> BALANCED when x's free fraction recovers.  Rebalancing is
# throttled by the logical operation counter (at least
# min_rebalance_interval_ops operations between migrations) and the step is
# bounded by migration_batch_size.  With no donor above threshold_high the
# allocator behaves as a static partition.
#
# Readings where the text is silent: migration_batch_size counts units of the
# RECIPIENT pool (the step gives the starving pool up to B units, limited by
# the donor's free units); one failing allocate() may take several transitions
# in a row (BALANCED -> X_PRESSURED -> REBALANCING -> BALANCED); after a
# migration the allocation is retried once.
#
# Text against figure.  The Method text starts a migration on a CapacityError
# with a donor above threshold_high; Fig. 2 reaches REBALANCING only through
# X_PRESSURED, i.e. only when the failing pool's own free fraction is below
# threshold_low.  The figure is followed: a multi-unit request that fails while
# its pool still has threshold_low or more free does not rebalance, and a
# failure in pool Y while the machine sits in X_PRESSURED is ignored until X
# recovers.
#
# Bytes that nobody owns.  When the gap between the pools already holds the B
# units the step would give (left-overs of earlier migrations, or an arena
# larger than the initial capacities), the step takes them from the gap: no
# donor is needed, so the threshold_high test does not apply, but it is a
# rebalance like any other (throttled, counted, REBALANCING -> BALANCED).
# ----------------------------------------------------------------------------
BALANCED = 0
KV_PRESSURED = 1
SSM_PRESSURED = 2
REBALANCING = 3


@dataclass(frozen=True)
class Policy:
    threshold_low: float = 0.05
    threshold_high: float = 0.30
    migration_batch_size: int = 128
    min_rebalance_interval_ops: int = 1000


class Rebalancer:
    def __init__(self, pools: Pools, policy: Policy = Policy()):
        if not (0.0 <= policy.threshold_low < policy.threshold_high <= 1.0):
            raise ValueError("threshold_low must be below threshold_high")
        if policy.migration_batch_size < 1 or policy.min_rebalance_interval_ops < 0:
            raise ValueError("bad migration_batch_size or min_rebalance_interval_ops")
        self.pools = pools
        self.policy = policy
        self.state = BALANCED
        self.last_rebalance_op: Optional[int] = None
        self.rebalance_count = 0
        self.oom_events = 0            # allocate() calls that finally failed

    def free_fraction(self, pool: int) -> float:
        cap = self.pools.capacity[pool]
        return self.pools.free_count(pool) / cap if cap else 0.0

    def allocate(self, pool: int, n: int) -> Tuple[int, List[int], int]:
        """Returns (code, handles, donor units migrated by this call)."""
        code, hs = self.pools.alloc(pool, n)
        if code != ERR_CAPACITY:
            return code, hs, 0
        moved = self._capacity_error_handler(pool)     # donor units, 0: no rebalance, -1: from the gap
        if moved:
            code, hs = self.pools.alloc(pool, n)
        if code == ERR_CAPACITY:
            self.oom_events += 1
        return code, hs, max(moved, 0)

    def _capacity_error_handler(self, pool: int) -> int:
        pol, p = self.policy, self.pools
        other = 1 - pool
        pressured = KV_PRESSURED if pool == POOL_KV else SSM_PRESSURED
        # free recovers
        if self.state == KV_PRESSURED and self.free_fraction(POOL_KV) >= pol.threshold_low:
            self.state = BALANCED
        if self.state == SSM_PRESSURED and self.free_fraction(POOL_SSM) >= pol.threshold_low:
            self.state = BALANCED
        if self.state == BALANCED and self.free_fraction(pool) < pol.threshold_low:
            self.state = pressured
        if self.state != pressured:
            return 0
        need_bytes = pol.migration_batch_size * p.unit[pool] - p.gap
        from_gap = need_bytes <= 0                     # the gap alone holds the step's B units
        if not from_gap and not (self.free_fraction(other) > pol.threshold_high):
            return 0                                   # no donor: static-partition behaviour
        if self.last_rebalance_op is not None and \
                p.ops - self.last_rebalance_op < pol.min_rebalance_interval_ops:
            return 0                                   # throttled
        donor_units = 0
        if not from_gap:
            donor_units = min(-(-need_bytes // p.unit[other]), p.free_count(other))
            if donor_units == 0:
                return 0
        self.state = REBALANCING
        res = p.absorb_gap(pool) if from_gap else p.migrate(other, donor_units)
        assert res.code == OK
        self.rebalance_count += 1
        self.last_rebalance_op = p.ops
        self.state = BALANCED                          # migration complete
        return -1 if from_gap else donor_units
