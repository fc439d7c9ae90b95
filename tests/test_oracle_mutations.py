"""Are the oracle's pins sharp?  Each case plants one plausible mistake in a
copy of the oracle's source (a wrong index, sign, operand, comparison or
rounding), points the pin tests at the mutated copy and requires that at least
one pin fails.  Mistakes are planted in the oracle only, on the CPU."""
import importlib
import os
import sys
import types

import pytest

import tests.helpers as helpers_mod
import tests.test_oracle_compute as pins_compute
import tests.test_oracle_policy as pins_policy
import tests.test_oracle_table as pins_table

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = open(os.path.join(ROOT, "oracle", "avmp_oracle.py")).read()

# (name, text to find, replacement)
MUTATIONS = [
    ("handle tag one bit lower", "return (pool_id << PAGE_ID_BITS) | page_id", "return (pool_id << (PAGE_ID_BITS - 1)) | page_id"),
    ("unit ignores V", "return 2 * self.n_kv_heads * self.head_dim * self.elem_bytes", "return self.n_kv_heads * self.head_dim * self.elem_bytes"),
    ("ssm slots ascend from the base", "return self.usable - (slot + 1) * self.unit[POOL_SSM]", "return slot * self.unit[POOL_SSM]"),
    ("alloc takes the worst-ranked slot", "return int(free[np.argmin(self.rank[pool][free])])", "return int(free[np.argmax(self.rank[pool][free])])"),
    ("alloc takes the highest free id", "return int(free[0]) if free.size else None", "return int(free[-1]) if free.size else None"),
    ("capacity check off by one", "if self.free_count(pool) < n or free_vids < n:", "if self.free_count(pool) <= n or free_vids < n:"),
    ("free forgets the reverse map", "            self.vid_of[pool][slot] = UNMAPPED\n        return OK", "        return OK"),
    ("duplicate handles accepted", "if self.resolve(h) is None or int(h) in seen:", "if self.resolve(h) is None:"),
    ("migrate skips the copy", "                self.arena[do: do + u] = self.arena[so: so + u]", "                pass"),
    ("migrate copies the wrong way", "                self.arena[do: do + u] = self.arena[so: so + u]", "                self.arena[so: so + u] = self.arena[do: do + u]"),
    ("migrate forgets the table", "            self.slot_of[donor][vid] = dst", "            pass"),
    ("gain in donor units", "        gain = avail // self.unit[recip]\n", "        gain = avail // self.unit[donor]\n"),
    ("waste modulo the donor unit", "        self.gap = avail % self.unit[recip]", "        self.gap = avail % self.unit[donor]"),
    ("old gap dropped", "        avail = self.gap + n * self.unit[donor]", "        avail = n * self.unit[donor]"),
    ("failed migrate still shrinks", "        if n > self.capacity[donor] or self.free_count(donor) < n:\n            return MigrateResult(ERR_CAPACITY)",
     "        if n > self.capacity[donor] or self.free_count(donor) < n:\n            self.capacity[donor] -= 1\n            return MigrateResult(ERR_CAPACITY)"),
    ("K chunk index swapped", "k = e[: G * T * D].reshape(G, D // x, T, x).transpose(2, 0, 1, 3).reshape(T, G, D)", "k = e[: G * T * D].reshape(G, T, D // x, x).transpose(1, 0, 2, 3).reshape(T, G, D)"),
    ("V read token-major", "v = e[G * T * D:].reshape(G, D, T).transpose(2, 0, 1)", "v = e[G * T * D:].reshape(G, T, D).transpose(1, 0, 2)"),
    ("query head to KV head by modulo", "g = j // (Hq // G)", "g = j % G"),
    ("scale 1/D", "s = (K[:, g, :] * qf[r, j][None, :]).sum(axis=1) / math.sqrt(D)", "s = (K[:, g, :] * qf[r, j][None, :]).sum(axis=1) / D"),
    ("tail slot of the last page counted", "K, V = K[:n_tok], V[:n_tok]", "K, V = K[:n_tok + 1], V[:n_tok + 1]" if False else "K, V = K[:max(n_tok - 1, 1)], V[:max(n_tok - 1, 1)]"),
    ("softmax not normalised", "                p /= p.sum()\n", ""),
    ("decay exp(dt + A)", "a = np.exp(dtf[r] * Af)", "a = np.exp(dtf[r] + Af)"),
    ("drive term uses C", "driven = (dtf[r][:, None] * xf[r])[:, :, None] * Bf[r][None, None, :]", "driven = (dtf[r][:, None] * xf[r])[:, :, None] * Cf[r][None, None, :]"),
    ("drive term without dt", "driven = (dtf[r][:, None] * xf[r])[:, :, None] * Bf[r][None, None, :]", "driven = (xf[r])[:, :, None] * Bf[r][None, None, :]"),
    ("y from the old state", "            S = decayed + driven\n            y[r] = (S * Cf[r][None, None, :]).sum(axis=2)", "            y[r] = (S * Cf[r][None, None, :]).sum(axis=2)\n            S = decayed + driven"),
    ("y summed over the wrong axis", "y[r] = (S * Cf[r][None, None, :]).sum(axis=2)", "y[r] = (S * Cf[r][None, None, :]).sum(axis=2).T.reshape(y[r].shape) if S.shape[0] != S.shape[1] else (S * Cf[r][None, None, :]).sum(axis=2).T"),
    ("bf16 rounds toward zero", "q = np.ldexp(np.rint(np.ldexp(v, -qe)), qe)", "q = np.ldexp(np.trunc(np.ldexp(v, -qe)), qe)"),
    ("append lands one slot late", "self.write_kv_token(int(handles[r, t // T]), t % T, k_new[r], v_new[r])", "self.write_kv_token(int(handles[r, (t + 1) // T]), (t + 1) % T, k_new[r], v_new[r])"),
    ("append without attending the new token", "o.append(self.paged_attention(kv_handles[ia], ctx + 1, q[ia]))", "o.append(self.paged_attention(kv_handles[ia], ctx, q[ia]))"),
    ("donor needs only threshold_low", "not (self.free_fraction(other) > pol.threshold_high):", "not (self.free_fraction(other) > pol.threshold_low):"),
    ("donor test not strict", "not (self.free_fraction(other) > pol.threshold_high):", "not (self.free_fraction(other) >= pol.threshold_high):"),
    ("gap step still asks for a donor", "if not from_gap and not (self.free_fraction(other)", "if not (self.free_fraction(other)"),
    ("gap step taken when the gap is short of B units", "from_gap = need_bytes <= 0", "from_gap = need_bytes <= p.unit[pool]"),
    ("gap step never taken", "from_gap = need_bytes <= 0", "from_gap = False"),
    ("gap step escapes the throttle", "        if self.last_rebalance_op is not None and \\\n", "        if not from_gap and self.last_rebalance_op is not None and \\\n"),
    ("absorbed units counted in the other pool's size", "        gain = self.gap // self.unit[pool]\n", "        gain = self.gap // self.unit[1 - pool]\n"),
    ("absorbing empties the gap", "        self.gap -= gain * self.unit[pool]", "        self.gap = 0"),
    ("absorbing a short gap is not refused", "        if gain == 0:\n            return MigrateResult(ERR_CAPACITY)", "        if gain < 0:\n            return MigrateResult(ERR_CAPACITY)"),
    ("throttle ignored", "                p.ops - self.last_rebalance_op < pol.min_rebalance_interval_ops:\n            return 0", "                False:\n            return 0"),
    ("throttle off by one", "p.ops - self.last_rebalance_op < pol.min_rebalance_interval_ops", "p.ops - self.last_rebalance_op <= pol.min_rebalance_interval_ops"),
    ("pressure test inverted", "if self.state == BALANCED and self.free_fraction(pool) < pol.threshold_low:", "if self.state == BALANCED and self.free_fraction(pool) > pol.threshold_low:"),
    ("batch bound in donor units", "need_bytes = pol.migration_batch_size * p.unit[pool] - p.gap", "need_bytes = pol.migration_batch_size * p.unit[other] - p.gap"),
    ("thresholds not validated", "if not (0.0 <= policy.threshold_low < policy.threshold_high <= 1.0):", "if False:"),
    ("migration before any failure", "        if code != ERR_CAPACITY:\n            return code, hs, 0\n        moved = self._capacity_error_handler(pool)",
     "        moved = self._capacity_error_handler(pool) if code != ERR_CAPACITY and self.pools.free_count(pool) == 0 else 0\n        if code != ERR_CAPACITY:\n            return code, hs, moved\n        moved = self._capacity_error_handler(pool)"),
    ("conv taps reversed", "                v += wf[k] * past[k]", "                v += wf[K - 2 - k] * past[k]"),
    ("conv newest token meets the oldest tap", "            v += wf[K - 1] * uf[r]", "            v += wf[0] * uf[r]"),
    ("conv forgets the bias", "            v = bf.copy()", "            v = np.zeros_like(bf)"),
    ("conv without activation", "            out[r] = v / (1.0 + np.exp(-v))", "            out[r] = v"),
    ("conv sigmoid of the wrong sign", "            out[r] = v / (1.0 + np.exp(-v))", "            out[r] = v / (1.0 + np.exp(v))"),
    ("conv window does not advance", "            rows[:-1] = rows[1:].copy()", "            pass"),
    ("conv window stores the token in the oldest row", "            rows[-1] = u_raw[r].view(np.uint8)", "            rows[0] = u_raw[r].view(np.uint8)"),
    ("conv hands out C as B", "        return x, out[:, H * P: H * P + N], out[:, H * P + N:]", "        return x, out[:, H * P + N:], out[:, H * P: H * P + N]"),
    ("block size ignores the conv window", "                raw += (self.conv_kernel - 1) * self.conv_dim * self.elem_bytes", "                raw += 0"),
    ("padding rounds down", "            unit = round_up(unit, self.unit_bytes(POOL_KV))", "            unit = max(unit // self.unit_bytes(POOL_KV), 1) * self.unit_bytes(POOL_KV)"),
    ("padding ignored", "        if pool == POOL_SSM and self.pad_ssm_to_kv_page:", "        if False:"),
    ("decode step skips the convolution", "            elif self.shape.conv_kernel:", "            elif False:"),
]

PIN_MODULES = (pins_table, pins_compute, pins_policy)


def _pin_functions():
    out = []
    for mod in PIN_MODULES:
        for name in sorted(dir(mod)):
            fn = getattr(mod, name)
            if name.startswith("test_") and callable(fn):
                out.append((mod, name, fn))
    return out


def _run_pins(mutated):
    """Run every oracle pin against `mutated`; return the names of those that fail."""
    import oracle.sampled as sampled_mod
    patched = [(m, "orc", getattr(m, "orc")) for m in PIN_MODULES + (helpers_mod, sampled_mod)]
    shapes = [(pins_table, n, getattr(pins_table, n)) for n in ("TINY", "JAMBA")] + \
             [(pins_policy, "TINY", pins_policy.TINY)]
    failed = []
    try:
        for m, attr, _ in patched:
            setattr(m, attr, mutated)
        # module-level Shape objects were built from the original class: rebuild them
        pins_table.TINY = pins_table._shape(pins_table.inputs.TINY)
        pins_table.JAMBA = pins_table._shape(pins_table.inputs.JAMBA_MINI)
        pins_policy.TINY = helpers_mod.oracle_shape(pins_policy.inputs.TINY)
        pins_policy.UK, pins_policy.US = pins_policy.TINY.unit_bytes(0), pins_policy.TINY.unit_bytes(1)
        for mod, name, fn in _pin_functions():
            params = getattr(fn, "pytestmark", [])
            arglists = [()]
            for mark in params:
                if mark.name == "parametrize":
                    vals = mark.args[1]
                    arglists = [v if isinstance(v, tuple) else (v,) for v in vals]
            for args in arglists:
                try:
                    fn(*args)
                except KeyboardInterrupt:
                    raise
                except BaseException:       # any failure of a pin counts (pytest's own Failed is a BaseException)
                    failed.append(name)
                    break
    finally:
        for m, attr, old in patched:
            setattr(m, attr, old)
        for m, attr, old in shapes:
            setattr(m, attr, old)
        pins_policy.UK, pins_policy.US = pins_policy.TINY.unit_bytes(0), pins_policy.TINY.unit_bytes(1)
    return failed


def _mutated_module(find, repl):
    assert SOURCE.count(find) >= 1, "mutation target not found in the oracle source: " + find[:50]
    mod = types.ModuleType("oracle_mutant")
    mod.__dict__["__name__"] = "oracle_mutant"
    sys.modules["oracle_mutant"] = mod          # dataclasses look their module up by name
    exec(compile(SOURCE.replace(find, repl, 1), "oracle_mutant.py", "exec"), mod.__dict__)
    return mod


def test_unmutated_oracle_passes_every_pin_through_this_runner():
    mod = _mutated_module("POOL_KV = 0", "POOL_KV = 0")
    assert _run_pins(mod) == []


@pytest.mark.parametrize("name,find,repl", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(name, find, repl):
    failed = _run_pins(_mutated_module(find, repl))
    assert failed, "no pin noticed: " + name
