"""Deterministic generator for the synthetic MoE-decode inputs.

Every array is a pure function of (config seed, stream id, indices): each
stream owns a counter-based Philox generator keyed through numpy's
SeedSequence, so any expert / sequence can be produced on its own, in any
order, on any machine.

Value recipe: all weight matrices N(0, 0.02^2); hidden states N(0, 1); one
preferred expert set per (layer, sequence) drawn without replacement, with a
constant logit bias `beta` on its members.  bf16 configs round every stored
value to bf16 (round-to-nearest-even) so that both consumers see exactly the
same numbers.

Top-K margin: a hidden state is kept only if, for every layer, the K-th and
(K+1)-th largest of  W_r x + bias  (evaluated here in fp64 from the stored
values) are at least `delta` apart; otherwise it is redrawn from a separate
stream.  This is a filter on the *inputs* that makes the selected expert set
independent of floating-point summation order; no value computed here is ever
used as an expected result.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np

from .configs import MoEConfig

# stream ids
_ST_ROUTER, _ST_EXPERT, _ST_SHARED, _ST_X, _ST_XPREFILL, _ST_PREF, _ST_RESAMPLE = range(1, 8)

WEIGHT_STD = 0.02
MAX_REDRAWS = 32


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern (uint16), round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def widen(a: np.ndarray) -> np.ndarray:
    """Stored array (uint16 bf16 bits or float32) -> float32 with identical values."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a)
    return np.ascontiguousarray(a, dtype=np.float32)


INT4_GROUP = 32


def quantize_int4(w_store: np.ndarray):
    """Input recipe for 4-bit experts: a stored bf16 matrix [rows][k] -> (codes uint8 [rows][k] in 0..15,
    scales uint16 bf16 bits [rows][k/32]).  Per group of 32 consecutive columns the scale is max|w| / 7 rounded to
    bf16 (1 for an all-zero group) and the code is round(w / scale) + 8, clipped to 0..15.  This only PRODUCES the
    quantised inputs; what the codes and scales mean (weight = scale * (code - 8)) is implemented separately by the
    library and by the oracle."""
    w = bf16_bits_to_f32(w_store).astype(np.float64)
    rows, k = w.shape
    assert k % INT4_GROUP == 0
    g = w.reshape(rows, k // INT4_GROUP, INT4_GROUP)
    s_bits = f32_to_bf16_bits((np.abs(g).max(axis=-1) / 7.0).astype(np.float32))
    s_bits[bf16_bits_to_f32(s_bits) == 0.0] = np.uint16(0x3F80)
    s = bf16_bits_to_f32(s_bits).astype(np.float64)
    codes = np.clip(np.rint(g / s[..., None]) + 8.0, 0.0, 15.0).astype(np.uint8).reshape(rows, k)
    return codes, s_bits


class Workload:
    def __init__(self, cfg: MoEConfig):
        self.cfg = cfg
        self._router_cache = {}
        self._tok_cache = {}
        self.redraws = 0

    # ------------------------------------------------------------------ rng
    def _rng(self, stream: int, *idx: int) -> np.random.Generator:
        ss = np.random.SeedSequence([self.cfg.seed, stream, *[int(i) for i in idx]])
        return np.random.Generator(np.random.Philox(ss))

    def _store(self, a32: np.ndarray) -> np.ndarray:
        if self.cfg.dtype == "bf16":
            return f32_to_bf16_bits(a32)
        return np.ascontiguousarray(a32, dtype=np.float32)

    def _normal(self, rng, shape, std) -> np.ndarray:
        a = rng.standard_normal(shape, dtype=np.float32)
        if std != 1.0:
            a *= np.float32(std)
        return self._store(a)

    # -------------------------------------------------------------- weights
    def router_w(self, layer: int) -> np.ndarray:
        """W_r of one layer, [E, d], storage dtype."""
        if layer not in self._router_cache:
            c = self.cfg
            self._router_cache[layer] = self._normal(self._rng(_ST_ROUTER, layer),
                                                     (c.n_experts, c.d_model), WEIGHT_STD)
        return self._router_cache[layer]

    def _ffn(self, rng):
        c = self.cfg
        wg = self._normal(rng, (c.d_ff, c.d_model), WEIGHT_STD)
        wu = self._normal(rng, (c.d_ff, c.d_model), WEIGHT_STD)
        wd = self._normal(rng, (c.d_model, c.d_ff), WEIGHT_STD)
        return wg, wu, wd

    def expert(self, layer: int, e: int):
        """(W_g [f,d], W_u [f,d], W_d [d,f]) of routed expert e, storage dtype."""
        return self._ffn(self._rng(_ST_EXPERT, layer, e))

    def shared(self, layer: int, s: int):
        return self._ffn(self._rng(_ST_SHARED, layer, s))

    def expert_int4(self, layer: int, e: int):
        """The same expert quantised to 4 bits: ((codes, scales) of W_g, of W_u, of W_d), see quantize_int4."""
        return tuple(quantize_int4(m) for m in self.expert(layer, e))

    def shared_int4(self, layer: int, s: int):
        return tuple(quantize_int4(m) for m in self.shared(layer, s))

    def experts_parallel(self, layer: int, ids, workers: int = 8):
        """[(W_g, W_u, W_d)] for several experts, generated on a thread pool."""
        with ThreadPoolExecutor(max_workers=workers) as ex:
            return list(ex.map(lambda e: self.expert(layer, e), ids))

    # -------------------------------------------------------------- routing
    def pref_set(self, layer: int, seq: int) -> np.ndarray:
        """Sorted preferred expert ids of (layer, sequence); may be empty."""
        c = self.cfg
        if c.pref_hi == 0:
            return np.zeros(0, dtype=np.int32)
        rng = self._rng(_ST_PREF, layer, seq)
        n = c.pref_lo + int(rng.integers(0, c.pref_hi - c.pref_lo + 1))
        perm = rng.permutation(c.n_experts)[:n]
        return np.sort(perm).astype(np.int32)

    def bias(self, layer: int, seq: int) -> np.ndarray:
        """Logit bias [E] fp32: beta on the preferred set, 0 elsewhere."""
        b = np.zeros(self.cfg.n_experts, dtype=np.float32)
        b[self.pref_set(layer, seq)] = np.float32(self.cfg.beta)
        return b

    # --------------------------------------------------------- hidden states
    def _margin_ok(self, x_store: np.ndarray, seq: int) -> np.ndarray:
        """Per-row bool: every layer's K-th/(K+1)-th logit gap >= delta (fp64)."""
        c = self.cfg
        ok = np.ones(x_store.shape[0], dtype=bool)
        if c.top_k >= c.n_experts:
            return ok
        x64 = widen(x_store).astype(np.float64)
        for l in range(c.n_layers):
            w64 = widen(self.router_w(l)).astype(np.float64)
            z = x64 @ w64.T + self.bias(l, seq).astype(np.float64)[None, :]
            zs = np.sort(z, axis=1)[:, ::-1]
            ok &= (zs[:, c.top_k - 1] - zs[:, c.top_k]) >= c.delta
        return ok

    def _filtered(self, stream: int, seq: int, n: int) -> np.ndarray:
        c = self.cfg
        x = self._normal(self._rng(stream, seq), (n, c.d_model), 1.0)
        for attempt in range(MAX_REDRAWS):
            bad = np.flatnonzero(~self._margin_ok(x, seq))
            if bad.size == 0:
                return x
            self.redraws += int(bad.size)
            fresh = self._normal(self._rng(_ST_RESAMPLE, stream, seq, attempt),
                                 (n, c.d_model), 1.0)
            x[bad] = fresh[bad]
        raise RuntimeError("top-K margin could not be met")

    def tokens(self, seq: int) -> np.ndarray:
        """Hidden states of the decode steps of one sequence, [T, d], storage dtype."""
        if seq not in self._tok_cache:
            self._tok_cache[seq] = self._filtered(_ST_X, seq, self.cfg.n_steps)
        return self._tok_cache[seq]

    def prefill_tokens(self, seq: int) -> np.ndarray:
        """Hidden states of the prompt of one sequence, [prefill_len, d]."""
        return self._filtered(_ST_XPREFILL, seq, self.cfg.prefill_len)

    # ---------------------------------------------------------- prefetch set
    def prefetch_list(self, layer: int, seq: int) -> np.ndarray:
        """Stand-in for the activation predictor's Top-C set (Section 3.2): the
        preferred set, padded to the capacity with the lowest-id other experts;
        listed so that preferred experts come last (most recently loaded)."""
        c = self.cfg
        cap = min(c.capacity, c.n_experts)
        pref = [int(e) for e in self.pref_set(layer, seq)]
        if len(pref) >= cap:
            return np.asarray(pref[:cap], dtype=np.int32)
        rest = [e for e in range(c.n_experts) if e not in pref][:cap - len(pref)]
        return np.asarray(rest + pref, dtype=np.int32)
