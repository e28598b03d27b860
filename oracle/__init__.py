"""CPU oracle for the MoE decode step (test infrastructure, never the product).

Thin ctypes binding over ``moe_oracle.c`` plus the per-layer orchestration in
the order of the paper's section 2: router logits -> softmax -> Top-K ->
gate weights (Eq. 1) -> cache lookups for the selected experts in a fixed
order -> SwiGLU experts (Eq. 3) -> weighted sum (Eq. 2).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It imports nothing from the HIP package.

Readings fixed here (the paper leaves them open):
  * Top-K is taken on the logits (monotone in p); equal values go to the lower id.
  * The K lookups of one token are made in ascending expert id; tokens of a
    batch in ascending row.
  * norm_topk=1 renormalises the K selected probabilities to sum to one;
    norm_topk=0 is Eq. 2 as printed.
  * Shared experts (not in the paper) are always resident, weight 1, not looked up.
  * Eviction drops the device copy; nothing is written back.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        l = C.CDLL(build())
        f32p, f64p, i32p, u64p = (C.POINTER(C.c_float), C.POINTER(C.c_double),
                                  C.POINTER(C.c_int32), C.POINTER(C.c_uint64))
        l.orc_set_threads.argtypes = [C.c_int]
        l.orc_get_threads.restype = C.c_int
        l.orc_router_logits.argtypes = [f32p, f32p, f32p, C.c_int, C.c_int, C.c_int, f64p]
        l.orc_softmax.argtypes = [f64p, C.c_int, C.c_int, f64p]
        l.orc_topk.argtypes = [f64p, C.c_int, C.c_int, C.c_int, i32p]
        l.orc_gate_weights.argtypes = [f64p, i32p, C.c_int, C.c_int, C.c_int, C.c_int, f64p]
        l.orc_expert_swiglu.argtypes = [f32p, f32p, f32p, f32p, C.c_int, C.c_int, f64p]
        l.orc_cache_new.argtypes = [C.c_int, C.c_int, C.c_int, C.c_double]
        l.orc_cache_new.restype = C.c_void_p
        l.orc_cache_free.argtypes = [C.c_void_p]
        l.orc_cache_reset.argtypes = [C.c_void_p, C.c_int]
        l.orc_cache_lookup.argtypes = [C.c_void_p, C.c_int, i32p]
        l.orc_cache_lookup.restype = C.c_int
        l.orc_cache_pin.argtypes = [C.c_void_p, i32p, C.c_int]
        l.orc_cache_end_token.argtypes = [C.c_void_p]
        l.orc_cache_resident.argtypes = [C.c_void_p, i32p]
        l.orc_cache_resident.restype = C.c_int
        l.orc_cache_stats.argtypes = [C.c_void_p, u64p, C.c_uint64]
        l.orc_cache_sim_loss.argtypes = [i32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, f64p, f64p, f64p]
        _lib = l
    return _lib


def set_threads(n: int) -> None:
    lib().orc_set_threads(int(n))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(C.POINTER(C.c_float))


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


# ----------------------------------------------------------------- Eq. 1
def router_logits(x, w_r, bias=None) -> np.ndarray:
    """logits[b,e] = sum_j W_r[e,j] x[b,j] (+ bias[b,e]); x [B,d], W_r [E,d] float32."""
    x, xp = _f32(x)
    w_r, wp = _f32(w_r)
    B, d = x.shape
    E = w_r.shape[0]
    assert w_r.shape[1] == d
    bp = None
    if bias is not None:
        bias, bp = _f32(bias)
        assert bias.shape == (B, E)
    out = np.empty((B, E), dtype=np.float64)
    lib().orc_router_logits(xp, wp, bp, B, E, d, out.ctypes.data_as(C.POINTER(C.c_double)))
    return out


def softmax(logits) -> np.ndarray:
    z, zp = _f64(logits)
    B, E = z.shape
    out = np.empty_like(z)
    lib().orc_softmax(zp, B, E, out.ctypes.data_as(C.POINTER(C.c_double)))
    return out


def topk(scores, K: int) -> np.ndarray:
    """Ids of the K largest entries per row, ascending id (ties -> lower id)."""
    z, zp = _f64(scores)
    B, E = z.shape
    assert 1 <= K <= E
    out = np.empty((B, K), dtype=np.int32)
    lib().orc_topk(zp, B, E, K, out.ctypes.data_as(C.POINTER(C.c_int32)))
    return out


def gate_weights(p, idx, norm_topk: int = 1) -> np.ndarray:
    p, pp = _f64(p)
    idx, ip = _i32(idx)
    B, E = p.shape
    K = idx.shape[1]
    out = np.empty((B, K), dtype=np.float64)
    lib().orc_gate_weights(pp, ip, B, E, K, int(norm_topk), out.ctypes.data_as(C.POINTER(C.c_double)))
    return out


# ----------------------------------------------------------------- Eq. 3
def expert_swiglu(x, w_g, w_u, w_d) -> np.ndarray:
    """E(x) = W_d (silu(W_g x) * (W_u x)) for one token x [d]; float64 result [d]."""
    x, xp = _f32(x)
    w_g, gp = _f32(w_g)
    w_u, up = _f32(w_u)
    w_d, dp = _f32(w_d)
    f, d = w_g.shape
    assert x.shape == (d,) and w_u.shape == (f, d) and w_d.shape == (d, f)
    out = np.empty(d, dtype=np.float64)
    lib().orc_expert_swiglu(xp, gp, up, dp, d, f, out.ctypes.data_as(C.POINTER(C.c_double)))
    return out


# ----------------------------------------------------------------- cache
POLICY_LRU = 0
POLICY_GAMMA = 1


class ExpertCache:
    """Per-layer expert cache with C slots (LRU, or the gamma-discounted
    count policy of Definition C.1; gamma=1 is LFU)."""

    def __init__(self, n_experts: int, capacity: int, policy: int = POLICY_LRU, gamma: float = 1.0):
        assert capacity >= 1 and n_experts >= 1
        self.E, self.C, self.policy, self.gamma = n_experts, capacity, policy, gamma
        self._h = C.c_void_p(lib().orc_cache_new(n_experts, capacity, policy, gamma))
        self.stream_loads = 0     # experts streamed past the cache by prompt processing

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.orc_cache_free(self._h)
            self._h = None

    def reset(self, clear_stats: bool = False):
        lib().orc_cache_reset(self._h, int(clear_stats))

    def lookup(self, e: int):
        """-> (hit: bool, evicted expert or -1)"""
        assert 0 <= e < self.E
        ev = C.c_int32(-1)
        hit = lib().orc_cache_lookup(self._h, int(e), C.byref(ev))
        return bool(hit), int(ev.value)

    def end_token(self):
        lib().orc_cache_end_token(self._h)

    def pin(self, ids):
        ids, ip = _i32(ids)
        assert len(set(ids.tolist())) == len(ids) <= self.C
        lib().orc_cache_pin(self._h, ip, len(ids))

    def resident(self):
        out = np.empty(self.E, dtype=np.int32)
        n = lib().orc_cache_resident(self._h, out.ctypes.data_as(C.POINTER(C.c_int32)))
        return out[:n].tolist()

    def stats(self, expert_bytes: int = 0) -> dict:
        out = np.zeros(6, dtype=np.uint64)
        lib().orc_cache_stats(self._h, out.ctypes.data_as(C.POINTER(C.c_uint64)), int(expert_bytes))
        d = dict(zip(("lookups", "hits", "misses", "evictions", "pin_loads", "bytes_h2d"), (int(v) for v in out)))
        d["stream_loads"] = self.stream_loads
        d["bytes_streamed"] = self.stream_loads * int(expert_bytes)
        return d


# ----------------------------------------------------------- whole layer
@dataclass
class LayerWeights:
    """float32 views of one layer's parameters (bf16 data widened exactly)."""
    router_w: np.ndarray                       # [E, d]
    expert: callable                           # e -> (W_g [f,d], W_u [f,d], W_d [d,f])
    shared: list = field(default_factory=list)  # [(W_g, W_u, W_d)] always-on experts


@dataclass
class DecodeResult:
    y: np.ndarray        # [B, d] float64
    idx: np.ndarray      # [B, K] int32, ascending id
    w: np.ndarray        # [B, K] float64 gate weights
    trace: list          # [(token, expert, hit, evicted)]
    logits: np.ndarray   # [B, E] float64
    p: np.ndarray        # [B, E] float64


def route(x, w_r, bias, K: int, norm_topk: int = 1):
    """Eq. 1 plus the gate weights of Eq. 2 -> (logits, p, idx, w)."""
    logits = router_logits(x, w_r, bias)
    p = softmax(logits)
    idx = topk(logits, K)
    w = gate_weights(p, idx, norm_topk)
    return logits, p, idx, w


def moe_layer_decode(weights: LayerWeights, cache: ExpertCache, x, bias, K: int,
                     norm_topk: int = 1, compute_y: bool = True) -> DecodeResult:
    """One MoE layer on a batch of tokens x [B,d] (float32 values)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, d = x.shape
    logits, p, idx, w = route(x, weights.router_w, bias, K, norm_topk)
    trace = []
    for b in range(B):
        for k in range(K):
            e = int(idx[b, k])
            hit, ev = cache.lookup(e)
            trace.append((b, e, int(hit), ev))
        cache.end_token()
    y = np.zeros((B, d), dtype=np.float64)
    if compute_y:
        for b in range(B):
            for k in range(K):
                wg, wu, wd = weights.expert(int(idx[b, k]))
                y[b] += w[b, k] * expert_swiglu(x[b], wg, wu, wd)
            for (wg, wu, wd) in weights.shared:
                y[b] += expert_swiglu(x[b], wg, wu, wd)
    return DecodeResult(y, idx, w, trace, logits, p)


def moe_layer_prefill(weights: LayerWeights, cache: ExpertCache, x, bias, K: int, norm_topk: int = 1,
                      rows=None) -> DecodeResult:
    """Prompt tokens through one layer in streaming mode: Eq. 1-3 as in decode, but the cache is only read.
    Selected experts that are not resident are counted as stream loads (once per call) and nothing is inserted.
    rows: token rows whose output is evaluated (default all)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, d = x.shape
    logits, p, idx, w = route(x, weights.router_w, bias, K, norm_topk)
    resident = set(cache.resident())
    cache.stream_loads += len(set(int(e) for e in idx.reshape(-1)) - resident)
    y = np.zeros((B, d), dtype=np.float64)
    for b in (range(B) if rows is None else rows):
        for k in range(K):
            wg, wu, wd = weights.expert(int(idx[b, k]))
            y[b] += w[b, k] * expert_swiglu(x[b], wg, wu, wd)
        for (wg, wu, wd) in weights.shared:
            y[b] += expert_swiglu(x[b], wg, wu, wd)
    return DecodeResult(y, idx, w, [], logits, p)


def moe_layer_dense(weights: LayerWeights, n_experts: int, x, bias, K: int, norm_topk: int = 1):
    """Brute force: every expert evaluated, then masked by the request vector r."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, d = x.shape
    logits, p, idx, w = route(x, weights.router_w, bias, K, norm_topk)
    r = np.zeros((B, n_experts))
    gate = np.zeros((B, n_experts))
    for b in range(B):
        r[b, idx[b]] = 1.0
        gate[b, idx[b]] = w[b]
    y = np.zeros((B, d), dtype=np.float64)
    for b in range(B):
        for e in range(n_experts):
            wg, wu, wd = weights.expert(e)
            out = expert_swiglu(x[b], wg, wu, wd)
            if r[b, e] == 1.0:
                y[b] += gate[b, e] * out
        for (wg, wu, wd) in weights.shared:
            y[b] += expert_swiglu(x[b], wg, wu, wd)
    return y


def cache_sim_loss(idx, n_experts: int, capacity: int, gamma: float, c1=None):
    """Forward value of the cache-simulation loss of section 3.1.1 / appendix C.1 over a routing trace.
    idx [L][T][K] selected experts.  Returns (L_cs, L_cs_hard): the soft loss with the soft cache of
    Proposition C.2 and the hard miss count of Definition C.1 (Top-C ties to the lower id), both divided by
    L*T.  c1 [L][E] is the first cache state (L1 norm C); None = uniform C/E."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    L, T, K = idx.shape
    soft_sum = hard_sum = 0.0
    for l in range(L):
        row = np.ascontiguousarray(idx[l])
        c1p = None
        if c1 is not None:
            c1l, c1p = _f64(np.asarray(c1)[l])
        so, ho = C.c_double(), C.c_double()
        lib().orc_cache_sim_loss(row.ctypes.data_as(C.POINTER(C.c_int32)), T, K, int(n_experts), int(capacity),
                                 float(gamma), c1p, C.byref(so), C.byref(ho))
        soft_sum += so.value
        hard_sum += ho.value
    return soft_sum / (L * T), hard_sum / (L * T)


def pooled_prefetch_set(scores, capacity: int) -> list:
    """Prefetch set of a cache shared by several sequences: section 3.2's Top-C of the predictor's scores, applied
    to the scores summed over the sequences (fp64, in row order).  Returned lowest total first, so that pinning in
    list order leaves the best-scored expert most recently used; equal totals rank the lower id higher."""
    scores = np.asarray(scores, dtype=np.float32)
    total = np.zeros(scores.shape[1], dtype=np.float64)
    for row in scores:
        total = total + row.astype(np.float64)
    ranked = sorted(range(scores.shape[1]), key=lambda e: (-total[e], e))
    return ranked[:min(capacity, scores.shape[1])][::-1]


def dequant_int4(codes, scale_bits) -> np.ndarray:
    """4-bit group-quantised matrix -> its weights (section 3.2 keeps experts in INT4; the format here is the
    generic symmetric one: 32 consecutive elements of a row share one bf16 scale, weight = scale * (code - 8)).
    codes [rows][k] integers 0..15, scale_bits [rows][k/32] bf16 bit patterns.  Exact in float32 (8 x 4 bits)."""
    codes = np.asarray(codes)
    scale = (np.asarray(scale_bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    rows, k = codes.shape
    assert scale.shape == (rows, k // 32) and k % 32 == 0
    grouped = codes.astype(np.float64).reshape(rows, k // 32, 32)            # [row][group][element of the group]
    out = scale.astype(np.float64)[:, :, None] * (grouped - 8.0)
    return out.reshape(rows, k).astype(np.float32)


def expert_bytes_int4(d: int, f: int) -> int:
    """Bytes of one 4-bit expert: 3 d f codes of 4 bits plus one 16-bit scale per 32 codes (4.5 bits per weight)."""
    return 3 * d * f // 2 + (3 * d * f // 32) * 2


def expert_bytes(d: int, f: int, elem_bytes: int) -> int:
    """Bytes of one expert's three projection matrices (Eq. 3 shapes)."""
    return 3 * d * f * elem_bytes
