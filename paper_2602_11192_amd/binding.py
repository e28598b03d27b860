"""ctypes binding of libmoe_cache.so (include/moe_cache.h).

Argument marshalling only: every step of the MoE decode path runs inside the
library's HIP kernels.  There is no fallback: if the shared library has not been
built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_cache.so")

MOE_OK = 0
MOE_ERR_INVALID_ARG = -1
MOE_ERR_CAPACITY_LT_TOPK = -2
MOE_ERR_OUT_OF_MEMORY = -3
MOE_ERR_HIP = -4
MOE_ERR_STAGING_EXHAUSTED = -5
MOE_ERR_UNSUPPORTED = -6
MOE_ERR_TIMEOUT = -7

MOE_DTYPE_FP32, MOE_DTYPE_BF16 = 0, 1
MOE_POLICY_LRU, MOE_POLICY_GAMMA = 0, 1
MOE_LAYOUT_ROWMAJOR, MOE_LAYOUT_TILED, MOE_LAYOUT_TILED_INT4 = 0, 1, 2
MOE_FETCH_COPY_ENGINE, MOE_FETCH_IN_KERNEL = 0, 1

EXPORTS = ["moe_expert_bytes", "moe_expert_block_bytes", "moe_pack_expert", "moe_pack_expert_int4", "moe_cache_create", "moe_cache_destroy", "moe_cache_reset",
           "moe_cache_prefill_pins", "moe_layer_decode", "moe_layer_prefill", "moe_cache_stats", "moe_cache_read_trace",
           "moe_cache_resident", "moe_cache_set_profiling", "moe_cache_timing", "moe_probe_stream",
           "moe_cache_sim_loss", "moe_pooled_prefetch_set", "moe_layer_decode_resident_noalloc", "moe_last_error",
           "moe_version"]


class moe_cache_config_t(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "n_experts", "n_shared", "top_k", "d_model", "d_ff", "capacity", "dtype", "norm_topk",
        "policy", "max_batch", "staging_buffers", "device_id", "trace_capacity", "pool_layout", "fetch_mode")
    ] + [("gamma", C.c_double)]


class moe_weights_t(C.Structure):
    _fields_ = [("router_w", C.c_void_p), ("expert_pool", C.c_void_p), ("shared_w", C.c_void_p),
                ("expert_pool_layers", C.POINTER(C.c_void_p))]


class moe_cache_stats_t(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("lookups", "hits", "misses", "evictions", "pin_loads", "bytes_h2d",
                                          "stream_loads", "bytes_streamed")]


class moe_trace_rec_t(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("token", "expert", "hit", "evicted")]


class moe_timing_t(C.Structure):
    _fields_ = [("ffn_launches", C.c_uint64), ("ffn_gate_up_ms", C.c_double), ("ffn_down_ms", C.c_double),
                ("ffn_fused_launches", C.c_uint64), ("ffn_fused_ms", C.c_double),
                ("route_launches", C.c_uint64), ("route_ms", C.c_double),
                ("fetch_launches", C.c_uint64), ("fetch_bytes", C.c_uint64), ("fetch_ms", C.c_double),
                ("decode_single_launches", C.c_uint64), ("decode_single_ms", C.c_double),
                ("copies", C.c_uint64), ("copy_bytes", C.c_uint64), ("copy_ms", C.c_double),
                ("decode_tiles_launches", C.c_uint64)]


class moe_resident_layer_t(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_experts", "n_shared", "top_k", "d_model", "d_ff", "dtype", "norm_topk",
                                         "pool_layout")] + [("router_w", C.c_void_p), ("experts", C.c_void_p),
                                                            ("shared_w", C.c_void_p)]


class MoeError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("moe_cache error %d: %s" % (code, text))
        self.code = code


def _load():
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "libmoe_cache.so is not built (expected %s); run `python -c 'import __graft_entry__ as g; g.build()'`"
            % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.moe_expert_bytes.argtypes = [i32, i32, i32]
    lib.moe_expert_bytes.restype = C.c_uint64
    lib.moe_pack_expert.argtypes = [vp, vp, i32, i32]
    lib.moe_expert_block_bytes.argtypes = [i32, i32, i32, i32]
    lib.moe_expert_block_bytes.restype = C.c_uint64
    lib.moe_pack_expert_int4.argtypes = [vp, vp, vp, i32, i32]
    lib.moe_cache_create.argtypes = [C.POINTER(moe_cache_config_t), C.POINTER(moe_weights_t), C.POINTER(vp)]
    lib.moe_cache_destroy.argtypes = [vp]
    lib.moe_cache_reset.argtypes = [vp, i32, i32, vp]
    lib.moe_cache_prefill_pins.argtypes = [vp, i32, C.POINTER(i32), i32, vp]
    lib.moe_layer_decode.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp, vp]
    lib.moe_layer_prefill.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp, vp]
    lib.moe_cache_stats.argtypes = [vp, i32, C.POINTER(moe_cache_stats_t)]
    lib.moe_cache_read_trace.argtypes = [vp, i32, C.POINTER(moe_trace_rec_t), i64, C.POINTER(i64), C.POINTER(i64)]
    lib.moe_cache_resident.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32)]
    lib.moe_cache_set_profiling.argtypes = [vp, i32]
    lib.moe_cache_timing.argtypes = [vp, C.POINTER(moe_timing_t), i32]
    lib.moe_probe_stream.argtypes = [vp, vp, C.c_uint64, i32, i32, vp, C.POINTER(C.c_double)]
    lib.moe_cache_sim_loss.argtypes = [vp, i32, i32, i32, i32, i32, C.c_double, vp, vp, vp, vp]
    lib.moe_pooled_prefetch_set.argtypes = [vp, i32, i32, i32, C.POINTER(i32), C.POINTER(i32)]
    lib.moe_layer_decode_resident_noalloc.argtypes = [C.POINTER(moe_resident_layer_t), vp, vp, i32, vp, vp, vp, vp]
    lib.moe_last_error.restype = C.c_char_p
    lib.moe_version.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("moe_expert_bytes", "moe_expert_block_bytes", "moe_last_error", "moe_version"):
            getattr(lib, name).restype = C.c_int
    return lib


lib = _load()


def _check(rc: int):
    if rc != MOE_OK:
        raise MoeError(rc, lib.moe_last_error().decode())


def moe_last_error() -> str:
    return lib.moe_last_error().decode()


def moe_version() -> str:
    return lib.moe_version().decode()


def moe_expert_bytes(d_model: int, d_ff: int, dtype: int) -> int:
    return int(lib.moe_expert_bytes(d_model, d_ff, dtype))


def moe_pack_expert(src: np.ndarray, dst: np.ndarray, d_model: int, d_ff: int) -> None:
    """Row-major W_g|W_u|W_d (uint16 bf16 bits, 3*d*f elements) -> tiled layout, host to host."""
    assert src.dtype == np.uint16 and dst.dtype == np.uint16
    assert src.size == dst.size == 3 * d_model * d_ff and src.flags.c_contiguous and dst.flags.c_contiguous
    _check(lib.moe_pack_expert(src.ctypes.data, dst.ctypes.data, d_model, d_ff))


def moe_expert_block_bytes(d_model: int, d_ff: int, dtype: int, pool_layout: int) -> int:
    return int(lib.moe_expert_block_bytes(d_model, d_ff, dtype, pool_layout))


def moe_pack_expert_int4(codes: np.ndarray, scales: np.ndarray, dst: np.ndarray, d_model: int, d_ff: int) -> None:
    """codes uint8 [3*d*f] (W_g | W_u | W_d row-major, one code per byte), scales uint16 bf16 bits [3*d*f/32]
    -> one INT4 tiled block in dst (uint8, moe_expert_block_bytes long), host to host."""
    assert codes.dtype == np.uint8 and scales.dtype == np.uint16 and dst.dtype == np.uint8
    assert codes.size == 3 * d_model * d_ff and scales.size * 32 == codes.size
    assert dst.size == moe_expert_block_bytes(d_model, d_ff, MOE_DTYPE_BF16, MOE_LAYOUT_TILED_INT4)
    assert codes.flags.c_contiguous and scales.flags.c_contiguous and dst.flags.c_contiguous
    _check(lib.moe_pack_expert_int4(codes.ctypes.data, scales.ctypes.data, dst.ctypes.data, d_model, d_ff))


def moe_pooled_prefetch_set(scores: np.ndarray, capacity: int) -> list:
    """scores [n_seqs][E] float32 -> ids of the Top-capacity experts by summed score, best last."""
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    n_seqs, E = scores.shape
    ids = (C.c_int32 * min(capacity, E))()
    n = C.c_int32()
    _check(lib.moe_pooled_prefetch_set(scores.ctypes.data, n_seqs, E, capacity, ids, C.byref(n)))
    return list(ids[:n.value])


def moe_probe_stream(src, dst, nbytes: int, mode: int, iters: int = 10, stream=None) -> float:
    """Average kernel time (ms) of a plain read (mode 0) or copy (mode 1) of nbytes between device tensors."""
    ms = C.c_double()
    rc = lib.moe_probe_stream(_ptr(src), _ptr(dst), nbytes, mode, iters, _stream(stream), C.byref(ms))
    if rc != MOE_OK:
        raise MoeError(rc, "moe_probe_stream failed")
    return ms.value


def moe_cache_sim_loss(idx, n_experts: int, capacity: int, gamma: float, c1=None, out=None, flag=None, stream=None):
    """Per-trace sums of the soft cache-simulation loss and of the hard miss count for device tensor
    idx [n_traces][T][K] (int32).  Returns (out [n_traces][2] fp64, flag [n_traces] int32) device tensors."""
    import torch
    assert idx.dtype == torch.int32 and idx.dim() == 3 and idx.is_contiguous() and idx.is_cuda
    n, T, K = idx.shape
    if out is None:
        out = torch.empty((n, 2), dtype=torch.float64, device=idx.device)
    if flag is None:
        flag = torch.empty((n,), dtype=torch.int32, device=idx.device)
    if c1 is not None:
        assert c1.dtype == torch.float64 and tuple(c1.shape) == (n, n_experts) and c1.is_contiguous()
    assert out.dtype == torch.float64 and out.numel() == 2 * n and flag.dtype == torch.int32 and flag.numel() == n
    _check(lib.moe_cache_sim_loss(_ptr(idx), n, T, K, n_experts, capacity, float(gamma), _ptr(c1), _ptr(out),
                                  _ptr(flag), _stream(stream)))
    return out, flag


def moe_layer_decode_resident_noalloc(*, n_experts, top_k, d_model, d_ff, dtype, pool_layout, router_w, experts, x, y,
                                      shared_w=None, n_shared=0, norm_topk=1, logit_bias=None, topk_idx=None,
                                      topk_w=None, stream=None):
    """One MoE block over device-resident experts through the entry point that allocates nothing.
    router_w [E, d], experts (flat, E blocks), x, y [B, d]: device tensors."""
    layer = moe_resident_layer_t(n_experts, n_shared, top_k, d_model, d_ff, dtype, norm_topk, pool_layout,
                                 _ptr(router_w), _ptr(experts), _ptr(shared_w))
    _check(lib.moe_layer_decode_resident_noalloc(C.byref(layer), _ptr(x), _ptr(logit_bias), x.shape[0], _ptr(y),
                                                 _ptr(topk_idx), _ptr(topk_w), _stream(stream)))


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


class MoECache:
    """Owner of one moe_cache_t.  Tensors passed in are borrowed: they are kept
    referenced here so they outlive the native object."""

    def __init__(self, *, n_layers, n_experts, top_k, d_model, d_ff, capacity, dtype, router_w, expert_pool,
                 shared_w=None, n_shared=0, norm_topk=1, policy=MOE_POLICY_LRU, gamma=1.0, max_batch=1,
                 staging_buffers=0, device_id=-1, trace_capacity=0, pool_layout=MOE_LAYOUT_ROWMAJOR,
                 fetch_mode=MOE_FETCH_COPY_ENGINE):
        self.cfg = moe_cache_config_t(n_layers, n_experts, n_shared, top_k, d_model, d_ff, capacity, dtype,
                                      norm_topk, policy, max_batch, staging_buffers, device_id, trace_capacity,
                                      pool_layout, fetch_mode, float(gamma))
        self._keep = (router_w, expert_pool, shared_w)
        if isinstance(expert_pool, (list, tuple)):         # one pinned tensor per layer
            arr = (C.c_void_p * len(expert_pool))(*[p.data_ptr() for p in expert_pool])
            w = moe_weights_t(_ptr(router_w), None, _ptr(shared_w), arr)
        else:
            w = moe_weights_t(_ptr(router_w), _ptr(expert_pool), _ptr(shared_w), None)
        self._h = C.c_void_p()
        _check(lib.moe_cache_create(C.byref(self.cfg), C.byref(w), C.byref(self._h)))

    # same names as the C entry points
    def moe_cache_destroy(self):
        if self._h:
            h, self._h = self._h, C.c_void_p()
            _check(lib.moe_cache_destroy(h))

    close = moe_cache_destroy

    def __del__(self):
        try:
            self.moe_cache_destroy()
        except Exception:
            pass

    def moe_cache_reset(self, layer=-1, clear_stats=False, stream=None):
        _check(lib.moe_cache_reset(self._h, layer, int(clear_stats), _stream(stream)))

    def moe_cache_prefill_pins(self, layer, expert_ids, stream=None):
        ids = np.ascontiguousarray(expert_ids, dtype=np.int32)
        _check(lib.moe_cache_prefill_pins(self._h, layer, ids.ctypes.data_as(C.POINTER(C.c_int32)), len(ids),
                                          _stream(stream)))

    def moe_layer_decode(self, layer, x, y, logit_bias=None, topk_idx=None, topk_w=None, stream=None):
        """x, y: device tensors [B, d] of the cache's dtype; logit_bias [B, E] fp32 or None."""
        _check(lib.moe_layer_decode(self._h, layer, _ptr(x), _ptr(logit_bias), x.shape[0], _ptr(y),
                                    _ptr(topk_idx), _ptr(topk_w), _stream(stream)))

    def moe_layer_prefill(self, layer, x, y, logit_bias=None, topk_idx=None, topk_w=None, stream=None):
        """Prompt tokens x [n, d] through one layer in streaming mode (the cache is read, never changed)."""
        _check(lib.moe_layer_prefill(self._h, layer, _ptr(x), _ptr(logit_bias), x.shape[0], _ptr(y),
                                     _ptr(topk_idx), _ptr(topk_w), _stream(stream)))

    def moe_cache_stats(self, layer=-1) -> dict:
        st = moe_cache_stats_t()
        _check(lib.moe_cache_stats(self._h, layer, C.byref(st)))
        return {n: int(getattr(st, n)) for n, _ in st._fields_}

    def moe_cache_read_trace(self, layer):
        """-> (records [n,4] int32 as (token, expert, hit, evicted), total produced)"""
        cap = max(int(self.cfg.trace_capacity), 1)
        buf = (moe_trace_rec_t * cap)()
        n, tot = C.c_int64(), C.c_int64()
        _check(lib.moe_cache_read_trace(self._h, layer, buf, cap, C.byref(n), C.byref(tot)))
        arr = np.frombuffer(buf, dtype=np.int32).reshape(cap, 4)[: n.value].copy()
        return arr, int(tot.value)

    def moe_cache_resident(self, layer) -> list:
        out = (C.c_int32 * max(int(self.cfg.capacity), 1))()
        n = C.c_int32()
        _check(lib.moe_cache_resident(self._h, layer, out, C.byref(n)))
        return list(out[: n.value])

    def moe_cache_set_profiling(self, enabled: bool):
        _check(lib.moe_cache_set_profiling(self._h, int(enabled)))

    def moe_cache_timing(self, clear=False) -> dict:
        t = moe_timing_t()
        _check(lib.moe_cache_timing(self._h, C.byref(t), int(clear)))
        return {n: getattr(t, n) for n, _ in t._fields_}
