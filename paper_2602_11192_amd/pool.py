"""Places a synthetic workload's parameters where the library expects them:
router weights and shared experts in HBM, routed experts in a pinned host pool
(optionally permuted into the tiled layout).  Data movement only."""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

from . import binding as B


def torch_dtype(cfg):
    return torch.float32 if cfg.dtype == "fp32" else torch.bfloat16


def moe_dtype(cfg):
    return B.MOE_DTYPE_FP32 if cfg.dtype == "fp32" else B.MOE_DTYPE_BF16


def to_device(arr: np.ndarray, device="cuda:0") -> torch.Tensor:
    """Stored numpy array (float32, or uint16 bf16 bit patterns) -> device tensor of the same values."""
    if arr.dtype == np.uint16:
        return torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr)).to(device)


def to_numpy(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> float32 numpy (bf16 widened exactly)."""
    return t.detach().float().cpu().numpy()


def _block(mats, cfg, tiled: bool) -> np.ndarray:
    flat = np.concatenate([m.reshape(-1) for m in mats])
    if not tiled:
        return flat
    out = np.empty_like(flat)
    B.moe_pack_expert(flat, out, cfg.d_model, cfg.d_ff)
    return out


def int4_block_bytes(cfg) -> int:
    return B.moe_expert_block_bytes(cfg.d_model, cfg.d_ff, B.MOE_DTYPE_BF16, B.MOE_LAYOUT_TILED_INT4)


def _block_int4(quantised, cfg) -> np.ndarray:
    """((codes, scales) x 3) of one expert -> one INT4 tiled block (uint8)."""
    codes = np.concatenate([q.reshape(-1) for q, _ in quantised])
    scales = np.concatenate([s.reshape(-1) for _, s in quantised])
    out = np.empty(int4_block_bytes(cfg), dtype=np.uint8)
    B.moe_pack_expert_int4(codes, scales, out, cfg.d_model, cfg.d_ff)
    return out


def build_pool(wl, tiled: bool, workers: int = 8, int4: bool = False, per_layer: bool = False):
    """Pinned host tensor [L][E] expert blocks (flat), storage dtype (uint8 for 4-bit experts); per_layer: a list
    of L such tensors of [E] blocks each, for stacks too large to pin in one allocation."""
    if per_layer:
        return [build_pool(_LayerView(wl, l), tiled, workers, int4) for l in range(wl.cfg.n_layers)]
    cfg = wl.cfg
    n = cfg.n_layers * cfg.n_experts
    if int4:
        per = int4_block_bytes(cfg)
        pool = torch.empty(n * per, dtype=torch.uint8, pin_memory=torch.cuda.is_available())
        view = pool.numpy()
    else:
        per = 3 * cfg.d_model * cfg.d_ff
        tdt = torch.float32 if cfg.dtype == "fp32" else torch.int16
        pool = torch.empty(n * per, dtype=tdt, pin_memory=torch.cuda.is_available())
        view = pool.numpy()
        if cfg.dtype != "fp32":
            view = view.view(np.uint16)

    def fill(i):
        l, e = divmod(i, cfg.n_experts)
        view[i * per:(i + 1) * per] = (_block_int4(wl.expert_int4(l, e), cfg) if int4
                                       else _block(wl.expert(l, e), cfg, tiled))

    with ThreadPoolExecutor(max_workers=workers) as ex:
        list(ex.map(fill, range(n)))
    return pool


class _LayerView:
    """One layer of a workload, seen as a single-layer workload (for building per-layer pools)."""

    def __init__(self, wl, layer):
        self._wl, self._layer = wl, layer
        self.cfg = wl.cfg.with_(n_layers=1)

    def expert(self, l, e):
        return self._wl.expert(self._layer, e)

    def expert_int4(self, l, e):
        return self._wl.expert_int4(self._layer, e)


def build_router(wl, device="cuda:0") -> torch.Tensor:
    cfg = wl.cfg
    return to_device(np.stack([wl.router_w(l) for l in range(cfg.n_layers)]), device)


def build_shared(wl, tiled: bool, device="cuda:0", int4: bool = False):
    cfg = wl.cfg
    if cfg.n_shared == 0:
        return None
    if int4:
        blocks = [_block_int4(wl.shared_int4(l, s), cfg) for l in range(cfg.n_layers) for s in range(cfg.n_shared)]
        return torch.from_numpy(np.concatenate(blocks)).to(device)
    blocks = [_block(wl.shared(l, s), cfg, tiled) for l in range(cfg.n_layers) for s in range(cfg.n_shared)]
    return to_device(np.concatenate(blocks), device)


def make_cache(wl, *, tiled=None, capacity=None, max_batch=1, staging_buffers=0, trace_capacity=0,
               policy=B.MOE_POLICY_LRU, gamma=1.0, norm_topk=None, device="cuda:0", pool=None,
               fetch_mode=B.MOE_FETCH_COPY_ENGINE, int4=False):
    """Build pool + router (+ shared) for `wl` and create the native cache (int4: 4-bit experts)."""
    cfg = wl.cfg
    if tiled is None:
        tiled = cfg.dtype == "bf16"
    pool = build_pool(wl, tiled, int4=int4) if pool is None else pool
    router = build_router(wl, device)
    shared = build_shared(wl, tiled, device, int4=int4)
    cache = B.MoECache(
        n_layers=cfg.n_layers, n_experts=cfg.n_experts, n_shared=cfg.n_shared, top_k=cfg.top_k,
        d_model=cfg.d_model, d_ff=cfg.d_ff, capacity=cfg.capacity if capacity is None else capacity,
        dtype=moe_dtype(cfg), norm_topk=cfg.norm_topk if norm_topk is None else norm_topk, policy=policy,
        gamma=gamma, max_batch=max_batch, staging_buffers=staging_buffers,
        device_id=torch.device(device).index or 0, trace_capacity=trace_capacity,
        pool_layout=B.MOE_LAYOUT_TILED_INT4 if int4 else B.MOE_LAYOUT_TILED if tiled else B.MOE_LAYOUT_ROWMAJOR,
        fetch_mode=fetch_mode,
        router_w=router, expert_pool=pool, shared_w=shared)
    return cache
