#!/usr/bin/env python3
"""Benchmark of the MoE decode hot path on one MI355X.

A step is one pass of the whole hot path over the OLMoE-like workload: 16
sequences, served one after the other at batch 1 (the paper's main setting);
per sequence the layer's cache is emptied, the prefetch set is preloaded, then
128 tokens are decoded through router -> gating -> cache lookup (+ host->device
fetch of missed experts) -> SwiGLU experts -> combine.  All inputs (hidden
states, biases, router, pinned expert pool) are resident before the timed
region.  The same schedules then run on a cut of the Mixtral-like stack (the
other configuration the bandwidth target names) and are reported under
"mixtral_like".  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published
PCIE_PEAK_GBPS = 64.0       # PCIe 5 x16, one direction, nominal


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="olmoe_like")
    ap.add_argument("--layers", type=int, default=None, help="cut the layer stack of the workload to this many layers")
    ap.add_argument("--seqs", type=int, default=None, help="use only this many sequences")
    ap.add_argument("--decode-steps", type=int, default=None, help="decode steps per sequence")
    ap.add_argument("--cpu-baseline-tokens", type=int, default=256)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fetch-mode", choices=["copy_engine", "in_kernel"], default="in_kernel",
                    help="how missed experts reach the device (see MOE_FETCH_* in include/moe_cache.h)")
    ap.add_argument("--batch-sweep", metavar="FILE", default=None,
                    help="also time the resident path at batch 1..1024 and write the table to FILE (JSON)")
    ap.add_argument("--int4", choices=["auto", "on", "off"], default="auto",
                    help="also run the workload with 4-bit group-quantised experts and report it under "
                         "'int4_experts' (auto: only when the whole pool has at most 5e8 weights)")
    ap.add_argument("--sweep-sizes", default=None, help="comma-separated batch sizes for --batch-sweep")
    ap.add_argument("--extras", metavar="FILE", default=None,
                    help="also measure the widened rows (eviction policies, shared-cache batched decode with pooled "
                         "prefetch, prompt streaming, cache-simulation loss) and write them to FILE (JSON)")
    ap.add_argument("--second-layers", type=int, default=12,
                    help="layers of the Mixtral-like section that follows the default workload (0 = leave it out)")
    ap.add_argument("--no-sweep", action="store_true", help="leave out the resident-path batch sweep")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run one plain 256 MiB copy kernel (reference dispatch for profiler memory counters)")
    return ap.parse_args()


class Runner:
    """Pre-marshalled arguments for the per-token calls (keeps the Python loop thin)."""

    def __init__(self, wl, cache, torch, P):
        cfg = wl.cfg
        self.cfg, self.cache, self.torch = cfg, cache, torch
        self.lib = P.B.lib
        self.h = cache._h
        self.x = [P.to_device(wl.tokens(s)) for s in range(cfg.n_seqs)]
        self.bias = [[torch.from_numpy(wl.bias(l, s)[None, :].copy()).cuda() for s in range(cfg.n_seqs)]
                     for l in range(cfg.n_layers)]
        self.y = torch.empty((cfg.n_seqs, cfg.d_model), dtype=P.torch_dtype(cfg), device="cuda:0")
        self.pins = [[wl.prefetch_list(l, s) for s in range(cfg.n_seqs)] for l in range(cfg.n_layers)]
        row = cfg.d_model * cfg.elem_bytes
        self.xp = [[C.c_void_p(x.data_ptr() + t * row) for t in range(cfg.n_steps)] for x in self.x]
        self.bp = [[C.c_void_p(b.data_ptr()) for b in bl] for bl in self.bias]
        self.yp = C.c_void_p(self.y.data_ptr())
        self.sp = C.c_void_p(torch.cuda.current_stream().cuda_stream)

    def _chk(self, rc):
        if rc != 0:
            raise RuntimeError("moe_layer_decode failed: %d %s" % (rc, self.lib.moe_last_error().decode()))

    def pass_sequence_serial(self, pins=True):
        """One step: every sequence, batch 1, reset + prefetch per sequence.  Returns tokens decoded."""
        cfg, dec, h, yp, sp = self.cfg, self.lib.moe_layer_decode, self.h, self.yp, self.sp
        for s in range(cfg.n_seqs):
            self.cache.moe_cache_reset(-1)
            if pins:
                for l in range(cfg.n_layers):
                    self.cache.moe_cache_prefill_pins(l, self.pins[l][s])
            xp = self.xp[s]
            for t in range(cfg.n_steps):
                for l in range(cfg.n_layers):
                    rc = dec(h, l, xp[t], self.bp[l][s], 1, yp, None, None, sp)
                    if rc:
                        self._chk(rc)
        return cfg.n_seqs * cfg.n_steps

    def pass_resident(self):
        """Same tokens, no resets: for a cache that holds every expert."""
        cfg, dec, h, yp, sp = self.cfg, self.lib.moe_layer_decode, self.h, self.yp, self.sp
        for s in range(cfg.n_seqs):
            xp = self.xp[s]
            for t in range(cfg.n_steps):
                for l in range(cfg.n_layers):
                    rc = dec(h, l, xp[t], self.bp[l][s], 1, yp, None, None, sp)
                    if rc:
                        self._chk(rc)
        return cfg.n_seqs * cfg.n_steps


def miss_path(torch, P, wl, pool, fetch_mode, n_tokens=48):
    """Every lookup misses: capacity = K and a logit bias that walks through disjoint sets of K experts, so each
    token evicts the whole cache.  Measures the pinned-pool -> device rate of the fetch path on its own."""
    import numpy as np
    cfg = wl.cfg
    E, K = cfg.n_experts, cfg.top_k
    n_sets = E // K
    if n_sets < 2:
        return None
    cache = P.make_cache(wl, tiled=True, pool=pool, capacity=K, fetch_mode=fetch_mode)
    bias = np.zeros((n_sets, E), dtype=np.float32)
    for i in range(n_sets):
        bias[i, i * K:(i + 1) * K] = 1.0e4
    bias_d = torch.from_numpy(bias).cuda()
    x = P.to_device(wl.tokens(0)[:min(n_tokens, cfg.n_steps)])
    y = torch.empty((1, cfg.d_model), dtype=P.torch_dtype(cfg), device="cuda:0")

    def one_pass():
        for t in range(x.shape[0]):
            cache.moe_layer_decode(0, x[t:t + 1], y, bias_d[t % n_sets:t % n_sets + 1])
        return x.shape[0]

    one_pass()
    cache.moe_cache_reset(-1, clear_stats=True)
    n, dt = timed(torch, one_pass, 1)
    st = cache.moe_cache_stats()
    cache.close()
    return {"schedule": "capacity = top-k = %d, consecutive tokens forced onto disjoint expert sets: every lookup misses" % K,
            "tokens": n, "lookups": st["lookups"], "misses": st["misses"], "bytes_h2d": st["bytes_h2d"],
            "ms_per_token": dt / n * 1e3, "pcie_GBps": st["bytes_h2d"] / dt / 1e9, "peak_GBps": PCIE_PEAK_GBPS}


def timed(torch, fn, steps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n = 0
    for _ in range(steps):
        n += fn()
    torch.cuda.synchronize()
    return n, time.perf_counter() - t0


def batch_sweep(torch, P, wl, pool, sizes=(1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024), reps=20):
    """Resident path (capacity = E) at growing batch: tokens/s, kernel times, distinct experts per call (U, from
    the routing the library returns), whole-call fraction of the HBM roofline, matrix-core rate of the FFN."""
    import numpy as np
    cfg = wl.cfg
    E, K, d = cfg.n_experts, cfg.top_k, cfg.d_model
    # row i of a batch is step i // S of sequence i % S: a batch takes one token of every sequence, then wraps
    toks = np.stack([wl.tokens(s) for s in range(cfg.n_seqs)], axis=1).reshape(-1, cfg.d_model)
    bias = np.tile(np.stack([wl.bias(0, s) for s in range(cfg.n_seqs)]), (cfg.n_steps, 1))
    rows = []
    for bsz in sizes:
        if bsz > toks.shape[0]:
            break
        cache = P.make_cache(wl, tiled=True, pool=pool, capacity=E, max_batch=bsz,
                             fetch_mode=P.B.MOE_FETCH_IN_KERNEL)
        cache.moe_cache_prefill_pins(0, list(range(E)))
        x = P.to_device(toks[:bsz])
        b = torch.from_numpy(bias[:bsz].copy()).cuda()
        y = torch.empty((bsz, d), dtype=P.torch_dtype(cfg), device="cuda:0")
        idx = torch.empty((bsz, K), dtype=torch.int32, device="cuda:0")
        for _ in range(3):
            cache.moe_layer_decode(0, x, y, b, idx)
        torch.cuda.synchronize()
        u = len(np.unique(idx.cpu().numpy()))
        t0 = time.perf_counter()
        for _ in range(reps):
            cache.moe_layer_decode(0, x, y, b)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / reps
        cache.moe_cache_set_profiling(True)
        cache.moe_cache_timing(clear=True)
        for _ in range(reps):
            cache.moe_layer_decode(0, x, y, b)
        tm = cache.moe_cache_timing(clear=True)
        n = max(1, tm["ffn_launches"] + tm["ffn_fused_launches"] + tm["decode_single_launches"])
        ffn_us = (tm["ffn_gate_up_ms"] + tm["ffn_down_ms"] + tm["ffn_fused_ms"] + tm["decode_single_ms"]) / n * 1e3
        flops = 6.0 * d * cfg.d_ff * bsz * (K + cfg.n_shared)
        call_bytes = (u + cfg.n_shared) * cfg.expert_bytes + E * d * cfg.elem_bytes + 2 * bsz * d * cfg.elem_bytes + bsz * E * 4
        rows.append({"batch": bsz, "call_us": dt * 1e6, "tokens_per_s": bsz / dt, "distinct_experts": u,
                     "frac_of_hbm_peak_whole_call": call_bytes / dt / 1e9 / HBM_PEAK_GBPS,
                     "route_cache_us": tm["route_ms"] / max(1, tm["route_launches"]) * 1e3, "ffn_us": ffn_us,
                     "ffn_us_over_weight_stream_at_6.1TBps": ffn_us / ((u + cfg.n_shared) * cfg.expert_bytes / 6.1e6),
                     "ffn_TFLOPs": flops / ffn_us / 1e6,
                     "ffn_kernel": ("router + experts in one launch" if tm["decode_single_launches"] else
                                    "single-launch decode FFN" if tm["ffn_fused_launches"] else "grouped GEMM, two kernels")})
        cache.close()
    return {"workload": cfg.name, "layer": 0, "capacity": E, "rows": rows}


def extras(torch, P, wl, pool, a):
    """Measurements of the rows beyond the batch-1 LRU decode step, on the same workload (layer stack as given)."""
    import numpy as np
    B = P.B
    cfg = wl.cfg
    K, E, S = cfg.top_k, cfg.n_experts, cfg.n_seqs
    out = {"workload": cfg.name}

    # eviction policies on the sequence-serial schedule (Definition C.1: gamma -> 0 is LRU, gamma = 1 is LFU)
    pol = []
    for name, policy, gamma in (("LRU", B.MOE_POLICY_LRU, 0.0), ("gamma=1 (LFU)", B.MOE_POLICY_GAMMA, 1.0),
                                ("gamma=0.9", B.MOE_POLICY_GAMMA, 0.9)):
        cache = P.make_cache(wl, tiled=True, pool=pool, fetch_mode=B.MOE_FETCH_IN_KERNEL, policy=policy, gamma=gamma)
        run = Runner(wl, cache, torch, P)
        run.pass_sequence_serial()
        cache.moe_cache_reset(-1, clear_stats=True)
        n, dt = timed(torch, run.pass_sequence_serial, 2)
        st = cache.moe_cache_stats()
        pol.append({"policy": name, "tokens_per_s": n / dt, "hit_rate": st["hits"] / max(1, st["lookups"]),
                    "misses_per_token": st["misses"] / n})
        cache.close()
    out["eviction_policies"] = pol

    # all sequences decode together on one cache per layer, preloaded with the pooled prefetch set
    rows = []
    xs = [P.to_device(np.stack([wl.tokens(s)[t] for s in range(S)])) for t in range(cfg.n_steps)]
    bias = [torch.from_numpy(np.stack([wl.bias(l, s) for s in range(S)])).cuda() for l in range(cfg.n_layers)]
    y = torch.empty((S, cfg.d_model), dtype=P.torch_dtype(cfg), device="cuda:0")
    for cap in sorted({cfg.capacity, min(E, 2 * cfg.capacity), E}):
        cache = P.make_cache(wl, tiled=True, pool=pool, capacity=cap, max_batch=S, staging_buffers=min(E - cap, S * K),
                             fetch_mode=B.MOE_FETCH_IN_KERNEL)
        sets = [B.moe_pooled_prefetch_set(np.stack([wl.bias(l, s) for s in range(S)]), cap)
                for l in range(cfg.n_layers)]

        def one_pass():
            cache.moe_cache_reset(-1)
            for l in range(cfg.n_layers):
                cache.moe_cache_prefill_pins(l, sets[l])
            for t in range(cfg.n_steps):
                for l in range(cfg.n_layers):
                    cache.moe_layer_decode(l, xs[t], y, bias[l])
            return S * cfg.n_steps

        one_pass()
        cache.moe_cache_reset(-1, clear_stats=True)
        n, dt = timed(torch, one_pass, 2)
        st = cache.moe_cache_stats()
        rows.append({"capacity": cap, "batch": S, "tokens_per_s": n / dt,
                     "hit_rate": st["hits"] / max(1, st["lookups"]), "misses_per_call": st["misses"] / (2 * cfg.n_steps * cfg.n_layers)})
        cache.close()
    out["shared_cache_batched_decode"] = rows

    # prompt streaming: a prompt through every layer with the cache read-only (missing experts read from the pool)
    n_p = min(512, S * cfg.n_steps)
    toks = np.concatenate([wl.tokens(s) for s in range(S)])[:n_p]
    xp = P.to_device(toks)
    yp = torch.empty((n_p, cfg.d_model), dtype=P.torch_dtype(cfg), device="cuda:0")
    cache = P.make_cache(wl, tiled=True, pool=pool, max_batch=n_p)
    for l in range(cfg.n_layers):
        cache.moe_cache_prefill_pins(l, wl.prefetch_list(l, 0))

    def prompt_pass():
        for l in range(cfg.n_layers):
            cache.moe_layer_prefill(l, xp, yp)
        return n_p

    prompt_pass()
    cache.moe_cache_reset(-1, clear_stats=True)
    for l in range(cfg.n_layers):
        cache.moe_cache_prefill_pins(l, wl.prefetch_list(l, 0))
    n, dt = timed(torch, prompt_pass, 3)
    st = cache.moe_cache_stats()
    out["prompt_streaming"] = {"prompt_tokens": n_p, "tokens_per_s": n / dt, "ms_per_layer": dt / 3 / cfg.n_layers * 1e3,
                               "experts_streamed_per_layer": st["stream_loads"] / (3 * cfg.n_layers),
                               "pcie_GBps_lower_bound": st["bytes_streamed"] / dt / 1e9,
                               "ffn_TFLOPs_incl_routing": 6.0 * cfg.d_model * cfg.d_ff * n_p * (K + cfg.n_shared) * 3 * cfg.n_layers / dt / 1e12}
    cache.close()

    # cache-simulation loss of the routing traces of the workload (one trace per sequence and layer)
    idx_all = torch.empty((S, cfg.n_steps, K), dtype=torch.int32, device="cuda:0")
    cache = P.make_cache(wl, tiled=True, pool=pool, capacity=E, max_batch=S)
    cache.moe_cache_prefill_pins(0, list(range(E)))
    idx_t = torch.empty((S, K), dtype=torch.int32, device="cuda:0")
    for t in range(cfg.n_steps):
        cache.moe_layer_decode(0, xs[t], y, bias[0], idx_t)
        idx_all[:, t, :] = idx_t
    cache.close()
    reps = 64
    big = idx_all.repeat(reps, 1, 1).contiguous()                  # reps * S traces
    outb, flag = B.moe_cache_sim_loss(big, E, cfg.capacity, 0.9)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        B.moe_cache_sim_loss(big, E, cfg.capacity, 0.9, out=outb, flag=flag)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 10
    res = outb[:S].cpu().numpy()
    out["cache_simulation_loss"] = {"traces": reps * S, "tokens_per_trace": cfg.n_steps, "gamma": 0.9,
                                    "capacity": cfg.capacity, "ms_per_launch": ms,
                                    "token_steps_per_s": reps * S * cfg.n_steps / (ms * 1e-3),
                                    "L_cs": float(res[:, 0].sum() / (S * cfg.n_steps)),
                                    "L_cs_hard": float(res[:, 1].sum() / (S * cfg.n_steps)),
                                    "note": "layer 0 routing of the workload; uniform first state"}
    return out


def int4_section(torch, P, wl, a):
    """The same schedule on 4-bit experts (a separate, lower-precision configuration: never the headline value)."""
    cfg = wl.cfg
    K, d = cfg.top_k, cfg.d_model
    qb = P.int4_block_bytes(cfg)
    pool = P.build_pool(wl, tiled=True, int4=True)
    cache = P.make_cache(wl, int4=True, pool=pool, fetch_mode=P.B.MOE_FETCH_IN_KERNEL)
    run = Runner(wl, cache, torch, P)
    run.pass_sequence_serial()
    cache.moe_cache_reset(-1, clear_stats=True)
    n_tok, dt = timed(torch, run.pass_sequence_serial, a.steps)
    st = cache.moe_cache_stats()
    cache.moe_cache_set_profiling(True)
    cache.moe_cache_timing(clear=True)
    timed(torch, run.pass_sequence_serial, a.steps)
    tm = cache.moe_cache_timing(clear=True)
    cache.close()
    rcache = P.make_cache(wl, int4=True, pool=pool, capacity=cfg.n_experts, fetch_mode=P.B.MOE_FETCH_IN_KERNEL)
    rrun = Runner(wl, rcache, torch, P)
    for l in range(cfg.n_layers):
        rcache.moe_cache_prefill_pins(l, list(range(cfg.n_experts)))
    rrun.pass_resident()
    n_r, dt_r = timed(torch, rrun.pass_resident, a.steps)
    rcache.close()
    # a prompt of up to 512 tokens through the stack with the cache read-only: missing experts stream in 4-bit form
    import numpy as np
    n_p = min(512, cfg.n_seqs * cfg.n_steps)
    xp = P.to_device(np.concatenate([wl.tokens(s) for s in range(cfg.n_seqs)])[:n_p])
    yp = torch.empty((n_p, d), dtype=torch.bfloat16, device="cuda:0")
    pcache = P.make_cache(wl, int4=True, pool=pool, max_batch=n_p)
    for l in range(cfg.n_layers):
        pcache.moe_cache_prefill_pins(l, wl.prefetch_list(l, 0))

    def prompt_pass():
        for l in range(cfg.n_layers):
            pcache.moe_layer_prefill(l, xp, yp)
        return n_p

    prompt_pass()
    pst0 = pcache.moe_cache_stats()
    n_pp, dt_pp = timed(torch, prompt_pass, 3)
    pst = pcache.moe_cache_stats()
    pcache.close()
    single = tm["decode_single_launches"] > 0
    k_bytes = (K + cfg.n_shared) * qb + d * 2 + (K + cfg.n_shared) * d * 4 + (cfg.n_experts * d * 2 + cfg.n_experts * 4 if single else 0)
    k_ms = (tm["decode_single_ms"] / tm["decode_single_launches"] if single
            else tm["ffn_fused_ms"] / max(1, tm["ffn_fused_launches"]))
    return {"prompt_streaming": {"prompt_tokens": n_p, "ms_per_layer": dt_pp / 3 / cfg.n_layers * 1e3,
                                 "tokens_per_s": n_pp / dt_pp,
                                 "pcie_GBps_lower_bound": (pst["bytes_streamed"] - pst0["bytes_streamed"]) / dt_pp / 1e9},
            "format": "groups of 32 along the contraction dimension, 4-bit codes + bf16 scale, weight = s * (q - 8)",
            "expert_bytes": qb, "tokens_per_s": n_tok / dt,
            "cache_hit_rate": st["hits"] / max(1, st["lookups"]), "misses_per_token": st["misses"] / max(1, n_tok),
            "pcie_GBps": tm["fetch_bytes"] / (tm["fetch_ms"] * 1e-3) / 1e9 if tm["fetch_ms"] > 0 else None,
            "main_kernel": {"kernel": ("decode_single_q4_kernel (router, gating, lookups and the 4-bit expert FFN in one "
                                       "launch)" if single else "ffn_fused_q4_kernel"),
                            "bytes_per_launch": k_bytes, "avg_launch_ms": k_ms,
                              "launches_timed": tm["decode_single_launches"] if single else tm["ffn_fused_launches"],
                              "achieved_GBps": k_bytes / (k_ms * 1e-3) / 1e9 if k_ms > 0 else None,
                              "frac_of_hbm_peak": k_bytes / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS if k_ms > 0 else None},
            "resident_path_tokens_per_s": n_r / dt_r,
            "resident_path_us_per_layer_call": dt_r / n_r / cfg.n_layers * 1e6,
            "note": "same capacity C in experts (a quarter of the bytes); in-kernel fetch; outputs differ from the "
                    "bf16 run by the quantisation error, parity is against the oracle on the same 4-bit values"}


def cpu_baseline(wl, n_tokens):
    """The oracle as it stands, all host cores through its OpenMP row loops, on the first tokens of the workload."""
    import numpy as np
    import oracle
    from tests.helpers import OracleStack
    from workload import widen
    cfg = wl.cfg
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
    cores = max(1, min(cores, 16))
    oracle.set_threads(cores)
    ost = OracleStack(wl, keep=cfg.n_experts * cfg.n_layers)
    for l in range(cfg.n_layers):                      # parameter conversion is not part of the timed work
        for e in range(cfg.n_experts):
            ost.expert(l, e)
    def run(limit):
        done, t_used = 0, 0.0
        for s in range(cfg.n_seqs):
            x32 = widen(wl.tokens(s))
            for c in ost.caches:
                c.reset()
            for l in range(cfg.n_layers):
                ost.caches[l].pin(wl.prefetch_list(l, s))
            biases = [wl.bias(l, s)[None, :] for l in range(cfg.n_layers)]
            t0 = time.perf_counter()
            for t in range(cfg.n_steps):
                for l in range(cfg.n_layers):
                    ost.decode(l, x32[t:t + 1], biases[l])
                done += 1
                if done >= limit:
                    break
            t_used += time.perf_counter() - t0
            if done >= limit:
                break
        return done, t_used

    done, t_used = run(n_tokens)
    oracle.set_threads(1)
    done1, t1 = run(max(1, n_tokens // 8))             # the same loops on one thread, shorter sample
    return {"value": done / t_used, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "first %d decode tokens of the workload (sequence-serial, batch 1, all %d layer(s)), "
                      "fp64 oracle with OpenMP over output rows" % (done, cfg.n_layers),
            "single_thread": {"value": done1 / t1, "unit": "tokens/s", "cores": 1,
                              "sample": "first %d decode tokens, same loops on one thread" % done1}}


def kernel_roofline(cfg, tm, traffic):
    """Roofline entry of the dominant kernel from the HIP-event sums of a profiled pass (calls without a miss)."""
    K, d, f, s_el, E = cfg.top_k, cfg.d_model, cfg.d_ff, cfg.elem_bytes, cfg.n_experts
    KS_ = K + cfg.n_shared
    experts = KS_ * 3 * d * f * s_el
    if tm["decode_single_launches"] > 0:
        # one launch = router + gating + cache lookups + the K selected (and shared) experts' FFN: the experts'
        # three matrices, the router matrix, the token and its bias in, one output row per expert out
        k_bytes = experts + E * d * s_el + d * s_el + E * 4 + KS_ * d * 4
        k_ms = tm["decode_single_ms"] / tm["decode_single_launches"]
        k_n = tm["decode_single_launches"]
        k_name = (("decode_tiles_kernel" if tm.get("decode_tiles_launches", 0) > 0 else "decode_single_kernel") +
                  " (router GEMV, Top-K gating, cache lookups and gate/up + SiLU*mul + down "
                  "projection of the K selected experts in one launch)")
    elif tm["ffn_fused_launches"] > 0:
        k_bytes = experts + d * s_el + KS_ * d * 4
        k_ms = tm["ffn_fused_ms"] / tm["ffn_fused_launches"]
        k_n = tm["ffn_fused_launches"]
        k_name = "ffn_fused_kernel (gate/up + SiLU*mul + down projection of the K selected experts, one launch)"
    else:
        k_bytes = KS_ * 2 * d * f * s_el + d * s_el + KS_ * f * s_el
        k_ms = tm["ffn_gate_up_ms"] / max(1, tm["ffn_launches"])
        k_n = tm["ffn_launches"]
        k_name = "ffn_tiled_kernel<2,...> (gate/up + SiLU*mul of the K selected experts)"
    achieved = k_bytes / (k_ms * 1e-3) / 1e9 if k_ms > 0 else 0.0
    return {"bound": "hbm", "kernel": k_name, "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "bytes_per_launch": k_bytes,
            "avg_launch_ms": k_ms, "launches_timed": k_n,
            "source": "HIP events attached to the kernel's dispatch on the launch stream (hipExtLaunchKernelGGL "
                      "start/stop), same steps re-run with event timing on; launches of calls without a miss"}


def stored_traffic(name):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary (not measured in
    this run: counters need the profiler)."""
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(tpath):
        return None, None
    t = json.load(open(tpath)).get(name)
    if not t:
        return None, None
    return t.get("bytes_per_launch"), {k: t.get(k) for k in ("commit", "date", "kernel", "note")}


def resident_batched(torch, P, wl, pool, reps=3):
    """Schedule R at B = S: every expert resident, one token of each sequence per call.  U = distinct experts a call
    touches, counted from the routing the library returns."""
    import numpy as np
    cfg = wl.cfg
    S, K, E, d = cfg.n_seqs, cfg.top_k, cfg.n_experts, cfg.d_model
    cache = P.make_cache(wl, tiled=True, pool=pool, capacity=E, max_batch=S, fetch_mode=P.B.MOE_FETCH_IN_KERNEL)
    for l in range(cfg.n_layers):
        cache.moe_cache_prefill_pins(l, list(range(E)))
    T = min(cfg.n_steps, 32)
    xs = [P.to_device(np.stack([wl.tokens(s)[t] for s in range(S)])) for t in range(T)]
    bias = [torch.from_numpy(np.stack([wl.bias(l, s) for s in range(S)])).cuda() for l in range(cfg.n_layers)]
    y = torch.empty((S, d), dtype=P.torch_dtype(cfg), device="cuda:0")
    idx = torch.empty((T, cfg.n_layers, S, K), dtype=torch.int32, device="cuda:0")

    def one_pass():
        for t in range(T):
            for l in range(cfg.n_layers):
                cache.moe_layer_decode(l, xs[t], y, bias[l], idx[t, l])
        return S * T

    one_pass()
    n, dt = timed(torch, one_pass, reps)
    u = float(np.mean([len(np.unique(c)) for c in idx.cpu().numpy().reshape(T * cfg.n_layers, S * K)]))
    cache.close()
    call_s = dt / (reps * T * cfg.n_layers)
    call_bytes = (u + cfg.n_shared) * cfg.expert_bytes + E * d * cfg.elem_bytes + 2 * S * d * cfg.elem_bytes + S * E * 4
    return {"batch": S, "tokens_per_s": n / dt, "call_us": call_s * 1e6, "distinct_experts_per_call": u,
            "algorithmic_GBps_whole_call": call_bytes / call_s / 1e9,
            "frac_of_hbm_peak_whole_call": call_bytes / call_s / 1e9 / HBM_PEAK_GBPS,
            "note": "capacity = E, all experts preloaded, one token of each of the %d sequences per call; bytes = "
                    "distinct experts touched x expert bytes + router + tokens in and out" % S}


def measure(torch, P, wl, pool, a, steps, warmup, full):
    """One workload through the schedules: capacity-C sequence-serial decode (the value), the same with kernel
    timing, the resident path at batch 1 and at batch S, the all-miss path; `full` adds the comparisons."""
    cfg = wl.cfg
    K, d, f, eb, s_el = cfg.top_k, cfg.d_model, cfg.d_ff, cfg.expert_bytes, cfg.elem_bytes
    fetch_mode = P.B.MOE_FETCH_IN_KERNEL if a.fetch_mode == "in_kernel" else P.B.MOE_FETCH_COPY_ENGINE
    cache = P.make_cache(wl, tiled=True, pool=pool, fetch_mode=fetch_mode)
    run = Runner(wl, cache, torch, P)
    for _ in range(warmup):
        run.pass_sequence_serial()
    cache.moe_cache_reset(-1, clear_stats=True)
    n_tok, dt = timed(torch, run.pass_sequence_serial, steps)
    st = cache.moe_cache_stats()

    # same steps again with HIP-event timing of the kernels and copies (events sit on the launch stream)
    cache.moe_cache_set_profiling(True)
    cache.moe_cache_timing(clear=True)
    n_tok_p, dt_p = timed(torch, run.pass_sequence_serial, max(1, steps // 2))
    tm = cache.moe_cache_timing(clear=True)
    cache.moe_cache_set_profiling(False)

    cold = None
    if full:    # the same schedule without the per-sequence prefetch: every sequence starts on an empty cache
        run.pass_sequence_serial(pins=False)
        cache.moe_cache_reset(-1, clear_stats=True)
        n_cold, dt_cold = timed(torch, lambda: run.pass_sequence_serial(pins=False), max(1, steps // 4))
        st_cold = cache.moe_cache_stats()
        cold = {"tokens_per_s": n_cold / dt_cold, "cache_hit_rate": st_cold["hits"] / max(1, st_cold["lookups"]),
                "misses_per_token": st_cold["misses"] / max(1, n_cold),
                "note": "no prefetch set: the first tokens of a sequence miss until its experts are resident"}
    cache.close()

    # the same workload with the copy-engine fetch (hipMemcpyAsync on the copy stream): router kernel, expert kernel
    # and combine are three launches there, which also times the expert kernel on its own
    other = None
    if a.fetch_mode == "in_kernel":
        ocache = P.make_cache(wl, tiled=True, pool=pool, fetch_mode=P.B.MOE_FETCH_COPY_ENGINE)
        orun = Runner(wl, ocache, torch, P)
        orun.pass_sequence_serial()
        n_o, dt_o = timed(torch, orun.pass_sequence_serial, max(1, steps // 2))
        ocache.moe_cache_set_profiling(True)
        ocache.moe_cache_timing(clear=True)
        timed(torch, orun.pass_sequence_serial, 1)
        otm = ocache.moe_cache_timing(clear=True)
        ocache.close()
        KS_ = K + cfg.n_shared
        e_bytes = KS_ * 3 * d * f * s_el + d * s_el + KS_ * d * 4
        e_ms = otm["ffn_fused_ms"] / max(1, otm["ffn_fused_launches"])
        other = {"tokens_per_s": n_o / dt_o,
                 "pcie_GBps": otm["copy_bytes"] / (otm["copy_ms"] * 1e-3) / 1e9 if otm["copy_ms"] > 0 else None,
                 "expert_kernel_alone": ({"kernel": "ffn_fused_kernel", "bytes_per_launch": e_bytes,
                                          "avg_launch_ms": e_ms, "launches_timed": otm["ffn_fused_launches"],
                                          "achieved_GBps": e_bytes / (e_ms * 1e-3) / 1e9,
                                          "frac_of_hbm_peak": e_bytes / (e_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
                                         if e_ms > 0 else None),
                 "route_cache_kernel_us": otm["route_ms"] / max(1, otm["route_launches"]) * 1e3,
                 "note": "fetch_mode copy_engine: hipMemcpyAsync per missed expert on the library's copy stream; "
                         "router + gating + lookups, expert FFN and combine are separate launches with a host "
                         "wait for the miss list in between"}

    # ---------------- resident path: every expert on the device, batch 1 ----------------
    rcache = P.make_cache(wl, tiled=True, pool=pool, capacity=cfg.n_experts, fetch_mode=fetch_mode)
    rrun = Runner(wl, rcache, torch, P)
    for l in range(cfg.n_layers):
        rcache.moe_cache_prefill_pins(l, list(range(cfg.n_experts)))
    for _ in range(max(1, warmup)):
        rrun.pass_resident()
    n_tok_r, dt_r = timed(torch, rrun.pass_resident, steps)
    rcache.moe_cache_set_profiling(True)
    rcache.moe_cache_timing(clear=True)
    timed(torch, rrun.pass_resident, max(1, steps // 2))
    rtm = rcache.moe_cache_timing(clear=True)
    rcache.close()

    traffic, traffic_src = stored_traffic(cfg.name)
    roofline = kernel_roofline(cfg, tm, traffic)
    if traffic_src:
        roofline["traffic_source"] = dict(traffic_src, kind="stored profile figure (rocprofv3 --pmc FETCH_SIZE + "
                                                            "WRITE_SIZE), not measured in this run")
    layer_bytes = (K + cfg.n_shared) * eb + cfg.n_experts * d * s_el + 2 * d * s_el + cfg.n_experts * 4
    res_tok_s = n_tok_r / dt_r
    r_launches = max(1, rtm["ffn_launches"] + rtm["ffn_fused_launches"] + rtm["decode_single_launches"])
    out = {
        "value": n_tok / dt, "ms_per_step": dt / steps * 1e3,
        "workload": "%s: %d layer(s), d=%d, d_ff=%d, E=%d, top-%d, capacity %d, %d sequences x %d decode steps, "
                    "sequence-serial batch 1 with per-sequence prefetch, LRU" %
                    (cfg.name, cfg.n_layers, d, f, cfg.n_experts, K, cfg.capacity, cfg.n_seqs, cfg.n_steps),
        "tokens_per_step": cfg.n_seqs * cfg.n_steps,
        "cache_hit_rate": st["hits"] / max(1, st["lookups"]),
        "misses_per_token": st["misses"] / max(1, n_tok),
        "roofline": roofline,
        "fetch_mode": a.fetch_mode,
        "pcie": ({"achieved": tm["fetch_bytes"] / (tm["fetch_ms"] * 1e-3) / 1e9 if tm["fetch_ms"] > 0 else None,
                  "peak": PCIE_PEAK_GBPS, "unit": "GB/s", "launches": tm["fetch_launches"],
                  "note": "bytes read from the pinned pool / duration of the expert kernels that fetched them "
                          "(fetch and compute of the resident experts overlap inside those launches)"}
                 if a.fetch_mode == "in_kernel" else
                 {"achieved": tm["copy_bytes"] / (tm["copy_ms"] * 1e-3) / 1e9 if tm["copy_ms"] > 0 else None,
                  "peak": PCIE_PEAK_GBPS, "unit": "GB/s", "copies": tm["copies"], "copy_ms_total": tm["copy_ms"]}),
        "resident_path": {"batch": 1, "tokens_per_s": res_tok_s, "us_per_token": 1e6 / res_tok_s,
                          "us_per_layer_call": 1e6 / res_tok_s / cfg.n_layers,
                          "algorithmic_GBps_whole_call": layer_bytes * cfg.n_layers * res_tok_s / 1e9,
                          "frac_of_hbm_peak_whole_call": layer_bytes * cfg.n_layers * res_tok_s / 1e9 / HBM_PEAK_GBPS,
                          "launches_per_call": (("decode_tiles_kernel" if rtm.get("decode_tiles_launches", 0) else
                                                 "decode_single_kernel") + " + combine_chunks_kernel"
                                                if rtm["decode_single_launches"] else
                                                "route_cache_kernel + expert FFN + combine"),
                          "main_kernel_us": (rtm["ffn_gate_up_ms"] + rtm["ffn_down_ms"] + rtm["ffn_fused_ms"] +
                                             rtm["decode_single_ms"]) / r_launches * 1e3,
                          "route_cache_us": rtm["route_ms"] / max(1, rtm["route_launches"]) * 1e3},
        "resident_path_batched": resident_batched(torch, P, wl, pool),
        "cold_start": cold,
        "copy_engine_fetch": other,
        "miss_path": miss_path(torch, P, wl, pool, fetch_mode),
        "profiled_rerun_tokens_per_s": n_tok_p / dt_p,
    }
    # the paper's latency model (Eq. 4) evaluated with this run's own terms
    rate = out["pcie"]["achieved"]
    if rate:
        t_compute = n_tok / res_tok_s
        t_transfer = eb / (rate * 1e9)
        n_tx = st["misses"] + st["pin_loads"]
        out["latency_model"] = {
            "equation": "Time_decode ~ Time_compute + N_miss * Time_transfer",
            "compute_s": t_compute, "n_miss": st["misses"], "n_prefetch_loads": st["pin_loads"],
            "transfer_s_per_expert": t_transfer,
            "predicted_s": t_compute + n_tx * t_transfer, "measured_s": dt,
            "measured_over_predicted": dt / (t_compute + n_tx * t_transfer),
            "predicted_s_at_nominal_pcie": t_compute + n_tx * eb / (PCIE_PEAK_GBPS * 1e9),
            "note": "Time_compute = tokens x resident-path time per token; Time_transfer = expert bytes / measured "
                    "pinned-pool rate; transfers = misses + the per-sequence prefetch loads, both inside the timed "
                    "region; a fetch overlaps the resident experts' compute inside the same launch"}
    return out


def build_workload(P, cfg, per_layer=None):
    from workload import Workload
    wl = Workload(cfg)
    t0 = time.perf_counter()
    # pools beyond 40 GB are pinned layer by layer (one allocation of the whole stack can be refused)
    if per_layer is None:
        per_layer = cfg.n_layers * cfg.n_experts * cfg.expert_bytes > 40e9
    pool = P.build_pool(wl, tiled=True, per_layer=per_layer)
    for s in range(cfg.n_seqs):
        wl.tokens(s)
    return wl, pool, time.perf_counter() - t0


def second_workload(torch, P, a):
    """The other configuration the bandwidth target names (Mixtral-8x7B-like MoE blocks), cut so that its pinned
    pool fits the host and the whole section takes about a minute: fewer layers, sequences and steps, all stated."""
    from workload import get_config
    base = get_config("mixtral_like")
    last = None
    import gc
    for layers in (a.second_layers, max(1, a.second_layers * 2 // 3), max(1, a.second_layers // 3)):
        cfg = base.with_(n_layers=layers, n_seqs=4, n_steps=16)
        gc.collect()
        torch._C._host_emptyCache()         # pinned blocks of the previous workload go back to the system
        try:
            wl, pool, t_gen = build_workload(P, cfg, per_layer=True)
        except RuntimeError as e:           # the host refused to pin that much memory (about 45 GB per process here)
            last = str(e).splitlines()[0]
            continue
        out = measure(torch, P, wl, pool, a, steps=2, warmup=1, full=False)
        out["setup_s"] = t_gen
        out["scope"] = ("%d of the stack's %d layers (host pool %.1f GB pinned), 4 of 8 sequences x 16 of 256 decode "
                        "steps; tokens/s is per token through these %d layers" %
                        (layers, base.n_layers, layers * cfg.n_experts * cfg.expert_bytes / 1e9, layers))
        out["roofline_tokens_per_s_this_cut"] = HBM_PEAK_GBPS * 1e9 / (layers * (cfg.top_k * cfg.expert_bytes))
        if not a.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline(Workload_view(wl, 1), 4)
            out["cpu_baseline"]["sample"] += "; ONE layer of the cut (tokens/s through one layer, not the stack)"
        del pool
        return out
    return {"error": "could not pin the expert pool: %s" % last}


def Workload_view(wl, n_layers):
    """The first n_layers layers of a workload (same seeds: layer l of the view is layer l of the original)."""
    from workload import Workload
    return Workload(wl.cfg.with_(n_layers=n_layers))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build is single-GPU (the hot path has no cross-GPU step); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2602_11192_amd.build import ensure_built
    ensure_built()
    from paper_2602_11192_amd import pool as P
    from workload import get_config
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)

    if a.calibrate_copy:
        n = 256 << 20
        src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty(n, dtype=torch.uint8, device="cuda")
        P.B.moe_probe_stream(src, dst, n, 1, 1)
        del src, dst

    # what a plain streaming read sustains on this GPU in this run (boxes differ by several percent)
    n_probe = 512 * 1000 * 1000
    probe_src = torch.empty(n_probe, dtype=torch.uint8, device="cuda").random_(0, 255)
    P.B.moe_probe_stream(probe_src, None, n_probe, 0, 3)
    probe_ms = P.B.moe_probe_stream(probe_src, None, n_probe, 0, 20)
    del probe_src
    hbm_probe = {"read_GBps": n_probe / probe_ms / 1e6, "bytes": n_probe,
                 "frac_of_peak": n_probe / probe_ms / 1e6 / HBM_PEAK_GBPS,
                 "note": "plain streaming read of 512 MB by the library's probe kernel, same GPU, same run: the "
                         "practical ceiling that roofline.achieved compares with"}

    cfg = get_config(a.workload)
    if a.layers:
        cfg = cfg.with_(n_layers=a.layers)
    if a.seqs:
        cfg = cfg.with_(n_seqs=a.seqs)
    if a.decode_steps:
        cfg = cfg.with_(n_steps=a.decode_steps)
    wl, pool, t_gen = build_workload(P, cfg)
    m = measure(torch, P, wl, pool, a, a.steps, a.warmup, full=True)

    out = {
        "metric": "decode tokens/sec per MoE layer stack at 1 MI355X",
        "value": m.pop("value"), "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": m.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": m.pop("workload"), "tokens_per_step": m.pop("tokens_per_step")},
    }
    out.update(m)
    out["hbm_probe"] = hbm_probe
    out["setup_s"] = t_gen
    sweep_sizes = tuple(int(v) for v in a.sweep_sizes.split(",")) if a.sweep_sizes else None
    if a.batch_sweep or (a.workload == "olmoe_like" and not a.no_sweep):
        kw = {"sizes": sweep_sizes} if sweep_sizes else {}
        sweep = batch_sweep(torch, P, wl, pool, **kw)
        if a.batch_sweep:
            json.dump(sweep, open(a.batch_sweep, "w"), indent=1)
        out["resident_batch_sweep"] = sweep
    if a.extras:
        json.dump(extras(torch, P, wl, pool, a), open(a.extras, "w"), indent=1)
    n_weights = cfg.n_layers * cfg.n_experts * 3 * cfg.d_model * cfg.d_ff
    if cfg.dtype == "bf16" and (a.int4 == "on" or (a.int4 == "auto" and n_weights <= 5e8)):
        del pool
        pool = None
        out["int4_experts"] = int4_section(torch, P, wl, a)
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, a.cpu_baseline_tokens)
    del pool
    if a.workload == "olmoe_like" and a.second_layers > 0:
        out["mixtral_like"] = second_workload(torch, P, a)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
