"""Drivers shared by the GPU parity tests: run the same seeded workload through
the HIP library and through the CPU oracle and collect comparable records."""
from __future__ import annotations

import numpy as np

import oracle
from workload import widen

TOL = {"fp32": 1e-4, "bf16": 2e-2}


class OracleStack:
    """Oracle-side state of a layer stack: float32 parameters and one cache per layer."""

    def __init__(self, wl, capacity=None, policy=oracle.POLICY_LRU, gamma=1.0, keep=40, int4=False):
        self.wl, self.cfg, self.int4 = wl, wl.cfg, int4
        c = self.cfg
        cap = min(c.capacity if capacity is None else capacity, c.n_experts)
        self.caches = [oracle.ExpertCache(c.n_experts, cap, policy, gamma) for _ in range(c.n_layers)]
        self.router = [widen(wl.router_w(l)) for l in range(c.n_layers)]
        if int4:        # the oracle sees the 4-bit experts through its own dequantisation
            self.shared = [[tuple(oracle.dequant_int4(q, s) for q, s in wl.shared_int4(l, sh))
                            for sh in range(c.n_shared)] for l in range(c.n_layers)]
        else:
            self.shared = [[tuple(widen(m) for m in wl.shared(l, s)) for s in range(c.n_shared)]
                           for l in range(c.n_layers)]
        self._experts, self._keep = {}, keep

    def expert(self, l, e):
        key = (l, e)
        if key not in self._experts:
            if len(self._experts) >= self._keep:
                self._experts.pop(next(iter(self._experts)))
            if self.int4:
                self._experts[key] = tuple(oracle.dequant_int4(q, s) for q, s in self.wl.expert_int4(l, e))
            else:
                self._experts[key] = tuple(widen(m) for m in self.wl.expert(l, e))
        return self._experts[key]

    def decode(self, l, x32, bias, compute_y=True, norm_topk=None):
        lw = oracle.LayerWeights(self.router[l], lambda e: self.expert(l, e), self.shared[l])
        return oracle.moe_layer_decode(lw, self.caches[l], x32, bias, self.cfg.top_k,
                                       self.cfg.norm_topk if norm_topk is None else norm_topk, compute_y)

    def prefill(self, l, x32, bias, rows=None):
        lw = oracle.LayerWeights(self.router[l], lambda e: self.expert(l, e), self.shared[l])
        return oracle.moe_layer_prefill(lw, self.caches[l], x32, bias, self.cfg.top_k, self.cfg.norm_topk, rows)


def rel_err(y, ref):
    """Per token: max_i |y_i - ref_i| / max_i |ref_i|."""
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return np.abs(y - ref).max(axis=-1) / np.abs(ref).max(axis=-1)


def elementwise_excess(y, ref, tol):
    """Second error measure: largest |y_i - ref_i| / (tol |ref_i| + tol rms(ref)) over the elements of each token;
    <= 1 means every element is within tol of its own magnitude plus the same share of the row's rms (a relative
    error alone is unbounded near zeros)."""
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True))
    return (np.abs(y - ref) / (tol * np.abs(ref) + tol * rms)).max(axis=-1)


WORST_ELEMENTWISE = {"value": 0.0}      # largest elementwise_excess seen by run_sequence_serial (reported by tests)


def run_sequence_serial(wl, cache, ostack, *, pins=True, y_every=1, seqs=None, steps=None, torch=None, pool=None,
                        y_layers=None, y_seqs=None):
    """Schedule of the paper's main setting: one sequence at a time, batch 1;
    per sequence: empty the caches, preload the prefetch set, then T decode
    steps through all layers.  Returns the worst output error and checks
    routing and traces on the way.  Outputs are compared every y_every-th step
    (of the layers / sequences in y_layers / y_seqs when given); routing, gate
    weights and the cache trace are compared for every call."""
    from paper_2602_11192_amd import pool as P
    cfg = wl.cfg
    dev = "cuda:0"
    seqs = range(cfg.n_seqs) if seqs is None else seqs
    steps = cfg.n_steps if steps is None else steps
    tdt = P.torch_dtype(cfg)
    y = torch.empty((1, cfg.d_model), dtype=tdt, device=dev)
    idx = torch.empty((1, cfg.top_k), dtype=torch.int32, device=dev)
    gw = torch.empty((1, cfg.top_k), dtype=torch.float32, device=dev)
    worst, n_y = 0.0, 0
    traces = [[] for _ in range(cfg.n_layers)]
    for s in seqs:
        cache.moe_cache_reset(-1)
        for c in ostack.caches:
            c.reset()
        if pins:
            for l in range(cfg.n_layers):
                ids = wl.prefetch_list(l, s)
                cache.moe_cache_prefill_pins(l, ids)
                ostack.caches[l].pin(ids)
        xs = wl.tokens(s)
        x_dev = P.to_device(xs, dev)
        x32 = widen(xs)
        biases = [wl.bias(l, s)[None, :] for l in range(cfg.n_layers)]
        biases_dev = [torch.from_numpy(b).to(dev) for b in biases]
        for t in range(steps):
            for l in range(cfg.n_layers):
                want_y = ((t % y_every) == 0 and (y_layers is None or l in y_layers) and
                          (y_seqs is None or s in y_seqs))
                cache.moe_layer_decode(l, x_dev[t:t + 1], y, biases_dev[l], idx, gw)
                res = ostack.decode(l, x32[t:t + 1], biases[l], compute_y=want_y)
                torch.cuda.synchronize()
                assert idx.cpu().numpy().tolist() == res.idx.tolist(), (s, t, l)
                np.testing.assert_allclose(gw.cpu().numpy(), res.w, rtol=0, atol=2e-5)
                traces[l].extend(res.trace)
                if want_y:
                    err = float(rel_err(P.to_numpy(y), res.y)[0])
                    assert err <= TOL[cfg.dtype], (s, t, l, err)
                    ex = float(elementwise_excess(P.to_numpy(y), res.y, TOL[cfg.dtype])[0])
                    assert ex <= 1.0, (s, t, l, ex)
                    WORST_ELEMENTWISE["value"] = max(WORST_ELEMENTWISE["value"], ex)
                    worst = max(worst, err)
                    n_y += 1
    return worst, n_y, traces


def compare_traces_and_stats(cache, ostack, traces, expert_bytes):
    for l, ref in enumerate(traces):
        got, total = cache.moe_cache_read_trace(l)
        assert total == len(ref)
        n = min(len(ref), len(got))
        assert got[:n].tolist() == [list(r) for r in ref[:n]], "trace of layer %d differs" % l
        assert cache.moe_cache_stats(l) == ostack.caches[l].stats(expert_bytes)
        assert cache.moe_cache_resident(l) == ostack.caches[l].resident()
