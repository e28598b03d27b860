"""Randomised parity: seeded mixes of shapes, policies, layouts, fetch modes, call sizes and spare-buffer counts,
with resets, preloads and prompt calls in between, through the C ABI against the oracle (routing and traces exact,
outputs within the bf16 tolerance)."""
import random

import numpy as np
import pytest

import oracle
from tests.helpers import TOL, OracleStack, compare_traces_and_stats, rel_err
from workload import Workload, widen
from workload.configs import MoEConfig

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as t
    if not t.cuda.is_available():
        pytest.skip("needs the GPU")
    return t


@pytest.fixture(scope="module")
def P():
    from paper_2602_11192_amd import pool
    return pool


def one_case(rng, torch, P):
    B = P.B
    d_model = rng.choice([128, 160, 256, 512, 1024])
    d_ff = rng.choice([32, 64, 96, 160])
    E = rng.randint(4, 40)
    K = rng.randint(1, min(E, 6))
    C = rng.randint(K, E)
    n_shared = rng.choice([0, 0, 1, 2])
    tiled = rng.random() < 0.75
    int4 = tiled and d_model % 256 == 0 and rng.random() < 0.3
    gamma = rng.choice([None, None, 1.0, 0.9, 0.5])
    fetch = B.MOE_FETCH_IN_KERNEL if (tiled and rng.random() < 0.5) else B.MOE_FETCH_COPY_ENGINE
    batches = [rng.choice([1, 1, 2, 3, 5, 8, 17, 33]) for _ in range(6)]
    mb = max(batches)
    staging = rng.randint(0, mb * K)       # too few spare buffers: the call runs as waves of tokens
    pref = rng.randint(0, min(E, 6))
    cfg = MoEConfig(name="mix", cfg_id=rng.randint(100, 100000), dtype="bf16", n_layers=1, d_model=d_model, d_ff=d_ff,
                    n_experts=E, n_shared=n_shared, top_k=K, capacity=C, n_seqs=mb, n_steps=len(batches),
                    prefill_len=0, beta=rng.choice([0.0, 1.0, 2.5]), pref_lo=pref, pref_hi=pref, delta=1e-3)
    what = (f"d={d_model} f={d_ff} E={E} K={K} C={C} shared={n_shared} tiled={tiled} int4={int4} gamma={gamma} "
            f"fetch={fetch} batches={batches} staging={staging} id={cfg.cfg_id}")
    wl = Workload(cfg)
    kw = dict(policy=B.MOE_POLICY_GAMMA, gamma=gamma) if gamma is not None else {}
    cache = P.make_cache(wl, tiled=tiled, int4=int4, max_batch=mb, staging_buffers=staging, trace_capacity=1 << 16,
                         fetch_mode=fetch, **kw)
    ost = OracleStack(wl, policy=oracle.POLICY_GAMMA if gamma is not None else oracle.POLICY_LRU,
                      gamma=1.0 if gamma is None else gamma, keep=E, int4=int4)
    trace = []
    for step, bsz in enumerate(batches):
        r = rng.random()
        if r < 0.15:                # drop the cache and preload a random set
            ids = rng.sample(range(E), rng.randint(0, C))
            cache.moe_cache_reset(0)
            ost.caches[0].reset()
            cache.moe_cache_prefill_pins(0, ids)
            ost.caches[0].pin(ids)
        elif r < 0.35 and tiled:    # a prompt through the layer: the cache is read, never changed
            n_p = min(mb, rng.choice([1, 3, 17, mb]))
            rows_p = [rng.randrange(mb) for _ in range(n_p)]
            xs = np.stack([wl.tokens(s)[step] for s in rows_p])
            bias = np.stack([wl.bias(0, s) for s in rows_p])
            y = torch.empty((n_p, d_model), dtype=torch.bfloat16, device="cuda:0")
            idx = torch.empty((n_p, K), dtype=torch.int32, device="cuda:0")
            cache.moe_layer_prefill(0, P.to_device(xs), y, torch.from_numpy(bias).cuda(), idx, None)
            res = ost.prefill(0, widen(xs), bias)
            torch.cuda.synchronize()
            assert idx.cpu().numpy().tolist() == res.idx.tolist(), what
            assert rel_err(P.to_numpy(y), res.y).max() <= TOL["bf16"], what
        rows = list(range(bsz))
        xs = np.stack([wl.tokens(s)[step] for s in rows])
        bias = np.stack([wl.bias(0, s) for s in rows])
        y = torch.empty((bsz, d_model), dtype=torch.bfloat16, device="cuda:0")
        idx = torch.empty((bsz, K), dtype=torch.int32, device="cuda:0")
        cache.moe_layer_decode(0, P.to_device(xs), y, torch.from_numpy(bias).cuda(), idx, None)
        res = ost.decode(0, widen(xs), bias)
        torch.cuda.synchronize()
        assert idx.cpu().numpy().tolist() == res.idx.tolist(), what
        err = rel_err(P.to_numpy(y), res.y)
        assert err.max() <= TOL["bf16"], (what, err)
        trace.extend(res.trace)
    compare_traces_and_stats(cache, ost, [trace], P.int4_block_bytes(cfg) if int4 else cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_mix_of_shapes_policies_and_modes(torch, P, seed):
    rng = random.Random(seed)
    for _ in range(100):
        one_case(rng, torch, P)
