"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the
same seeded inputs.  Routing indices, cache traces, statistics and resident sets
must match exactly; outputs within the stated tolerance (fp32 1e-4, bf16 2e-2 of
the token's largest output magnitude)."""
import numpy as np
import pytest

import oracle
from tests.helpers import TOL, OracleStack, compare_traces_and_stats, rel_err, run_sequence_serial
from workload import MoEConfig, Workload, get_config, widen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "these tests need the MI355X"
    return t


@pytest.fixture(scope="module")
def P():
    from paper_2602_11192_amd import pool
    return pool


def small_cfg(**kw):
    base = dict(name="small_bf16", cfg_id=11, dtype="bf16", n_layers=2, d_model=128, d_ff=96, n_experts=16,
                n_shared=0, top_k=4, capacity=6, n_seqs=3, n_steps=24, prefill_len=0, beta=2.0, pref_lo=4,
                pref_hi=4, delta=1e-3)
    base.update(kw)
    return MoEConfig(**base)


# ------------------------------------------------------------------ config 1
@pytest.mark.parametrize("pins", [True, False])
def test_tiny_fp32_full_workload(torch, P, pins):
    cfg = get_config("tiny_fp32")
    wl = Workload(cfg)
    cache = P.make_cache(wl, trace_capacity=4096)
    ost = OracleStack(wl)
    worst, n_y, traces = run_sequence_serial(wl, cache, ost, pins=pins, torch=torch)
    assert n_y == cfg.n_seqs * cfg.n_steps and worst <= TOL["fp32"]
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    st = cache.moe_cache_stats()
    assert st["hits"] + st["misses"] == st["lookups"] == cfg.n_seqs * cfg.n_steps * cfg.top_k
    cache.close()


# ------------------------------------------------- small bf16, both layouts
@pytest.mark.parametrize("tiled", [False, True])
@pytest.mark.parametrize("norm_topk", [1, 0])
def test_small_bf16_sequence_serial(torch, P, tiled, norm_topk):
    cfg = small_cfg(norm_topk=norm_topk)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=tiled, trace_capacity=4096)
    ost = OracleStack(wl)
    worst, n_y, traces = run_sequence_serial(wl, cache, ost, torch=torch)
    assert n_y == cfg.n_seqs * cfg.n_steps * cfg.n_layers
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("tiled", [False, True])
def test_small_bf16_shared_experts(torch, P, tiled):
    cfg = small_cfg(n_shared=2, d_ff=160, d_model=96)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=tiled, trace_capacity=4096)
    ost = OracleStack(wl)
    _, _, traces = run_sequence_serial(wl, cache, ost, torch=torch, seqs=[0, 1], steps=12)
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


def batched_step(torch, P, wl, cache, ost, layer, rows, step):
    """One call with one token from each sequence in `rows`."""
    cfg = wl.cfg
    xs = np.stack([wl.tokens(s)[step] for s in rows])
    bias = np.stack([wl.bias(layer, s) for s in rows])
    x_dev = P.to_device(xs)
    y = torch.empty((len(rows), cfg.d_model), dtype=P.torch_dtype(cfg), device="cuda:0")
    idx = torch.empty((len(rows), cfg.top_k), dtype=torch.int32, device="cuda:0")
    cache.moe_layer_decode(layer, x_dev, y, torch.from_numpy(bias).cuda(), idx, None)
    res = ost.decode(layer, widen(xs), bias)
    torch.cuda.synchronize()
    assert idx.cpu().numpy().tolist() == res.idx.tolist()
    err = rel_err(P.to_numpy(y), res.y)
    assert err.max() <= TOL[cfg.dtype], err
    return res.trace


@pytest.mark.parametrize("tiled", [False, True])
@pytest.mark.parametrize("batch", [3, 7])
def test_small_bf16_batched_with_evictions_inside_a_call(torch, P, tiled, batch):
    # batch * K > C: a call evicts experts that earlier tokens of the same call hit,
    # which exercises the spare-buffer indirection.
    cfg = small_cfg(n_seqs=7, n_steps=10, n_layers=1, capacity=5)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=tiled, max_batch=batch, staging_buffers=batch * cfg.top_k, trace_capacity=8192)
    ost = OracleStack(wl)
    traces = [[]]
    for step in range(cfg.n_steps):
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, list(range(batch)), step))
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("d_model,d_ff", [(256, 96), (512, 160), (1024, 64)])
@pytest.mark.parametrize("batch", [1, 4, 6, 7, 16, 17])
def test_single_launch_decode_ffn_shapes(torch, P, d_model, d_ff, batch):
    # hidden widths that are multiples of 256 take the single-launch decode FFN for calls of up to 6 tokens;
    # larger calls take the grouped GEMM on the same cache
    cfg = small_cfg(d_model=d_model, d_ff=d_ff, n_seqs=17, n_steps=4, n_layers=1, capacity=16, n_shared=1)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, max_batch=17, trace_capacity=4096)
    ost = OracleStack(wl, capacity=16, keep=16)
    traces = [[]]
    for step in range(cfg.n_steps):
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, list(range(batch)), step))
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("batch", [1, 3, 5, 7])
def test_in_kernel_fetch_matches_oracle(torch, P, batch):
    # missed experts are read from the pinned pool by the expert kernel itself and land in their buffers
    from paper_2602_11192_amd import binding as B
    cfg = small_cfg(n_seqs=7, n_steps=12, n_layers=2, capacity=5 if batch > 1 else 6, d_model=256, d_ff=96, beta=1.0)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, max_batch=batch, staging_buffers=batch * cfg.top_k if batch > 1 else 0,
                         trace_capacity=8192, fetch_mode=B.MOE_FETCH_IN_KERNEL)
    ost = OracleStack(wl)
    if batch == 1:
        _, _, traces = run_sequence_serial(wl, cache, ost, torch=torch, seqs=[0, 1, 2], pins=False)
    else:
        traces = [[], []]
        for step in range(cfg.n_steps):
            for l in range(2):
                traces[l].extend(batched_step(torch, P, wl, cache, ost, l, list(range(batch)), step))
    assert cache.moe_cache_stats()["misses"] > 10
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


def test_lru_table_larger_than_a_wave(torch, P):
    # capacity above 64 slots: the cache table is staged in LDS instead of registers
    cfg = small_cfg(n_experts=96, capacity=70, n_layers=1, n_seqs=2, n_steps=40, pref_lo=0, pref_hi=0, beta=0.0)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, trace_capacity=4096)
    ost = OracleStack(wl, keep=96)
    _, _, traces = run_sequence_serial(wl, cache, ost, torch=torch, pins=False, y_every=10)
    assert cache.moe_cache_stats(0)["evictions"] > 0
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


def test_alternating_small_and_large_batches_share_one_table(torch, P):
    # calls of 1-3 tokens use the register-resident table, calls of 17 tokens the LDS one
    cfg = small_cfg(n_seqs=17, n_steps=8, n_layers=1, capacity=8)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, max_batch=17, staging_buffers=17 * cfg.top_k, trace_capacity=8192)
    ost = OracleStack(wl)
    traces = [[]]
    for step in range(cfg.n_steps):
        rows = list(range(17)) if step % 2 else [step % 17, (step + 5) % 17, (step + 11) % 17][: 1 + step % 3]
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, rows, step))
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("gamma", [1.0, 0.7])
def test_gamma_policy_batched(torch, P, gamma):
    # batched calls under the discounted-count policy (table staged in LDS, general grouping)
    from paper_2602_11192_amd import binding as B
    cfg = small_cfg(n_seqs=20, n_steps=6, n_layers=1, capacity=7, n_shared=1)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, max_batch=20, staging_buffers=20 * cfg.top_k, trace_capacity=8192,
                         policy=B.MOE_POLICY_GAMMA, gamma=gamma)
    ost = OracleStack(wl, policy=oracle.POLICY_GAMMA, gamma=gamma)
    traces = [[]]
    for step in range(cfg.n_steps):
        rows = list(range(20)) if step % 2 == 0 else list(range(3, 9))
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, rows, step))
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


def test_resident_batch_with_64_buffers_and_shared_experts(torch, P):
    # 64 expert buffers plus shared experts: buffer ids run past 64; 40 tokens = 240 pairs in one call
    cfg = small_cfg(n_experts=64, capacity=64, top_k=4, n_shared=2, n_seqs=40, n_steps=3, n_layers=1,
                    d_model=256, d_ff=64)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, max_batch=40, trace_capacity=4096)
    ost = OracleStack(wl, capacity=64, keep=64)
    traces = [[]]
    for step in range(cfg.n_steps):
        rows = list(range(40)) if step != 1 else list(range(11))
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, rows, step))
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("d_model,d_ff", [(160, 96), (256, 128), (512, 96)])
@pytest.mark.parametrize("n_experts,top_k,batch", [(16, 4, 128), (4, 2, 300), (8, 2, 97), (2, 1, 520), (8, 2, 600)])
def test_many_tokens_per_expert_take_the_grouped_gemm(torch, P, n_experts, top_k, batch, d_model, d_ff):
    # enough tokens per expert for the LDS-staged grouped GEMM: 64- and 128-token tiles, and from ~100 tokens per
    # expert the 256-token tiles (300 tokens over 4 experts, 520 over 2: several tiles per expert, ragged last tile).
    # d_model a multiple of 256 / d_ff of 128: from a mean of 40 / 56 tokens per expert the gate/up / down pass runs the
    # ring variant on a work list (both at 256 x 128, only the gate/up pass at 512 x 96)
    cfg = small_cfg(n_experts=n_experts, top_k=top_k, capacity=n_experts, n_seqs=batch, n_steps=2, n_layers=1,
                    d_model=d_model, d_ff=d_ff, n_shared=1, pref_lo=1, pref_hi=1)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, max_batch=batch, trace_capacity=4096)
    ost = OracleStack(wl, capacity=n_experts, keep=n_experts)
    traces = [[]]
    for step in range(cfg.n_steps):
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, list(range(batch)), step))
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("n_tokens", [1, 40, 200])
def test_prompt_streaming_reads_the_cache_without_changing_it(torch, P, n_tokens):
    cfg = small_cfg(n_seqs=3, n_steps=8, n_layers=1, capacity=6, n_shared=1, prefill_len=n_tokens, d_model=160)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, max_batch=max(n_tokens, 2), trace_capacity=4096)
    ost = OracleStack(wl)
    pins = wl.prefetch_list(0, 0)[:4]
    cache.moe_cache_prefill_pins(0, pins)
    ost.caches[0].pin(pins)
    xs = wl.prefill_tokens(0)
    bias = np.tile(wl.bias(0, 0), (n_tokens, 1))
    y = torch.empty((n_tokens, cfg.d_model), dtype=torch.bfloat16, device="cuda:0")
    idx = torch.empty((n_tokens, cfg.top_k), dtype=torch.int32, device="cuda:0")
    gw = torch.empty((n_tokens, cfg.top_k), dtype=torch.float32, device="cuda:0")
    for _ in range(2):                                   # twice: the second call must see the same cache
        cache.moe_layer_prefill(0, P.to_device(xs), y, torch.from_numpy(bias).cuda(), idx, gw)
        res = ost.prefill(0, widen(xs), bias)
        torch.cuda.synchronize()
        assert idx.cpu().numpy().tolist() == res.idx.tolist()
        np.testing.assert_allclose(gw.cpu().numpy(), res.w, rtol=0, atol=2e-5)
        assert rel_err(P.to_numpy(y), res.y).max() <= TOL["bf16"]
    assert ost.caches[0].stream_loads > 0 or n_tokens == 1
    # the cache is as the pins left it, and decoding afterwards follows the oracle's trace
    traces = [[]]
    for step in range(cfg.n_steps):
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, [0], step))
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("staging", [0, 3])
@pytest.mark.parametrize("tiled", [False, True])
def test_calls_that_do_not_fit_the_spare_buffers_run_as_waves(torch, P, tiled, staging):
    # 8 tokens x K = 4 lookups against 4 slots and few spare buffers: the call is split into waves of tokens;
    # trace, statistics and outputs equal the oracle's, which knows nothing of buffers
    cfg = small_cfg(n_seqs=8, n_steps=6, n_layers=1, capacity=4, pref_lo=0, pref_hi=0, beta=0.0)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=tiled, max_batch=8, staging_buffers=staging, trace_capacity=1024)
    ost = OracleStack(wl)
    traces = [[]]
    for step in range(cfg.n_steps):
        rows = list(range(8)) if step % 2 == 0 else [1, 4, 6]
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, rows, step))
    assert cache.moe_cache_stats(0)["evictions"] > 20
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


def test_shared_cache_with_pooled_prefetch(torch, P):
    # 6 sequences decode together on one cache, preloaded with the Top-C of their summed preference scores
    from paper_2602_11192_amd import binding as B
    cfg = small_cfg(n_seqs=6, n_steps=10, n_layers=2, capacity=8, beta=2.5)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, max_batch=6, staging_buffers=4, trace_capacity=4096)
    ost = OracleStack(wl)
    for l in range(cfg.n_layers):
        scores = np.stack([wl.bias(l, s) for s in range(6)])
        ids = B.moe_pooled_prefetch_set(scores, cfg.capacity)
        assert ids == oracle.pooled_prefetch_set(scores, cfg.capacity)
        cache.moe_cache_prefill_pins(l, ids)
        ost.caches[l].pin(ids)
    traces = [[], []]
    for step in range(cfg.n_steps):
        for l in range(cfg.n_layers):
            traces[l].extend(batched_step(torch, P, wl, cache, ost, l, list(range(6)), step))
    st = cache.moe_cache_stats()
    assert st["pin_loads"] == 16 and st["hits"] > st["misses"]
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("gamma", [0.3, 0.49])
def test_gamma_policy_below_one_half_gives_the_lru_trace(torch, P, gamma):
    """Remark after Definition C.1 on the device: one expert per token, gamma < 1/2 - the discounted-count policy
    and LRU must produce the same trace, which is also the oracle's LRU trace."""
    from paper_2602_11192_amd import binding as B
    cfg = small_cfg(top_k=1, n_experts=12, capacity=5, n_layers=1, n_seqs=2, n_steps=150, pref_lo=0, pref_hi=0,
                    beta=0.0, cfg_id=17)
    wl = Workload(cfg)
    traces = {}
    for name, kw in (("gamma", dict(policy=B.MOE_POLICY_GAMMA, gamma=gamma)), ("lru", {})):
        cache = P.make_cache(wl, tiled=True, trace_capacity=4096, **kw)
        ost = OracleStack(wl)                       # the oracle runs LRU in both cases
        _, _, tr = run_sequence_serial(wl, cache, ost, torch=torch, pins=False, y_every=50)
        got, total = cache.moe_cache_read_trace(0)
        assert total == len(tr[0]) and got.tolist() == [list(r) for r in tr[0]]
        assert cache.moe_cache_resident(0) == ost.caches[0].resident()
        traces[name] = got.tolist()
        assert cache.moe_cache_stats(0)["evictions"] > 50
        cache.close()
    assert traces["gamma"] == traces["lru"]


@pytest.mark.parametrize("gamma", [1.0, 0.9])
def test_small_bf16_gamma_policy(torch, P, gamma):
    from paper_2602_11192_amd import binding as B
    cfg = small_cfg(n_layers=1, n_steps=40)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, trace_capacity=4096, policy=B.MOE_POLICY_GAMMA, gamma=gamma)
    ost = OracleStack(wl, policy=oracle.POLICY_GAMMA, gamma=gamma)
    _, _, traces = run_sequence_serial(wl, cache, ost, torch=torch, y_every=8)
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("tiled", [False, True])
@pytest.mark.parametrize("E,K,C", [(1, 1, 1),       # a single expert
                                   (4, 4, 4),       # every expert selected by every token (K = E)
                                   (16, 1, 1),      # one slot: every change of expert evicts
                                   (16, 4, 4),      # capacity = K: a token can evict all of the previous one's
                                   (16, 4, 100),    # capacity above E is clamped: misses are first touches only
                                   (64, 8, 63)])    # all but one expert fit
def test_degenerate_cache_shapes(torch, P, tiled, E, K, C):
    cfg = small_cfg(n_experts=E, top_k=K, capacity=C, n_layers=1, n_seqs=2, n_steps=20, pref_lo=0, pref_hi=0,
                    beta=0.0, d_model=256, d_ff=64)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=tiled, trace_capacity=4096)
    ost = OracleStack(wl, keep=64)
    _, _, traces = run_sequence_serial(wl, cache, ost, torch=torch, pins=False, y_every=4)
    st = cache.moe_cache_stats(0)
    if C >= E:
        assert st["evictions"] == 0
    if K == E:
        assert st["misses"] == E * 2                                  # each sequence starts cold: E first touches
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("d_model,d_ff", [(8, 1), (40, 7), (264, 33)])
def test_odd_widths_take_the_generic_kernels(torch, P, d_model, d_ff):
    # widths that fit no tile: row-major layout, generic kernels
    cfg = small_cfg(d_model=d_model, d_ff=d_ff, n_layers=1, n_seqs=2, n_steps=10)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=False, max_batch=3, staging_buffers=12, trace_capacity=2048)
    ost = OracleStack(wl)
    traces = [[]]
    for step in range(cfg.n_steps):
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, [0, 1] if step % 2 else [1], step))
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("E,K,C,n_shared,batch,policy", [
    (16, 4, 16, 1, 130, "lru"),      # everything resident: parallel all-hit path, shared expert
    (16, 4, 6, 0, 128, "lru"),       # constrained: misses inside the call, in-order routine, waves of tokens
    (8, 2, 8, 0, 300, "lru"),        # fewer experts than one tile of 16
    (100, 6, 100, 0, 200, "lru"),    # 64 < E <= 256, table larger than a wave (LDS table)
    (64, 8, 64, 2, 144, "lru"),      # 64 slots, 64 buffers, shared experts
    (16, 4, 8, 0, 140, "gamma"),     # discounted-count policy
    (32, 4, 32, 0, 113, "lru"),      # just above the size from which the tile kernel is used, ragged last tile
])
def test_large_calls_route_in_tiles_of_16_tokens(torch, P, E, K, C, n_shared, batch, policy):
    # calls of 112 tokens and more: router logits of 16 tokens per workgroup on the matrix cores, cache phase on
    # all waves of the last workgroup; routing, traces and outputs must not depend on which kernel ran
    from paper_2602_11192_amd import binding as B
    cfg = small_cfg(n_experts=E, top_k=K, capacity=C, n_shared=n_shared, n_seqs=batch, n_steps=3, n_layers=1,
                    d_model=256, d_ff=64, beta=1.0, pref_lo=min(4, K), pref_hi=min(4, K))
    wl = Workload(cfg)
    kw = dict(policy=B.MOE_POLICY_GAMMA, gamma=0.9) if policy == "gamma" else {}
    cache = P.make_cache(wl, tiled=True, max_batch=batch, staging_buffers=max(0, min(E, 64) - C), trace_capacity=1 << 15,
                         **kw)
    ost = OracleStack(wl, keep=128, **(dict(policy=oracle.POLICY_GAMMA, gamma=0.9) if policy == "gamma" else {}))
    traces = [[]]
    for step in range(cfg.n_steps):
        rows = list(range(batch)) if step != 1 else list(range(3))          # a small call in between
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, rows, step))
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("fetch", ["copy_engine", "in_kernel"])
def test_one_pinned_pool_per_layer(torch, P, fetch):
    # the expert pool handed over as L separate pinned allocations (expert_pool_layers)
    from paper_2602_11192_amd import binding as B
    cfg = small_cfg(n_layers=3, n_seqs=2, n_steps=12, d_model=256, d_ff=96, beta=1.0)
    wl = Workload(cfg)
    pools = P.build_pool(wl, tiled=True, per_layer=True)
    assert isinstance(pools, list) and len(pools) == 3
    cache = P.make_cache(wl, tiled=True, pool=pools, trace_capacity=4096,
                         fetch_mode=B.MOE_FETCH_IN_KERNEL if fetch == "in_kernel" else B.MOE_FETCH_COPY_ENGINE)
    ost = OracleStack(wl)
    _, _, traces = run_sequence_serial(wl, cache, ost, torch=torch)
    assert cache.moe_cache_stats()["misses"] > 10
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


def test_error_paths_on_device(torch, P):
    from paper_2602_11192_amd import binding as B
    cfg = small_cfg(n_layers=1)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, max_batch=2)
    x = torch.zeros((3, cfg.d_model), dtype=torch.bfloat16, device="cuda:0")
    y = torch.zeros_like(x)
    for call in (lambda: cache.moe_layer_decode(0, x, y),                       # batch > max_batch
                 lambda: cache.moe_layer_decode(1, x[:1], y[:1]),               # layer out of range
                 lambda: cache.moe_cache_prefill_pins(0, [1, 1]),               # duplicate ids
                 lambda: cache.moe_cache_prefill_pins(0, [cfg.n_experts]),      # id out of range
                 lambda: cache.moe_cache_prefill_pins(0, list(range(cfg.capacity + 1)))):
        with pytest.raises(B.MoeError) as ei:
            call()
        assert ei.value.code == B.MOE_ERR_INVALID_ARG
    cache.close()


# ------------------------------------------------------------- cache-simulation loss (section 3.1.1, appendix C.1)
@pytest.mark.gpu
@pytest.mark.parametrize("E,K,C,T,gamma,init", [
    (64, 8, 16, 300, 0.9, "uniform"), (8, 2, 5, 257, 1.0, "uniform"), (16, 2, 10, 200, 0.0, "prefetch"),
    (1000, 6, 100, 120, 0.5, "uniform"), (64, 6, 12, 64, 0.97, "prefetch"), (5, 1, 1, 33, 0.3, "uniform"),
    (130, 64, 65, 40, 0.8, "prefetch"), (64, 64, 32, 20, 0.7, "uniform"), (33, 7, 33, 90, 0.6, "prefetch")])
def test_cache_sim_loss_matches_oracle(torch, E, K, C, T, gamma, init):
    from paper_2602_11192_amd import binding as B
    n = 5
    r = np.random.default_rng(E * 1000 + K)
    w = 1.0 / np.arange(1, E + 1) ** 0.8
    w /= w.sum()
    idx = np.array([[np.sort(r.choice(E, size=K, replace=False, p=w)) for _ in range(T)] for _ in range(n)],
                   dtype=np.int32)
    c1 = None
    if init == "prefetch":
        c1 = np.zeros((n, E))
        for i in range(n):
            c1[i, r.choice(E, size=C, replace=False)] = 1.0
    out, flag = B.moe_cache_sim_loss(torch.from_numpy(idx).cuda(), E, C, gamma,
                                     None if c1 is None else torch.from_numpy(c1).cuda())
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    assert flag.cpu().numpy().tolist() == [0] * n
    for i in range(n):
        soft, hard = oracle.cache_sim_loss(idx[i:i + 1], E, C, gamma, None if c1 is None else c1[i:i + 1])
        assert out[i, 1] == round(hard * T)                       # miss count: exact
        assert out[i, 0] == pytest.approx(soft * T, rel=1e-12, abs=1e-12)


@pytest.mark.gpu
def test_cache_sim_loss_edges(torch):
    from paper_2602_11192_amd import binding as B
    idx = torch.zeros((2, 0, 2), dtype=torch.int32, device="cuda")            # no tokens
    out, flag = B.moe_cache_sim_loss(idx, 8, 4, 0.9)
    torch.cuda.synchronize()
    assert out.cpu().numpy().tolist() == [[0.0, 0.0], [0.0, 0.0]] and flag.cpu().tolist() == [0, 0]
    bad = torch.tensor([[[0, 1], [1, 9]], [[2, 3], [4, 5]]], dtype=torch.int32, device="cuda")
    out, flag = B.moe_cache_sim_loss(bad, 8, 4, 0.9)                           # id 9 is outside 0..7
    torch.cuda.synchronize()
    assert flag.cpu().tolist() == [1, 0]
    for args in [(0, 4, 0.9), (8, 0, 0.9), (8, 9, 0.9), (8, 4, 1.5), (2000, 4, 0.9)]:
        with pytest.raises(B.MoeError):
            B.moe_cache_sim_loss(bad, *args)
    with pytest.raises(B.MoeError):
        B.moe_cache_sim_loss(torch.zeros((1, 2, 9), dtype=torch.int32, device="cuda"), 8, 4, 0.9)   # K > E
