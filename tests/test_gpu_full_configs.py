"""GPU parity at the full layer shapes of the five workloads.

Routing indices, cache traces, statistics and resident sets are compared for
every lookup; outputs are compared on a sample of the tokens (the oracle needs
3*d*d_ff double-precision multiply-adds per expert and token).  Layer stacks are
cut to one layer here: the layers of a stack are independent problems of the
same shape, and one layer of the Mixtral-like stack already holds 2.8 GB of
expert weights."""
import numpy as np
import pytest

import oracle
from tests.helpers import TOL, OracleStack, compare_traces_and_stats, rel_err, run_sequence_serial
from workload import Workload, get_config, widen

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


@pytest.fixture(autouse=True)
def oracle_threads():
    oracle.set_threads(16)
    yield
    oracle.set_threads(1)


@pytest.fixture(scope="module")
def olmoe(P):
    wl = Workload(get_config("olmoe_like"))
    return wl, P.build_pool(wl, tiled=True)


def test_olmoe_like_full_workload_sequence_serial(torch, P, olmoe):
    """The benchmark's configuration: 16 sequences x 128 steps, capacity 16, prefetch per sequence."""
    wl, pool = olmoe
    cfg = wl.cfg
    cache = P.make_cache(wl, pool=pool, trace_capacity=cfg.n_seqs * cfg.n_steps * cfg.top_k)
    ost = OracleStack(wl, keep=cfg.n_experts)
    worst, n_y, traces = run_sequence_serial(wl, cache, ost, torch=torch, y_every=16)
    assert n_y == cfg.n_seqs * cfg.n_steps // 16
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    st = cache.moe_cache_stats()
    assert st["lookups"] == cfg.n_seqs * cfg.n_steps * cfg.top_k
    assert 0.7 < st["hits"] / st["lookups"] < 0.95        # the concentrated regime of the fine-tuned models
    print("olmoe_like: worst rel err %.3e over %d tokens, hit rate %.3f" % (worst, n_y, st["hits"] / st["lookups"]))
    cache.close()


def test_olmoe_like_in_kernel_fetch(torch, P, olmoe):
    from paper_2602_11192_amd import binding as B
    wl, pool = olmoe
    cfg = wl.cfg
    cache = P.make_cache(wl, pool=pool, trace_capacity=6 * cfg.n_steps * cfg.top_k, fetch_mode=B.MOE_FETCH_IN_KERNEL)
    ost = OracleStack(wl, keep=cfg.n_experts)
    worst, n_y, traces = run_sequence_serial(wl, cache, ost, torch=torch, y_every=8, seqs=[0, 3, 7, 8, 12, 15])
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    assert cache.moe_cache_stats()["misses"] > 100
    cache.close()


def test_olmoe_like_cold_start_without_prefetch(torch, P, olmoe):
    wl, pool = olmoe
    cfg = wl.cfg
    cache = P.make_cache(wl, pool=pool, trace_capacity=4 * cfg.n_steps * cfg.top_k)
    ost = OracleStack(wl, keep=cfg.n_experts)
    _, _, traces = run_sequence_serial(wl, cache, ost, torch=torch, pins=False, y_every=32, seqs=[0, 5, 9, 15])
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("batch", [16, 5])
def test_olmoe_like_resident_path_batched(torch, P, olmoe, batch):
    """Every expert resident (capacity = E), one token of each sequence per call."""
    wl, pool = olmoe
    cfg = wl.cfg
    cache = P.make_cache(wl, pool=pool, capacity=cfg.n_experts, max_batch=batch, trace_capacity=8192)
    ost = OracleStack(wl, capacity=cfg.n_experts, keep=cfg.n_experts)
    ids = list(range(cfg.n_experts))
    cache.moe_cache_prefill_pins(0, ids)
    ost.caches[0].pin(ids)
    y = torch.empty((batch, cfg.d_model), dtype=torch.bfloat16, device="cuda:0")
    idx = torch.empty((batch, cfg.top_k), dtype=torch.int32, device="cuda:0")
    bias = np.stack([wl.bias(0, s) for s in range(batch)])
    bias_dev = torch.from_numpy(bias).cuda()
    trace = []
    for step in (0, 1, 50, 127):
        xs = np.stack([wl.tokens(s)[step] for s in range(batch)])
        cache.moe_layer_decode(0, P.to_device(xs), y, bias_dev, idx)
        res = ost.decode(0, widen(xs), bias)
        torch.cuda.synchronize()
        assert idx.cpu().numpy().tolist() == res.idx.tolist()
        assert rel_err(P.to_numpy(y), res.y).max() <= TOL["bf16"]
        trace += res.trace
    compare_traces_and_stats(cache, ost, [trace], cfg.expert_bytes)
    assert cache.moe_cache_stats()["misses"] == 0
    cache.close()


@pytest.mark.parametrize("fetch", ["copy_engine", "in_kernel"])
@pytest.mark.parametrize("name", ["mixtral_like", "phi35_like_concentrated", "phi35_like_diverse", "deepseek_like"])
def test_one_layer_of_the_large_stacks(torch, P, name, fetch):
    cfg = get_config(name).with_(n_layers=1, n_seqs=2, n_steps=24)
    wl = Workload(cfg)
    mode = P.B.MOE_FETCH_IN_KERNEL if fetch == "in_kernel" else P.B.MOE_FETCH_COPY_ENGINE
    cache = P.make_cache(wl, trace_capacity=4096, fetch_mode=mode)
    ost = OracleStack(wl, keep=min(cfg.n_experts, 16))
    worst, n_y, traces = run_sequence_serial(wl, cache, ost, torch=torch, y_every=8)
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    st = cache.moe_cache_stats()
    print("%s: worst rel err %.3e over %d tokens, hit rate %.3f" % (name, worst, n_y, st["hits"] / st["lookups"]))
    cache.close()


@pytest.mark.parametrize("fetch", ["copy_engine", "in_kernel"])
def test_launch_smaller_than_the_gpu(torch, P, fetch):
    # 2 selected experts x 32 chunks: fewer workgroups than the GPU has compute units
    cfg = get_config("olmoe_like").with_(n_experts=8, top_k=2, capacity=4, n_seqs=3, n_steps=24, pref_lo=2, pref_hi=2)
    wl = Workload(cfg)
    mode = P.B.MOE_FETCH_IN_KERNEL if fetch == "in_kernel" else P.B.MOE_FETCH_COPY_ENGINE
    cache = P.make_cache(wl, trace_capacity=4096, fetch_mode=mode)
    ost = OracleStack(wl, keep=cfg.n_experts)
    worst, n_y, traces = run_sequence_serial(wl, cache, ost, torch=torch, y_every=4)
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    assert cache.moe_cache_stats()["misses"] > 0
    cache.close()


@pytest.mark.parametrize("batch", [8, 12])
def test_mixtral_like_batched_resident_decode(torch, P, batch):
    """Several tokens per call on the Mixtral-like layer (d_ff = 14336): 8 tokens still take the single-launch
    kernel, 12 the grouped GEMM, whose down pass runs four k-blocks per step on this long contraction."""
    cfg = get_config("mixtral_like").with_(n_layers=1, n_seqs=batch, n_steps=2, capacity=8)
    wl = Workload(cfg)
    cache = P.make_cache(wl, max_batch=batch, trace_capacity=4096)
    ost = OracleStack(wl, capacity=8, keep=8)
    ids = list(range(cfg.n_experts))
    cache.moe_cache_prefill_pins(0, ids)
    ost.caches[0].pin(ids)
    trace = []
    for step in range(cfg.n_steps):
        xs = np.stack([wl.tokens(s)[step] for s in range(batch)])
        bias = np.stack([wl.bias(0, s) for s in range(batch)])
        y = torch.empty((batch, cfg.d_model), dtype=torch.bfloat16, device="cuda:0")
        idx = torch.empty((batch, cfg.top_k), dtype=torch.int32, device="cuda:0")
        cache.moe_layer_decode(0, P.to_device(xs), y, torch.from_numpy(bias).cuda(), idx, None)
        res = ost.decode(0, widen(xs), bias)
        torch.cuda.synchronize()
        assert idx.cpu().numpy().tolist() == res.idx.tolist()
        assert rel_err(P.to_numpy(y), res.y).max() <= TOL["bf16"]
        trace += res.trace
    compare_traces_and_stats(cache, ost, [trace], cfg.expert_bytes)
    cache.close()


def test_phi_like_batched_resident_decode(torch, P):
    """All 32 sequences of the Phi-like workload decode together on a resident layer: the grouped GEMM at
    d = 4096, d_ff = 6400 (100 row blocks of 64, ragged against the 128-row workgroups of larger calls)."""
    cfg = get_config("phi35_like_concentrated").with_(n_layers=1, n_steps=1, capacity=16)
    wl = Workload(cfg)
    B_ = cfg.n_seqs
    cache = P.make_cache(wl, max_batch=B_, trace_capacity=4096)
    ost = OracleStack(wl, capacity=16, keep=16)
    ids = list(range(cfg.n_experts))
    cache.moe_cache_prefill_pins(0, ids)
    ost.caches[0].pin(ids)
    xs = np.stack([wl.tokens(s)[0] for s in range(B_)])
    bias = np.stack([wl.bias(0, s) for s in range(B_)])
    y = torch.empty((B_, cfg.d_model), dtype=torch.bfloat16, device="cuda:0")
    idx = torch.empty((B_, cfg.top_k), dtype=torch.int32, device="cuda:0")
    cache.moe_layer_decode(0, P.to_device(xs), y, torch.from_numpy(bias).cuda(), idx, None)
    res = ost.decode(0, widen(xs), bias)
    torch.cuda.synchronize()
    assert idx.cpu().numpy().tolist() == res.idx.tolist()
    assert rel_err(P.to_numpy(y), res.y).max() <= TOL["bf16"]
    compare_traces_and_stats(cache, ost, [res.trace], cfg.expert_bytes)
    cache.close()


def test_deepseek_like_batched_shared_cache(torch, P):
    """Eight sequences decode together through one capacity-12 cache with two shared experts."""
    cfg = get_config("deepseek_like").with_(n_layers=1, n_seqs=8, n_steps=6)
    wl = Workload(cfg)
    B = cfg.n_seqs
    cache = P.make_cache(wl, max_batch=B, staging_buffers=B * cfg.top_k, trace_capacity=4096)
    ost = OracleStack(wl, keep=cfg.n_experts)
    y = torch.empty((B, cfg.d_model), dtype=torch.bfloat16, device="cuda:0")
    idx = torch.empty((B, cfg.top_k), dtype=torch.int32, device="cuda:0")
    bias = np.stack([wl.bias(0, s) for s in range(B)])
    bias_dev = torch.from_numpy(bias).cuda()
    trace = []
    for step in range(cfg.n_steps):
        xs = np.stack([wl.tokens(s)[step] for s in range(B)])
        cache.moe_layer_decode(0, P.to_device(xs), y, bias_dev, idx)
        res = ost.decode(0, widen(xs), bias, compute_y=step % 3 == 0)
        torch.cuda.synchronize()
        assert idx.cpu().numpy().tolist() == res.idx.tolist()
        if step % 3 == 0:
            assert rel_err(P.to_numpy(y), res.y).max() <= TOL["bf16"]
        trace += res.trace
    compare_traces_and_stats(cache, ost, [trace], cfg.expert_bytes)
    cache.close()


def test_deepseek_like_prompt_then_decode(torch, P):
    """A 512-token prompt streams through the layer (grouped GEMM, missing experts read from the host pool);
    the prefetch set is the Top-C of the mean router probability over the prompt - the activation predictor's
    own training target (section 3.1.2) standing in for the predictor; then the sequence decodes."""
    cfg = get_config("deepseek_like").with_(n_layers=1, n_seqs=1, n_steps=16)
    wl = Workload(cfg)
    cache = P.make_cache(wl, max_batch=cfg.prefill_len, trace_capacity=4096)
    ost = OracleStack(wl, keep=cfg.n_experts)
    xs = wl.prefill_tokens(0)
    n = xs.shape[0]
    bias = np.tile(wl.bias(0, 0), (n, 1))
    y = torch.empty((n, cfg.d_model), dtype=torch.bfloat16, device="cuda:0")
    idx = torch.empty((n, cfg.top_k), dtype=torch.int32, device="cuda:0")
    cache.moe_layer_prefill(0, P.to_device(xs), y, torch.from_numpy(bias).cuda(), idx)
    rows = list(range(0, n, 37))
    res = ost.prefill(0, widen(xs), bias, rows=rows)
    torch.cuda.synchronize()
    assert idx.cpu().numpy().tolist() == res.idx.tolist()
    assert rel_err(P.to_numpy(y)[rows], res.y[rows]).max() <= TOL["bf16"]
    st = cache.moe_cache_stats(0)
    assert st["stream_loads"] == ost.caches[0].stream_loads == len(set(res.idx.reshape(-1).tolist()))
    assert st["lookups"] == 0 and cache.moe_cache_resident(0) == []
    # prefetch set from the prompt's mean router probability, best expert loaded last
    score = res.p.mean(axis=0)
    pins = np.argsort(score, kind="stable")[-cfg.capacity:].astype(np.int32)
    cache.moe_cache_prefill_pins(0, pins)
    ost.caches[0].pin(pins)
    trace = []
    yd = torch.empty((1, cfg.d_model), dtype=torch.bfloat16, device="cuda:0")
    idd = torch.empty((1, cfg.top_k), dtype=torch.int32, device="cuda:0")
    toks = wl.tokens(0)
    b1 = wl.bias(0, 0)[None, :]
    b1_dev = torch.from_numpy(b1).cuda()
    for t in range(cfg.n_steps):
        cache.moe_layer_decode(0, P.to_device(toks[t:t + 1]), yd, b1_dev, idd)
        r = ost.decode(0, widen(toks[t:t + 1]), b1, compute_y=t % 4 == 0)
        torch.cuda.synchronize()
        assert idd.cpu().numpy().tolist() == r.idx.tolist()
        if t % 4 == 0:
            assert rel_err(P.to_numpy(yd), r.y).max() <= TOL["bf16"]
        trace += r.trace
    compare_traces_and_stats(cache, ost, [trace], cfg.expert_bytes)
    st = cache.moe_cache_stats(0)
    print("deepseek_like prompt+decode: streamed %d experts, decode hit rate %.3f" % (st["stream_loads"], st["hits"] / st["lookups"]))
    cache.close()
