"""MI355X parity of the decode path on 4-bit group-quantised experts (section 3.2 keeps experts in INT4): the HIP
path sees packed codes and scales, the oracle sees its own dequantisation of the same codes and scales."""
import numpy as np
import pytest

import oracle
from tests.helpers import OracleStack, compare_traces_and_stats, run_sequence_serial
from tests.test_gpu_parity import batched_step, small_cfg
from workload import Workload, get_config

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


def q4_bytes(cfg):
    return oracle.expert_bytes_int4(cfg.d_model, cfg.d_ff)


@pytest.mark.parametrize("fetch", ["copy_engine", "in_kernel"])
@pytest.mark.parametrize("d_model,d_ff", [(256, 96), (512, 64), (768, 32), (1024, 160)])
def test_int4_sequence_serial(torch, P, fetch, d_model, d_ff):
    from paper_2602_11192_amd import binding as B
    cfg = small_cfg(d_model=d_model, d_ff=d_ff, n_seqs=2, n_steps=16, beta=1.0)
    wl = Workload(cfg)
    mode = B.MOE_FETCH_IN_KERNEL if fetch == "in_kernel" else B.MOE_FETCH_COPY_ENGINE
    cache = P.make_cache(wl, int4=True, trace_capacity=4096, fetch_mode=mode)
    ost = OracleStack(wl, int4=True)
    worst, n_y, traces = run_sequence_serial(wl, cache, ost, torch=torch)
    assert n_y == cfg.n_seqs * cfg.n_steps * cfg.n_layers
    st = cache.moe_cache_stats()
    assert st["misses"] > 5 and st["bytes_h2d"] == (st["misses"] + st["pin_loads"]) * q4_bytes(cfg)
    compare_traces_and_stats(cache, ost, traces, q4_bytes(cfg))
    cache.close()


@pytest.mark.parametrize("fetch", ["copy_engine", "in_kernel"])
@pytest.mark.parametrize("batch", [2, 5, 16])
def test_int4_batched_with_shared_experts(torch, P, fetch, batch):
    from paper_2602_11192_amd import binding as B
    cfg = small_cfg(d_model=512, d_ff=96, n_seqs=16, n_steps=6, n_layers=1, capacity=7, n_shared=2)
    wl = Workload(cfg)
    mode = B.MOE_FETCH_IN_KERNEL if fetch == "in_kernel" else B.MOE_FETCH_COPY_ENGINE
    cache = P.make_cache(wl, int4=True, max_batch=batch, staging_buffers=batch * cfg.top_k, trace_capacity=8192,
                         fetch_mode=mode)
    ost = OracleStack(wl, int4=True)
    traces = [[]]
    for step in range(cfg.n_steps):
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, list(range(batch)), step))
    compare_traces_and_stats(cache, ost, traces, q4_bytes(cfg))
    cache.close()


def test_int4_limits_are_reported(torch, P):
    from paper_2602_11192_amd import binding as B
    with pytest.raises(B.MoeError):
        P.make_cache(Workload(small_cfg(d_model=128, d_ff=96)), int4=True)      # d_model % 256 != 0
    assert B.moe_expert_block_bytes(256, 48, B.MOE_DTYPE_BF16, B.MOE_LAYOUT_TILED_INT4) == 0    # d_ff % 32 != 0


@pytest.mark.parametrize("d_model,d_ff", [(256, 96), (512, 160)])
@pytest.mark.parametrize("batch", [17, 40, 150])
def test_int4_many_tokens_take_the_grouped_gemm(torch, P, d_model, d_ff, batch):
    # more than 16 tokens per call: the 4-bit grouped GEMM (up to several token tiles per expert, ragged tails)
    cfg = small_cfg(d_model=d_model, d_ff=d_ff, n_experts=8, top_k=2, n_seqs=150, n_steps=3, n_layers=1, capacity=8,
                    n_shared=1, beta=1.0)
    wl = Workload(cfg)
    cache = P.make_cache(wl, int4=True, max_batch=batch, trace_capacity=4096)
    ost = OracleStack(wl, int4=True, capacity=8, keep=16)
    traces = [[]]
    for step in range(cfg.n_steps):
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, list(range(batch)), step))
    compare_traces_and_stats(cache, ost, traces, q4_bytes(cfg))
    cache.close()


def test_int4_batched_gemm_with_evictions(torch, P):
    # constrained cache, 24 tokens per call: copy-engine fetches, then the grouped GEMM over the fetched experts
    cfg = small_cfg(d_model=256, d_ff=96, n_seqs=24, n_steps=5, n_layers=1, capacity=6)
    wl = Workload(cfg)
    cache = P.make_cache(wl, int4=True, max_batch=24, staging_buffers=10, trace_capacity=8192)
    ost = OracleStack(wl, int4=True)
    traces = [[]]
    for step in range(cfg.n_steps):
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, list(range(24)), step))
    assert cache.moe_cache_stats(0)["evictions"] > 10
    compare_traces_and_stats(cache, ost, traces, q4_bytes(cfg))
    cache.close()


@pytest.mark.parametrize("n_tokens", [1, 37, 200])
def test_int4_prompt_streaming(torch, P, n_tokens):
    from tests.helpers import TOL, rel_err
    from workload import widen
    cfg = small_cfg(n_seqs=2, n_steps=6, n_layers=1, capacity=6, n_shared=1, prefill_len=n_tokens, d_model=256,
                    d_ff=96)
    wl = Workload(cfg)
    cache = P.make_cache(wl, int4=True, max_batch=max(n_tokens, 2), trace_capacity=4096)
    ost = OracleStack(wl, int4=True)
    pins = wl.prefetch_list(0, 0)[:4]
    cache.moe_cache_prefill_pins(0, pins)
    ost.caches[0].pin(pins)
    xs = wl.prefill_tokens(0)
    bias = np.tile(wl.bias(0, 0), (n_tokens, 1))
    y = torch.empty((n_tokens, cfg.d_model), dtype=torch.bfloat16, device="cuda:0")
    idx = torch.empty((n_tokens, cfg.top_k), dtype=torch.int32, device="cuda:0")
    for _ in range(2):
        cache.moe_layer_prefill(0, P.to_device(xs), y, torch.from_numpy(bias).cuda(), idx)
        res = ost.prefill(0, widen(xs), bias)
        torch.cuda.synchronize()
        assert idx.cpu().numpy().tolist() == res.idx.tolist()
        assert rel_err(P.to_numpy(y), res.y).max() <= TOL["bf16"]
    traces = [[]]
    for step in range(cfg.n_steps):
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, [0], step))
    compare_traces_and_stats(cache, ost, traces, q4_bytes(cfg))
    cache.close()


def test_int4_olmoe_like_sampled(torch, P):
    # full-size layer of the OLMoE-like workload with 4-bit experts: two sequences, outputs checked every 8th step
    from paper_2602_11192_amd import binding as B
    cfg = get_config("olmoe_like")
    wl = Workload(cfg)
    cache = P.make_cache(wl, int4=True, trace_capacity=1 << 16, fetch_mode=B.MOE_FETCH_IN_KERNEL)
    ost = OracleStack(wl, int4=True, keep=64)
    worst, n_y, traces = run_sequence_serial(wl, cache, ost, torch=torch, seqs=[0, 1], steps=64, y_every=8)
    print("int4 olmoe_like worst rel err", worst, "outputs", n_y)
    compare_traces_and_stats(cache, ost, traces, q4_bytes(cfg))
    cache.close()


def test_two_caches_interleaved_on_a_side_stream(torch, P):
    # two independent caches (bf16 with in-kernel fetch, 4-bit with the copy engine) driven alternately on a
    # non-default stream: no state may leak between them
    from paper_2602_11192_amd import binding as B
    cfg_a = small_cfg(cfg_id=21, d_model=256, d_ff=96, n_layers=1, n_seqs=4, n_steps=10, beta=1.0)
    cfg_b = small_cfg(cfg_id=22, d_model=512, d_ff=64, n_layers=1, n_seqs=4, n_steps=10, capacity=5, n_shared=1)
    wl_a, wl_b = Workload(cfg_a), Workload(cfg_b)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        cache_a = P.make_cache(wl_a, tiled=True, max_batch=2, staging_buffers=8, trace_capacity=2048,
                               fetch_mode=B.MOE_FETCH_IN_KERNEL)
        cache_b = P.make_cache(wl_b, int4=True, max_batch=2, staging_buffers=8, trace_capacity=2048)
        ost_a, ost_b = OracleStack(wl_a), OracleStack(wl_b, int4=True)
        tr_a, tr_b = [[]], [[]]
        for step in range(cfg_a.n_steps):
            rows = [0, 1] if step % 3 else [2]
            tr_a[0].extend(batched_step(torch, P, wl_a, cache_a, ost_a, 0, rows, step))
            tr_b[0].extend(batched_step(torch, P, wl_b, cache_b, ost_b, 0, rows[::-1], step))
        compare_traces_and_stats(cache_a, ost_a, tr_a, cfg_a.expert_bytes)
        compare_traces_and_stats(cache_b, ost_b, tr_b, q4_bytes(cfg_b))
        cache_a.close()
        cache_b.close()
