"""GPU parity of the single-launch decode call (router, gating, cache lookups, expert FFN and combine in one
kernel, no host wait) against the oracle: batch 1 on a constrained cache with in-kernel fetch, and small batches on
a cache that holds every expert.  Routing, traces, statistics and resident sets exact; outputs within tolerance."""
import numpy as np
import pytest

from tests.helpers import TOL, OracleStack, compare_traces_and_stats, rel_err, run_sequence_serial
from tests.test_gpu_parity import batched_step, small_cfg
from workload import Workload, widen

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


def timing_counts(cache, fn):
    """Run fn with kernel timing on and return how many calls went through the single launch."""
    cache.moe_cache_set_profiling(True)
    cache.moe_cache_timing(clear=True)
    fn()
    tm = cache.moe_cache_timing(clear=True)
    cache.moe_cache_set_profiling(False)
    return tm


# experts, top-k, capacity, shared, d_model, d_ff: one and several logit tiles, shared experts, both wave counts
SHAPES = [(16, 4, 6, 0, 256, 96), (8, 2, 3, 0, 512, 128), (64, 8, 16, 0, 256, 64), (40, 6, 12, 2, 256, 96),
          (128, 4, 9, 0, 256, 64), (16, 2, 2, 1, 1024, 2048),
          # more than 256 chunk workgroups per call: the tile kernel (one workgroup per compute unit, two or three
          # 16-row tiles each, k-blocks shared between neighbours)
          (16, 4, 6, 1, 256, 2400), (8, 2, 3, 0, 512, 5760), (16, 8, 10, 2, 1024, 1152)]


@pytest.mark.parametrize("E,K,cap,ns,d,f", SHAPES)
@pytest.mark.parametrize("pins", [True, False])
def test_batch1_constrained_cache(torch, P, E, K, cap, ns, d, f, pins):
    B = P.B
    cfg = small_cfg(n_experts=E, top_k=K, capacity=cap, n_shared=ns, d_model=d, d_ff=f, n_layers=2, n_seqs=3,
                    n_steps=20, pref_lo=min(K, 4), pref_hi=min(K + 1, E), beta=1.5, cfg_id=41)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, trace_capacity=8192, fetch_mode=B.MOE_FETCH_IN_KERNEL)
    ost = OracleStack(wl, keep=min(E, 24))
    worst, n_y, traces = run_sequence_serial(wl, cache, ost, torch=torch, pins=pins, y_every=1 if f < 512 else 5)
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    st = cache.moe_cache_stats()
    assert st["misses"] > 0 and st["hits"] > 0 and st["hits"] + st["misses"] == st["lookups"]
    # and the calls really were single launches
    x = P.to_device(wl.tokens(0)[:1])
    y = torch.empty((1, d), dtype=torch.bfloat16, device="cuda:0")
    tm = timing_counts(cache, lambda: [cache.moe_layer_decode(0, x, y) for _ in range(4)])
    assert tm["decode_single_launches"] + tm["fetch_launches"] == 4 and tm["route_launches"] == 0
    # more chunk workgroups than compute units: the resident calls among them ran the tile kernel
    assert tm["decode_tiles_launches"] == (tm["decode_single_launches"] if (f // 32) * (K + ns) > 256 else 0)
    cache.close()


@pytest.mark.parametrize("batch", [2, 4, 5])
@pytest.mark.parametrize("E,K,ns,d,f", [(16, 4, 0, 256, 96), (64, 8, 0, 512, 64), (24, 3, 2, 256, 128)])
def test_small_batches_on_a_cache_that_holds_everything(torch, P, batch, E, K, ns, d, f):
    B = P.B
    cfg = small_cfg(n_experts=E, top_k=K, capacity=E, n_shared=ns, d_model=d, d_ff=f, n_layers=1, n_seqs=6,
                    n_steps=10, cfg_id=42)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, max_batch=batch, trace_capacity=8192, fetch_mode=B.MOE_FETCH_IN_KERNEL)
    ost = OracleStack(wl, keep=E)
    traces = [[]]
    for step in range(cfg.n_steps):         # starts empty: the first calls fetch inside the launch
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, list(range(batch)), step))
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    x = P.to_device(np.stack([wl.tokens(s)[0] for s in range(batch)]))
    y = torch.empty((batch, d), dtype=torch.bfloat16, device="cuda:0")
    tm = timing_counts(cache, lambda: [cache.moe_layer_decode(0, x, y) for _ in range(3)])
    if batch <= 4:          # the single launch takes up to four tokens; larger calls route in a kernel of their own
        assert tm["decode_single_launches"] + tm["fetch_launches"] == 3 and tm["route_launches"] == 0
    else:
        assert tm["decode_single_launches"] == 0 and tm["route_launches"] == 3
    cache.close()


@pytest.mark.parametrize("E,K,d,f", [(64, 8, 2048, 1024), (8, 2, 512, 5760)], ids=["chunk kernel", "tile kernel"])
def test_results_do_not_depend_on_timing(torch, P, E, K, d, f):
    """The partial sums are added in a fixed order (in LDS, then by the combine): repeated calls give identical bits."""
    B = P.B
    cfg = small_cfg(n_experts=E, top_k=K, capacity=E, d_model=d, d_ff=f, n_layers=1, n_seqs=2, n_steps=2,
                    cfg_id=43)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, fetch_mode=B.MOE_FETCH_IN_KERNEL)
    cache.moe_cache_prefill_pins(0, list(range(E)))
    x = P.to_device(wl.tokens(0)[:1])
    ys = []
    for _ in range(20):
        y = torch.empty((1, cfg.d_model), dtype=torch.bfloat16, device="cuda:0")
        cache.moe_layer_decode(0, x, y)
        ys.append(y)
    torch.cuda.synchronize()
    for y in ys[1:]:
        assert torch.equal(y.view(torch.int16), ys[0].view(torch.int16))
    ost = OracleStack(wl, capacity=E, keep=E)
    res = ost.decode(0, widen(wl.tokens(0)[:1]), None)
    assert float(rel_err(P.to_numpy(ys[0]), res.y)[0]) <= TOL["bf16"]
    cache.close()


def test_mixing_single_launch_calls_with_the_other_paths(torch, P):
    """Batch 1 (single launch), a batch of 9 (router kernel + grouped GEMM) and prefill_pins alternate on one
    cache: all of them read and write the same table."""
    B = P.B
    cfg = small_cfg(n_experts=16, top_k=4, capacity=16, d_model=256, d_ff=96, n_layers=1, n_seqs=9, n_steps=12,
                    cfg_id=44)
    wl = Workload(cfg)
    cache = P.make_cache(wl, tiled=True, max_batch=9, trace_capacity=8192, fetch_mode=B.MOE_FETCH_IN_KERNEL)
    ost = OracleStack(wl, capacity=16, keep=16)
    traces = [[]]
    for step in range(cfg.n_steps):
        if step == 5:
            cache.moe_cache_prefill_pins(0, [1, 3, 5])
            ost.caches[0].pin([1, 3, 5])
        rows = list(range(9)) if step % 3 == 2 else [step % 9] if step % 3 == 0 else [1, 4, 7]
        traces[0].extend(batched_step(torch, P, wl, cache, ost, 0, rows, step))
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    cache.close()


@pytest.mark.parametrize("E,K,cap,ns,d,f", [(16, 4, 6, 0, 256, 96), (64, 8, 16, 0, 512, 64), (24, 3, 7, 2, 256, 128)])
def test_int4_batch1_constrained_cache(torch, P, E, K, cap, ns, d, f):
    """The same single launch on 4-bit experts (values compared with the oracle's own dequantisation)."""
    B = P.B
    cfg = small_cfg(n_experts=E, top_k=K, capacity=cap, n_shared=ns, d_model=d, d_ff=f, n_layers=2, n_seqs=3,
                    n_steps=16, pref_lo=min(K, 4), pref_hi=min(K + 1, E), beta=1.5, cfg_id=45)
    wl = Workload(cfg)
    cache = P.make_cache(wl, int4=True, trace_capacity=8192, fetch_mode=B.MOE_FETCH_IN_KERNEL)
    ost = OracleStack(wl, keep=min(E, 24), int4=True)
    _, _, traces = run_sequence_serial(wl, cache, ost, torch=torch, pins=True)
    compare_traces_and_stats(cache, ost, traces, P.int4_block_bytes(cfg))
    assert cache.moe_cache_stats()["misses"] > 0
    x = P.to_device(wl.tokens(0)[:1])
    y = torch.empty((1, d), dtype=torch.bfloat16, device="cuda:0")
    tm = timing_counts(cache, lambda: [cache.moe_layer_decode(0, x, y) for _ in range(4)])
    assert tm["decode_single_launches"] + tm["fetch_launches"] == 4 and tm["route_launches"] == 0
    cache.close()
