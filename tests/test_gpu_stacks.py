"""GPU parity over the stated schedules of the three large configurations, cut to four layers (their full pools do
not fit the host's pinned memory): EVERY sequence and EVERY decode step goes through the library and the oracle;
routing, gate weights, the cache trace, the statistics and the resident sets of every layer must match exactly,
outputs are compared on a subsample (the oracle's fp64 expert FFN at these widths takes a second per token).
Then the DeepSeekMoE-like schedule as written: per sequence a 512-token prompt streamed through the layers, the
prefetch set taken from the prompt's mean router probability, then the decode steps."""
import numpy as np
import pytest

from tests.helpers import (TOL, WORST_ELEMENTWISE, OracleStack, compare_traces_and_stats, elementwise_excess, rel_err,
                           run_sequence_serial)
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


# name, step stride of the output checks (layer 0, sequences 0 and 1; every call is checked for routing and trace)
STACKS = [("mixtral_like", 32), ("phi35_like_concentrated", 16), ("phi35_like_diverse", 16), ("deepseek_like", 8)]


@pytest.mark.parametrize("name,y_every", STACKS)
def test_every_token_of_four_layers(torch, P, name, y_every):
    cfg = get_config(name).with_(n_layers=4)
    wl = Workload(cfg)
    print("%s: %d sequences x %d steps x %d layers" % (name, cfg.n_seqs, cfg.n_steps, cfg.n_layers), flush=True)
    lookups = cfg.n_seqs * cfg.n_steps * cfg.top_k
    cache = P.make_cache(wl, trace_capacity=lookups, fetch_mode=P.B.MOE_FETCH_IN_KERNEL)
    ost = OracleStack(wl, keep=cfg.n_experts)
    WORST_ELEMENTWISE["value"] = 0.0
    worst, n_y, traces = run_sequence_serial(wl, cache, ost, torch=torch, y_every=y_every, y_layers=(0,),
                                             y_seqs=(0, 1))
    assert n_y == 2 * ((cfg.n_steps + y_every - 1) // y_every)
    assert all(len(tr) == lookups for tr in traces)
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    st = cache.moe_cache_stats()
    assert st["lookups"] == lookups * cfg.n_layers and st["hits"] + st["misses"] == st["lookups"]
    print("%s: %d lookups, hit rate %.3f, %d outputs compared, worst error %.2e of the row maximum, "
          "worst element-wise error %.2f of its allowance (2e-2 |ref_i| + 2e-2 rms(ref))"
          % (name, st["lookups"], st["hits"] / st["lookups"], n_y, worst, WORST_ELEMENTWISE["value"]), flush=True)
    cache.close()


def test_deepseek_like_schedule_as_written(torch, P):
    """Per sequence: empty caches -> the 512-token prompt through every layer in streaming mode -> per layer the
    Top-C of the prompt's mean router probability (the predictor's training target, section 3.1.2) is preloaded ->
    64 decode steps.  Four sequences, two layers."""
    B = P.B
    cfg = get_config("deepseek_like").with_(n_layers=2, n_seqs=4)
    wl = Workload(cfg)
    L, K, d, C = cfg.n_layers, cfg.top_k, cfg.d_model, cfg.capacity
    n_p = cfg.prefill_len
    cache = P.make_cache(wl, max_batch=n_p, trace_capacity=cfg.n_seqs * cfg.n_steps * K,
                         fetch_mode=B.MOE_FETCH_IN_KERNEL)
    ost = OracleStack(wl, keep=cfg.n_experts)
    yp = torch.empty((n_p, d), dtype=torch.bfloat16, device="cuda:0")
    ip = torch.empty((n_p, K), dtype=torch.int32, device="cuda:0")
    yd = torch.empty((1, d), dtype=torch.bfloat16, device="cuda:0")
    idd = torch.empty((1, K), dtype=torch.int32, device="cuda:0")
    gwd = torch.empty((1, K), dtype=torch.float32, device="cuda:0")
    traces = [[] for _ in range(L)]
    streamed = 0
    for s in range(cfg.n_seqs):
        print("deepseek_like schedule: sequence %d" % s, flush=True)
        cache.moe_cache_reset(-1)
        for c in ost.caches:
            c.reset()
        xs = wl.prefill_tokens(s)
        xs_dev, xs32 = P.to_device(xs), widen(xs)
        rows = list(range(s, n_p, 97))
        for l in range(L):
            bias = np.tile(wl.bias(l, s), (n_p, 1))
            cache.moe_layer_prefill(l, xs_dev, yp, torch.from_numpy(bias).cuda(), ip)
            res = ost.prefill(l, xs32, bias, rows=rows if l == 0 else [])
            torch.cuda.synchronize()
            assert ip.cpu().numpy().tolist() == res.idx.tolist(), (s, l)
            if l == 0:
                assert rel_err(P.to_numpy(yp)[rows], res.y[rows]).max() <= TOL["bf16"]
            streamed += len(set(res.idx.reshape(-1).tolist()))          # the cache is empty during the prompt
            assert cache.moe_cache_resident(l) == []
            pins = B.moe_pooled_prefetch_set(res.p.mean(axis=0, keepdims=True).astype(np.float32), C)
            cache.moe_cache_prefill_pins(l, pins)
            ost.caches[l].pin(pins)
        toks = wl.tokens(s)
        t_dev, t32 = P.to_device(toks), widen(toks)
        b1 = [wl.bias(l, s)[None, :] for l in range(L)]
        b1_dev = [torch.from_numpy(b).cuda() for b in b1]
        for t in range(cfg.n_steps):
            for l in range(L):
                want_y = l == 0 and t % 16 == 0
                cache.moe_layer_decode(l, t_dev[t:t + 1], yd, b1_dev[l], idd, gwd)
                r = ost.decode(l, t32[t:t + 1], b1[l], compute_y=want_y)
                torch.cuda.synchronize()
                assert idd.cpu().numpy().tolist() == r.idx.tolist(), (s, t, l)
                np.testing.assert_allclose(gwd.cpu().numpy(), r.w, rtol=0, atol=2e-5)
                if want_y:
                    assert rel_err(P.to_numpy(yd), r.y).max() <= TOL["bf16"]
                    assert elementwise_excess(P.to_numpy(yd), r.y, TOL["bf16"]).max() <= 1.0
                traces[l] += r.trace
    compare_traces_and_stats(cache, ost, traces, cfg.expert_bytes)
    st = cache.moe_cache_stats()
    assert st["stream_loads"] == streamed and st["pin_loads"] == cfg.n_seqs * L * C
    assert st["lookups"] == cfg.n_seqs * cfg.n_steps * K * L
    print("deepseek_like schedule: %d experts streamed by the prompts, decode hit rate %.3f"
          % (st["stream_loads"], st["hits"] / st["lookups"]), flush=True)
    cache.close()
