"""The entry point that allocates nothing (moe_layer_decode_resident_noalloc) against moe_layer_decode on a cache
that holds every expert: same kernels, so routing, gate weights and outputs must be bit-identical; one call is also
checked against the oracle.  Every case makes calls in a row on the shared device array, later ones smaller."""
import numpy as np
import pytest

from tests.helpers import TOL, OracleStack, rel_err
from workload import MoEConfig, Workload, widen

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


def cfg_of(**kw):
    base = dict(name="noalloc_bf16", cfg_id=31, dtype="bf16", n_layers=1, d_model=256, d_ff=128, n_experts=16,
                n_shared=0, top_k=4, capacity=16, n_seqs=40, n_steps=2, prefill_len=0, beta=2.0, pref_lo=4,
                pref_hi=4, delta=1e-3)
    base.update(kw)
    return MoEConfig(**base)


CASES = [
    ("bf16 tiled", cfg_of(), True, False, [40, 3, 1]),              # grouped GEMM, then the single-launch kernel
    ("bf16 tiled + shared", cfg_of(cfg_id=32, n_shared=2, top_k=3), True, False, [5, 2]),
    ("bf16 row-major", cfg_of(cfg_id=33, d_ff=96), False, False, [7, 1]),
    ("fp32 row-major", cfg_of(cfg_id=34, dtype="fp32", d_model=64, delta=1e-5), False, False, [9, 4]),
    ("int4", cfg_of(cfg_id=35), True, True, [20, 16, 2]),
]


@pytest.mark.parametrize("name,cfg,tiled,int4,batches", CASES, ids=[c[0] for c in CASES])
def test_noalloc_equals_cached_decode(torch, P, name, cfg, tiled, int4, batches):
    B = P.B
    wl = Workload(cfg)
    E, K, d = cfg.n_experts, cfg.top_k, cfg.d_model
    pool = P.build_pool(wl, tiled, int4=int4)
    experts_dev = pool.cuda()
    router = P.build_router(wl)
    shared = P.build_shared(wl, tiled, int4=int4)
    cache = P.make_cache(wl, tiled=tiled, pool=pool, capacity=E, max_batch=max(batches), int4=int4)
    cache.moe_cache_prefill_pins(0, list(range(E)))
    layout = B.MOE_LAYOUT_TILED_INT4 if int4 else B.MOE_LAYOUT_TILED if tiled else B.MOE_LAYOUT_ROWMAJOR
    toks = np.stack([wl.tokens(s)[0] for s in range(cfg.n_seqs)])
    bias = np.stack([wl.bias(0, s) for s in range(cfg.n_seqs)])
    tdt = P.torch_dtype(cfg)
    ost = OracleStack(wl, capacity=E, int4=int4)
    for i, bsz in enumerate(batches):
        print("noalloc case %s batch %d" % (name, bsz), flush=True)
        rows = slice(i, i + bsz)
        x = P.to_device(toks[rows])
        b = torch.from_numpy(bias[rows].copy()).cuda()
        y0 = torch.empty((bsz, d), dtype=tdt, device="cuda:0")
        y1 = torch.full((bsz, d), 7.0, dtype=tdt, device="cuda:0")
        i0 = torch.empty((bsz, K), dtype=torch.int32, device="cuda:0")
        i1 = torch.full((bsz, K), -1, dtype=torch.int32, device="cuda:0")
        w0 = torch.empty((bsz, K), dtype=torch.float32, device="cuda:0")
        w1 = torch.full((bsz, K), -1.0, dtype=torch.float32, device="cuda:0")
        cache.moe_layer_decode(0, x, y0, b, i0, w0)
        B.moe_layer_decode_resident_noalloc(
            n_experts=E, n_shared=cfg.n_shared, top_k=K, d_model=d, d_ff=cfg.d_ff, dtype=P.moe_dtype(cfg),
            norm_topk=cfg.norm_topk, pool_layout=layout, router_w=router, experts=experts_dev, shared_w=shared,
            x=x, y=y1, logit_bias=b, topk_idx=i1, topk_w=w1)
        torch.cuda.synchronize()
        assert torch.equal(i0, i1)
        assert torch.equal(w0, w1)
        assert torch.equal(y0.view(torch.int16 if tdt == torch.bfloat16 else torch.int32),
                           y1.view(torch.int16 if tdt == torch.bfloat16 else torch.int32))
        if i == 0:      # and the values themselves, against the oracle
            res = ost.decode(0, widen(toks[rows]), bias[rows])
            assert i1.cpu().numpy().tolist() == res.idx.tolist()
            assert float(rel_err(P.to_numpy(y1), res.y).max()) <= TOL[cfg.dtype]
    cache.close()


def test_noalloc_beside_the_tile_kernel(torch, P):
    """A one-token call on large experts: the cached decode runs its tile kernel, this entry point the chunk kernel.
    Same routing bit for bit; the outputs differ at most by the order of the fp32 partial sums."""
    B = P.B
    cfg = cfg_of(cfg_id=37, d_model=512, d_ff=5760, n_experts=8, top_k=2, capacity=8, n_seqs=4, pref_lo=2, pref_hi=2)
    wl = Workload(cfg)
    E, K, d = cfg.n_experts, cfg.top_k, cfg.d_model
    pool = P.build_pool(wl, True)
    experts_dev = pool.cuda()
    router = P.build_router(wl)
    cache = P.make_cache(wl, tiled=True, pool=pool, capacity=E, fetch_mode=B.MOE_FETCH_IN_KERNEL)
    cache.moe_cache_prefill_pins(0, list(range(E)))
    ost = OracleStack(wl, capacity=E)
    for s in range(cfg.n_seqs):
        print("noalloc beside the tile kernel, sequence %d" % s, flush=True)
        tok = wl.tokens(s)[:1]
        x = P.to_device(tok)
        y0 = torch.empty((1, d), dtype=torch.bfloat16, device="cuda:0")
        y1 = torch.full((1, d), 7.0, dtype=torch.bfloat16, device="cuda:0")
        i0 = torch.empty((1, K), dtype=torch.int32, device="cuda:0")
        i1 = torch.full((1, K), -1, dtype=torch.int32, device="cuda:0")
        w0 = torch.empty((1, K), dtype=torch.float32, device="cuda:0")
        w1 = torch.full((1, K), -1.0, dtype=torch.float32, device="cuda:0")
        cache.moe_cache_set_profiling(True)
        cache.moe_cache_timing(clear=True)
        cache.moe_layer_decode(0, x, y0, None, i0, w0)
        tm = cache.moe_cache_timing(clear=True)
        cache.moe_cache_set_profiling(False)
        assert tm["decode_tiles_launches"] == 1
        B.moe_layer_decode_resident_noalloc(
            n_experts=E, n_shared=0, top_k=K, d_model=d, d_ff=cfg.d_ff, dtype=P.moe_dtype(cfg),
            norm_topk=cfg.norm_topk, pool_layout=B.MOE_LAYOUT_TILED, router_w=router, experts=experts_dev,
            shared_w=None, x=x, y=y1, logit_bias=None, topk_idx=i1, topk_w=w1)
        torch.cuda.synchronize()
        assert torch.equal(i0, i1) and torch.equal(w0, w1)
        res = ost.decode(0, widen(tok), None)
        assert float(rel_err(P.to_numpy(y0), res.y).max()) <= TOL["bf16"]
        assert float(rel_err(P.to_numpy(y1), res.y).max()) <= TOL["bf16"]
        assert float(rel_err(P.to_numpy(y1), P.to_numpy(y0).astype(np.float64)).max()) <= TOL["bf16"]
    cache.close()


def test_noalloc_rejects_what_does_not_fit(torch, P):
    B = P.B
    cfg = cfg_of(cfg_id=36)
    wl = Workload(cfg)
    pool = P.build_pool(wl, True)
    experts_dev = pool.cuda()
    router = P.build_router(wl)
    n = 1 << 16                    # 65536 tokens x 4 experts x 256 fp32 outputs exceed the 32 MiB array
    x = torch.zeros((n, cfg.d_model), dtype=torch.bfloat16, device="cuda:0")
    y = torch.zeros_like(x)
    with pytest.raises(B.MoeError) as ei:
        B.moe_layer_decode_resident_noalloc(
            n_experts=cfg.n_experts, top_k=cfg.top_k, d_model=cfg.d_model, d_ff=cfg.d_ff, dtype=B.MOE_DTYPE_BF16,
            pool_layout=B.MOE_LAYOUT_TILED, router_w=router, experts=experts_dev, x=x, y=y)
    assert ei.value.code == B.MOE_ERR_UNSUPPORTED and "scratch" in str(ei.value)
