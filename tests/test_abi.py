"""CPU-only checks of the C ABI: the library loads, exports every function the
header declares, validates arguments before touching the GPU, and its host-side
helpers (byte model, tiled-layout permutation) are right."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2602_11192_amd import binding
    return binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "moe_cache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(B):
    names = declared_functions()
    assert {"moe_cache_create", "moe_cache_prefill_pins", "moe_layer_decode", "moe_cache_stats"} <= set(names)
    for n in names:
        assert hasattr(B.lib, n), n
    assert sorted(B.EXPORTS) == names
    assert "gfx950" in B.moe_version()


def test_struct_sizes_match_header(B):
    assert C.sizeof(B.moe_cache_config_t) == 16 * 4 + 8
    assert C.sizeof(B.moe_cache_stats_t) == 64
    assert C.sizeof(B.moe_trace_rec_t) == 16
    assert C.sizeof(B.moe_weights_t) == 32


def test_expert_bytes(B):
    assert B.moe_expert_bytes(4096, 14336, B.MOE_DTYPE_BF16) == 352_321_536
    assert B.moe_expert_bytes(64, 128, B.MOE_DTYPE_FP32) == 98_304
    assert B.moe_expert_bytes(0, 128, B.MOE_DTYPE_FP32) == 0
    assert B.moe_expert_bytes(64, 128, 7) == 0


def good_cfg(B, **kw):
    f = dict(n_layers=1, n_experts=8, n_shared=0, top_k=2, d_model=64, d_ff=128, capacity=2, dtype=B.MOE_DTYPE_FP32,
             norm_topk=1, policy=B.MOE_POLICY_LRU, max_batch=1, staging_buffers=0, device_id=-1, trace_capacity=0,
             pool_layout=B.MOE_LAYOUT_ROWMAJOR, fetch_mode=0, gamma=1.0)
    f.update(kw)
    return B.moe_cache_config_t(**f)


def create(B, cfg, router=0x1000, pool=0x2000, shared=None):
    w = B.moe_weights_t(router, pool, shared)
    h = C.c_void_p()
    rc = B.lib.moe_cache_create(C.byref(cfg), C.byref(w), C.byref(h))
    assert not h.value or rc == 0
    return rc, h


@pytest.mark.parametrize("kw,code", [
    (dict(n_layers=0), "MOE_ERR_INVALID_ARG"), (dict(n_experts=0), "MOE_ERR_INVALID_ARG"),
    (dict(n_experts=2000), "MOE_ERR_INVALID_ARG"), (dict(top_k=0), "MOE_ERR_INVALID_ARG"),
    (dict(top_k=9), "MOE_ERR_INVALID_ARG"), (dict(capacity=1), "MOE_ERR_CAPACITY_LT_TOPK"),
    (dict(capacity=0), "MOE_ERR_INVALID_ARG"), (dict(dtype=3), "MOE_ERR_INVALID_ARG"),
    (dict(policy=5), "MOE_ERR_INVALID_ARG"), (dict(policy=1, gamma=1.5), "MOE_ERR_INVALID_ARG"),
    (dict(max_batch=0), "MOE_ERR_INVALID_ARG"), (dict(staging_buffers=-1), "MOE_ERR_INVALID_ARG"),
    (dict(trace_capacity=-1), "MOE_ERR_INVALID_ARG"), (dict(fetch_mode=2), "MOE_ERR_INVALID_ARG"),
    (dict(fetch_mode=1), "MOE_ERR_UNSUPPORTED"),               # in-kernel fetch needs the tiled bf16 layout
    (dict(pool_layout=1), "MOE_ERR_UNSUPPORTED"),              # tiled needs bf16
    (dict(dtype=1, pool_layout=1, d_ff=100), "MOE_ERR_UNSUPPORTED"),
    (dict(d_model=66), "MOE_ERR_UNSUPPORTED"), (dict(norm_topk=2), "MOE_ERR_INVALID_ARG"),
    (dict(n_shared=1), "MOE_ERR_INVALID_ARG"),                 # shared_w missing
])
def test_create_rejects_bad_config_before_touching_the_gpu(B, kw, code):
    rc, _ = create(B, good_cfg(B, **kw))
    assert rc == getattr(B, code), B.moe_last_error()
    assert B.moe_last_error()


def test_create_null_and_misaligned_pointers(B):
    cfg = good_cfg(B)
    assert create(B, cfg, router=None)[0] == B.MOE_ERR_INVALID_ARG
    assert create(B, cfg, pool=None)[0] == B.MOE_ERR_INVALID_ARG
    assert create(B, cfg, router=0x1004)[0] == B.MOE_ERR_INVALID_ARG
    assert B.lib.moe_cache_create(None, None, None) == B.MOE_ERR_INVALID_ARG


def test_null_handles_are_errors_not_crashes(B):
    st = B.moe_cache_stats_t()
    assert B.lib.moe_cache_stats(None, 0, C.byref(st)) == B.MOE_ERR_INVALID_ARG
    assert B.lib.moe_layer_decode(None, 0, None, None, 1, None, None, None, None) == B.MOE_ERR_INVALID_ARG
    assert B.lib.moe_cache_prefill_pins(None, 0, None, 0, None) == B.MOE_ERR_INVALID_ARG
    assert B.lib.moe_cache_reset(None, 0, 0, None) == B.MOE_ERR_INVALID_ARG
    assert B.lib.moe_cache_destroy(None) == B.MOE_OK


def test_valid_config_without_gpu_fails_loudly(B):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    rc, _ = create(B, good_cfg(B))
    assert rc == B.MOE_ERR_HIP and "HIP" in B.moe_last_error()


def test_pack_expert_is_the_documented_permutation(B):
    d, f = 64, 96
    src = np.arange(3 * d * f, dtype=np.uint32).astype(np.uint16)        # distinct enough per neighbourhood
    rng = np.random.default_rng(0)
    src = rng.integers(0, 65536, size=3 * d * f, dtype=np.uint16)
    dst = np.zeros_like(src)
    B.moe_pack_expert(src, dst, d, f)
    wg, wu, wd = src[:f * d].reshape(f, d), src[f * d:2 * f * d].reshape(f, d), src[2 * f * d:].reshape(d, f)
    gu = dst[:2 * f * d].reshape(f // 16, d // 32, 2, 64, 8)
    dn = dst[2 * f * d:].reshape(f // 32, d // 16, 64, 8)
    lane = np.arange(64)
    for ft in range(f // 16):
        for kb in range(d // 32):
            for m, w in enumerate((wg, wu)):
                for j in range(8):
                    np.testing.assert_array_equal(gu[ft, kb, m, :, j],
                                                  w[ft * 16 + lane % 16, kb * 32 + (lane // 16) * 8 + j])
    for dt in range(d // 16):
        for kb in range(f // 32):
            for j in range(8):
                np.testing.assert_array_equal(dn[kb, dt, :, j], wd[dt * 16 + lane % 16, kb * 32 + (lane // 16) * 8 + j])
    assert sorted(dst.tolist()) == sorted(src.tolist())
    bad = np.zeros(3 * 48 * 64, dtype=np.uint16)
    assert B.lib.moe_pack_expert(bad.ctypes.data, bad.ctypes.data, 48, 64) == B.MOE_ERR_UNSUPPORTED


def test_pooled_prefetch_set_hand_example_and_oracle(B):
    import oracle
    # totals: e0 = 1.0, e1 = 3.0, e2 = 3.0, e3 = 0.5 -> ranking 1, 2 (tie: lower id first), 0, 3
    scores = np.array([[1.0, 1.0, 2.0, 0.5], [0.0, 2.0, 1.0, 0.0]], dtype=np.float32)
    assert B.moe_pooled_prefetch_set(scores, 3) == [0, 2, 1] == oracle.pooled_prefetch_set(scores, 3)
    assert B.moe_pooled_prefetch_set(scores, 9) == [3, 0, 2, 1]
    r = np.random.default_rng(3)
    for _ in range(20):
        sc = r.integers(0, 4, size=(5, 17)).astype(np.float32)        # many ties
        cap = int(r.integers(1, 20))
        assert B.moe_pooled_prefetch_set(sc, cap) == oracle.pooled_prefetch_set(sc, cap)
    with pytest.raises(B.MoeError):
        B.moe_pooled_prefetch_set(scores, 0)


def test_noalloc_entry_point_validates_before_touching_the_gpu(B):
    """Shapes, null pointers and batches beyond the fixed device array are refused on the host."""
    def call(batch=1, x=0x1000, y=0x2000, **kw):
        f = dict(n_experts=16, n_shared=0, top_k=4, d_model=256, d_ff=128, dtype=B.MOE_DTYPE_BF16, norm_topk=1,
                 pool_layout=B.MOE_LAYOUT_TILED, router_w=0x3000, experts=0x4000, shared_w=None)
        f.update(kw)
        layer = B.moe_resident_layer_t(**f)
        return B.lib.moe_layer_decode_resident_noalloc(C.byref(layer), x, None, batch, y, None, None, None)
    assert call(top_k=0) == B.MOE_ERR_INVALID_ARG
    assert call(x=None) == B.MOE_ERR_INVALID_ARG
    assert call(experts=None) == B.MOE_ERR_INVALID_ARG
    assert call(n_shared=1) == B.MOE_ERR_INVALID_ARG
    assert call(d_ff=100) == B.MOE_ERR_UNSUPPORTED
    assert call(batch=0) == B.MOE_ERR_INVALID_ARG
    assert call(batch=1 << 16) == B.MOE_ERR_UNSUPPORTED and "scratch" in B.moe_last_error()
    assert C.sizeof(B.moe_resident_layer_t) == 8 * 4 + 3 * 8
