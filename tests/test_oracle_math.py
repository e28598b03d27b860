"""Pins for the oracle's layer arithmetic (Eq. 1-3): closed forms, invariants,
brute force and library routines - none of them the oracle's own code."""
import math

import numpy as np
import pytest
import scipy.special
import torch

import oracle
from tests.golden.load import paper_constants
from workload import CONFIGS, Workload, get_config, widen


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------- router logits
def test_router_logits_matches_library_matmul_nonsquare():
    r = rng(1)
    x = r.standard_normal((5, 48)).astype(np.float32)
    w = r.standard_normal((7, 48)).astype(np.float32)
    b = r.standard_normal((5, 7)).astype(np.float32)
    got = oracle.router_logits(x, w, b)
    ref = x.astype(np.float64) @ w.astype(np.float64).T + b.astype(np.float64)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.router_logits(x, w), ref - b, rtol=0, atol=1e-12)


def test_router_logits_hand_values():
    # W_r = [[1,2],[3,-1],[0,0.5]], x = [2, -1] -> [0, 7, -0.5]; bias adds.
    w = np.array([[1, 2], [3, -1], [0, 0.5]], dtype=np.float32)
    x = np.array([[2, -1]], dtype=np.float32)
    np.testing.assert_array_equal(oracle.router_logits(x, w), [[0.0, 7.0, -0.5]])
    bias = np.array([[0.25, -1.0, 2.0]], dtype=np.float32)
    np.testing.assert_array_equal(oracle.router_logits(x, w, bias), [[0.25, 6.0, 1.5]])


# ------------------------------------------------------------------ softmax
def test_softmax_invariants_and_library():
    z = rng(2).standard_normal((9, 33)) * 4
    p = oracle.softmax(z)
    np.testing.assert_allclose(p.sum(1), 1.0, atol=1e-14)
    assert (p > 0).all()
    np.testing.assert_allclose(oracle.softmax(z + 123.456), p, atol=1e-13)
    np.testing.assert_allclose(p, scipy.special.softmax(z, axis=1), atol=1e-14)
    # order preserved
    assert (np.argsort(p, axis=1) == np.argsort(z, axis=1)).all()


def test_softmax_hand_values():
    # softmax([0, ln 3]) = [1/4, 3/4]; equal logits -> uniform
    p = oracle.softmax(np.array([[0.0, math.log(3.0)]]))
    np.testing.assert_allclose(p, [[0.25, 0.75]], atol=1e-15)
    np.testing.assert_allclose(oracle.softmax(np.full((1, 8), -7.0)), np.full((1, 8), 0.125), atol=1e-16)
    # huge logits do not overflow
    assert np.isfinite(oracle.softmax(np.array([[1e4, 1e4 - 1.0]]))).all()


# -------------------------------------------------------------------- top-K
def test_topk_brute_force_argsort():
    r = rng(3)
    for E, K in [(8, 2), (64, 8), (16, 2), (5, 5), (64, 6), (7, 1)]:
        z = r.standard_normal((50, E))
        got = oracle.topk(z, K)
        ref = np.sort(np.argsort(-z, axis=1, kind="stable")[:, :K], axis=1)
        np.testing.assert_array_equal(got, ref)
        assert got.shape == (50, K)
        # ||r||_1 = K, ids distinct and ascending
        assert (np.diff(got, axis=1) > 0).all()


def test_topk_ties_go_to_lower_id_and_uniform_case():
    z = np.array([[1.0, 3.0, 3.0, 3.0, 0.0]])
    np.testing.assert_array_equal(oracle.topk(z, 2), [[1, 2]])
    np.testing.assert_array_equal(oracle.topk(np.zeros((1, 8)), 3), [[0, 1, 2]])


def test_topk_permutation_equivariance():
    r = rng(4)
    z = r.standard_normal((20, 16))
    perm = r.permutation(16)
    a = oracle.topk(z, 4)
    b = oracle.topk(z[:, perm], 4)
    for row in range(20):
        assert set(perm[b[row]].tolist()) == set(a[row].tolist())


def test_topk_on_logits_equals_topk_on_probabilities():
    z = rng(5).standard_normal((40, 64)) * 2
    np.testing.assert_array_equal(oracle.topk(z, 8), oracle.topk(oracle.softmax(z), 8))


# -------------------------------------------------------------- gate weights
def test_gate_weights_sum_rules():
    z = rng(6).standard_normal((30, 16))
    p = oracle.softmax(z)
    idx = oracle.topk(z, 4)
    w1 = oracle.gate_weights(p, idx, 1)
    w0 = oracle.gate_weights(p, idx, 0)
    np.testing.assert_allclose(w1.sum(1), 1.0, atol=1e-14)
    sel = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    np.testing.assert_array_equal(w0, sel)                      # Eq. 2 as printed
    np.testing.assert_allclose(w1, sel / sel.sum(1, keepdims=True), atol=1e-15)
    # K = E: the renormalised mixture is the full softmax
    full = oracle.gate_weights(p, oracle.topk(z, 16), 1)
    np.testing.assert_allclose(full, p, atol=1e-14)


def test_gate_weights_hand_values():
    # logits [0, ln3, ln4, -inf-ish]: p = [1,3,4,~0]/8 ; top-2 = {1,2} -> 3/7, 4/7
    z = np.array([[0.0, math.log(3.0), math.log(4.0), -50.0]])
    p = oracle.softmax(z)
    idx = oracle.topk(z, 2)
    np.testing.assert_array_equal(idx, [[1, 2]])
    np.testing.assert_allclose(oracle.gate_weights(p, idx, 1), [[3 / 7, 4 / 7]], atol=1e-14)
    np.testing.assert_allclose(oracle.gate_weights(p, idx, 0), [[3 / 8, 4 / 8]], atol=1e-12)


# --------------------------------------------------------------- expert FFN
def test_expert_scalar_closed_form():
    # d = f = 1: E(t) = c * silu(a t) * (b t)
    a, b, c, t = 1.5, -0.75, 2.0, 0.5
    got = oracle.expert_swiglu(np.array([t]), np.array([[a]]), np.array([[b]]), np.array([[c]]))
    z = a * t
    assert got[0] == pytest.approx(c * (z / (1 + math.exp(-z))) * (b * t), rel=1e-15)
    # silu(1) and silu(-2), typed in from the definition z / (1 + e^-z)
    one = oracle.expert_swiglu(np.array([1.0]), np.array([[1.0]]), np.array([[1.0]]), np.array([[1.0]]))
    assert one[0] == pytest.approx(0.7310585786300049, rel=1e-15)
    neg = oracle.expert_swiglu(np.array([1.0]), np.array([[-2.0]]), np.array([[1.0]]), np.array([[1.0]]))
    assert neg[0] == pytest.approx(-0.2384058440442351, rel=1e-14)


def test_expert_identity_and_zero_gate():
    r = rng(7)
    x = r.standard_normal(12).astype(np.float32)
    eye = np.eye(12, dtype=np.float32)
    got = oracle.expert_swiglu(x, eye, eye, eye)
    x64 = x.astype(np.float64)
    np.testing.assert_allclose(got, x64 / (1 + np.exp(-x64)) * x64, rtol=1e-15)
    wu = r.standard_normal((20, 12)).astype(np.float32)
    wd = r.standard_normal((12, 20)).astype(np.float32)
    np.testing.assert_array_equal(oracle.expert_swiglu(x, np.zeros((20, 12), np.float32), wu, wd), np.zeros(12))


def test_expert_matches_torch_cpu_nonsquare():
    # d != f and distinct W_g / W_u so that a swapped or transposed operand fails
    r = rng(8)
    d, f = 24, 40
    x = r.standard_normal(d).astype(np.float32)
    wg, wu = (r.standard_normal((f, d)).astype(np.float32) for _ in range(2))
    wd = r.standard_normal((d, f)).astype(np.float32)
    got = oracle.expert_swiglu(x, wg, wu, wd)
    tx, tg, tu, td = (torch.from_numpy(a).double() for a in (x, wg, wu, wd))
    ref = td @ (torch.nn.functional.silu(tg @ tx) * (tu @ tx))
    np.testing.assert_allclose(got, ref.numpy(), rtol=1e-12, atol=1e-12)
    # swapping gate and up must change the result (the nonlinearity sits on the gate)
    swapped = oracle.expert_swiglu(x, wu, wg, wd)
    assert np.abs(swapped - got).max() > 1e-3


def test_expert_linearity_in_up_and_down():
    r = rng(9)
    d, f = 10, 14
    x = r.standard_normal(d).astype(np.float32)
    wg, wu = (r.standard_normal((f, d)).astype(np.float32) for _ in range(2))
    wd = r.standard_normal((d, f)).astype(np.float32)
    base = oracle.expert_swiglu(x, wg, wu, wd)
    np.testing.assert_allclose(oracle.expert_swiglu(x, wg, 2 * wu, wd), 2 * base, rtol=1e-13)
    np.testing.assert_allclose(oracle.expert_swiglu(x, wg, wu, -4 * wd), -4 * base, rtol=1e-13)


# ---------------------------------------------------- sparse path vs dense
@pytest.mark.parametrize("norm_topk", [1, 0])
def test_sparse_equals_dense_masked_exactly(norm_topk):
    cfg = get_config("tiny_fp32")
    wl = Workload(cfg)
    experts = [tuple(widen(m) for m in wl.expert(0, e)) for e in range(cfg.n_experts)]
    lw = oracle.LayerWeights(widen(wl.router_w(0)), lambda e: experts[e])
    for s in range(2):
        x = widen(wl.tokens(s))[:4]
        bias = np.tile(wl.bias(0, s), (4, 1))
        cache = oracle.ExpertCache(cfg.n_experts, cfg.capacity)
        res = oracle.moe_layer_decode(lw, cache, x, bias, cfg.top_k, norm_topk)
        dense = oracle.moe_layer_dense(lw, cfg.n_experts, x, bias, cfg.top_k, norm_topk)
        np.testing.assert_array_equal(res.y, dense)
        assert np.abs(res.y).max() > 0
        np.testing.assert_allclose(res.w.sum(1), 1.0 if norm_topk else
                                   np.take_along_axis(res.p, res.idx.astype(np.int64), 1).sum(1), atol=1e-14)


def test_layer_with_k_equal_e_is_full_mixture_and_shared_adds():
    r = rng(10)
    E, d, f = 3, 6, 5
    ex = [(r.standard_normal((f, d)).astype(np.float32), r.standard_normal((f, d)).astype(np.float32),
           r.standard_normal((d, f)).astype(np.float32)) for _ in range(E + 1)]
    wr = r.standard_normal((E, d)).astype(np.float32)
    x = r.standard_normal((2, d)).astype(np.float32)
    lw = oracle.LayerWeights(wr, lambda e: ex[e])
    res = oracle.moe_layer_decode(lw, oracle.ExpertCache(E, E), x, None, E)
    p = scipy.special.softmax(x.astype(np.float64) @ wr.astype(np.float64).T, axis=1)
    ref = np.zeros((2, d))
    for b in range(2):
        for e in range(E):
            ref[b] += p[b, e] * oracle.expert_swiglu(x[b], *ex[e])
    np.testing.assert_allclose(res.y, ref, rtol=1e-12, atol=1e-13)
    lw2 = oracle.LayerWeights(wr, lambda e: ex[e], shared=[ex[E]])
    res2 = oracle.moe_layer_decode(lw2, oracle.ExpertCache(E, E), x, None, E)
    for b in range(2):
        np.testing.assert_allclose(res2.y[b] - res.y[b], oracle.expert_swiglu(x[b], *ex[E]), atol=1e-12)


def test_prefill_streaming_is_the_same_layer_with_a_read_only_cache():
    cfg = get_config("tiny_fp32")
    wl = Workload(cfg)
    experts = [tuple(widen(m) for m in wl.expert(0, e)) for e in range(cfg.n_experts)]
    lw = oracle.LayerWeights(widen(wl.router_w(0)), lambda e: experts[e])
    x = widen(wl.tokens(0))[:6]
    bias = np.tile(wl.bias(0, 0), (6, 1))
    cache = oracle.ExpertCache(cfg.n_experts, 3)
    cache.pin([1, 4, 6])
    before = (cache.resident(), cache.stats(8))
    res = oracle.moe_layer_prefill(lw, cache, x, bias, cfg.top_k)
    np.testing.assert_array_equal(res.y, oracle.moe_layer_dense(lw, cfg.n_experts, x, bias, cfg.top_k))
    assert cache.resident() == before[0]                       # nothing inserted, nothing evicted
    used = set(res.idx.reshape(-1).tolist())
    st = cache.stats(8)
    assert st["stream_loads"] == len(used - {1, 4, 6}) and st["bytes_streamed"] == 8 * st["stream_loads"]
    assert {k: st[k] for k in before[1] if "stream" not in k} == {k: v for k, v in before[1].items() if "stream" not in k}
    # rows=... evaluates a subset only
    sub = oracle.moe_layer_prefill(lw, cache, x, bias, cfg.top_k, rows=[2, 5])
    np.testing.assert_array_equal(sub.y[[2, 5]], res.y[[2, 5]])
    assert not sub.y[[0, 1, 3, 4]].any()


# ------------------------------------------------------------- byte model
def test_expert_bytes_against_paper_transfer_time():
    k = paper_constants()
    nbytes = oracle.expert_bytes(4096, 14336, 2)          # Mixtral-8x7B expert, 16-bit
    assert nbytes == 352_321_536
    ms = nbytes / (k["pcie5_x16_gbps"] * 1e9) * 1e3
    assert k["mixtral_expert_transfer_ms_lo"] <= ms <= k["mixtral_expert_transfer_ms_hi"]
    for cfg in CONFIGS.values():
        assert cfg.expert_bytes == oracle.expert_bytes(cfg.d_model, cfg.d_ff, cfg.elem_bytes)


# ------------------------------------------------------- generator sanity
def test_generator_margin_and_concentration():
    cfg = get_config("olmoe_like").with_(n_seqs=2, n_steps=64)
    wl = Workload(cfg)
    wr = widen(wl.router_w(0))
    for s in range(2):
        x = widen(wl.tokens(s))
        bias = np.tile(wl.bias(0, s), (x.shape[0], 1))
        z = oracle.router_logits(x, wr, bias)
        zs = np.sort(z, axis=1)[:, ::-1]
        assert (zs[:, cfg.top_k - 1] - zs[:, cfg.top_k] >= cfg.delta).all()
        idx = oracle.topk(z, cfg.top_k)
        share = np.isin(idx, wl.pref_set(0, s)).mean()
        assert share > 0.5          # biased routing concentrates on the preferred set
    # reproducible
    np.testing.assert_array_equal(Workload(cfg).tokens(1), wl.tokens(1))
    np.testing.assert_array_equal(Workload(cfg).expert(0, 5)[2][:4], wl.expert(0, 5)[2][:4])
