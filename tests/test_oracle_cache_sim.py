"""Pins for the oracle's cache-simulation loss (section 3.1.1, appendix C.1): Proposition C.2's closed form,
the expansion in the proof of Lemma C.3 evaluated directly, limiting cases with closed forms, bounds, the norm invariant, and the hard count against an explicit Top-C simulation and against LRU."""
import numpy as np
import pytest

import oracle


def trace(seed, L, T, K, E, zipf=None):
    r = np.random.default_rng(seed)
    w = None
    if zipf:
        w = 1.0 / np.arange(1, E + 1) ** zipf
        w /= w.sum()
    return np.array([[np.sort(r.choice(E, size=K, replace=False, p=w)) for _ in range(T)] for _ in range(L)],
                    dtype=np.int32)


def soft_by_unrolled_sum(idx, E, C, gamma, c1=None):
    """Lemma C.3's proof: c^(t) = (Gamma^(t))^-1 (sum_{i<t} gamma^(t-1-i) r^(i) + gamma^(t-1) c^(1)),
    Gamma^(t) from Proposition C.2's closed form - no recursion anywhere."""
    L, T, K = idx.shape
    total = 0.0
    for l in range(L):
        r = np.zeros((T, E))
        for t in range(T):
            r[t, idx[l, t]] = 1.0
        c_first = np.full(E, C / E) if c1 is None else np.asarray(c1[l], dtype=np.float64)
        for t in range(1, T + 1):                                   # 1-based as in the paper
            Gamma = gamma ** (t - 1) + (K / C) * sum(gamma ** (t - i - 1) for i in range(1, t))
            ct = sum(gamma ** (t - 1 - i) * r[i - 1] for i in range(1, t)) + gamma ** (t - 1) * c_first
            total += K - (r[t - 1] @ ct) / Gamma
    return total / (L * T)


@pytest.mark.parametrize("gamma", [0.9, 0.5, 1.0, 0.0])
def test_soft_loss_equals_the_unrolled_expansion(gamma):
    E, C, K = 16, 4, 2
    idx = trace(1, 2, 40, K, E, zipf=1.0)
    soft, _ = oracle.cache_sim_loss(idx, E, C, gamma)
    assert soft == pytest.approx(soft_by_unrolled_sum(idx, E, C, gamma), rel=1e-12)
    c1 = np.zeros((2, E))
    c1[:, [1, 3, 5, 7]] = 1.0                                        # a prefetch set as first state
    soft, _ = oracle.cache_sim_loss(idx, E, C, gamma, c1)
    assert soft == pytest.approx(soft_by_unrolled_sum(idx, E, C, gamma, c1), rel=1e-12)


def test_gamma_zero_closed_form():
    # gamma = 0: c^(t+1) = (C/K) r^(t), so the loss of token t+1 is K - (C/K) <r^(t+1), r^(t)>
    E, C, K, T = 12, 3, 3, 50
    idx = trace(2, 1, T, K, E)
    soft, _ = oracle.cache_sim_loss(idx, E, C, 0.0)
    expect = K - K * (C / E)                                         # first token, uniform start
    for t in range(1, T):
        expect += K - (C / K) * len(set(idx[0, t]) & set(idx[0, t - 1]))
    assert soft == pytest.approx(expect / T, rel=1e-13)


def test_constant_routing_closed_form_and_bounds():
    # every token requests the same K experts, uniform start: <r, c^(t)> follows from Proposition C.2
    E, C, K, T, gamma = 10, 5, 2, 30, 0.8
    idx = np.tile(np.array([2, 7], dtype=np.int32), (1, T, 1))
    soft, hard = oracle.cache_sim_loss(idx, E, C, gamma)
    expect = 0.0
    for t in range(1, T + 1):
        geo = sum(gamma ** (t - i - 1) for i in range(1, t))
        Gamma = gamma ** (t - 1) + (K / C) * geo
        expect += K - (K * geo + gamma ** (t - 1) * K * C / E) / Gamma
    assert soft == pytest.approx(expect / T, rel=1e-13)
    # the soft state has L1 norm C and K requested entries, so <r, c> <= C: K - C <= L_cs <= K (the soft loss goes
    # negative for concentrated routing: entries of c grow up to C / K); the hard count lies in [0, K]
    for zipf in (0.7, 3.0):
        idx2 = trace(3, 3, 60, 4, 32, zipf=zipf)
        for g in (0.0, 0.3, 0.9, 1.0):
            s, h = oracle.cache_sim_loss(idx2, 32, 8, g)
            assert 4.0 - 8.0 <= s <= 4.0 and 0.0 <= h <= 4.0
    # constant routing drives the requested entries to C / K each: the per-token loss tends to K - C
    long_idx = np.tile(np.array([2, 7], dtype=np.int32), (1, 400, 1))
    s_all, _ = oracle.cache_sim_loss(long_idx, E, C, gamma)
    s_head, _ = oracle.cache_sim_loss(long_idx[:, :200], E, C, gamma)
    assert (400 * s_all - 200 * s_head) / 200 == pytest.approx(K - C, abs=1e-9)


def test_constant_routing_hard_count_by_hand():
    # E=10, C=5, uniform first state: Top-5 with ties to the lower id is {0,1,2,3,4}; tokens request {2,7}.
    # token 1 misses expert 7 only; from token 2 on both have the largest counts and are cached.
    idx = np.tile(np.array([2, 7], dtype=np.int32), (1, 6, 1))
    _, hard = oracle.cache_sim_loss(idx, 10, 5, 0.8)
    assert hard == pytest.approx(1.0 / 6.0)


def test_norm_of_soft_cache_stays_at_capacity():
    # Proposition C.2: ||c^(t)||_1 = C for every t.  Requesting ALL experts (K = E) reads the norm off the loss:
    # <1, 1 - c^(t)> = E - C for every token, whatever gamma is.
    E, C, T = 8, 3, 25
    idx = np.tile(np.arange(E, dtype=np.int32), (2, T, 1))
    for g in (0.0, 0.6, 1.0):
        soft, _ = oracle.cache_sim_loss(idx, E, C, g)
        assert soft == pytest.approx(E - C, rel=1e-13)


def hard_reference(idx_l, E, C, gamma):
    ct = np.full(E, C / E)
    misses = 0
    for tok in idx_l:
        order = sorted(range(E), key=lambda e: (-ct[e], e))[:C]
        misses += sum(1 for e in tok if e not in order)
        ct = gamma * ct
        ct[tok] += 1.0
    return misses


@pytest.mark.parametrize("gamma", [1.0, 0.9, 0.4])
def test_hard_count_equals_explicit_top_c(gamma):
    E, C, K = 20, 5, 2
    idx = trace(5, 3, 70, K, E, zipf=0.9)
    _, hard = oracle.cache_sim_loss(idx, E, C, gamma)
    ref = sum(hard_reference(idx[l], E, C, gamma) for l in range(3)) / (3 * 70)
    assert hard == pytest.approx(ref, rel=1e-14)


def test_hard_count_small_gamma_is_lru_after_warm_up():
    # gamma < 1/2, K = 1: once C distinct experts have been seen the Top-C set is the LRU content
    E, C, T = 9, 3, 200
    idx = trace(6, 1, T, 1, E, zipf=0.8)
    cache = oracle.ExpertCache(E, C)
    seen, warm, lru_misses, sim_misses = set(), None, 0, 0
    ct = np.full(E, C / E)
    for t in range(T):
        e = int(idx[0, t, 0])
        top = sorted(range(E), key=lambda x: (-ct[x], x))[:C]
        hit, _ = cache.lookup(e)
        if warm is not None:
            lru_misses += 0 if hit else 1
            sim_misses += 0 if e in top else 1
        seen.add(e)
        if warm is None and len(seen) >= C:
            warm = t
        ct = 0.3 * ct
        ct[e] += 1.0
    assert warm is not None and lru_misses == sim_misses and lru_misses > 10
