"""Pins for the fp64 CPU oracle: what the paper and the mathematics fix.

None of these tests re-types the oracle's own loop and compares; each route is
a closed form, a library routine (scipy), finite differences of a scalar,
exact-arithmetic brute force, or an invariant.  References are to Tree
Attention (arXiv 2408.04093).
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

import oracle

RNG = np.random.default_rng(20240804)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_problem(L, d, scale_q=1.0, dtype=np.float64, rng=RNG):
    q = (rng.standard_normal(d) * scale_q).astype(dtype)
    K = rng.standard_normal((L, d)).astype(dtype)
    V = rng.standard_normal((L, d)).astype(dtype)
    return q, K, V


def decode1(q, K, V, scale, L=None):
    """Single-head call through the batched entry point."""
    out, lse = oracle.decode(q[None, None], K[None, None], V[None, None], scale,
                             valid_len=None if L is None else [L], nthreads=1)
    return out[0, 0], lse[0, 0]


# ---------------------------------------------------------------- golden, hand-derived
def _read_golden(name):
    rec = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split(":")
            rec[k.strip()] = [float(x) for x in v.split()]
    return rec


def test_golden_rational_weights():
    """Section 3 definition with scores ln w: weights are w / sum(w) by hand."""
    g = _read_golden("rational_weights.txt")
    q = np.array(g["q"])
    K = np.stack([np.log(np.array(g["w"])), np.array(g["junk"])], axis=1)
    V = np.array([g["v0"], g["v1"], g["v2"], g["v3"]])
    out, lse = decode1(q, K, V, 1.0)
    np.testing.assert_allclose(out, g["out"], rtol=0, atol=1e-14)
    assert abs(lse - math.log(g["lse_is_log_of"][0])) < 1e-14


# ---------------------------------------------------------------- closed forms
def test_single_key_returns_its_value_and_score():
    q, K, V = rand_problem(1, 16)
    out, lse = decode1(q, K, V, 0.37)
    np.testing.assert_array_equal(out, V[0])
    assert lse == pytest.approx(0.37 * float(np.dot(q, K[0])), rel=1e-15)


def test_zero_query_gives_mean_and_log_count():
    q, K, V = rand_problem(37, 8)
    q[:] = 0
    out, lse = decode1(q, K, V, 1.0)
    np.testing.assert_allclose(out, V.mean(axis=0), atol=1e-15)
    assert lse == pytest.approx(math.log(37), abs=1e-15)


def test_equal_keys_give_mean_and_shifted_log_count():
    q, K, V = rand_problem(50, 8)
    K[:] = K[0]
    out, lse = decode1(q, K, V, 0.5)
    np.testing.assert_allclose(out, V.mean(axis=0), atol=1e-14)
    assert lse == pytest.approx(0.5 * float(q @ K[0]) + math.log(50), abs=1e-13)


def test_dominant_key_wins():
    q, K, V = rand_problem(20, 8)
    K[7] = 200.0 * q / np.dot(q, q)          # score 200, others O(1)
    out, lse = decode1(q, K, V, 1.0)
    np.testing.assert_allclose(out, V[7], atol=1e-60 + 1e-14)
    assert lse == pytest.approx(200.0, abs=1e-12)


def test_convex_combination_bounds():
    q, K, V = rand_problem(64, 12, scale_q=3.0)
    out, _ = decode1(q, K, V, 1.0)
    assert np.all(out <= V.max(axis=0) + 1e-15) and np.all(out >= V.min(axis=0) - 1e-15)


def test_constant_shift_of_scores_moves_only_lse():
    """Appendix F: subtracting a constant inside the exponent leaves the gradient
    unchanged.  Adding u to every key shifts every score by scale*q.u."""
    q, K, V = rand_problem(33, 8)
    u = RNG.standard_normal(8)
    o1, l1 = decode1(q, K, V, 0.7)
    o2, l2 = decode1(q, K + u, V, 0.7)
    np.testing.assert_allclose(o2, o1, atol=1e-13)
    assert l2 - l1 == pytest.approx(0.7 * float(q @ u), abs=1e-12)


def test_duplicating_the_cache_adds_log2():
    q, K, V = rand_problem(21, 8)
    o1, l1 = decode1(q, K, V, 1.0)
    o2, l2 = decode1(q, np.concatenate([K, K]), np.concatenate([V, V]), 1.0)
    np.testing.assert_allclose(o2, o1, atol=1e-14)
    assert l2 - l1 == pytest.approx(math.log(2), abs=1e-13)


def test_overflow_stability_large_scores():
    """Scores of +-700 would overflow an unshifted exp; the shifted form must not."""
    q = np.array([1.0, 0.0])
    K = np.array([[700.0, 0], [699.0, 0], [-700.0, 0]])
    V = np.array([[1.0, 0], [0, 1.0], [5, 5]])
    out, lse = decode1(q, K, V, 1.0)
    w0 = 1 / (1 + math.exp(-1))
    np.testing.assert_allclose(out, [w0, 1 - w0], atol=1e-15)
    assert lse == pytest.approx(700 + math.log1p(math.exp(-1)), abs=1e-12)


# ---------------------------------------------------------------- library routines
@pytest.mark.parametrize("L,d,scale", [(5, 3, 1.0), (64, 16, 0.25), (1000, 64, 0.125)])
def test_matches_scipy_softmax_and_logsumexp(L, d, scale):
    q, K, V = rand_problem(L, d)
    s = scale * (K @ q)
    out, lse = decode1(q, K, V, scale)
    np.testing.assert_allclose(out, scipy.special.softmax(s) @ V, rtol=0, atol=1e-13)
    assert lse == pytest.approx(float(scipy.special.logsumexp(s)), abs=1e-12)


def test_energy_matches_scipy_logsumexp():
    q, K, V = rand_problem(40, 6)
    zeta = RNG.standard_normal(6) * 0.3
    F = oracle.energy(q, K, V, 0.8, zeta)
    ref = float(scipy.special.logsumexp(0.8 * (K @ q) + V @ zeta))
    assert F == pytest.approx(ref, abs=1e-13)


# ---------------------------------------------------------------- brute force, exact
def test_bruteforce_exact_rational_small():
    """N <= 64: weights exp(s) with s = ln(integer) are integers, so the
    definition can be evaluated in exact rational arithmetic."""
    d, L = 3, 48
    ints = RNG.integers(1, 40, size=L)
    q = np.array([1.0, 0.0, 0.0])
    K = np.zeros((L, d))
    K[:, 0] = np.log(ints)
    K[:, 1:] = RNG.standard_normal((L, 2))
    Vint = RNG.integers(-9, 10, size=(L, d))
    out, lse = decode1(q, K, Vint.astype(np.float64), 1.0)
    Z = Fraction(int(ints.sum()))
    for c in range(d):
        exact = sum(Fraction(int(w)) * int(v) for w, v in zip(ints, Vint[:, c])) / Z
        assert out[c] == pytest.approx(float(exact), abs=1e-13)
    assert lse == pytest.approx(math.log(int(ints.sum())), abs=1e-13)


@pytest.mark.parametrize("L", [1, 2, 17, 64])
def test_bruteforce_unshifted_python_loops(L):
    """N <= 64, small scores: plain sums of math.exp with no max shift."""
    d = 8
    q, K, V = rand_problem(L, d)
    out, lse = decode1(q, K, V, 0.35)
    e = [math.exp(0.35 * math.fsum(q[c] * K[a, c] for c in range(d))) for a in range(L)]
    Z = math.fsum(e)
    for c in range(d):
        assert out[c] == pytest.approx(math.fsum(e[a] * V[a, c] for a in range(L)) / Z, abs=1e-14)
    assert lse == pytest.approx(math.log(Z), abs=1e-14)


# ---------------------------------------------------------------- Observation 1
@pytest.mark.parametrize("scale", [1.0, 0.3])
def test_output_is_gradient_of_energy(scale):
    """out = dF/dzeta at zeta = 0 and lse = F(0), by central differences."""
    d, L = 6, 50
    q, K, V = rand_problem(L, d)
    out, lse = decode1(q, K, V, scale)
    assert oracle.energy(q, K, V, scale, np.zeros(d)) == pytest.approx(lse, abs=1e-13)
    h = 1e-5
    for c in range(d):
        e = np.zeros(d)
        e[c] = h
        fd = (oracle.energy(q, K, V, scale, e) - oracle.energy(q, K, V, scale, -e)) / (2 * h)
        assert fd == pytest.approx(out[c], abs=2e-9)


# ---------------------------------------------------------------- associativity / chunking
def _random_tree_merges(P, rng, fan_in=2):
    """Random tree over a random leaf order: repeatedly fold `fan_in` live nodes."""
    live = list(rng.permutation(P))
    merges = []
    while len(live) > 1:
        k = min(fan_in, len(live))
        pick = [live.pop(int(rng.integers(len(live)))) for _ in range(k)]
        for src in pick[1:]:
            merges.append((int(pick[0]), int(src)))
        live.append(pick[0])
    return merges, int(live[0])


def _partials(q, K, V, scale, bounds):
    ms, ls, os_ = [], [], []
    for lo, hi in zip(bounds[:-1], bounds[1:]):
        m, l, o = oracle.partial(q, K, V, scale, int(lo), int(hi))
        ms.append(m), ls.append(l), os_.append(o)
    return np.array(ms), np.array(ls), np.array(os_)


@pytest.mark.parametrize("fan_in", [2, 3, 8, 64])
def test_any_chunking_and_tree_shape_gives_the_direct_result(fan_in):
    """Section 5.1 associativity: result independent of chunking and tree."""
    d, L, P = 16, 777, 23
    rng = np.random.default_rng(7 + fan_in)
    q, K, V = rand_problem(L, d, scale_q=2.0, rng=rng)
    direct_out, direct_lse = decode1(q, K, V, 0.5)
    cuts = np.sort(rng.choice(np.arange(0, L + 1), size=P - 1, replace=True))  # empty chunks allowed
    bounds = np.concatenate([[0], cuts, [L]])
    m, l, o = _partials(q, K, V, 0.5, bounds)
    merges, root = _random_tree_merges(P, rng, fan_in)
    out, lse = oracle.combine(m, l, o, merges, root)
    np.testing.assert_allclose(out, direct_out, rtol=0, atol=1e-13)
    assert lse == pytest.approx(direct_lse, abs=1e-12)


def test_full_range_partial_is_the_direct_result():
    q, K, V = rand_problem(100, 8)
    m, l, o = oracle.partial(q, K, V, 1.0, 0, 100)
    out, lse = decode1(q, K, V, 1.0)
    assert m == pytest.approx(float((K @ q).max()), rel=1e-15)
    np.testing.assert_allclose(o / l, out, atol=1e-14)
    assert m + math.log(l) == pytest.approx(lse, abs=1e-13)


def test_empty_partial_is_identity_and_all_empty_is_zero():
    q, K, V = rand_problem(10, 4)
    m, l, o = oracle.partial(q, K, V, 1.0, 3, 3)
    assert m == -math.inf and l == 0.0 and not o.any()
    out, lse = oracle.combine([m, m], [l, l], [o, o])
    assert not out.any() and lse == -math.inf


def test_algorithm3_form_equals_mlo_form():
    """Alg. 3 carries (o/l, m + log l) and takes the max over lse values."""
    d, L, P = 8, 300, 7
    q, K, V = rand_problem(L, d, scale_q=1.5)
    bounds = np.linspace(0, L, P + 1).astype(int)
    m, l, o = _partials(q, K, V, 1.0, bounds)
    out_a, lse_a = oracle.combine(m, l, o)
    out_b, lse_b = oracle.combine_alg3(o / l[:, None], m + np.log(l))
    np.testing.assert_allclose(out_b, out_a, atol=1e-14)
    assert lse_b == pytest.approx(lse_a, abs=1e-13)
    direct_out, direct_lse = decode1(q, K, V, 1.0)
    np.testing.assert_allclose(out_b, direct_out, atol=1e-13)
    assert lse_b == pytest.approx(direct_lse, abs=1e-12)


def test_algorithms_1_and_2_equal_the_definition():
    d, L, P = 8, 257, 5
    q, K, V = rand_problem(L, d, scale_q=2.0)
    bounds = np.array([0, 10, 10, 100, 200, L])
    out, lse = oracle.two_pass(q, K, V, 0.6, bounds)
    direct_out, direct_lse = decode1(q, K, V, 0.6)
    np.testing.assert_allclose(out, direct_out, atol=1e-13)
    assert lse == pytest.approx(direct_lse, abs=1e-12)


def test_section3_recurrence_equals_definition_on_small_scores():
    q, K, V = rand_problem(90, 8)
    np.testing.assert_allclose(oracle.recurrence(q, K, V, 0.3), decode1(q, K, V, 0.3)[0], atol=1e-14)


# ---------------------------------------------------------------- batching, GQA, lengths, storage types
def test_gqa_head_mapping_is_consecutive_groups():
    """Query head h reads KV head h // g: constant-valued V heads reveal the mapping."""
    B, Hq, Hkv, d, N = 2, 6, 3, 4, 9
    q = RNG.standard_normal((B, Hq, d))
    K = RNG.standard_normal((B, Hkv, N, d))
    V = np.empty((B, Hkv, N, d))
    for b in range(B):
        for h in range(Hkv):
            V[b, h] = 10 * b + h + 1
    out, _ = oracle.decode(q, K, V, 1.0)
    for b in range(B):
        for h in range(Hq):
            np.testing.assert_allclose(out[b, h], 10 * b + h // 2 + 1, atol=1e-13)


def test_batched_equals_per_head_calls_and_thread_count_is_irrelevant():
    B, Hq, Hkv, d, N = 2, 4, 2, 8, 31
    q = RNG.standard_normal((B, Hq, d))
    K = RNG.standard_normal((B, Hkv, N, d))
    V = RNG.standard_normal((B, Hkv, N, d))
    o1, l1 = oracle.decode(q, K, V, 0.4, nthreads=1)
    o4, l4 = oracle.decode(q, K, V, 0.4, nthreads=4)
    np.testing.assert_array_equal(o1, o4)
    np.testing.assert_array_equal(l1, l4)
    for b in range(B):
        for h in range(Hq):
            s = 0.4 * (K[b, h // 2] @ q[b, h])
            np.testing.assert_allclose(o1[b, h], scipy.special.softmax(s) @ V[b, h // 2], atol=1e-13)


def test_valid_len_hides_padding_and_zero_length_is_defined():
    B, Hq, Hkv, d, N = 4, 4, 2, 4, 12
    q = RNG.standard_normal((B, Hq, d))
    K = RNG.standard_normal((B, Hkv, N, d))
    V = RNG.standard_normal((B, Hkv, N, d))
    vl = [5, 0, 7, 99]                       # 99 > N: clamped to N
    for b, L in enumerate(vl):
        K[b, :, L:] = 1e30                   # padding must never be touched
        V[b, :, L:] = np.nan
    out, lse = oracle.decode(q, K, V, 1.0, valid_len=vl)
    for b in (0, 2, 3):
        L = min(vl[b], N)
        ref, ref_lse = oracle.decode(q[b:b + 1], K[b:b + 1, :, :L].copy(), V[b:b + 1, :, :L].copy(), 1.0)
        np.testing.assert_array_equal(out[b], ref[0])
        np.testing.assert_array_equal(lse[b], ref_lse[0])
        for h in range(Hq):
            s = K[b, h // 2, :L] @ q[b, h]
            np.testing.assert_allclose(out[b, h], scipy.special.softmax(s) @ V[b, h // 2, :L], atol=1e-13)
    assert not out[1].any() and np.all(lse[1] == -np.inf)


def test_bf16_and_fp32_storage_are_widened_exactly():
    # bf16 bit patterns: 1.0, 2.0, -1.0, 1.5, 0.10009765625
    bits = np.array([0x3F80, 0x4000, 0xBF80, 0x3FC0, 0x3DCD], dtype=np.uint16)
    vals = np.array([1.0, 2.0, -1.0, 1.5, 0.10009765625])
    d = 5
    q = np.zeros((1, 1, d), np.uint16)          # q = 0 -> out = mean of V rows
    K = np.zeros((1, 1, 2, d), np.uint16)
    V = np.stack([bits, bits[::-1]])[None, None]
    out, lse = oracle.decode(q, K, V, 1.0)
    np.testing.assert_array_equal(out[0, 0], (vals + vals[::-1]) / 2)
    # same numbers through the fp32 path and through the score (q = e_0, one key)
    q32 = np.zeros((1, 1, d), np.float32)
    q32[0, 0, 0] = 1
    K32 = np.float32(0.1) * np.ones((1, 1, 1, d), np.float32)
    out, lse = oracle.decode(q32, K32, K32, 3.0)
    assert lse[0, 0] == 3.0 * float(np.float32(0.1))
    qb = np.zeros((1, 1, d), np.uint16)
    qb[0, 0, 0] = 0x3F80
    Kb = np.full((1, 1, 1, d), 0x3DCD, np.uint16)
    out, lse = oracle.decode(qb, Kb, Kb, 1.0)
    assert lse[0, 0] == 0.10009765625 and out[0, 0, 0] == 0.10009765625


def test_torch_bf16_tensor_conversion_is_bit_exact():
    import torch
    t = torch.tensor([1.0, -2.5, 0.1, 3e38, 1e-38], dtype=torch.bfloat16)
    a = oracle.as_oracle_array(t)
    assert a.dtype == np.uint16
    back = (a.astype(np.uint32) << 16).view(np.float32)
    np.testing.assert_array_equal(back, t.float().numpy())


# ---------------------------------------------------------------- several query tokens, causal (Appendix C.1)
def test_causal_multi_token_equals_single_token_on_each_prefix():
    """Token t of Sq sees keys 0..L-Sq+t: the single-token result with that valid length."""
    B, Sq, Hq, Hkv, d, N = 2, 5, 4, 2, 8, 23
    q = RNG.standard_normal((B, Sq, Hq, d))
    K = RNG.standard_normal((B, Hkv, N, d))
    V = RNG.standard_normal((B, Hkv, N, d))
    vl = [23, 9]
    out, lse = oracle.decode_causal(q, K, V, 0.6, valid_len=vl)
    for t in range(Sq):
        ref, ref_lse = oracle.decode(q[:, t].copy(), K, V, 0.6, valid_len=[L - Sq + t + 1 for L in vl])
        np.testing.assert_array_equal(out[:, t], ref)
        np.testing.assert_array_equal(lse[:, t], ref_lse)
    # and against the library routine on an explicit slice
    s = 0.6 * (K[1, 1, :9 - 5 + 2 + 1] @ q[1, 2, 3])
    np.testing.assert_allclose(out[1, 2, 3], scipy.special.softmax(s) @ V[1, 1, :7], atol=1e-13)
    assert lse[1, 2, 3] == pytest.approx(float(scipy.special.logsumexp(s)), abs=1e-12)


def test_causal_single_token_is_plain_decode_and_short_caches_are_defined():
    q = RNG.standard_normal((1, 1, 2, 4))
    K = RNG.standard_normal((1, 1, 6, 4))
    V = RNG.standard_normal((1, 1, 6, 4))
    a = oracle.decode_causal(q, K, V, 1.0)
    b = oracle.decode(q[:, 0].copy(), K, V, 1.0)
    np.testing.assert_array_equal(a[0][:, 0], b[0])
    # 3 query tokens but only 2 cached keys: token 0 sees nothing, token 1 one key, token 2 both
    q3 = RNG.standard_normal((1, 3, 2, 4))
    out, lse = oracle.decode_causal(q3, K, V, 1.0, valid_len=[2])
    assert not out[0, 0].any() and np.all(lse[0, 0] == -np.inf)
    np.testing.assert_array_equal(out[0, 1], np.broadcast_to(V[0, 0, 0], (2, 4)))
    assert np.isfinite(lse[0, 2]).all()


def test_causal_output_is_gradient_of_the_total_energy():
    """d F_tot / d zeta_t at zeta = 0 is the output of token t; F_tot(0) = sum of the lse."""
    d, L, Sq = 5, 14, 3
    q = RNG.standard_normal((Sq, d))
    K = RNG.standard_normal((L, d))
    V = RNG.standard_normal((L, d))
    out, lse = oracle.decode_causal(q[None, :, None], K[None, None], V[None, None], 0.7)
    out, lse = out[0, :, 0], lse[0, :, 0]
    z0 = np.zeros((Sq, d))
    assert oracle.energy_causal(q, K, V, 0.7, z0) == pytest.approx(lse.sum(), abs=1e-12)
    h = 1e-5
    for t in range(Sq):
        for c in range(d):
            e = np.zeros((Sq, d))
            e[t, c] = h
            fd = (oracle.energy_causal(q, K, V, 0.7, e) - oracle.energy_causal(q, K, V, 0.7, -e)) / (2 * h)
            assert fd == pytest.approx(out[t, c], abs=2e-9)
    # the total energy itself against the library routine
    zeta = RNG.standard_normal((Sq, d)) * 0.2
    ref = sum(float(scipy.special.logsumexp(0.7 * (K[:L - Sq + t + 1] @ q[t]) + V[:L - Sq + t + 1] @ zeta[t]))
              for t in range(Sq))
    assert oracle.energy_causal(q, K, V, 0.7, zeta) == pytest.approx(ref, abs=1e-12)
