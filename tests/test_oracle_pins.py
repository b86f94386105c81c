"""Pins of the fp64 oracle against what the paper and the mathematics fix.

The paper (arxiv 2406.13035) prints no worked numeric example of the method's state, so
there are no paper values to store; the pins are closed forms, invariants stated in the
text, reductions to library routines, and brute force on tiny inputs (tests/brute.py)."""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import d2o_ref as ref
from tests import brute

rng = np.random.default_rng(7)


def _rand(n, d, seed):
    g = np.random.default_rng(seed)
    return g.standard_normal((n, d))


# ------------------------------------------------------------------ attention (Eq. 3, Eq. 4)

def test_attention_equals_library_sdpa():
    q, k, v = _rand(97, 16, 1) * 2, _rand(97, 16, 2), _rand(97, 16, 3)
    o, s = ref.prefill_attention_head(q, k, v, causal=True, row_block=32)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None],
        is_causal=True)[0].numpy()
    np.testing.assert_allclose(o, want, rtol=1e-12, atol=1e-13)
    assert abs(s.sum() - 97) < 1e-10          # every row of A sums to 1


def test_attention_row_block_invariance():
    q, k, v = _rand(70, 8, 4), _rand(70, 8, 5), _rand(70, 8, 6)
    o1, s1 = ref.prefill_attention_head(q, k, v, row_block=7)
    o2, s2 = ref.prefill_attention_head(q, k, v, row_block=1000)
    np.testing.assert_allclose(o1, o2, rtol=0, atol=1e-14)
    np.testing.assert_allclose(s1, s2, rtol=0, atol=1e-13)


def test_attention_row_range_is_a_slice_of_the_full_result():
    """Rows are independent: a row range gives exactly those rows of O (checked against the
    library SDPA on the same rows), its column sums are the dense matrix's sums over those
    rows, and with hi = N they are complete for every column j >= lo."""
    n, d = 70, 8
    q, k, v = _rand(n, d, 14), _rand(n, d, 15), _rand(n, d, 16)
    full_o, full_s = ref.prefill_attention_head(q, k, v)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None],
        is_causal=True)[0].numpy()
    A = np.array(brute.attention_matrix(q.tolist(), k.tolist()))
    for lo, hi in [(0, 13), (20, 51), (50, 70)]:
        o, s = ref.prefill_attention_head(q, k, v, row_block=9, row_range=(lo, hi))
        np.testing.assert_allclose(o, want[lo:hi], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(s, A[lo:hi].sum(axis=0), rtol=0, atol=1e-13)
    np.testing.assert_allclose(s[50:], full_s[50:], rtol=0, atol=1e-13)


def test_zero_query_causal_gives_harmonic_column_sums():
    # Q = 0: A[i, j] = 1/(i+1) for j <= i, so s[j] = H_N - H_j (0-based j) exactly.
    n = 40
    k, v = _rand(n, 4, 8), _rand(n, 4, 9)
    o, s = ref.prefill_attention_head(np.zeros((n, 4)), k, v)
    H = [Fraction(0)]
    for i in range(1, n + 1):
        H.append(H[-1] + Fraction(1, i))
    want = [H[n] - H[j] for j in range(n)]
    np.testing.assert_allclose(s, [float(x) for x in want], rtol=1e-13)
    mu = sum(want) / n
    var = sum((x - mu) ** 2 for x in want) / n
    assert abs(ref.head_variance(s) - float(var)) < 1e-13
    # row i of O is the mean of v[0..i]
    np.testing.assert_allclose(o[9], v[:10].mean(axis=0), rtol=1e-12)


def test_zero_query_noncausal_is_uniform():
    n = 33
    o, s = ref.prefill_attention_head(np.zeros((n, 4)), _rand(n, 4, 1), _rand(n, 4, 2),
                                      causal=False)
    np.testing.assert_allclose(s, np.ones(n), rtol=1e-13)
    assert ref.head_variance(s) < 1e-26
    assert ref.layer_density([s, s]) < 1e-26


def test_layer_density_is_the_mean_of_the_head_variances():
    """Eq. 4 with the per-head form of App. A.8: three heads whose column sums have the exact
    population variances 1, 8 and 0 (by hand: [1, 3] -> mean 2, deviations +-1; [0, 0, 6] ->
    mean 2, squared deviations 4, 4, 16; a constant vector) give F = (1 + 8 + 0) / 3 = 3.
    A sum over heads (9), a sample variance (2, 12, 0 -> 14 / 3) or a variance of the pooled
    values would all miss 3."""
    heads = [np.array([1.0, 3.0]), np.array([0.0, 0.0, 6.0]), np.full(5, 2.5)]
    assert ref.head_variance(heads[0]) == 1.0 and ref.head_variance(heads[1]) == 8.0
    assert ref.layer_density(heads) == 3.0
    assert ref.layer_density(heads[:2]) == 4.5
    # a harmonic head (Q = 0, causal) next to a uniform one: half the closed-form variance
    n = 12
    Hn = [Fraction(0)]
    for i in range(1, n + 1):
        Hn.append(Hn[-1] + Fraction(1, i))
    s = [Hn[n] - Hn[j] for j in range(n)]
    mu = sum(s) / n
    var = sum((x - mu) ** 2 for x in s) / n
    got = ref.layer_density([np.array([float(x) for x in s]), np.ones(n)])
    assert abs(got - float(var) / 2) < 1e-14


def test_constant_values_give_constant_output():
    v = np.tile(np.array([[1.5, -2.0, 0.25]]), (20, 1))
    o, _ = ref.prefill_attention_head(_rand(20, 3, 3) * 3, _rand(20, 3, 4), v)
    np.testing.assert_allclose(o, v, rtol=1e-13)


def test_attention_matches_brute_force_matrix():
    n, d = 24, 5
    q, k, v = _rand(n, d, 10) * 2, _rand(n, d, 11), _rand(n, d, 12)
    o, s = ref.prefill_attention_head(q, k, v, row_block=5)
    A = brute.attention_matrix(q.tolist(), k.tolist())
    np.testing.assert_allclose(s, brute.column_sums(A), rtol=1e-12)
    np.testing.assert_allclose(o, brute.attend(A, v.tolist()), rtol=1e-11, atol=1e-13)
    assert abs(ref.head_variance(s) - brute.variance(brute.column_sums(A))) < 1e-13
    assert abs(ref.head_variance(s) - np.var(s)) < 1e-13
    # a transposed operand or a missing mask would break these two:
    assert A[0][1] == 0.0 and abs(s[n - 1] - A[n - 1][n - 1]) < 1e-15


# ------------------------------------------------------------------ allocation (Eq. 5, App. A.2)

def test_allocation_uniform_when_densities_equal():
    S = ref.allocate_budgets(np.full(32, 3.7), 4096, round(0.2 * 4096 * 32), 64)
    assert S.sum() == round(0.2 * 4096 * 32)
    assert S.max() - S.min() <= 1                      # uniform alpha_l = rho
    S = ref.allocate_budgets(np.full(8, 0.1), 1000, 1600, 10)
    assert list(S) == [200] * 8


def test_allocation_two_layer_closed_form():
    F = np.array([0.3, 1.1])
    tot = 1000
    S = ref.allocate_budgets(F, 10_000, tot, 1)
    p0 = 1.0 / (1.0 + math.exp(F[0] - F[1]))           # softmax(-F)[0]
    assert S.sum() == tot and abs(S[0] - p0 * tot) <= 1.0
    assert S[0] > S[1]                                 # lower variance => larger cache


def test_allocation_matches_library_softmax_before_clamping():
    from scipy.special import softmax
    F = rng.uniform(0.0, 2.0, size=16)
    tot = 16 * 300
    S = ref.allocate_budgets(F, 4000, tot, 1)
    want = softmax(-F) * tot
    assert S.sum() == tot
    assert np.all(np.abs(S - want) < 1.0)
    order = np.argsort(F)
    assert np.all(np.diff(S[order]) <= 0)              # F_a < F_b  =>  S_a >= S_b


def test_allocation_clamps_and_conserves():
    F = np.array([0.0, 5.0, 500.0, 2000.0, 1e6, 3.0])  # exp(-F) underflows for some layers
    tot = 6 * 200
    S = ref.allocate_budgets(F, 512, tot, 64)
    assert S.sum() == tot and S.min() >= 64 and S.max() <= 512
    assert S[0] == 512                                 # the densest layer saturates at seq_len
    assert list(S[2:5]) == [64, 64, 64]
    with pytest.raises(ValueError):
        ref.allocate_budgets(F, 512, 6 * 64 - 1, 64)
    with pytest.raises(ValueError):
        ref.allocate_budgets(F, 512, 6 * 512 + 1, 64)


def test_allocation_integer_remainder_goes_to_largest_fractions():
    # equal densities, 3 layers, 10 units: shares 3.33.. each, the extra unit to layer 0
    assert list(ref.allocate_budgets(np.zeros(3), 100, 10, 0)) == [4, 3, 3]
    assert list(ref.allocate_budgets(np.zeros(3), 100, 11, 0)) == [4, 4, 3]


def test_allocation_policies_of_the_policy_analysis():
    """The four designs of alpha_l that Sec. 5 (dynamic allocation policy analysis) compares,
    pinned to their closed forms on inputs whose shares are exact."""
    # reciprocal of variance: weights 1 : 1/2 : 1/4 -> shares 4 : 2 : 1, exact for a multiple of 7
    S = ref.allocate_budgets(np.array([1.0, 2.0, 4.0]), 10_000, 7 * 123, 1, policy="reciprocal")
    assert list(S) == [4 * 123, 2 * 123, 123]
    # uniform: every layer gets rho * S whatever its variance
    S = ref.allocate_budgets(np.array([0.1, 9.0, 3.0, 50.0]), 4096, 4 * 819, 64, policy="uniform")
    assert list(S) == [819] * 4
    assert list(ref.allocate_budgets(np.array([5.0, 0.0, 1.0]), 100, 11, 0, policy="uniform")) == [4, 4, 3]
    # exponential decay: alpha_l = exp(-F_l) is the layer's own ratio, no sum constraint
    F = -np.log(np.array([0.3, 0.0625, 1.0, 1e-9]))
    S = ref.allocate_budgets(F, 1005, 0, 8, policy="exp_decay")
    assert list(S) == [301, 62, 1005, 8]               # 301.5, 62.8, all of it, clipped from 0
    # the three normalised designs spend the same budget and are monotone in the variance;
    # the softmax design is the one without a policy argument
    F = rng.uniform(0.2, 3.0, size=12)
    tot = 12 * 500
    for pol in ("softmax", "reciprocal", "uniform"):
        S = ref.allocate_budgets(F, 4000, tot, 16, policy=pol)
        assert S.sum() == tot and S.min() >= 16 and S.max() <= 4000
        assert np.all(np.diff(S[np.argsort(F)]) <= (1 if pol == "uniform" else 0))
    assert np.array_equal(ref.allocate_budgets(F, 4000, tot, 16), ref.allocate_budgets(F, 4000, tot, 16, policy="softmax"))
    want = (1.0 / F) / (1.0 / F).sum() * tot
    assert np.all(np.abs(ref.allocate_budgets(F, 4000, tot, 1, policy="reciprocal") - want) < 1.0)
    with pytest.raises(ValueError):
        ref.allocate_budgets(np.array([1.0, 0.0]), 100, 50, 1, policy="reciprocal")
    with pytest.raises(ValueError):
        ref.allocate_budgets(np.array([1.0, 2.0]), 100, 50, 1, policy="softmin")


# ------------------------------------------------------------------ selection (Eq. 7-8)

@pytest.mark.parametrize("n,budget,recent,sink", [(30, 12, 3, 0), (30, 12, 4, 2), (17, 6, 6, 0),
                                                  (25, 9, 0, 1), (12, 12, 3, 0), (12, 40, 3, 1)])
def test_selection_matches_repeated_removal(n, budget, recent, sink):
    g = np.random.default_rng(n * 100 + budget)
    for trial in range(20):
        score = g.integers(0, 6, size=n).astype(float) if trial % 2 else g.random(n)
        ret, evi = ref.select(score, budget, recent, sink)
        alive, dropped = brute.choose_retained(score.tolist(), budget, recent, sink)
        assert list(ret) == alive and list(evi) == dropped
        assert len(ret) == min(budget, n)
        assert sorted(list(ret) + list(evi)) == list(range(n))


def test_selection_without_heavy_hitters_is_sink_plus_window():
    ret, evi = ref.select(rng.random(50), 10, 7, 3)
    assert list(ret) == [0, 1, 2] + list(range(43, 50))
    with pytest.raises(ValueError):
        ref.select(rng.random(50), 5, 4, 2)


def test_selection_tie_keeps_lower_index():
    score = np.array([9.0, 1.0, 1.0, 1.0, 1.0, 9.0])
    ret, evi = ref.select(score, 3, 1, 0)              # window = {5}; top-2 of [0..4]
    assert list(ret) == [0, 1, 5] and list(evi) == [2, 3, 4]


# ------------------------------------------------------------------ matching (Eq. 9)

def test_cosine_properties_and_library_value():
    from scipy.spatial.distance import cosine as cosine_distance
    Ke, Kc = _rand(9, 6, 20), _rand(7, 6, 21)
    U = ref.cosine_matrix(Ke, Kc)
    assert np.all(U <= 1 + 1e-15) and np.all(U >= -1 - 1e-15)
    for i in range(9):
        for j in range(7):
            assert abs(U[i, j] - (1.0 - cosine_distance(Ke[i], Kc[j]))) < 1e-14
            assert abs(U[i, j] - brute.cosine(Ke[i].tolist(), Kc[j].tolist())) < 1e-14
    np.testing.assert_allclose(np.diag(ref.cosine_matrix(Kc, Kc)), 1.0, rtol=1e-15)
    U2 = ref.cosine_matrix(Ke * 3.5, Kc * 0.01)        # scale invariance
    np.testing.assert_allclose(U2, U, rtol=1e-13, atol=1e-15)
    assert np.all(ref.cosine_matrix(np.zeros((2, 6)), Kc) == 0.0)


def test_matching_finds_planted_twins_and_first_maximum():
    Kc = _rand(10, 8, 30)
    Kc[7] = Kc[2]                                       # duplicate retained keys
    Ke = np.vstack([Kc[4] * 2.0, Kc[2], _rand(1, 8, 31)])
    u, t = ref.match(Ke, Kc)
    assert t[0] == 4 and abs(u[0] - 1) < 1e-15
    assert t[1] == 2 and abs(u[1] - 1) < 1e-15          # first maximum, not index 7
    bu, bj = brute.nearest(np.vstack([Kc, Ke]).tolist(), list(range(10)), [10, 11, 12])
    assert bj == list(t)
    np.testing.assert_allclose(u, bu, rtol=1e-14)


# ------------------------------------------------------------------ threshold (Eq. 10)

def test_threshold_prefill_and_ema_closed_form():
    u = rng.random(25)
    tau, passed = ref.prefill_threshold(u)
    assert u.min() <= tau <= u.max() and abs(tau - math.fsum(u) / 25) < 1e-15
    assert list(passed) == [x >= tau for x in u]
    assert math.isnan(ref.prefill_threshold(np.zeros(0))[0])
    beta, tau0 = 0.7, 0.4
    us = rng.random(12)
    t = tau0
    for x in us:
        t = ref.ema_threshold(t, x, beta)
    T = len(us)
    closed = (1 - beta) ** T * tau0 + beta * sum((1 - beta) ** (T - 1 - k) * us[k]
                                                 for k in range(T))
    assert abs(t - closed) < 1e-14
    assert ref.ema_threshold(0.83, 0.83, 0.6) == pytest.approx(0.83, abs=1e-16)
    assert ref.ema_threshold(float("nan"), 0.31, 0.6) == 0.31


# ------------------------------------------------------------------ merge (Eq. 11-12)

def test_merge_two_token_hand_example():
    # kept k=[1,0], evicted k=[0,1], u=0: weights e/(e+1) and 1/(e+1)
    Kc, Vc = np.array([[1.0, 0.0]]), np.array([[2.0, 4.0]])
    Ke, Ve = np.array([[0.0, 1.0]]), np.array([[-1.0, 1.0]])
    K2, V2, n = ref.merge(Kc, Vc, Ke, Ve, np.array([0.0]), np.array([0]), np.array([True]))
    wc, we = math.e / (math.e + 1), 1 / (math.e + 1)
    np.testing.assert_allclose(K2[0], [wc, we], rtol=1e-15)
    np.testing.assert_allclose(V2[0], [2 * wc - we, 4 * wc + we], rtol=1e-15)
    assert n[0] == 1 and wc > we                        # the kept token has the largest weight


def test_merge_copies_of_twin_average_the_values():
    m = 5
    Kc, Vc = _rand(3, 4, 40), _rand(3, 4, 41)
    Ke = np.tile(Kc[1], (m, 1))
    Ve = _rand(m, 4, 42)
    K2, V2, n = ref.merge(Kc, Vc, Ke, Ve, np.ones(m), np.full(m, 1), np.ones(m, bool))
    np.testing.assert_allclose(K2[1], Kc[1], rtol=1e-14)                 # weights sum to 1
    np.testing.assert_allclose(V2[1], (Vc[1] + Ve.sum(0)) / (m + 1), rtol=1e-14)
    assert np.array_equal(K2[[0, 2]], Kc[[0, 2]]) and list(n) == [0, m, 0]


def test_average_merging_is_the_plain_mean_of_the_group():
    """The merge-policy ablation's alternative (Sec. 5): every member of a group weighs the same,
    whatever its similarity."""
    Kc, Vc, Ke, Ve = _rand(4, 6, 60), _rand(4, 6, 61), _rand(9, 6, 62), _rand(9, 6, 63)
    u = rng.uniform(-1, 1, size=9)
    t = np.array([0, 2, 2, 3, 2, 0, 3, 3, 3])
    passed = np.array([1, 1, 0, 1, 1, 1, 1, 0, 1], bool)
    K2, V2, n = ref.merge(Kc, Vc, Ke, Ve, u, t, passed, weighted=False)
    for j in range(4):
        src = [i for i in range(9) if passed[i] and t[i] == j]
        np.testing.assert_allclose(K2[j], np.vstack([Kc[j:j + 1], Ke[src]]).mean(0), rtol=1e-14)
        np.testing.assert_allclose(V2[j], np.vstack([Vc[j:j + 1], Ve[src]]).mean(0), rtol=1e-14)
        assert n[j] == len(src)
    assert np.array_equal(K2[1], Kc[1])                  # no source: untouched
    # two tokens: the midpoint, where Eq. 11-12 lean towards the kept token
    Km, _, _ = ref.merge(np.array([[1.0, 0.0]]), np.zeros((1, 2)), np.array([[0.0, 1.0]]), np.zeros((1, 2)),
                         np.array([0.3]), np.array([0]), np.array([True]), weighted=False)
    assert list(Km[0]) == [0.5, 0.5]
    Kw, _, _ = ref.merge(np.array([[1.0, 0.0]]), np.zeros((1, 2)), np.array([[0.0, 1.0]]), np.zeros((1, 2)),
                         np.array([0.3]), np.array([0]), np.array([True]))
    assert Kw[0][0] > 0.5 > Kw[0][1]


def test_merge_convex_hull_mask_and_brute_force():
    Kc, Vc, Ke, Ve = _rand(6, 5, 50), _rand(6, 5, 51), _rand(14, 5, 52), _rand(14, 5, 53)
    u, t = ref.match(Ke, Kc)
    tau, passed = ref.prefill_threshold(u)
    K2, V2, n = ref.merge(Kc, Vc, Ke, Ve, u, t, passed)
    assert n.sum() == passed.sum()
    for j in range(6):
        src = [i for i in range(14) if passed[i] and t[i] == j]
        grpK = np.vstack([Kc[j:j + 1], Ke[src]])
        grpV = np.vstack([Vc[j:j + 1], Ve[src]])
        assert np.all(K2[j] <= grpK.max(0) + 1e-15) and np.all(K2[j] >= grpK.min(0) - 1e-15)
        assert np.all(V2[j] <= grpV.max(0) + 1e-15) and np.all(V2[j] >= grpV.min(0) - 1e-15)
    allK, allV = np.vstack([Kc, Ke]).tolist(), np.vstack([Vc, Ve]).tolist()
    bK, bV = brute.merged_rows(allK, allV, list(range(6)), list(range(6, 20)), list(u),
                               list(t), list(passed))
    np.testing.assert_allclose(K2, [bK[j] for j in range(6)], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(V2, [bV[j] for j in range(6)], rtol=1e-13, atol=1e-15)
    # failed tokens are discarded: with nothing passing the cache rows are bit copies
    K3, V3, n3 = ref.merge(Kc, Vc, Ke, Ve, u, t, np.zeros(14, bool))
    assert np.array_equal(K3, Kc) and np.array_equal(V3, Vc) and n3.sum() == 0


def test_round_storage_bf16_matches_torch_and_is_idempotent():
    x = np.concatenate([rng.standard_normal(4000) * 10, [0.0, 1.0, -1.0, 1.00390625, 3.0e-3]])
    got = ref.round_storage(x, "bf16")
    # torch rounds fp32 -> bf16 to nearest even; feed it values exactly representable in fp32
    x32 = x.astype(np.float32).astype(np.float64)
    want = torch.from_numpy(x32.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(ref.round_storage(x32, "bf16"), want)
    np.testing.assert_array_equal(ref.round_storage(got, "bf16"), got)
    assert np.all(np.abs(got - x) <= np.abs(x) * 2.0 ** -8)
    # a tie: 1 + 2^-8 lies midway between 1 and 1 + 2^-7 and must go to the even mantissa
    assert ref.round_storage(np.array([1.0 + 2.0 ** -8]), "bf16")[0] == 1.0
    assert ref.round_storage(np.array([1.0 + 3 * 2.0 ** -8]), "bf16")[0] == 1.0 + 2.0 ** -6


# ------------------------------------------------------------------ whole method, brute force

@pytest.mark.parametrize("n,d,G,budget,recent,sink,steps", [
    (40, 6, 1, 12, 3, 0, 6), (33, 4, 2, 10, 4, 1, 5), (48, 8, 1, 16, 8, 2, 4),
    (20, 4, 1, 7, 0, 0, 4), (20, 4, 3, 6, 6, 0, 3), (16, 4, 1, 40, 5, 0, 3)])
def test_whole_method_matches_brute_force(n, d, G, budget, recent, sink, steps):
    g = np.random.default_rng(n + 17 * d + budget)
    cen = g.standard_normal((3, d)) * 2
    K = cen[g.integers(0, 3, n)] + 0.3 * g.standard_normal((n, d))
    V = g.standard_normal((n, d))
    Q = cen[g.integers(0, 3, (G, n))] + 0.5 * g.standard_normal((G, n, d))
    O, score, var = ref.prefill_kv_head(Q, K, V)
    A = [brute.attention_matrix(Q[h].tolist(), K.tolist()) for h in range(G)]
    bscore = [math.fsum(brute.column_sums(A[h])[j] for h in range(G)) for j in range(n)]
    np.testing.assert_allclose(score, bscore, rtol=1e-12)
    np.testing.assert_allclose(var, [brute.variance(brute.column_sums(a)) for a in A],
                               rtol=1e-10, atol=1e-14)
    cache, ev = ref.compress_head(K, V, score, budget, recent, sink)
    st, bev = brute.compress(K.tolist(), V.tolist(), bscore, budget, recent, sink)
    assert list(ev.retained) == bev["ret"] and list(ev.evicted) == bev["evi"]
    assert list(ev.target) == bev["t"] and list(ev.passed) == bev["passed"]
    np.testing.assert_allclose(ev.u_star, bev["u"], rtol=1e-13)
    np.testing.assert_allclose(cache.K, st["K"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(cache.V, st["V"], rtol=1e-12, atol=1e-14)
    assert len(ev.retained) + ev.passed.sum() + (~ev.passed).sum() == n
    for t in range(steps):
        q = cen[g.integers(0, 3, G)] + 0.5 * g.standard_normal((G, d))
        kn = cen[g.integers(0, 3)] + 0.3 * g.standard_normal(d)
        vn = g.standard_normal(d)
        out, e = ref.decode_step_head(cache, q, kn, vn, n + t, budget, recent, sink, 0.6)
        bout, be = brute.decode_step(st, q.tolist(), kn.tolist(), vn.tolist(), n + t, budget,
                                     recent, sink, 0.6)
        np.testing.assert_allclose(out, bout, rtol=1e-11, atol=1e-13)
        assert (e.evicted_pos, e.target_pos) == (be[0], be[1])
        assert list(cache.pos) == st["pos"]
        np.testing.assert_allclose(cache.K, st["K"], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(cache.score, st["score"], rtol=1e-12)
        if not math.isnan(cache.tau):
            assert abs(cache.tau - st["tau"]) < 1e-13


# ------------------------------------------------------------------ reductions and decode invariants

def _small_case(seed=3, n=64, d=8, G=2):
    g = np.random.default_rng(seed)
    cen = g.standard_normal((4, d)) * 2
    K = cen[g.integers(0, 4, n)] + 0.3 * g.standard_normal((n, d))
    V = g.standard_normal((n, d))
    Q = cen[g.integers(0, 4, (G, n))] + 0.5 * g.standard_normal((G, n, d))
    return g, cen, Q, K, V


def test_budget_at_least_prompt_length_is_full_attention():
    g, cen, Q, K, V = _small_case()
    n, d = K.shape
    _, score, _ = ref.prefill_kv_head(Q, K, V)
    cache, ev = ref.compress_head(K, V, score, n + 10, 4, 0)
    assert len(ev.evicted) == 0 and math.isnan(cache.tau) and np.array_equal(cache.K, K)
    Ks, Vs = K.copy(), V.copy()
    for t in range(5):
        q, kn, vn = g.standard_normal((2, d)), g.standard_normal(d), g.standard_normal(d)
        out, e = ref.decode_step_head(cache, q, kn, vn, n + t, n + 10, 4, 0, 0.7)
        Ks, Vs = np.vstack([Ks, kn]), np.vstack([Vs, vn])
        want = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(q)[:, None, :], torch.from_numpy(Ks)[None].expand(2, -1, -1),
            torch.from_numpy(Vs)[None].expand(2, -1, -1))[:, 0].numpy()
        np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-14)
        assert e.evicted_pos == -1
        assert abs(cache.score.sum() - 2 * (n + t + 1)) < 1e-9   # +G per step, nothing lost


def test_never_merging_is_pure_heavy_hitter_eviction():
    g, cen, Q, K, V = _small_case(5)
    _, score, _ = ref.prefill_kv_head(Q, K, V)
    cache, ev = ref.compress_head(K, V, score, 20, 5, 1, tau_force=float("inf"))
    assert not ev.passed.any()
    assert np.array_equal(cache.K, K[ev.retained]) and np.array_equal(cache.V, V[ev.retained])
    cache2, ev2 = ref.compress_head(K, V, score, 20, 5, 1, tau_force=float("-inf"))
    assert ev2.passed.all() and np.array_equal(ev2.retained, ev.retained)
    for t in range(4):
        out, e = ref.decode_step_head(cache, g.standard_normal((2, 8)), g.standard_normal(8),
                                      g.standard_normal(8), 64 + t, 20, 5, 1, 0.7,
                                      tau_force=float("inf"))
        assert e.target_pos == -1 and e.evicted_pos >= 0


def test_decode_zero_query_uniform_scores_and_window():
    g, cen, Q, K, V = _small_case(9)
    n, d, G = 64, 8, 2
    _, score, _ = ref.prefill_kv_head(Q, K, V)
    budget, recent = 16, 4
    cache, _ = ref.compress_head(K, V, score, budget, recent, 0)
    for t in range(8):
        before = cache.score.copy()
        pos_before = cache.pos.copy()
        vn = g.standard_normal(d)
        want_out = np.vstack([cache.V, vn]).mean(axis=0)
        out, e = ref.decode_step_head(cache, np.zeros((G, d)), g.standard_normal(d), vn,
                                      n + t, budget, recent, 0, 0.7)
        # uniform p = 1/(c+1): every surviving old slot gained G/(c+1)
        keep = np.isin(pos_before, cache.pos)
        np.testing.assert_allclose(cache.score[:-1] - before[keep], G / (budget + 1), rtol=1e-12)
        assert cache.pos.size == budget and cache.pos[-1] == n + t
        assert e.evicted_pos >= 0 and e.evicted_pos <= n + t - recent   # window is protected
        assert set(range(n + t - recent + 1, n + t + 1)) <= set(cache.pos.tolist())
        np.testing.assert_allclose(out[0], want_out, rtol=1e-12, atol=1e-14)


def test_decode_merge_is_two_term_weighted_mean():
    d = 4
    K = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0], [0.9, 0.1, 0, 0], [0, 0, 1.0, 0]])
    V = np.arange(16, dtype=float).reshape(4, 4)
    cache = ref.HeadCache(K.copy(), V.copy(), np.array([5.0, 4.0, 0.1, 3.0]),
                          np.arange(4), 0.2, "f64")
    q = np.zeros((1, d))
    out, e = ref.decode_step_head(cache, q, np.array([0, 0, 0, 1.0]), np.ones(4), 4, 4, 1, 0, 0.5)
    assert e.evicted_pos == 2 and e.target_pos == 0      # nearest to [0.9, 0.1] is [1, 0]
    u = 0.9 / math.sqrt(0.82)
    assert abs(e.u_star - u) < 1e-15 and abs(e.tau - (0.5 * u + 0.5 * 0.2)) < 1e-15
    w = math.exp(u)
    np.testing.assert_allclose(cache.K[0], (math.e * K[0] + w * K[2]) / (math.e + w), rtol=1e-15)
    np.testing.assert_allclose(cache.V[0], (math.e * V[0] + w * V[2]) / (math.e + w), rtol=1e-15)
    assert list(cache.pos) == [0, 1, 3, 4]


def test_allocation_is_the_clipped_proportional_solution():
    # Independent check by bisection on lambda: S_l = clip(lambda * exp(-F_l), lo, hi).
    g = np.random.default_rng(11)
    for trial in range(30):
        L = int(g.integers(2, 12))
        F = g.uniform(0, 12, size=L) * g.choice([0.1, 1.0, 30.0])
        lo, hi = 8, 300
        tot = int(g.integers(L * lo, L * hi + 1))
        S = ref.allocate_budgets(F, hi, tot, lo)
        w = np.exp(-(F - F.min()))
        a, b = 0.0, 1e300
        for _ in range(2000):
            mid = 0.5 * (a + b) if b < 1e299 else max(1.0, a * 2)
            if np.clip(mid * w, lo, hi).sum() < tot:
                a = mid
            else:
                b = mid
        want = np.clip(b * w, lo, hi)
        assert S.sum() == tot and S.min() >= lo and S.max() <= hi
        assert np.all(np.abs(S - want) <= 1.0 + 1e-6), (F, tot, S, want)


def test_per_head_allocation_is_the_softmax_over_all_layers_and_heads():
    """App. A.8: S_l^h = S_total * exp(-F^{l,h}) / sum over all (l, h); the layer proportions are the
    sums over heads and add up to 1; with every head of a layer alike and one KV head per query
    head the layer totals are those of Eq. 5 scaled by the head count."""
    from scipy.special import softmax
    g = np.random.default_rng(31)
    L, H = 6, 4
    F = g.uniform(0.0, 2.0, size=(L, H))
    total = L * H * 300
    S = ref.allocate_budgets_heads(F, 1, 5000, total, 1)
    want = softmax(-F.reshape(-1)).reshape(L, H) * total
    assert S.sum() == total and np.all(np.abs(S - want) < 1.0)
    alpha_l = softmax(-F.reshape(-1)).reshape(L, H).sum(axis=1)
    assert abs(alpha_l.sum() - 1.0) < 1e-12 and np.all(np.abs(S.sum(axis=1) - alpha_l * total) < H)
    # heads of a layer alike: the per-layer form of Eq. 5, H times over
    Fl = g.uniform(0.0, 2.0, size=L)
    Sh = ref.allocate_budgets_heads(np.repeat(Fl[:, None], H, axis=1), 1, 5000, total, 1)
    Sl = ref.allocate_budgets(Fl, 5000, total // H, 1)
    assert np.all(np.abs(Sh - Sl[:, None]) <= 1)
    # grouped-query: a KV head's statistic is the mean of its query heads' variances
    Fq = g.uniform(0.0, 2.0, size=(L, 8))
    Sg = ref.allocate_budgets_heads(Fq, 4, 5000, L * 2 * 300, 1)
    assert Sg.shape == (L, 2)
    assert np.array_equal(Sg, ref.allocate_budgets_heads(Fq.reshape(L, 2, 4).mean(axis=2), 1, 5000, L * 2 * 300, 1))
    # lower variance, larger cache - across layers AND heads
    order = np.argsort(Fq.reshape(L, 2, 4).mean(axis=2).reshape(-1))
    assert np.all(np.diff(Sg.reshape(-1)[order]) <= 0)


# ------------------------------------------------------------------ multi-token append

def _random_head_state(n, d, budget, recent, sink, seed, G=2):
    g = np.random.default_rng(seed)
    K, V = g.standard_normal((n, d)), g.standard_normal((n, d))
    Q = g.standard_normal((G, n, d)) * 1.5
    _, score, _ = ref.prefill_kv_head(Q, K, V)
    cache, _ = ref.compress_head(K, V, score, budget, recent, sink)
    return cache, g


def _copy_cache(c):
    return ref.HeadCache(c.K.copy(), c.V.copy(), c.score.copy(), c.pos.copy(), c.tau, c.storage)


def test_append_of_one_token_is_a_generation_step():
    """m = 1: the block form must be the generation step of Eq. 6-12, bit for bit."""
    d, G, budget, recent, sink, beta = 6, 2, 12, 3, 1, 0.6
    cache, g = _random_head_state(30, d, budget, recent, sink, 3, G)
    a, b = _copy_cache(cache), _copy_cache(cache)
    for t in range(9):
        q, k, v = g.standard_normal((G, d)) * 2, g.standard_normal(d), g.standard_normal(d)
        out1, e1 = ref.decode_step_head(a, q, k, v, 30 + t, budget, recent, sink, beta)
        out2, e2 = ref.append_chunk_head(b, q[:, None, :], k[None], v[None], 30 + t, budget, recent, sink, beta)
        assert np.array_equal(out1, out2[:, 0])
        assert list(e2.evicted) == ([e1.evicted_pos] if e1.evicted_pos >= 0 else [])
        if e1.evicted_pos >= 0:
            assert e2.u_star[0] == e1.u_star and e2.tau == e1.tau
            assert (int(e2.target[0]) if e2.passed[0] else -1) == e1.target_pos
        assert np.array_equal(a.K, b.K) and np.array_equal(a.V, b.V)
        assert np.array_equal(a.score, b.score) and np.array_equal(a.pos, b.pos)


def test_append_to_an_empty_cache_is_prompt_encoding():
    """A block appended to an empty cache with no threshold yet is prompt encoding: causal
    attention over the block, column sums as scores (Eq. 6, prompt case), and the token-level
    operation with tau_0 = mean best similarity (Eq. 10, t = 0)."""
    n, d, G, budget, recent, sink = 40, 5, 2, 14, 4, 2
    g = np.random.default_rng(11)
    K, V = g.standard_normal((n, d)), g.standard_normal((n, d))
    Q = g.standard_normal((G, n, d)) * 2
    O, score, _ = ref.prefill_kv_head(Q, K, V)
    want, ev = ref.compress_head(K, V, score, budget, recent, sink)
    empty = ref.HeadCache(np.zeros((0, d)), np.zeros((0, d)), np.zeros(0), np.zeros(0, dtype=np.int64),
                          float("nan"))
    out, ae = ref.append_chunk_head(empty, Q, K, V, 0, budget, recent, sink, 0.7)
    np.testing.assert_allclose(out, O, rtol=1e-12, atol=1e-14)
    assert np.array_equal(empty.pos, want.pos) and np.array_equal(ae.evicted, ev.evicted)
    assert np.array_equal(ae.target, ev.target) and np.array_equal(ae.passed, ev.passed)
    np.testing.assert_allclose(empty.score, want.score, rtol=1e-12)
    np.testing.assert_allclose(ae.u_star, ev.u_star, rtol=0, atol=1e-15)
    assert abs(ae.tau - ev.tau) < 1e-14
    np.testing.assert_allclose(empty.K, want.K, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(empty.V, want.V, rtol=1e-12, atol=1e-14)


def test_append_within_budget_is_full_causal_attention_over_cache_and_block():
    """budget >= count: nothing is evicted, outputs equal the library's attention of the block's
    queries over [cache; block] with a causal mask inside the block, and the scores grow by G per
    token in total (every softmax row sums to 1)."""
    d, G, m = 8, 3, 7
    g = np.random.default_rng(5)
    c0 = 20
    Kc, Vc = g.standard_normal((c0, d)), g.standard_normal((c0, d))
    cache = ref.HeadCache(Kc.copy(), Vc.copy(), g.random(c0), np.arange(c0, dtype=np.int64), 0.4)
    q, k, v = g.standard_normal((G, m, d)) * 2, g.standard_normal((m, d)), g.standard_normal((m, d))
    before = cache.score.sum()
    out, ev = ref.append_chunk_head(cache, q, k, v, c0, 100, 5, 0, 0.7)
    assert ev.evicted.size == 0 and cache.pos.size == c0 + m and cache.tau == 0.4
    assert abs(cache.score.sum() - before - G * m) < 1e-10
    Kall, Vall = np.vstack([Kc, k]), np.vstack([Vc, v])
    mask = torch.ones(m, c0 + m, dtype=torch.bool)
    for i in range(m):
        mask[i, c0 + i + 1:] = False
    for h in range(G):
        want = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(q[h])[None], torch.from_numpy(Kall)[None], torch.from_numpy(Vall)[None],
            attn_mask=mask[None])[0].numpy()
        np.testing.assert_allclose(out[h], want, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("n,d,G,budget,recent,sink,m,rounds", [
    (24, 4, 1, 10, 3, 0, 5, 3),
    (30, 3, 2, 9, 2, 1, 4, 4),
    (16, 5, 2, 12, 0, 2, 9, 2),       # no recent window, a block almost as large as the budget
    (20, 4, 1, 8, 8, 0, 3, 3),        # no heavy hitters: sinks + window only
])
def test_append_matches_brute_force(n, d, G, budget, recent, sink, m, rounds):
    g = np.random.default_rng(n * 100 + m)
    K, V = g.standard_normal((n, d)), g.standard_normal((n, d))
    Q = g.standard_normal((G, n, d)) * 1.5
    _, score, _ = ref.prefill_kv_head(Q, K, V)
    cache, _ = ref.compress_head(K, V, score, budget, recent, sink)
    A = [brute.attention_matrix(Q[h].tolist(), K.tolist()) for h in range(G)]
    bscore = [math.fsum(brute.column_sums(A[h])[j] for h in range(G)) for j in range(n)]
    state, _ = brute.compress(K.tolist(), V.tolist(), bscore, budget, recent, sink)
    pos = n
    for r in range(rounds):
        q, k, v = g.standard_normal((G, m, d)) * 2, g.standard_normal((m, d)), g.standard_normal((m, d))
        out, ev = ref.append_chunk_head(cache, q, k, v, pos, budget, recent, sink, 0.7)
        bout, bev = brute.append_chunk(state, [[q[h, i].tolist() for h in range(G)] for i in range(m)],
                                       k.tolist(), v.tolist(), pos, budget, recent, sink, 0.7)
        pos += m
        assert list(ev.evicted) == bev["evi"] and list(ev.target) == bev["t"]
        assert list(ev.passed) == bev["passed"]
        np.testing.assert_allclose(ev.u_star, bev["u"], rtol=0, atol=1e-14)
        for i in range(m):
            for h in range(G):
                np.testing.assert_allclose(out[h, i], bout[i][h], rtol=1e-11, atol=1e-13)
        assert list(cache.pos) == state["pos"] and abs(cache.tau - state["tau"]) < 1e-13
        np.testing.assert_allclose(cache.K, np.array(state["K"]), rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(cache.V, np.array(state["V"]), rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(cache.score, np.array(state["score"]), rtol=1e-11)
        assert cache.pos.size == budget


def test_append_threshold_is_the_ema_of_the_mean_best_similarity():
    """Eq. 10 for a step with several evicted tokens: tau <- beta * mean(u*) + (1 - beta) * tau, and
    the flags test against the updated value; a forced threshold leaves tau alone."""
    d, G, budget, recent, sink, beta, m = 6, 1, 10, 2, 0, 0.3, 6
    cache, g = _random_head_state(25, d, budget, recent, sink, 8, G)
    tau0 = cache.tau
    q, k, v = g.standard_normal((G, m, d)), g.standard_normal((m, d)), g.standard_normal((m, d))
    forced = _copy_cache(cache)
    _, ev = ref.append_chunk_head(cache, q, k, v, 25, budget, recent, sink, beta)
    assert ev.evicted.size == m
    want = beta * float(np.mean(ev.u_star)) + (1 - beta) * tau0
    assert abs(cache.tau - want) < 1e-15 and np.array_equal(ev.passed, ev.u_star >= cache.tau)
    _, evf = ref.append_chunk_head(forced, q, k, v, 25, budget, recent, sink, beta, tau_force=float("inf"))
    assert forced.tau == tau0 and not evf.passed.any() and np.array_equal(evf.evicted, ev.evicted)


# ------------------------------------------------------------------ upstream: projection and rotary embedding

def test_rope_is_a_complex_rotation_and_depends_on_relative_position_only():
    g = np.random.default_rng(4)
    d, n = 16, 9
    x = g.standard_normal((3, n, d))
    pos = np.array([0, 1, 2, 5, 17, 100, 1000, 4095, 131071])
    y = ref.rope_rotate(x, pos, 10000.0)
    # independent formulation: the pair (x_i, x_{i+d/2}) as a complex number times exp(i * angle)
    z = (x[..., :d // 2] + 1j * x[..., d // 2:]) * np.exp(1j * pos[:, None] * 10000.0 ** (-2.0 * np.arange(d // 2) / d))
    np.testing.assert_allclose(y, np.concatenate([z.real, z.imag], axis=-1), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(y[:, 0], x[:, 0], rtol=0, atol=0)                    # position 0: identity
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)
    # <rope(q, p), rope(k, p')> depends on p - p' only
    q, k = g.standard_normal(d), g.standard_normal(d)
    def dot_at(p, pp):
        return float(ref.rope_rotate(q[None], [p], 500000.0)[0] @ ref.rope_rotate(k[None], [pp], 500000.0)[0])
    assert abs(dot_at(7, 3) - dot_at(1007, 1003)) < 1e-9 and abs(dot_at(7, 3) - dot_at(4, 0)) < 1e-10
    assert abs(dot_at(7, 3) - dot_at(3, 7)) > 1e-3                                  # but on its sign


def test_qkv_projection_layout_and_library_matmul():
    g = np.random.default_rng(9)
    n, hidden, Hq, Hkv, d = 7, 12, 4, 2, 6
    X, W = g.standard_normal((n, hidden)), g.standard_normal(((Hq + 2 * Hkv) * d, hidden))
    Q, K, V = ref.qkv_project(X, W, Hq, Hkv, d, pos0=0, base=10000.0)
    assert Q.shape == (Hq, n, d) and K.shape == (Hkv, n, d) and V.shape == (Hkv, n, d)
    lin = torch.nn.functional.linear(torch.from_numpy(X), torch.from_numpy(W)).numpy()     # library routine
    np.testing.assert_allclose(V[1], lin[:, (Hq + Hkv + 1) * d:(Hq + Hkv + 2) * d], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(Q[2, 0], lin[0, 2 * d:3 * d], rtol=1e-12, atol=1e-13)       # position 0: no rotation
    np.testing.assert_allclose(K[1], ref.rope_rotate(lin[:, (Hq + 1) * d:(Hq + 2) * d], np.arange(n)), rtol=1e-12, atol=1e-13)
    # a position offset shifts the rotation, not the projection
    Q5, K5, V5 = ref.qkv_project(X, W, Hq, Hkv, d, pos0=5)
    np.testing.assert_array_equal(V5, V)
    np.testing.assert_allclose(Q5[3], ref.rope_rotate(lin[:, 3 * d:4 * d], np.arange(5, 5 + n)), rtol=1e-12, atol=1e-13)
    # one hot hidden state picks a column of W: X = e_j gives feature f the value W[f, j]
    E = np.zeros((1, hidden)); E[0, 3] = 1.0
    Qe, Ke, Ve = ref.qkv_project(E, W, Hq, Hkv, d)
    np.testing.assert_allclose(Ve[0, 0], W[(Hq + Hkv) * d:(Hq + Hkv + 1) * d, 3], rtol=0, atol=0)


# ------------------------------------------------------------------ fp8 cache encoding

def _e4m3_values():
    """Every finite value of the 8-bit format E4M3 (sign, 4 exponent bits with bias 7, 3 fraction
    bits; exponent field 0 = subnormal; the all-ones code with fraction 7 is NaN), built from the
    format's definition, not from the oracle."""
    vals = []
    for code in range(256):
        sign, ef, fr = code >> 7, (code >> 3) & 15, code & 7
        if ef == 15 and fr == 7:
            continue
        mag = fr / 8.0 * 2.0 ** -6 if ef == 0 else (1.0 + fr / 8.0) * 2.0 ** (ef - 7)
        vals.append(-mag if sign else mag)
    return np.array(sorted(set(vals)))


def test_fp8_rows_grid_values_are_fixed_points_and_midpoints_round_to_even():
    grid = _e4m3_values()
    assert grid.size == 253 and grid.max() == 448.0 and grid[grid > 0].min() == 2.0 ** -9
    # a row whose largest magnitude is 448 gets the scale 2^0: every grid value must come back unchanged
    for v in grid:
        assert ref.quantise_fp8_rows(np.array([v, 448.0]))[0] == v
    pos = grid[grid >= 0]
    for a, b in zip(pos[:-1], pos[1:]):
        got = ref.quantise_fp8_rows(np.array([(a + b) / 2, 448.0]))[0]
        # ties go to the value with the even fraction: of two neighbours exactly one is an even multiple of the spacing
        even = a if round(a / (b - a)) % 2 == 0 else b
        assert got == even, (a, b, got)
        assert ref.quantise_fp8_rows(np.array([a + 0.49 * (b - a), 448.0]))[0] == a
        assert ref.quantise_fp8_rows(np.array([a + 0.51 * (b - a), 448.0]))[0] == b
        assert ref.quantise_fp8_rows(np.array([-(a + 0.51 * (b - a)), 448.0]))[0] == -b


def test_fp8_rows_match_the_library_cast_scale_is_minimal_and_commutes_with_powers_of_two():
    rng = np.random.default_rng(11)
    x = rng.standard_normal((500, 128)) * np.exp(3 * rng.standard_normal((500, 1)))
    x = ref.round_storage(x, "bf16")                       # what enters the cache: bf16 rows
    x[7] = 0.0                                             # an all-zero row stays zero
    x[8, :] = 0.0
    x[8, 5] = -3.0                                         # a row with one element
    q = ref.quantise_fp8_rows(x)
    assert np.array_equal(q[7], np.zeros(128)) and q[8, 5] == -3.0
    amax = np.abs(x).max(-1)
    nz = amax > 0
    # the scale: the smallest power of two that brings the row's largest magnitude to 448 or below
    # (found here by search), and every encoded element is a grid value times that power
    grid = set(_e4m3_values().tolist())
    for r, qr, a in zip(x[nz][:100], q[nz][:100], amax[nz][:100]):
        e = next(k for k in range(-80, 80) if a * 2.0 ** -k <= 448.0)
        assert a * 2.0 ** -(e - 1) > 448.0
        assert all(v in grid for v in (qr * 2.0 ** -e).tolist())
    # against torch's float8_e4m3fn cast of the scaled row (bf16 inputs: the scaled values are exact in fp32)
    for r in x[nz][:200]:
        a = np.abs(r).max()
        fr, ex = np.frexp(a)
        e = int(ex - 9 if fr <= 0.875 else ex - 8)
        y = torch.tensor(np.ldexp(r, -e), dtype=torch.float32)
        assert float(y.abs().max()) <= 448.0 and float(y.abs().max()) > 224.0
        want = np.ldexp(y.to(torch.float8_e4m3fn).to(torch.float64).numpy(), e)
        assert np.array_equal(ref.quantise_fp8_rows(r), want)
    # error bound: half a spacing, i.e. 2^-4 relative for normal results, 2^-10 of the scale below
    err = np.abs(q - x)
    assert np.all(err <= np.maximum(2.0 ** -4 * np.abs(x), 2.0 ** -10 * (np.abs(q).max(-1, keepdims=True) / 224.0)))
    # idempotent, odd, and commuting with powers of two
    assert np.array_equal(ref.quantise_fp8_rows(q), q)
    assert np.array_equal(ref.quantise_fp8_rows(-x), -q)
    assert np.array_equal(ref.quantise_fp8_rows(x * 2.0 ** -7), q * 2.0 ** -7)
    assert np.array_equal(ref.round_storage(x, "fp8"), q)


def test_fp8_cache_every_row_is_encoded_and_decode_reads_the_encoded_rows():
    """storage = "fp8": after prompt compression every cache row (merged or not) is a fixed point
    of the encoding; a generation step encodes the new row before attending to it, so its
    output is full attention over the encoded rows (the library's SDPA on them); with the
    threshold at +inf (pure eviction) the surviving rows are never rewritten."""
    rng = np.random.default_rng(5)
    n, d, budget, recent = 90, 16, 30, 8
    K = ref.round_storage(rng.standard_normal((n, d)) * 2, "bf16")
    V = ref.round_storage(rng.standard_normal((n, d)), "bf16")
    score = rng.random(n)
    cache, ev = ref.compress_head(K, V, score, budget, recent, 0, "fp8")
    assert np.array_equal(ref.quantise_fp8_rows(cache.K), cache.K) and np.array_equal(ref.quantise_fp8_rows(cache.V), cache.V)
    same, _ = ref.compress_head(K, V, score, budget, recent, 0, "bf16")
    assert np.array_equal(cache.pos, same.pos)                                  # selection does not depend on storage
    assert np.array_equal(cache.K, ref.round_storage(same.K, "fp8"))            # the encoded bf16 rows
    pure, _ = ref.compress_head(K, V, score, budget, recent, 0, "fp8", tau_force=float("inf"))
    assert np.array_equal(pure.K, ref.quantise_fp8_rows(K[pure.pos]))
    q = ref.round_storage(rng.standard_normal((1, d)), "bf16")
    k_new = ref.round_storage(rng.standard_normal(d) * 2, "bf16")
    v_new = ref.round_storage(rng.standard_normal(d), "bf16")
    rows_K = np.vstack([pure.K, ref.quantise_fp8_rows(k_new)[None]])
    rows_V = np.vstack([pure.V, ref.quantise_fp8_rows(v_new)[None]])
    out, e = ref.decode_step_head(pure, q, k_new, v_new, n, budget, recent, 0, 0.5, tau_force=float("inf"))
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.tensor(q)[None], torch.tensor(rows_K)[None], torch.tensor(rows_V)[None]).numpy()[0]
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-14)
    assert e.evicted_pos >= 0 and e.target_pos == -1
    assert np.array_equal(ref.quantise_fp8_rows(pure.K), pure.K) and pure.K.shape[0] == budget


def test_append_of_one_token_on_an_fp8_cache_is_a_generation_step_on_it():
    """storage = "fp8": the block form with m = 1 and the generation step must agree bit for bit,
    and both leave a cache whose every row is a fixed point of the encoding."""
    d, G, budget, recent, sink, beta = 16, 2, 12, 3, 1, 0.6
    g = np.random.default_rng(9)
    n = 40
    K = ref.round_storage(g.standard_normal((n, d)) * 2, "bf16")
    V = ref.round_storage(g.standard_normal((n, d)), "bf16")
    cache, _ = ref.compress_head(K, V, g.random(n) * 3, budget, recent, sink, "fp8")
    a, b = _copy_cache(cache), _copy_cache(cache)
    merged = 0
    for t in range(12):
        q = ref.round_storage(g.standard_normal((G, d)) * 2, "bf16")
        k, v = ref.round_storage(g.standard_normal(d) * 2, "bf16"), ref.round_storage(g.standard_normal(d), "bf16")
        out1, e1 = ref.decode_step_head(a, q, k, v, n + t, budget, recent, sink, beta)
        out2, e2 = ref.append_chunk_head(b, q[:, None, :], k[None], v[None], n + t, budget, recent, sink, beta)
        assert np.array_equal(out1, out2[:, 0]) and list(e2.evicted) == [e1.evicted_pos]
        assert (int(e2.target[0]) if e2.passed[0] else -1) == e1.target_pos
        merged += e1.target_pos >= 0
        assert np.array_equal(a.K, b.K) and np.array_equal(a.V, b.V) and np.array_equal(a.score, b.score)
        assert np.array_equal(ref.quantise_fp8_rows(a.K), a.K) and np.array_equal(ref.quantise_fp8_rows(a.V), a.V)
    assert 0 < merged < 12   # both branches (merge and discard) were taken
