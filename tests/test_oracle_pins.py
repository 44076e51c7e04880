"""Pins of the CPU oracle against what the paper and the mathematics fix.

Each test checks an oracle function against something other than its own
formula: brute force on tiny inputs, closed forms, library routines reached by a
special case, values printed in the paper (tests/golden/), and invariants.
None of these needs a GPU.
"""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import rdkv_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16_round(x):
    """Round float32 to the nearest bf16 (ties to even), returned as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def rand_bf16(rng, shape, scale=1.0):
    return bf16_round(rng.standard_normal(shape).astype(np.float32) * np.float32(scale))


# ----------------------------------------------------------------------------
# O1 token weights (Prop. 3.1, Eq. 2, Alg. 1 Stage 1)
# ----------------------------------------------------------------------------
def _softmax_list(z):
    m = max(z)
    e = [math.exp(v - m) for v in z]
    s = sum(e)
    return [v / s for v in e]


def test_token_weights_equal_summed_tv_distance_bruteforce():
    # Prop. 3.1: evicting token t changes query tau's attention by TV distance a_{tau,t};
    # w_t is that distance summed over queries.  Pure-Python loops, renormalised softmax.
    rng = np.random.default_rng(1)
    Hkv, g, T, Sw, d = 2, 2, 11, 3, 8
    K = rand_bf16(rng, (Hkv, T, d))
    Q = rand_bf16(rng, (Hkv * g, Sw, d))
    w = O.token_weights(K, Q, causal=True)
    for h in range(Hkv):
        for t in range(T):
            tv_sum = 0.0
            for j in range(g):
                for i in range(Sw):
                    last = T - Sw + i                      # causal: keys 0..last
                    z = [sum(float(Q[h * g + j, i, c]) * float(K[h, u, c]) for c in range(d)) / math.sqrt(d)
                         for u in range(last + 1)]
                    a = _softmax_list(z)
                    if t > last:
                        continue                            # token not visible: no change
                    if last == 0:
                        continue
                    a_hat = [0.0 if u == t else a[u] / (1.0 - a[t]) for u in range(last + 1)]
                    tv_sum += 0.5 * sum(abs(x - y) for x, y in zip(a, a_hat))
            assert w[h, t] == pytest.approx(tv_sum, rel=1e-10, abs=1e-12)


def test_token_weights_mass_and_causal_edge():
    rng = np.random.default_rng(2)
    Hkv, g, T, Sw, d = 2, 4, 300, 32, 16
    K = rand_bf16(rng, (Hkv, T, d))
    Q = rand_bf16(rng, (Hkv * g, Sw, d))
    w = O.token_weights(K, Q, causal=True)
    # every softmax row sums to one: total mass = number of rows
    np.testing.assert_allclose(w.sum(axis=1), g * Sw, rtol=1e-12)
    # the last key is visible to the last window row only
    for h in range(Hkv):
        exp = 0.0
        for j in range(g):
            z = K[h].astype(np.float64) @ Q[h * g + j, Sw - 1].astype(np.float64) / math.sqrt(d)
            exp += _softmax_list(list(z))[T - 1]
        assert w[h, T - 1] == pytest.approx(exp, rel=1e-10)
    # without the mask every row sees all keys: more mass lands on the last keys
    w_nc = O.token_weights(K, Q, causal=False)
    np.testing.assert_allclose(w_nc.sum(axis=1), g * Sw, rtol=1e-12)
    assert not np.allclose(w_nc[:, -Sw:], w[:, -Sw:])
    # keys before the window are unaffected by the mask only through normalisation:
    # with one window row (Sw = 1) the mask is void
    w1 = O.token_weights(K, Q[:, -1:, :], causal=True)
    w1n = O.token_weights(K, Q[:, -1:, :], causal=False)
    np.testing.assert_allclose(w1, w1n, rtol=1e-13)


def test_token_weights_uniform_when_keys_identical():
    # identical keys -> uniform attention over the visible prefix (closed form)
    Hkv, g, T, Sw, d = 1, 1, 9, 2, 4
    K = np.ones((Hkv, T, d), dtype=np.float32)
    Q = rand_bf16(np.random.default_rng(3), (1, Sw, d))
    w = O.token_weights(K, Q, causal=True)
    exp = np.zeros(T)
    for i in range(Sw):
        last = T - Sw + i
        exp[:last + 1] += 1.0 / (last + 1)
    np.testing.assert_allclose(w[0], exp, rtol=1e-12)


def test_avg_pool_against_convolution_and_mass():
    rng = np.random.default_rng(4)
    w = rng.random((3, 50))
    p = O.avg_pool(w, 5)
    for r in range(3):
        np.testing.assert_allclose(p[r], np.convolve(w[r], np.ones(5) / 5.0, mode="same"), rtol=1e-12)
    # a unit impulse away from the edges spreads to five taps of 1/5 and keeps its mass
    e = np.zeros(20)
    e[10] = 1.0
    pe = O.avg_pool(e, 5)
    assert pe[8:13].tolist() == [0.2] * 5 and pe.sum() == pytest.approx(1.0)
    # at the edge the zero padding loses mass (divisor stays 5)
    e0 = np.zeros(20)
    e0[0] = 1.0
    assert O.avg_pool(e0, 5).sum() == pytest.approx(0.6)
    np.testing.assert_array_equal(O.avg_pool(w, 1), w)


# ----------------------------------------------------------------------------
# O2 channel weights (Prop. 3.2, Eq. 3-4)
# ----------------------------------------------------------------------------
def test_channel_weight_is_spectral_and_frobenius_norm_of_logit_deviation():
    rng = np.random.default_rng(5)
    Hkv, g, T, Sw, d = 2, 2, 40, 5, 8
    K = rand_bf16(rng, (Hkv, T, d))
    Q = rand_bf16(rng, (Hkv * g, Sw, d))
    wc = O.channel_weights(K, Q)
    for h in range(Hkv):
        Qg = Q[h * g:(h + 1) * g].reshape(-1, d).astype(np.float64)
        Kh = K[h].astype(np.float64)
        Z = Qg @ Kh.T / math.sqrt(d)
        for c in range(d):
            K0 = Kh.copy()
            K0[:, c] = 0.0
            dZ = Qg @ K0.T / math.sqrt(d) - Z                 # zeroing channel c (Eq. 3)
            sv = np.linalg.svd(dZ, compute_uv=False)
            assert sv[0] == pytest.approx(wc[h, c], rel=1e-9)
            assert np.linalg.norm(dZ, "fro") == pytest.approx(wc[h, c], rel=1e-9)   # Remark after Prop. 3.2
            assert sv[1] < 1e-9 * max(sv[0], 1e-30) + 1e-12   # rank one


# ----------------------------------------------------------------------------
# O3 continuous reverse water-filling (Thm 3.3)
# ----------------------------------------------------------------------------
def test_water_filling_worked_example():
    # c = (8, 2, 0.5), B = 4: water level theta = 1 -> b = (3, 1, 0), D = c 2^-b = (1, 1, 0.5)
    b, theta, lam = O.water_filling([8.0, 2.0, 0.5], 4.0)
    assert theta == pytest.approx(1.0)
    np.testing.assert_allclose(b, [3.0, 1.0, 0.0], atol=1e-12)
    np.testing.assert_allclose(np.array([8.0, 2.0, 0.5]) * 2.0 ** (-b), [1.0, 1.0, 0.5])
    assert lam == pytest.approx(math.log(2.0))


def test_water_filling_matches_classical_reverse_water_filling():
    # Classical form (Cover & Thomas): R_i = max(0, 1/2 log2(sigma_i^2 / theta_c)),
    # D_i = min(theta_c, sigma_i^2) with sigma_i = c_u and theta_c = theta^2.
    rng = np.random.default_rng(6)
    c = np.exp(rng.normal(0, 2.0, 200))
    B = 300.0
    b, theta, lam = O.water_filling(c, B)
    assert b.sum() == pytest.approx(B, rel=1e-10)                  # budget binds
    D = c * 2.0 ** (-b)
    np.testing.assert_allclose(D, np.minimum(theta, c), rtol=1e-10)
    R = np.maximum(0.0, 0.5 * np.log2(c ** 2 / theta ** 2))
    np.testing.assert_allclose(b, R, atol=1e-10)
    # phase transition at c_u = lam / ln 2
    assert np.all((b > 0) == (c > lam / math.log(2.0) * (1 + 1e-12)))
    # KKT/optimality: moving a little rate between any two units cannot lower the objective
    obj = D.sum()
    for _ in range(200):
        i, j = rng.integers(0, len(c), 2)
        if i == j:
            continue
        b2 = b.copy()
        delta = min(0.05, b2[i])
        b2[i] -= delta
        b2[j] += delta
        assert (c * 2.0 ** (-b2)).sum() >= obj - 1e-12


# ----------------------------------------------------------------------------
# O4 discrete allocation (Eq. 6, Alg. 2, Prop. A.3)
# ----------------------------------------------------------------------------
def _read_fig2():
    rows = {}
    with open(os.path.join(GOLDEN, "fig2_thresholds.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            p = line.split()
            rows[p[0]] = ([float(x) for x in p[1:5]], [float(x) for x in p[5:13]], [int(x) for x in p[13:21]])
    return rows


def test_fig2_four_thresholds_five_zones():
    # The figure's thresholds (16, 8, 4, 2 from the top) and bar heights: classification
    # with thresholds lam * r_k must reproduce the printed zones.
    for kind, (thr, scores, bits) in _read_fig2().items():
        r = list(reversed(thr))                       # ascending: thresholds into tiers 2, 4, 8, 16
        got = O.classify(np.array(scores, dtype=np.float32), 1.0, [0, 2, 4, 8, 16], r)
        assert got.tolist() == bits, kind
    tok_bits = _read_fig2()["token"][2]
    assert [i + 1 for i, b in enumerate(tok_bits) if b > 0] == [1, 2, 4, 5, 7, 8]   # T_kept in the caption


def _read_table9():
    tab = {}
    with open(os.path.join(GOLDEN, "table9_eps.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            p = line.split()
            tab[p[0]] = ([1.0] + [float(x) for x in p[1:4]] + [0.0], [1.0] + [float(x) for x in p[4:7]] + [0.0])
    return tab


def test_default_tables_are_the_printed_llama31_row_and_convex():
    tab = _read_table9()
    ek, ev = tab["LLaMA-3.1-8B"]
    assert list(O.EPS_K_LLAMA31_8B) == ek and list(O.EPS_V_LLAMA31_8B) == ev
    for name, (ek, ev) in tab.items():
        for e in (ek, ev):
            hb, r = O.hull_thresholds(O.TIERS, e)
            assert hb == [0, 2, 4, 8, 16], name          # every printed table is convex: all tiers on the hull
            assert all(r[i] < r[i + 1] for i in range(3))


def test_hull_drops_dominated_tiers():
    # a tier above the chord between its neighbours is never optimal
    hb, r = O.hull_thresholds([0, 2, 4, 8, 16], [1.0, 0.9, 0.1, 0.05, 0.0])
    assert hb == [0, 4, 8, 16]
    assert r[0] == pytest.approx(4 / np.float64(np.float32(1.0) - np.float32(0.1)), rel=1e-7)
    # and then argmin never selects it
    rng = np.random.default_rng(7)
    w = rng.random(500).astype(np.float32) * 10
    for lam in (0.01, 0.1, 0.5, 2.0):
        assert 2 not in O.argmin_bits(w, lam, [0, 2, 4, 8, 16], [1.0, 0.9, 0.1, 0.05, 0.0])


@pytest.mark.parametrize("eps", [O.EPS_V_LLAMA31_8B, O.EPS_K_LLAMA31_8B, O.EPS_BENNETT])
def test_threshold_form_equals_printed_argmin_form(eps):
    rng = np.random.default_rng(8)
    w = np.exp(rng.normal(0, 3, 4000)).astype(np.float32)
    hb, r = O.hull_thresholds(O.TIERS, eps)
    for lam in (1e-4, 1e-2, 0.3, 1.0, 7.0, 200.0):
        a = O.classify(w, lam, hb, r)
        b = O.argmin_bits(w, lam, O.TIERS, eps)
        # away from exact ties the two forms agree
        near_tie = np.zeros(len(w), dtype=bool)
        for rk in r:
            near_tie |= np.abs(w.astype(np.float64) - lam * rk) <= 1e-9 * lam * rk
        assert np.array_equal(a[~near_tie], b[~near_tie])


def test_exact_ties_take_the_lower_bit_width_in_both_forms():
    """Alg. 2's per-unit step at an exact tie.  With the dyadic table eps = (1, 1/2, 1/4, 1/8, 0) every quantity is
    exact in fp64: the hull ratios are r = (4, 8, 32, 64), and at lam = 1 a unit of weight r_k pays the same cost at
    tiers k-1 and k (w = 4: 4*1 + 0 = 4*1/2 + 2; w = 8: 8/2 + 2 = 8/4 + 4; w = 32: 32/4 + 4 = 32/8 + 8;
    w = 64: 64/8 + 8 = 0 + 16).  The printed argmin keeps the lower bit-width there, and so must the threshold form
    (strict '>'); one ulp above the tie both move up."""
    eps = (1.0, 0.5, 0.25, 0.125, 0.0)
    hb, r = O.hull_thresholds(O.TIERS, eps)
    assert hb == [0, 2, 4, 8, 16] and r == [4.0, 8.0, 32.0, 64.0]
    ties = np.array([4.0, 8.0, 32.0, 64.0], np.float32)
    above = np.nextafter(ties, np.float32(np.inf))
    below = np.nextafter(ties, np.float32(0))
    for lam, scale in ((1.0, 1.0), (0.25, 0.25), (8.0, 8.0)):            # powers of two keep the ties exact
        for form in (lambda w: O.argmin_bits(w, lam, O.TIERS, eps), lambda w: O.classify(w, lam, hb, r)):
            assert form(ties * np.float32(scale)).tolist() == [0, 2, 4, 8]
            assert form(above * np.float32(scale)).tolist() == [2, 4, 8, 16]
            assert form(below * np.float32(scale)).tolist() == [0, 2, 4, 8]
    # inside the bisection: weights sitting exactly on the thresholds of the multiplier the search visits.
    # 12 units, budget 2 bits per unit = 24 bits.  lam runs 32, 16, 8, 4, ...; at lam = 8 the units of weight 32 and
    # 64 tie between 0 and 2 bits (r_1 lam = 32) resp. 2 and 4 bits (r_2 lam = 64) and must take the lower one.
    w = np.array([64.0] * 4 + [32.0] * 4 + [1.0] * 4, np.float32)
    bits, info = O.mckp_bisect(w, np.float32(2.0), O.TIERS, eps, rel_tol=np.float32(0.0), max_iters=3, return_info=True)
    assert info["lam"] == 8.0 and bits.tolist() == [2] * 4 + [0] * 8
    bits, info = O.mckp_bisect(w, np.float32(2.0), O.TIERS, eps, rel_tol=np.float32(0.0), max_iters=4, return_info=True)
    # lam = 4: weight 64 ties between 4 and 8 bits (r_3 lam = 128 not reached; r_2 lam = 32 < 64 -> 4 bits), weight 32
    # ties between 2 and 4 bits -> 2 bits: 4*4 + 4*2 = 24 = the budget
    assert info["lam"] == 4.0 and bits.tolist() == [4] * 4 + [2] * 4 + [0] * 4


def test_bisection_runs_the_printed_per_unit_step():
    """mckp_bisect must return, for the multiplier it reports, exactly the printed argmin of every unit -- and the
    threshold form must reproduce the whole search on ordinary (tie-free) weights."""
    rng = np.random.default_rng(77)
    for eps in (O.EPS_V_LLAMA31_8B, O.EPS_K_LLAMA31_8B, O.EPS_BENNETT):
        w = np.exp(rng.normal(0, 2, 3000)).astype(np.float32)
        for avg in (0.4, 1.0, 3.0, 7.5):
            bits, info = O.mckp_bisect(w, np.float32(avg), O.TIERS, eps, return_info=True)
            assert np.array_equal(bits, O.argmin_bits(w, info["lam"], O.TIERS, eps))
            hb, r = O.hull_thresholds(O.TIERS, eps)
            assert np.array_equal(bits, O.classify(w, info["lam"], hb, r))
            assert int(bits.astype(np.int64).sum()) <= info["B_int"]


def test_mckp_bruteforce_optimality_and_weak_duality():
    # tiny instances: enumerate all 5^U allocations (Eq. 6) and check
    #   g(lam) <= OPT(B) <= primal(returned)                       (Prop. A.3)
    #   returned allocation is optimal for the bits it actually uses (Lagrangian optimality)
    rng = np.random.default_rng(9)
    tiers = list(O.TIERS)
    for trial in range(25):
        U = int(rng.integers(3, 8))
        w = np.exp(rng.normal(0, 1.5, U)).astype(np.float32)
        eps = [O.EPS_V_LLAMA31_8B, O.EPS_BENNETT][trial % 2]
        e = np.array([np.float64(np.float32(x)) for x in eps])
        avg = np.float32(rng.choice([0.7, 1.5, 3.0, 6.0, 11.0]))
        bits, info = O.mckp_bisect(w, avg, tiers, eps, return_info=True)
        B = info["B_int"]
        S = int(bits.sum())
        assert S <= B
        cost = lambda alloc: sum(float(w[u]) * e[tiers.index(int(alloc[u]))] for u in range(U))
        best_B, best_S = math.inf, math.inf
        for alloc in itertools.product(tiers, repeat=U):
            s = sum(alloc)
            c = cost(alloc)
            if s <= B:
                best_B = min(best_B, c)
            if s <= S:
                best_S = min(best_S, c)
        primal = cost(bits)
        assert primal >= best_B - 1e-12
        assert primal == pytest.approx(best_S, rel=1e-12, abs=1e-15)
        if info["lam"] is not None:
            lam = info["lam"]
            g_lam = sum(min(float(w[u]) * e[k] + lam * tiers[k] for k in range(5)) for u in range(U)) - lam * B
            assert g_lam <= best_B + 1e-12


def test_mckp_feasible_monotone_and_within_band_on_smooth_weights():
    rng = np.random.default_rng(10)
    U = 20000
    w = np.exp(rng.normal(0, 2.0, U)).astype(np.float32)
    prev = None
    for avg in (0.4, 1.0, 2.0, 4.0, 8.0, 12.0):
        bits, info = O.mckp_bisect(w, np.float32(avg), return_info=True)
        S = int(bits.astype(np.int64).sum())
        assert set(np.unique(bits)) <= set(O.TIERS)
        assert S <= info["B_int"]
        assert S >= math.ceil(0.99 * info["B_int"]) - 16            # smooth weights: the 1 % band is reached
        assert info["iters"] <= 64
        # a unit's bit-width is a non-decreasing function of its weight
        order = np.argsort(w, kind="stable")
        assert np.all(np.diff(bits[order].astype(int)) >= 0)
        if prev is not None:
            assert np.all(bits >= prev)                             # a larger budget takes bits from no unit
        prev = bits


def test_mckp_shortcuts_and_degenerate_inputs():
    w = np.array([3.0, 1.0, 0.0, 2.0], dtype=np.float32)
    assert O.mckp_bisect(w, np.float32(16.0)).tolist() == [16] * 4      # budget covers everything
    assert O.mckp_bisect(w, np.float32(20.0)).tolist() == [16] * 4
    assert O.mckp_bisect(w, np.float32(0.0)).tolist() == [0] * 4        # zero budget: no division by zero
    assert O.mckp_bisect(w, np.float32(0.3)).tolist() == [0] * 4        # floor(1.2) = 1 < 2 bits
    assert O.mckp_bisect(np.zeros(0, np.float32), np.float32(2.0)).shape == (0,)
    # equal weights: units move together, so only all-or-nothing is feasible
    we = np.ones(10, dtype=np.float32)
    b = O.mckp_bisect(we, np.float32(3.0))
    assert len(set(b.tolist())) == 1 and int(b.sum()) <= 30
    # all-zero weights: nothing is worth a bit
    assert O.mckp_bisect(np.zeros(5, np.float32), np.float32(4.0)).tolist() == [0] * 5
    # budget for exactly one 2-bit unit goes to the heaviest unit
    assert O.mckp_bisect(w, np.float32(0.5)).tolist() == [2, 0, 0, 0]


def test_mckp_on_fine_grid_approaches_water_filling():
    # With tiers {0,1,...,16} and eps(b) = 2^-b the discrete problem is Eq. 5 on a grid:
    # the allocation stays within about one bit of Thm 3.3's closed form.
    rng = np.random.default_rng(11)
    U = 5000
    w = np.exp(rng.normal(0, 2.0, U)).astype(np.float32)
    tiers = list(range(17))
    eps = [2.0 ** (-b) for b in tiers]
    avg = np.float32(3.0)
    bits = O.mckp_bisect(w, avg, tiers, eps).astype(np.float64)
    b_cont, theta, lam = O.water_filling(w.astype(np.float64), float(bits.sum()))
    b_cont = np.minimum(b_cont, 16.0)
    assert np.max(np.abs(bits - b_cont)) <= 1.25
    assert abs(np.mean(bits - b_cont)) < 0.05


def test_mixed_budgets_match_alg1_bookkeeping():
    # Alg. 1: B_head = 2 B_tok d 16; B_V = B_K = B_head / 2; Bbar_V = B_V / d per token-unit sum;
    # k_avg = B_K / (n_kept d).
    d, T, B_tok = 128, 1000, 64
    B_head = 2 * B_tok * d * 16
    avg_bits = B_head / (2 * T * d)                  # average over all K and V scalars
    n_kept = 300
    v_avg, k_avg = O.mixed_budgets(np.float32(avg_bits), np.float32(0.5), T, n_kept, d)
    assert v_avg * T == pytest.approx((B_head / 2) / d, rel=1e-6)
    assert k_avg == pytest.approx((B_head / 2) / (n_kept * d), rel=1e-6)
    assert O.mixed_budgets(np.float32(8.0), np.float32(0.5), T, 10, d)[1] == 16.0   # capped at full precision


# ----------------------------------------------------------------------------
# O5 reference quantizer
# ----------------------------------------------------------------------------
def test_quantizer_hand_worked_groups_and_ties_to_even():
    # 2-bit, range [0, 3]: s = 1, m = 0, codes are the values
    c, s, m = O.quantize_groups(np.array([[0.0, 1.0, 2.0, 3.0]], np.float32), 2)
    assert c.tolist() == [[0, 1, 2, 3]] and float(s[0]) == 1.0 and float(m[0]) == 0.0
    # ties go to the even code: (x - m)/s = 0.5 -> 0, 1.5 -> 2, 2.5 -> 2
    c, s, m = O.quantize_groups(np.array([[-1.5, -1.0, 0.0, 1.0, 1.5]], np.float32), 2)
    assert float(s[0]) == 1.0 and float(m[0]) == -1.5
    assert c.tolist() == [[0, 0, 2, 2, 3]]
    # 4-bit: 16 levels over [-7.5, 7.5] -> s = 1, code = x + 7.5 rounded to even on ties
    x = np.array([[-7.5, -7.0, 0.0, 0.5, 7.5]], np.float32)
    c, s, m = O.quantize_groups(x, 4)
    assert float(s[0]) == 1.0 and c.tolist() == [[0, 0, 8, 8, 15]]
    # 8-bit: 256 levels over [0, 255]
    x = np.arange(0, 256, 17, dtype=np.float32)[None, :]
    c, s, m = O.quantize_groups(x, 8)
    assert float(s[0]) == 1.0 and c[0].tolist() == list(range(0, 256, 17))
    # constant group: zero scale, exact reconstruction
    c, s, m = O.quantize_groups(np.full((1, 32), 2.5, np.float32), 4)
    assert float(s[0]) == 0.0 and not c.any()
    assert np.all(O.dequantize_groups(c, s, m) == 2.5)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_quantizer_error_bound_and_ranges(bits):
    rng = np.random.default_rng(12 + bits)
    x = rand_bf16(rng, (2000, 4, 32))
    x[:, 1, 5] *= 10.0                                  # outlier channel inside a group
    x = bf16_round(x)
    c, s, m = O.quantize_groups(x, bits)
    Q = (1 << bits) - 1
    assert c.min() >= 0 and c.max() <= Q
    assert np.all(c.max(axis=-1) == Q) and np.all(c.min(axis=-1) == 0)      # both ends of the range are hit
    # bf16 inputs are exact in fp16's normal range: the offset is the group minimum itself
    np.testing.assert_array_equal(m.astype(np.float32), x.min(axis=-1))
    xh = O.dequantize_groups(c, s, m)
    err = np.abs(xh - x.astype(np.float64))
    bound = 0.5 * s.astype(np.float64)[..., None] * (1 + 2.0 ** -10)
    assert np.all(err <= bound)
    # scale is the fp16 rounding of range / Q
    rng_over_q = (x.max(-1).astype(np.float64) - x.min(-1).astype(np.float64)) / Q
    assert np.all(np.abs(s.astype(np.float64) - rng_over_q) <= rng_over_q * 2.0 ** -11 + 1e-12)


def test_quantizer_uniform_data_has_bennett_mse():
    # Lemma A.1: a uniform quantizer of cell width Delta has per-coordinate MSE Delta^2 / 12.
    rng = np.random.default_rng(15)
    x = bf16_round(rng.uniform(-4, 4, (4000, 32)).astype(np.float32))
    for bits in (4, 8):
        c, s, m = O.quantize_groups(x, bits)
        xh = O.dequantize_groups(c, s, m)
        mse = np.mean((xh - x) ** 2)
        delta2 = np.mean(s.astype(np.float64) ** 2)
        # bf16 inputs at 8 bits sit on a grid comparable to the cell width, so allow a wide band there
        tol = 0.08 if bits == 4 else 0.35
        assert mse == pytest.approx(delta2 / 12.0, rel=tol)


# ----------------------------------------------------------------------------
# O6 packing
# ----------------------------------------------------------------------------
def test_pack_bit_positions_as_printed():
    # App. B: 2-bit -> four elements per byte at offsets 0,2,4,6; 4-bit -> two at offsets 0,4
    assert O.pack_codes(np.array([[1, 2, 3, 0]], np.uint8), 2).tolist() == [[1 | (2 << 2) | (3 << 4)]]
    assert O.pack_codes(np.array([[0, 0, 0, 3]], np.uint8), 2).tolist() == [[0xC0]]
    assert O.pack_codes(np.array([[0xA, 0x5]], np.uint8), 4).tolist() == [[0x5A]]
    assert O.pack_codes(np.array([[7, 200]], np.uint8), 8).tolist() == [[7, 200]]
    rng = np.random.default_rng(16)
    for bits in (2, 4, 8):
        codes = rng.integers(0, 1 << bits, (37, 128)).astype(np.uint8)
        data = O.pack_codes(codes, bits)
        assert data.shape == (37, 128 * bits // 8)
        np.testing.assert_array_equal(O.unpack_codes(data, bits), codes)


def _small_case(rng, Hkv=2, T=150, d=128, batch=1):
    Ks = [rand_bf16(rng, (Hkv, T + 7 * s, d)) for s in range(batch)]
    Vs = [rand_bf16(rng, (Hkv, T + 7 * s, d)) for s in range(batch)]
    for K in Ks:
        K[:, :, 3] = bf16_round(K[:, :, 3] * 10)
    return Ks, Vs


def test_cache_layout_counts_offsets_and_bytes():
    rng = np.random.default_rng(17)
    Ks, Vs = _small_case(rng, batch=2)
    bits = [rng.choice(np.array([0, 2, 4, 8, 16], np.uint8), size=K.shape[:2], p=[.4, .25, .2, .1, .05]) for K in Ks]
    cache = O.build_cache_tokenwise(Ks, Vs, bits)
    n_items = 4
    assert cache["counts"].shape == (n_items, 4)
    it = 0
    pos_cursor = 0
    for s in range(2):
        for h in range(2):
            for ti, b in enumerate(O.PACK_ORDER):
                pos = np.nonzero(bits[s][h] == b)[0]
                n = len(pos)
                assert cache["counts"][it, ti] == n
                np.testing.assert_array_equal(cache["tier_idx"][pos_cursor:pos_cursor + n], pos)   # ascending, stable
                pos_cursor += n
                assert np.all(cache["seg_off"][it, ti] % 256 == 0)
            it += 1
    assert pos_cursor == len(cache["tier_idx"])
    # closed-form stored bytes: 2 * (16 b + 16) per row for b in {2,4,8}, 512 for b = 16
    c = cache["counts"].sum(axis=0)
    assert O.stored_bytes(cache["counts"]) == c[0] * 512 + c[1] * 2 * 144 + c[2] * 2 * 80 + c[3] * 2 * 48
    # segments do not overlap and the arena is just large enough
    spans = []
    for i in range(n_items):
        for ti, b in enumerate(O.PACK_ORDER):
            npad = (int(cache["counts"][i, ti]) + 63) // 64 * 64          # whole 64-row tiles
            sizes = [npad * O.row_bytes(b), npad * O.meta_bytes(b)] * 2
            for si in range(4):
                if sizes[si]:
                    spans.append((int(cache["seg_off"][i, ti, si]), sizes[si]))
    spans.sort()
    for (o0, s0), (o1, _) in zip(spans, spans[1:]):
        assert o0 + s0 <= o1
    assert spans[-1][0] + spans[-1][1] <= len(cache["arena"]) < spans[-1][0] + spans[-1][1] + 256


def test_physical_roundtrip_equals_canonical_dequant():
    rng = np.random.default_rng(18)
    Ks, Vs = _small_case(rng)
    bits = [rng.choice(np.array([0, 2, 4, 8, 16], np.uint8), size=Ks[0].shape[:2])]
    cache = O.build_cache_tokenwise(Ks, Vs, bits)
    for item in range(2):
        Kh, Vh = O.unpack_item(cache, item)
        rec = cache["canon"][item]
        rows_k, rows_v = [], []
        for b in O.PACK_ORDER:
            ent = rec[b]
            n = len(ent["pos"])
            if b == 16:
                rows_k.append(Ks[0][item][ent["pos"]].astype(np.float64))
                rows_v.append(Vs[0][item][ent["pos"]].astype(np.float64))
            else:
                for name, dst in (("k", rows_k), ("v", rows_v)):
                    s = ent[name + "_scale"].view(np.float16).astype(np.float64)
                    m = ent[name + "_off"].view(np.float16).astype(np.float64)
                    codes = ent[name + "_codes"].reshape(n, 4, 32).astype(np.float64)
                    dst.append((codes * s[:, :, None] + m[:, :, None]).reshape(n, 128))
        np.testing.assert_array_equal(Kh, np.concatenate(rows_k))
        np.testing.assert_array_equal(Vh, np.concatenate(rows_v))


# ----------------------------------------------------------------------------
# O7 decode (Sec. 3.3, Eq. 7)
# ----------------------------------------------------------------------------
def _bruteforce_attention(q, K, V):
    """softmax(q K^T / sqrt(d)) V with Python loops."""
    n, d = K.shape
    z = [sum(float(q[c]) * float(K[t, c]) for c in range(d)) / math.sqrt(d) for t in range(n)]
    a = _softmax_list(z)
    return [sum(a[t] * float(V[t, c]) for t in range(n)) for c in range(d)], max(z) + math.log(sum(math.exp(v - max(z)) for v in z))


def test_all_16_bit_cache_reproduces_bruteforce_attention():
    rng = np.random.default_rng(19)
    Hkv, g, T, d = 2, 2, 70, 128
    Ks, Vs = [rand_bf16(rng, (Hkv, T, d))], [rand_bf16(rng, (Hkv, T, d))]
    q = rand_bf16(rng, (1, Hkv * g, d))
    cache = O.build_cache_tokenwise(Ks, Vs, [np.full((Hkv, T), 16, np.uint8)])
    out, lse = O.decode(cache, q)
    for j in range(Hkv * g):
        o, l = _bruteforce_attention(q[0, j], Ks[0][j // g], Vs[0][j // g])
        np.testing.assert_allclose(out[0, j], o, rtol=1e-11, atol=1e-13)
        assert lse[0, j] == pytest.approx(l, rel=1e-12)
    out_d, lse_d = O.decode_dense(Ks, Vs, q)
    np.testing.assert_allclose(out, out_d, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, lse_d, rtol=1e-12)


def test_zero_bit_units_are_exactly_eviction():
    rng = np.random.default_rng(20)
    Hkv, g, T, d = 1, 4, 90, 128
    Ks, Vs = [rand_bf16(rng, (Hkv, T, d))], [rand_bf16(rng, (Hkv, T, d))]
    q = rand_bf16(rng, (1, g, d))
    bits = np.where(rng.random((Hkv, T)) < 0.6, 0, 16).astype(np.uint8)
    cache = O.build_cache_tokenwise(Ks, Vs, [bits])
    out, lse = O.decode(cache, q)
    keep = np.nonzero(bits[0])[0]
    for j in range(g):
        o, l = _bruteforce_attention(q[0, j], Ks[0][0][keep], Vs[0][0][keep])
        np.testing.assert_allclose(out[0, j], o, rtol=1e-11, atol=1e-13)
        assert lse[0, j] == pytest.approx(l, rel=1e-12)
    # a head whose tokens are all evicted: zero output, lse = -inf
    cache0 = O.build_cache_tokenwise(Ks, Vs, [np.zeros((Hkv, T), np.uint8)])
    o0, l0 = O.decode(cache0, q)
    assert not o0.any() and np.all(np.isneginf(l0))


def test_decode_over_quantized_tiers_equals_attention_over_dequantized_rows_any_order():
    # Eq. 7: the zone sums are dense attention over (K_hat, V_hat); softmax attention does not
    # depend on the order of the rows, on a shift of the logits, or on how the rows are split
    # (LSE merge of partial results).
    rng = np.random.default_rng(21)
    Hkv, g, T, d = 1, 2, 200, 128
    Ks, Vs = _small_case(rng, Hkv=Hkv, T=T)
    q = rand_bf16(rng, (1, g, d))
    bits = rng.choice(np.array([0, 2, 4, 8, 16], np.uint8), size=(Hkv, T))
    cache = O.build_cache_tokenwise(Ks, Vs, [bits])
    out, lse = O.decode(cache, q)
    Kh, Vh = O.unpack_item(cache, 0)
    perm = rng.permutation(len(Kh))
    o_p, l_p = O.attention_rows(q[0], Kh[perm], Vh[perm])
    np.testing.assert_allclose(out[0], o_p, rtol=1e-11, atol=1e-13)
    # split into three parts and merge with log-sum-exp weights
    parts = np.array_split(np.arange(len(Kh)), 3)
    os_, ls_ = zip(*[O.attention_rows(q[0], Kh[p], Vh[p]) for p in parts])
    ls_ = np.stack(ls_)
    lmax = ls_.max(axis=0)
    wts = np.exp(ls_ - lmax)
    merged = sum(wts[i][:, None] * os_[i] for i in range(3)) / wts.sum(axis=0)[:, None]
    np.testing.assert_allclose(merged, out[0], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(lmax + np.log(wts.sum(axis=0)), lse[0], rtol=1e-12)
    # the quantised rows differ from the originals by at most scale/2 per element, so the result is close
    # to (but not equal to) attention over the original kept rows
    bits8 = np.where(bits == 0, 0, np.where(bits == 16, 16, 8)).astype(np.uint8)
    out8, _ = O.decode(O.build_cache_tokenwise(Ks, Vs, [bits8]), q)
    keep = np.concatenate([np.nonzero(bits8[0] == b)[0] for b in O.PACK_ORDER])
    o_ref, _ = O.attention_rows(q[0], Ks[0][0][keep].astype(np.float64), Vs[0][0][keep].astype(np.float64))
    assert 0 < np.max(np.abs(o_ref - out8[0])) < 0.02


def test_k_dequant_fusion_identity():
    # App. B: q . k_hat = sum_c (s q_c) code_c - sum_c s z q_c; with offsets m = -s z per group
    # this reads sum_g s_g (q_g . code_g) + sum_g m_g sum(q_g).
    rng = np.random.default_rng(22)
    x = rand_bf16(rng, (50, 4, 32))
    q = rand_bf16(rng, (4, 32)).astype(np.float64)
    for bits in (2, 4, 8):
        c, s, m = O.quantize_groups(x, bits)
        xh = O.dequantize_groups(c, s, m)
        lhs = (xh * q[None]).sum(axis=(1, 2))
        rhs = (s.astype(np.float64) * (c.astype(np.float64) * q[None]).sum(-1)).sum(-1) \
            + (m.astype(np.float64) * q.sum(-1)[None]).sum(-1)
        np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-12)


def test_compress_tokenwise_equals_its_stages_and_brute_force_attention():
    """The whole token-wise pass (Alg. 1 with K sharing the token map) against its stages called one by one, and the
    decode of its result against brute-force attention over rows dequantized straight from the canonical records."""
    rng = np.random.default_rng(29)
    Hkv, g, d, Sw = 2, 2, 128, 16
    seq = [300, 131]
    Ks = [rand_bf16(rng, (Hkv, T, d)) for T in seq]
    Vs = [rand_bf16(rng, (Hkv, T, d)) for T in seq]
    for K in Ks:
        K[:, :, 7] *= np.float32(8.0)                          # an outlier channel
    Qo = [rand_bf16(rng, (Hkv * g, Sw, d)) for _ in seq]
    budgets = [np.float32(7.0), np.float32(1.5)]
    cache = O.compress_tokenwise(Ks, Vs, Qo, budgets, eps=O.EPS_BENNETT)
    bits_list = []
    for s_, T in enumerate(seq):
        w = O.avg_pool(O.token_weights(Ks[s_], Qo[s_]), 5).astype(np.float32)      # Stage 1
        assert np.array_equal(cache["weights"][s_], w)
        # before pooling every window row is a probability vector: total mass g * S_w per KV head
        np.testing.assert_allclose(O.token_weights(Ks[s_], Qo[s_]).sum(axis=1), g * Sw, rtol=1e-12)
        bits = np.stack([O.mckp_bisect(w[h], budgets[s_], O.TIERS, O.EPS_BENNETT) for h in range(Hkv)])   # Stage 2
        assert np.array_equal(cache["bits"][s_], bits)
        for h in range(Hkv):
            assert int(bits[h].astype(np.int64).sum()) <= int(np.floor(float(budgets[s_]) * T))
        bits_list.append(bits)
    assert len({int(b) for bb in bits_list for b in np.unique(bb)}) >= 4         # the case spans the tiers
    staged = O.build_cache_tokenwise(Ks, Vs, bits_list)                          # Stage 4
    assert np.array_equal(cache["arena"], staged["arena"]) and np.array_equal(cache["counts"], staged["counts"])
    assert np.array_equal(cache["tier_idx"], staged["tier_idx"])
    assert O.stored_bytes(cache["counts"]) == sum(
        int((bb == b).sum()) * 2 * (16 * b + (16 if b < 16 else 0)) for bb in bits_list for b in (2, 4, 8, 16))
    # decode = softmax attention over the retained rows, dequantized here from a quantizer call of this test's own
    q = rand_bf16(rng, (len(seq), Hkv * g, d))
    out, lse = O.decode(cache, q)
    for s_, T in enumerate(seq):
        for h in range(Hkv):
            Kh, Vh = [], []
            for b in (16, 8, 4, 2):
                idx = np.nonzero(bits_list[s_][h] == b)[0]
                for X, dst in ((Ks[s_][h][idx], Kh), (Vs[s_][h][idx], Vh)):
                    if b == 16:
                        dst.append(X.astype(np.float64))
                    else:
                        c, sc, m = O.quantize_groups(X.reshape(-1, 4, 32), b)
                        dst.append(O.dequantize_groups(c, sc, m).reshape(-1, d))
            Kh, Vh = np.concatenate(Kh), np.concatenate(Vh)
            for j in range(g):
                o, l = _bruteforce_attention(q[s_, h * g + j], Kh, Vh)
                np.testing.assert_allclose(out[s_, h * g + j], o, rtol=1e-11, atol=1e-12)
                assert abs(lse[s_, h * g + j] - l) < 1e-10


def test_compress_tokenwise_end_to_end_small():
    rng = np.random.default_rng(23)
    Hkv, g, T, d, Sw = 2, 2, 400, 128, 32
    Ks, Vs = _small_case(rng, Hkv=Hkv, T=T)
    Qo = [rand_bf16(rng, (Hkv * g, Sw, d))]
    cache = O.compress_tokenwise(Ks, Vs, Qo, [np.float32(2.0)])
    for h in range(Hkv):
        assert int(cache["bits"][0][h].astype(int).sum()) <= 2 * T
    assert O.stored_bytes(cache["counts"]) > 0
    q = rand_bf16(rng, (1, Hkv * g, d))
    out, lse = O.decode(cache, q)
    assert np.all(np.isfinite(out)) and np.all(np.isfinite(lse))


# ----------------------------------------------------------------------------
# 64-row tiles of the token-wise mode
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("which", ["k", "v"])
def test_tile64_positions_are_a_bijection_onto_the_tile(bits, which):
    byte_off, shift = O.tile64_code_positions(bits, which)
    tb = O.tile64_data_bytes(bits)
    assert tb == 64 * 128 * bits // 8
    pos = byte_off * 8 + shift
    assert pos.min() == 0 and pos.max() == tb * 8 - bits
    assert len(np.unique(pos)) == 64 * 128                      # no two codes share a field
    assert np.all(shift % bits == 0)                            # App. B: fields at offsets 0,2,4,6 / 0,4 / 0
    sc, of = O.tile64_meta_positions(which)
    both = np.concatenate([sc.reshape(-1), of.reshape(-1)])
    assert sorted(both.tolist()) == list(range(512))            # 16 bytes per token, each fp16 slot used once


def test_tile64_positions_hand_checked():
    # word W of lane L sits at 1024*(W//4) + 16*L + 4*(W%4); a lane owns 4*bits words, `bits` words per group.
    # K, 2-bit (2 words per group, 8 fields per half): token r = lane r.  ch 0 = group 0, step 0, code 0 -> word 0 bit 0;
    # ch 1 = code 1 -> high half of word 0 -> byte 2; ch 2 = code 2 -> word 1 -> byte 4; ch 4 = step 1 -> field 1 -> bit 2;
    # ch 28 = step 7 -> field 7 -> bit 14 -> byte 1, shift 6; ch 32 = group 1 -> word 2 -> byte 8; ch 96 -> word 6 ->
    # second 16-byte chunk -> byte 1024 + 8; token 1 -> lane 1 -> byte 16
    bo, sh = O.tile64_code_positions(2, "k")
    assert [(int(bo[0, c]), int(sh[0, c])) for c in (0, 1, 2, 4, 28, 32, 96)] == \
        [(0, 0), (2, 0), (4, 0), (0, 2), (1, 6), (8, 0), (1032, 0)]
    assert bo[1, 0] == 16 and bo[63, 0] == 16 * 63
    # K, 4-bit (4 words per group, 4 fields per half): steps 0..3 use the word pair (0, 1), steps 4..7 the pair (2, 3)
    bo, sh = O.tile64_code_positions(4, "k")
    assert [(int(bo[0, c]), int(sh[0, c])) for c in (0, 4, 12, 16, 18, 32)] == \
        [(0, 0), (0, 4), (1, 4), (8, 0), (12, 0), (1024, 0)]
    # K, 8-bit (8 words per group, 2 fields per half): step s uses the pair s // 2, byte s % 2 of each half
    bo, sh = O.tile64_code_positions(8, "k")
    assert [int(bo[0, c]) for c in (0, 1, 2, 3, 4, 8, 32)] == [0, 2, 4, 6, 1, 8, 2048]
    assert not sh.any()
    # V, 2-bit: lane = 32*(r // 32) + c % 32 holds one channel for 32 tokens; the token index plays the role the
    # channel index plays for K: token 1 = code 1 -> byte 2; token 4 = step 1 -> bit 2; token 32 -> lane 32 -> byte 512;
    # channel 1 -> lane 1 -> byte 16; channel 32 = group 1 -> word 2 -> byte 8
    bo, sh = O.tile64_code_positions(2, "v")
    assert [(int(bo[r, c]), int(sh[r, c])) for r, c in ((0, 0), (1, 0), (4, 0), (32, 0), (0, 1), (0, 32), (33, 33))] == \
        [(0, 0), (2, 0), (0, 2), (512, 0), (16, 0), (8, 0), (512 + 16 + 8 + 2, 0)]
    # metadata: K row-major [4 scales][4 offsets] per token; V per 4-token block, per group: 4 scales then 4 offsets
    sc, of = O.tile64_meta_positions("k")
    assert sc[0].tolist() == [0, 1, 2, 3] and of[0].tolist() == [4, 5, 6, 7] and sc[5, 2] == 42 and of[63, 3] == 511
    sc, of = O.tile64_meta_positions("v")
    assert sc[0].tolist() == [0, 8, 16, 24] and sc[1, 0] == 1 and of[0, 0] == 4 and sc[4, 0] == 32 and of[63, 3] == 511


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_tile64_pack_roundtrip_and_padding(bits):
    rng = np.random.default_rng(60 + bits)
    n = 150                                                      # two full tiles and a ragged third
    codes = rng.integers(0, 1 << bits, (n, 128)).astype(np.uint8)
    sc = rng.integers(0, 65536, (n, 4)).astype(np.uint16)
    of = rng.integers(0, 65536, (n, 4)).astype(np.uint16)
    for which in ("k", "v"):
        data, meta = O.pack_tiles64(codes, sc, of, bits, which)
        assert data.size == 3 * O.tile64_data_bytes(bits) and meta.size == 3 * 1024
        c2, s2, o2 = O.unpack_tiles64(data, meta, n, bits, which)
        np.testing.assert_array_equal(c2, codes)
        np.testing.assert_array_equal(s2, sc)
        np.testing.assert_array_equal(o2, of)
        c3, s3, o3 = O.unpack_tiles64(data, meta, 192, bits, which)
        assert not c3[n:].any() and not s3[n:].any() and not o3[n:].any()
    one = np.zeros((1, 128), np.uint8)
    one[0, 77] = (1 << bits) - 1
    data, _ = O.pack_tiles64(one, np.zeros((1, 4), np.uint16), np.zeros((1, 4), np.uint16), bits, "v")
    assert int(np.unpackbits(data).sum()) == bits


# ----------------------------------------------------------------------------
# mixed mode: V token-wise, K channel-wise on the retained tokens (Sec. 3.2 Stages 2-3, App. B)
# ----------------------------------------------------------------------------
def _mixed_case(rng, T=150, hkv=2, p_tok=(.3, .3, .2, .1, .1), p_ch=(.1, .4, .3, .15, .05)):
    K = rand_bf16(rng, (hkv, T, 128))
    K[:, :, 7] *= 10.0
    K = bf16_round(K)
    V = rand_bf16(rng, (hkv, T, 128))
    bt = rng.choice([0, 2, 4, 8, 16], (hkv, T), p=p_tok).astype(np.uint8)
    bc = rng.choice([0, 2, 4, 8, 16], (hkv, 128), p=p_ch).astype(np.uint8)
    return K, V, bt, bc


def test_mixed_all_16_bit_reproduces_bruteforce_attention():
    rng = np.random.default_rng(41)
    K, V, _, _ = _mixed_case(rng, T=70)
    bt = np.full((2, 70), 16, np.uint8)
    bc = np.full((2, 128), 16, np.uint8)
    cache = O.build_cache_mixed([K], [V], [bt], [bc])
    q = rand_bf16(rng, (1, 8, 128))
    out, lse = O.decode(cache, q)
    for j in range(8):
        o, l = _bruteforce_attention(q[0, j], K[j // 4], V[j // 4])
        np.testing.assert_allclose(out[0, j], o, rtol=1e-12, atol=1e-13)
        assert abs(lse[0, j] - l) < 1e-12


def test_zero_bit_channel_is_a_zeroed_key_column_and_zero_bit_token_is_eviction():
    # Sec. 3.2: a channel with b_c = 0 is removed (its K column contributes nothing to q.k);
    # a token with b_t = 0 is evicted.  With every other unit at 16 bits the result is exact.
    rng = np.random.default_rng(42)
    K, V, _, _ = _mixed_case(rng, T=90)
    bt = np.where(rng.random((2, 90)) < 0.4, 0, 16).astype(np.uint8)
    bc = np.where(rng.random((2, 128)) < 0.3, 0, 16).astype(np.uint8)
    cache = O.build_cache_mixed([K], [V], [bt], [bc])
    q = rand_bf16(rng, (1, 8, 128))
    out, lse = O.decode(cache, q)
    for j in range(8):
        h = j // 4
        keep = np.nonzero(bt[h])[0]
        Kz = K[h][keep].astype(np.float64) * (bc[h] > 0)[None, :]
        o, l = _bruteforce_attention(q[0, j], Kz, V[h][keep])
        np.testing.assert_allclose(out[0, j], o, rtol=1e-12, atol=1e-13)
        assert abs(lse[0, j] - l) < 1e-12


def test_channelwise_quantizer_groups_are_32_tokens_of_one_channel():
    rng = np.random.default_rng(43)
    n = 75
    X = rand_bf16(rng, (n, 128), scale=2.0)
    bc = np.tile(np.array([16, 8, 4, 2, 0, 8, 4, 2], np.uint8), 16)
    codes, sc, of = O.quantize_channelwise(X, bc)
    Xh = O.dequantize_channelwise(codes, sc, of, bc)
    assert sc.shape == (3, 128) and of.shape == (3, 128)
    for c in range(128):
        b = int(bc[c])
        if b == 16:
            np.testing.assert_array_equal(Xh[:, c], X[:, c].astype(np.float64))      # input bits kept
        elif b == 0:
            assert not Xh[:, c].any() and not codes[:, c].any()
        else:
            assert codes[:, c].max() <= (1 << b) - 1
            for t in range(3):
                rows = slice(32 * t, min(n, 32 * t + 32))
                s = float(sc[t, c:c + 1].view(np.float16)[0])
                m = float(of[t, c:c + 1].view(np.float16)[0])
                # offset = the group's minimum (bf16 values of this size are exact in fp16)
                assert m == float(X[rows, c].min())
                # error bound of a round-to-nearest uniform quantizer (fp16 rounding of s may clamp the top element)
                assert np.abs(Xh[rows, c] - X[rows, c]).max() <= 0.5 * s * (1 + 2 ** -10) + 0.125 * s * (b == 8)
    # a group is one tile of one channel: changing tile 1 of channel 1 leaves every other (tile, channel) alone
    X2 = X.copy()
    X2[40, 1] = np.float32(50.0)
    c2, s2, o2 = O.quantize_channelwise(X2, bc)
    same = np.ones((3, 128), bool)
    same[1, 1] = False
    assert np.array_equal(s2[same], sc[same]) and np.array_equal(o2[same], of[same]) and s2[1, 1] != sc[1, 1]
    keep = np.ones((n, 128), bool)
    keep[32:64, 1] = False
    assert np.array_equal(c2[keep], codes[keep])


def test_per_channel_dequantization_fusion_identity():
    # App. B: q.k_hat = sum_c (s_c q_c) code_c - sum_c s_c z_c q_c with k_hat = s (code - z), here z = -m / s
    rng = np.random.default_rng(44)
    X = rand_bf16(rng, (32, 128))
    bc = rng.choice([2, 4, 8], 128).astype(np.uint8)
    codes, sc, of = O.quantize_channelwise(X, bc)
    s = sc[0].copy().view(np.float16).astype(np.float64)
    m = of[0].copy().view(np.float16).astype(np.float64)
    q = rng.standard_normal(128)
    fused = codes.astype(np.float64) @ (s * q) + np.dot(m, q)            # -s z = m
    direct = O.dequantize_channelwise(codes, sc, of, bc) @ q
    np.testing.assert_allclose(fused, direct, rtol=1e-12, atol=1e-12)


def _hand_bits_ch():
    bc = np.zeros(128, np.uint8)
    bc[[5, 70, 100]] = 8
    bc[[0, 1]] = 16
    bc[10:21] = 4                      # 11 channels -> two words of 8 slots, five padding slots
    bc[[30, 31, 32]] = 2
    return bc


def test_channel_slots_hand_worked():
    sl = O.channel_slots(_hand_bits_ch())
    assert sl["npad"] == {16: 4, 8: 4, 4: 16, 2: 16} and sl["nw"] == {16: 2, 8: 1, 4: 2, 2: 1}
    assert sl["slot_ch"].tolist() == [0, 1, -1, -1] + [5, 70, 100, -1] + list(range(10, 21)) + [-1] * 5 \
        + [30, 31, 32] + [-1] * 13
    assert (sl["n_words"], sl["n_words_padded"], sl["n_steps16"], sl["n_qsteps"]) == (6, 6, 1, 9)
    assert O.k_tile_bytes_mixed(sl) == 64 * 6 * 4 and O.k_meta_bytes_mixed(sl) == 2 * 9 * 16
    # an odd word count is padded to an even one; no channels at all -> no bytes
    bc = np.zeros(128, np.uint8)
    bc[:4] = 8
    sl = O.channel_slots(bc)
    assert (sl["n_words"], sl["n_words_padded"]) == (1, 2)
    sl = O.channel_slots(np.zeros(128, np.uint8))
    assert O.k_tile_bytes_mixed(sl) == 0 and O.k_meta_bytes_mixed(sl) == 0 and sl["slot_ch"].size == 0
    # every channel at 16 bits: 64 words per token, 32 steps, no padding
    sl = O.channel_slots(np.full(128, 16, np.uint8))
    assert (sl["n_words"], sl["n_steps16"], sl["n_qsteps"]) == (64, 32, 0) and (sl["slot_ch"] >= 0).all()


def test_mixed_k_tile_layout_hand_checked_and_roundtrip():
    rng = np.random.default_rng(45)
    bc = _hand_bits_ch()
    n = 75
    X = rand_bf16(rng, (n, 128))
    codes, sc, of = O.quantize_channelwise(X, bc)
    data, meta = O.pack_k_tiles_mixed(codes, sc, of, bc)
    tb = 1536
    assert data.size == 2 * tb and meta.size == 2 * 288
    d16 = data.view("<u2")
    # six words per token: words 0..3 of token r at byte 16 r, words 4, 5 at byte 1024 + 8 r.
    # words 0, 1 = the 16-bit step: channels 0, 1 in the halves of word 0, two padding slots in word 1
    assert d16[0] == codes[0, 0] and d16[1] == codes[0, 1] and d16[2] == 0 and d16[3] == 0 and d16[8] == codes[1, 0]
    # word 2 = the 8-bit step (channels 5, 70, 100, padding): elements 0, 1 in the low bytes of the halves,
    # elements 2, 3 in their high bytes
    assert data[8] == codes[0, 5] and data[10] == codes[0, 70] and data[9] == codes[0, 100] and data[11] == 0
    assert data[16 + 8] == codes[1, 5]
    # word 3 = 4-bit channels 10..17: step 0 = (10, 11, 12, 13) in the low byte of each half, step 1 in the high byte;
    # inside a byte the low nibble is element 0 / 1, the high nibble element 2 / 3
    assert (int(data[12]) & 15, int(data[12]) >> 4) == (int(codes[0, 10]), int(codes[0, 12]))
    assert (int(data[14]) & 15, int(data[14]) >> 4) == (int(codes[0, 11]), int(codes[0, 13]))
    assert (int(data[13]) & 15, int(data[13]) >> 4) == (int(codes[0, 14]), int(codes[0, 16]))
    assert (int(data[15]) & 15, int(data[15]) >> 4) == (int(codes[0, 15]), int(codes[0, 17]))
    # word 4 (second run) = 4-bit channels 18, 19, 20 and five padding slots
    assert (int(data[1024]) & 15, int(data[1024]) >> 4) == (int(codes[0, 18]), int(codes[0, 20]))
    assert int(data[1026]) == int(codes[0, 19]) and data[1025] == 0 and data[1027] == 0
    # word 5 = 2-bit channels 30, 31, 32: elements 0, 1 at bits 0-1 of the halves, element 2 at bits 2-3
    w = int(data[1028:1032].view("<u4")[0])
    assert (w & 3, (w >> 16) & 3, (w >> 2) & 3, w >> 18, (w >> 4) & 0xFFF) == \
        (int(codes[0, 30]), int(codes[0, 31]), int(codes[0, 32]), 0, 0)
    assert (int(data[1024 + 8 + 4]) & 3) == int(codes[1, 30])
    # second tile: rows 64..74, zero rows after them
    assert data[tb + 8] == codes[64, 5] and data[tb + 16 * 10 + 8] == codes[74, 5] and data[tb + 16 * 11 + 8] == 0
    # metadata: per token group and quantized step 4 scales then 4 offsets; 9 steps = 1 (8-bit) + 4 + 4
    m16 = meta.view("<u2")
    assert m16[:8].tolist() == [sc[0, 5], sc[0, 70], sc[0, 100], 0, of[0, 5], of[0, 70], of[0, 100], 0]
    assert m16[8:12].tolist() == [sc[0, c] for c in (10, 11, 12, 13)] and m16[12] == of[0, 10]
    assert m16[40:44].tolist() == [sc[0, 30], sc[0, 31], sc[0, 32], 0]
    assert m16[72] == sc[1, 5] and m16[144] == sc[2, 5] and m16[144 + 72] == 0       # group 1; tile 1; no rows in group 3
    c2, s2, o2 = O.unpack_k_tiles_mixed(data, meta, n, bc)
    np.testing.assert_array_equal(c2, codes)
    np.testing.assert_array_equal(s2, sc)
    np.testing.assert_array_equal(o2, of)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_mixed_k_tile_fields_are_disjoint_and_cover_the_tile(seed):
    rng = np.random.default_rng(seed)
    bc = rng.choice([0, 2, 4, 8, 16], 128, p=[.1, .4, .3, .15, .05]).astype(np.uint8)
    sl = O.channel_slots(bc)
    # all-ones codes of every real slot: set bits = sum of widths x 64 tokens, so no two fields overlap
    codes = np.zeros((64, 128), np.uint16)
    for c in range(128):
        codes[:, c] = (1 << int(bc[c])) - 1 if bc[c] else 0
    ng = 2
    data, _ = O.pack_k_tiles_mixed(codes, np.zeros((ng, 128), np.uint16), np.zeros((ng, 128), np.uint16), bc)
    assert data.size == O.k_tile_bytes_mixed(sl)
    assert int(np.unpackbits(data).sum()) == 64 * int(bc.astype(np.int64).sum())
    # a quantized code never reaches the exponent bits of its 16-bit half once its step's shift is applied:
    # fields of one half are 2b apart per step and b apart inside a step
    for b in (2, 4, 8):
        bits = sorted(O._k_code_bit(b, j) % 16 for j in range(0, 32 // b, 2))
        assert bits == list(range(0, 16, b))


def test_v16_tile_roundtrip_and_positions():
    rng = np.random.default_rng(46)
    vb = rng.integers(0, 65536, (70, 128)).astype(np.uint16)
    data = O.pack_v16_tiles(vb)
    assert data.size == 2 * 16384
    w = data.view("<u2")
    # lane 0 = (token half 0, channel 0): its first 16-byte unit holds tokens 0..7, the next unit (1 KiB on) 8..15
    assert [int(x) for x in w[:8]] == [int(vb[r, 0]) for r in range(8)] and w[512] == vb[8, 0]
    # lane 1 = channel 1; lane 32 = token half 1; channel 32 = group 1 = unit 4
    assert w[8] == vb[0, 1] and w[256] == vb[32, 0] and w[2048] == vb[0, 32]
    assert w[8192] == vb[64, 0] and w[8192 + 6] == 0                                # second tile: rows 64..69, then zeros
    np.testing.assert_array_equal(O.unpack_v16_tiles(data, 70), vb)


def test_mixed_cache_bytes_and_decode_from_physical_bytes():
    rng = np.random.default_rng(47)
    K, V, bt, bc = _mixed_case(rng)
    cache = O.build_cache_mixed([K], [V], [bt], [bc])
    # closed-form segment sizes
    for item in range(2):
        sl = O.channel_slots(bc[item])
        for ti, b in enumerate(O.PACK_ORDER):
            n = int((bt[item] == b).sum())
            assert cache["counts"][item, ti] == n
            nt = (n + 63) // 64
            sizes = [nt * O.k_tile_bytes_mixed(sl), nt * O.k_meta_bytes_mixed(sl),
                     nt * (16384 if b == 16 else 1024 * b), 0 if b == 16 else nt * 1024]
            offs = cache["seg_off"][item, ti]
            assert all(int(o) % 256 == 0 for o in offs)
            nxt = list(offs[1:]) + [cache["seg_off"][item, ti + 1, 0] if ti < 3 else
                                    (cache["seg_off"][item + 1, 0, 0] if item == 0 else cache["arena"].size)]
            for o, sz, o2 in zip(offs, sizes, nxt):
                assert int(o) + sz <= int(o2) < int(o) + sz + 256
    # decoding the physical bytes equals attention over the canonical dequantized rows
    q = rand_bf16(rng, (1, 8, 128))
    out, lse = O.decode(cache, q)
    for j in range(8):
        h = j // 4
        rec = cache["canon"][h]
        Kh = np.concatenate([O.dequantize_channelwise(rec[b]["k_codes"], rec[b]["k_scale"], rec[b]["k_off"], bc[h])
                             for b in O.PACK_ORDER])
        Vh = np.concatenate([O.bf16_from_bits(rec[16]["v_codes"]).astype(np.float64)] +
                            [O.dequantize_groups(rec[b]["v_codes"].reshape(-1, 4, 32), rec[b]["v_scale"].view(np.float16),
                                                 rec[b]["v_off"].view(np.float16)).reshape(-1, 128) for b in (8, 4, 2)])
        o, l = _bruteforce_attention(q[0, j], Kh, Vh)
        np.testing.assert_allclose(out[0, j], o, rtol=1e-11, atol=1e-12)
    assert O.stored_bytes_mixed(cache["counts"], cache["bits_ch"]) < cache["arena"].size


def test_stored_bytes_mixed_hand_computed():
    """Bytes a mixed-mode decode step reads, worked by hand for the channel map of _hand_bits_ch(): 2 channels at 16
    bits, 3 at 8, 11 at 4, 3 at 2 -> 32 + 24 + 44 + 6 = 106 bits = 13.25 bytes of K codes per retained token, 17
    quantized channels of 4 metadata bytes (fp16 scale + fp16 offset) per group of 32 retained tokens; V rows as in
    token-wise mode (256 / 144 / 80 / 48 bytes at 16 / 8 / 4 / 2 bits)."""
    bc = _hand_bits_ch()
    counts = np.array([[3, 40, 65, 0]])                # rows per V tier 16, 8, 4, 2
    # tier 16:  3 rows: K floor(3 * 13.25) = 39,  1 group -> 68;   V 3 * 256  = 768   -> 875
    # tier  8: 40 rows: K 530,                    2 groups -> 136; V 40 * 144 = 5760  -> 6426
    # tier  4: 65 rows: K floor(861.25) = 861,    3 groups -> 204; V 65 * 80  = 5200  -> 6265
    assert O.stored_bytes_mixed(counts, [bc]) == 875 + 6426 + 6265 == 13566
    # one scale per channel over all retained tokens: one 68-byte record per non-empty tier segment
    assert O.stored_bytes_mixed(counts, [bc], k_per_channel_scale=True) == (39 + 68 + 768) + (530 + 68 + 5760) + (861 + 68 + 5200) == 13362
    # second item with no quantized channel (all 16-bit: 256 bytes per K row, no metadata) and 2-bit V rows only
    bc16 = np.full(128, 16, np.uint8)
    two = np.array([[3, 40, 65, 0], [0, 0, 0, 10]])
    assert O.stored_bytes_mixed(two, [bc, bc16]) == 13566 + 10 * 256 + 10 * 48
    # every channel evicted: only the V rows remain
    assert O.stored_bytes_mixed(np.array([[1, 1, 1, 1]]), [np.zeros(128, np.uint8)]) == 256 + 144 + 80 + 48
    # cross-check against the packed form on real data: the arena of a cache whose segments are all whole tiles and
    # 256-byte multiples holds exactly the stored bytes plus the zero padding of the sorted-channel rows
    rng = np.random.default_rng(91)
    T = 64 * 4
    K, V = rand_bf16(rng, (1, T, 128)), rand_bf16(rng, (1, T, 128))
    bt = np.repeat(np.array([16, 8, 4, 2], np.uint8), 64)[None]
    cache = O.build_cache_mixed([K], [V], [bt], [bc[None]])
    sl = O.channel_slots(bc)
    pad_k = 4 * (O.k_tile_bytes_mixed(sl) - 64 * 106 // 8)            # padding slots inside the four K tiles
    pad_meta = 4 * 2 * (4 * 9 - 17) * 4                               # 9 quantized steps = 36 slots for 17 channels
    align = 4 * (512 - O.k_meta_bytes_mixed(sl))                      # each tile's 288 metadata bytes end a 256-byte unit
    assert cache["arena"].size - pad_k - pad_meta - align == O.stored_bytes_mixed(cache["counts"], cache["bits_ch"])


def test_allocate_mixed_meets_both_budgets():
    # Sec. 3.2: B_V = B_K = B_head / 2; the K budget is spread over the retained tokens only
    rng = np.random.default_rng(48)
    T, d = 3000, 128
    w_tok = (1.0 + rng.pareto(1.2, T)).astype(np.float32)
    w_ch = np.exp(rng.standard_normal(d)).astype(np.float32)
    for avg in (0.5, 1.0, 2.0):
        bt, bc = O.allocate_mixed(w_tok, w_ch, np.float32(avg))
        n_kept = int((bt > 0).sum())
        assert int(bt.astype(np.int64).sum()) <= math.floor(avg * T)                    # V: mean b_t <= avg
        k_avg = min(16.0, avg * T / n_kept)
        assert int(bc.astype(np.int64).sum()) <= math.floor(np.float32(k_avg) * d)      # K: mean b_c <= k_avg
        # whole-cache budget: nominal bits of V plus K never exceed avg bits per cache scalar
        total_bits = int(bt.astype(np.int64).sum()) * d + int(bc.astype(np.int64).sum()) * n_kept
        assert total_bits <= avg * 2 * T * d
        assert set(np.unique(bt)) <= {0, 2, 4, 8, 16} and set(np.unique(bc)) <= {0, 2, 4, 8, 16}
    bt, bc = O.allocate_mixed(w_tok, w_ch, np.float32(0.0))
    assert not bt.any() and not bc.any()


# ----------------------------------------------------------------------------
# Zone C: tokens appended after the compression pass (third term of Eq. 7)
# ----------------------------------------------------------------------------
def test_appended_tokens_on_an_all_16_bit_cache_reproduce_bruteforce_attention():
    rng = np.random.default_rng(61)
    Hkv, g, T, n_new = 2, 4, 150, 5
    Ks, Vs = _small_case(rng, Hkv=Hkv, T=T)
    cache = O.build_cache_tokenwise(Ks, Vs, [np.full((Hkv, T), 16, np.uint8)])
    kn = rand_bf16(rng, (n_new, 1, Hkv, 128))
    vn = rand_bf16(rng, (n_new, 1, Hkv, 128))
    for i in range(n_new):
        O.append_tokens(cache, kn[i], vn[i])
    q = rand_bf16(rng, (1, Hkv * g, 128))
    out, lse = O.decode(cache, q)
    for j in range(Hkv * g):
        h = j // g
        Kall = np.concatenate([Ks[0][h], kn[:, 0, h]])
        Vall = np.concatenate([Vs[0][h], vn[:, 0, h]])
        o, l = _bruteforce_attention(q[0, j], Kall, Vall)
        np.testing.assert_allclose(out[0, j], o, rtol=1e-12, atol=1e-13)
        assert abs(lse[0, j] - l) < 1e-12


def test_appended_zone_is_the_lse_merge_of_the_two_zones_and_survives_full_eviction():
    # Eq. 7: the output over (compressed rows, new rows) is the softmax-weighted merge of the two zones
    rng = np.random.default_rng(62)
    Hkv, g, T = 2, 2, 200
    Ks, Vs = _small_case(rng, Hkv=Hkv, T=T)
    bits = rng.choice([0, 2, 4, 8, 16], (Hkv, T)).astype(np.uint8)
    bits[1, :] = 0                                                 # head 1 keeps nothing of the prompt
    cache = O.build_cache_tokenwise(Ks, Vs, [bits])
    q = rand_bf16(rng, (1, Hkv * g, 128))
    out_a, lse_a = O.decode(cache, q)
    kn = rand_bf16(rng, (3, 1, Hkv, 128))
    vn = rand_bf16(rng, (3, 1, Hkv, 128))
    for i in range(3):
        O.append_tokens(cache, kn[i], vn[i])
    out, lse = O.decode(cache, q)
    for j in range(Hkv * g):
        h = j // g
        o_c, l_c = _bruteforce_attention(q[0, j], kn[:, 0, h], vn[:, 0, h])
        o_c = np.asarray(o_c)
        if h == 1:                                                 # only the new tokens are left
            np.testing.assert_allclose(out[0, j], o_c, rtol=1e-12, atol=1e-13)
            assert abs(lse[0, j] - l_c) < 1e-12 and np.isneginf(lse_a[0, j])
        else:
            m = max(lse_a[0, j], l_c)
            wa, wc = np.exp(lse_a[0, j] - m), np.exp(l_c - m)
            np.testing.assert_allclose(out[0, j], (wa * out_a[0, j] + wc * o_c) / (wa + wc), rtol=1e-11, atol=1e-12)
            assert abs(lse[0, j] - (m + np.log(wa + wc))) < 1e-11


# ----------------------------------------------------------------------------
# the paper's own K format: one scale and zero-point per channel over all retained tokens (App. B)
# ----------------------------------------------------------------------------
def test_per_channel_scale_is_one_group_over_the_whole_unit():
    rng = np.random.default_rng(71)
    n = 100
    X = rand_bf16(rng, (n, 128), scale=2.0)
    bc = rng.choice([0, 2, 4, 8, 16], 128).astype(np.uint8)
    codes, sc, of = O.quantize_channelwise(X, bc, None)
    assert sc.shape == (1, 128) and of.shape == (1, 128)
    Xh = O.dequantize_channelwise(codes, sc, of, bc, None)
    q = rng.standard_normal(128)
    s = sc[0].copy().view(np.float16).astype(np.float64)
    m = of[0].copy().view(np.float16).astype(np.float64)
    for c in range(128):
        b = int(bc[c])
        if b in (2, 4, 8):
            assert m[c] == float(X[:, c].min())                           # offset = minimum of the whole unit
            assert np.abs(Xh[:, c] - X[:, c]).max() <= 0.5 * s[c] * (1 + 2 ** -10) + 0.125 * s[c] * (b == 8)
            assert codes[:, c].max() <= (1 << b) - 1 and codes[:, c].min() == 0
    # fusion identity with a single scaled query for every token (App. B): q.k_hat = sum (s q) code + sum m q
    quant = np.isin(bc, (2, 4, 8))
    raw16 = np.where(bc == 16)[0]
    fused = codes[:, quant].astype(np.float64) @ (s[quant] * q[quant]) + np.dot(m[quant], q[quant]) \
        + X[:, raw16].astype(np.float64) @ q[raw16]
    np.testing.assert_allclose(fused, Xh @ q, rtol=1e-12, atol=1e-12)
    # a unit of at most 32 tokens is the same thing in both formats
    c32, s32, o32 = O.quantize_channelwise(X[:32], bc)
    c1, s1, o1 = O.quantize_channelwise(X[:32], bc, None)
    assert np.array_equal(c32, c1) and np.array_equal(s32, s1) and np.array_equal(o32, o1)


def test_mixed_cache_with_per_channel_scale_bytes_and_decode():
    rng = np.random.default_rng(72)
    K, V, bt, bc = _mixed_case(rng)
    cache = O.build_cache_mixed([K], [V], [bt], [bc], k_per_channel_scale=True)
    for item in range(2):
        sl = O.channel_slots(bc[item])
        keep = np.concatenate([np.nonzero(bt[item] == b)[0] for b in O.PACK_ORDER])
        codes, sc, of = O.quantize_channelwise(K[item][keep], bc[item], None)
        for ti, b in enumerate(O.PACK_ORDER):
            n = int((bt[item] == b).sum())
            offs = cache["seg_off"][item, ti]
            # the metadata segment of a non-empty tier is one record: 16 bytes per quantized step
            nxt = int(offs[2])
            assert int(offs[1]) + (16 * sl["n_qsteps"] if n else 0) <= nxt < int(offs[1]) + 16 * sl["n_qsteps"] + 256
            if n:
                m16 = cache["arena"][int(offs[1]):int(offs[1]) + 16 * sl["n_qsteps"]].view("<u2")
                q0 = int(np.nonzero(sl["slot_ch"][sl["npad"][16]:] >= 0)[0][0])          # first real quantized slot
                ch = int(sl["slot_ch"][sl["npad"][16] + q0])
                assert m16[8 * (q0 // 4) + q0 % 4] == sc[0, ch] and m16[8 * (q0 // 4) + 4 + q0 % 4] == of[0, ch]
    q = rand_bf16(rng, (1, 8, 128))
    out, lse = O.decode(cache, q)
    for j in range(8):
        h = j // 4
        keep = np.concatenate([np.nonzero(bt[h] == b)[0] for b in O.PACK_ORDER])
        codes, sc, of = O.quantize_channelwise(K[h][keep], bc[h], None)
        Kh = O.dequantize_channelwise(codes, sc, of, bc[h], None)
        rec = cache["canon"][h]
        Vh = np.concatenate([O.bf16_from_bits(rec[16]["v_codes"]).astype(np.float64)] +
                            [O.dequantize_groups(rec[b]["v_codes"].reshape(-1, 4, 32), rec[b]["v_scale"].view(np.float16),
                                                 rec[b]["v_off"].view(np.float16)).reshape(-1, 128) for b in (8, 4, 2)])
        o, l = _bruteforce_attention(q[0, j], Kh, Vh)
        np.testing.assert_allclose(out[0, j], o, rtol=1e-11, atol=1e-12)
    full = O.build_cache_mixed([K], [V], [bt], [bc])
    assert O.stored_bytes_mixed(cache["counts"], cache["bits_ch"], k_per_channel_scale=True) < \
        O.stored_bytes_mixed(full["counts"], full["bits_ch"])


# ---- distortion-table calibration (App. B "Calibration", App. "Calibrated Distortion Tables") --------------------------------------------------
def _grid_group(bits, rng):
    """32 values m + s (code + delta), s a power of two, delta = +-1/4 except on the two end points: the quantizer
    must find exactly these codes, and every inner element is off by exactly s/4.  All values are bf16-exact."""
    Q = (1 << bits) - 1
    s = 2.0 ** -7
    pool = list(range(1, min(Q, 64)))               # codes whose 4 code +- 1 still fits 8 significant bits
    inner = rng.choice(pool, size=30, replace=True)
    delta = rng.choice([-0.25, 0.25], size=30)
    x = np.concatenate([[0.0], s * (inner + delta), [s * Q]]).astype(np.float32)
    rng.shuffle(x)
    return x, 30 * (s / 4) ** 2


@pytest.mark.parametrize("channelwise", [False, True])
def test_calibration_closed_form_on_grid_data(channelwise):
    rng = np.random.default_rng(11)
    T, d = 64, 128
    for bi, bits in enumerate(O.CALIB_BITS):
        X = np.zeros((T, d), dtype=np.float32)
        err = 0.0
        for a in range(T):                            # row a, group grp (token-wise view)
            for grp in range(4):
                X[a, 32 * grp:32 * grp + 32], e = _grid_group(bits, rng)
                err += e
        want = err / float((X.astype(np.float64) ** 2).sum())
        assert np.array_equal(bf16_round(X), X)
        if channelwise:                               # the same groups laid along the token axis of a channel
            Kc = X.reshape(T, 4, 32).transpose(1, 2, 0).reshape(128, T)          # token = 32 grp + i, channel = a
            Kc = np.concatenate([Kc, Kc], axis=1)                               # d = 128 channels
            want = 2 * err / float((Kc.astype(np.float64) ** 2).sum())
            ek, _ = O.calibrate_eps([Kc[None]], [Kc[None]], k_channelwise=True)
        else:
            ek, ev = O.calibrate_eps([X[None]], [X[None]])
            assert ev[0, bi] == pytest.approx(want, rel=1e-12)
        assert ek[0, bi] == pytest.approx(want, rel=1e-12)


def test_calibration_axes_transposition_and_unit_scale():
    # channel-wise K in groups of 32 tokens is token-wise quantization of the transposed matrix
    rng = np.random.default_rng(12)
    X = bf16_round(rng.standard_normal((128, 128)).astype(np.float32) * np.float32(3.0))
    ek_ch, ev = O.calibrate_eps([X[None]], [X[None]], k_channelwise=True)
    ek_tr, _ = O.calibrate_eps([X.T.copy()[None]], [X[None]])
    np.testing.assert_allclose(ek_ch, ek_tr, rtol=1e-13)
    # with at most 32 tokens a channel's only group is the whole unit: both K formats agree
    Y = X[:29]
    a, _ = O.calibrate_eps([Y[None]], [Y[None]], k_channelwise=True)
    b_, _ = O.calibrate_eps([Y[None]], [Y[None]], k_channelwise=True, k_per_channel_scale=True)
    np.testing.assert_array_equal(a, b_)
    # one scale over a long unit is coarser than one per 32 tokens
    c, _ = O.calibrate_eps([X[None]], [X[None]], k_channelwise=True, k_per_channel_scale=True)
    assert (c > ek_ch).all()
    # powers of two scale the data, the scales and the errors alike
    e1 = O.calibrate_eps([X[None]], [X[None]])
    e2 = O.calibrate_eps([(X * np.float32(0.25))[None]], [(X * np.float32(0.25))[None]])
    np.testing.assert_allclose(e1[0], e2[0], rtol=1e-12)
    np.testing.assert_allclose(e1[1], e2[1], rtol=1e-12)


def test_calibration_on_gaussian_data_has_the_printed_order_of_magnitude():
    # uniform quantization noise: a step of range / Q gives a mean squared error of step^2 / 12; Table 9's entries
    # (five models) span 0.149-0.347, 0.0062-0.0164 and 2.2e-5-1.5e-4 (one outlier at 4.4e-3)
    tab = _read_table9()
    lo = [min(min(ek[i], ev[i]) for ek, ev in tab.values()) for i in (1, 2, 3)]
    hi = [max(max(ek[i], ev[i]) for ek, ev in tab.values()) for i in (1, 2, 3)]
    rng = np.random.default_rng(13)
    K = bf16_round(rng.standard_normal((2, 512, 128)).astype(np.float32))
    V = bf16_round(rng.standard_normal((2, 512, 128)).astype(np.float32))
    ek, ev = O.calibrate_eps([K], [V])
    assert ek.shape == (2, 3) and ev.shape == (2, 3)
    for e in (ek, ev):
        assert (e[:, 0] > e[:, 1]).all() and (e[:, 1] > e[:, 2]).all()
        for i in range(3):
            assert (e[:, i] > 0.5 * lo[i]).all() and (e[:, i] < 2.0 * hi[i]).all()
    # and against the noise model itself: E[step^2] / 12 with the measured group ranges
    x = V[0].reshape(512, 4, 32)
    rng_g = x.max(-1).astype(np.float64) - x.min(-1).astype(np.float64)
    for i, b in enumerate(O.CALIB_BITS[1:], start=1):     # 2-bit noise is far from uniform; 4- and 8-bit are close
        model = float((32 * (rng_g / ((1 << b) - 1)) ** 2 / 12).sum() / (V[0].astype(np.float64) ** 2).sum())
        assert ev[0, i] == pytest.approx(model, rel=0.1)


def test_calibration_degenerate_slices():
    Z = np.zeros((1, 40, 128), dtype=np.float32)
    C = np.full((1, 40, 128), 1.5, dtype=np.float32)      # constant groups: scale 0, offset = the value: exact
    for kw in ({}, {"k_channelwise": True}, {"k_channelwise": True, "k_per_channel_scale": True}):
        ek, ev = O.calibrate_eps([Z, C], [Z, C], **kw)
        assert not ek.any() and not ev.any()


# ----------------------------------------------------------------------------
# streaming re-budgeting: the appended tokens go through the same pass (App. "Limitations and Future Work")
# ----------------------------------------------------------------------------
def _cache_with_tail(rng, Hkv, g, T, n_new, mixed=False):
    Ks, Vs = _small_case(rng, Hkv=Hkv, T=T)
    bits = rng.choice([0, 2, 4, 8, 16], (Hkv, T)).astype(np.uint8)
    if mixed:
        cache = O.build_cache_mixed(Ks, Vs, [bits], [rng.choice([0, 2, 4, 8, 16], (Hkv, 128)).astype(np.uint8)])
    else:
        cache = O.build_cache_tokenwise(Ks, Vs, [bits])
    kn = rand_bf16(rng, (n_new, 1, Hkv, 128))
    vn = rand_bf16(rng, (n_new, 1, Hkv, 128))
    for i in range(n_new):
        O.append_tokens(cache, kn[i], vn[i])
    return cache, kn, vn


@pytest.mark.parametrize("mixed", [False, True])
def test_rebudget_at_16_bits_changes_nothing_and_at_0_bits_forgets_the_tail(mixed):
    rng = np.random.default_rng(81)
    Hkv, g, T, n_new, S_w = 2, 2, 120, 70, 8
    q = rand_bf16(rng, (1, Hkv * g, 128))
    Qobs = [rand_bf16(rng, (Hkv * g, S_w, 128))]
    cache, kn, vn = _cache_with_tail(rng, Hkv, g, T, n_new, mixed)
    before, lse_before = O.decode(cache, q)
    child = O.rebudget_tail(cache, Qobs, [np.float32(16.0)])
    assert (np.concatenate([b.ravel() for b in child["bits"]]) == 16).all()      # every row kept verbatim
    assert not mixed or (child["bits_ch"] == 16).all()
    assert all(t[0].shape[0] == 0 for t in cache["tail"])                       # the tail is empty again
    after, lse_after = O.decode(cache, q)
    np.testing.assert_allclose(after, before, rtol=1e-12, atol=1e-13)            # same rows, other order
    np.testing.assert_allclose(lse_after, lse_before, rtol=0, atol=1e-12)

    cache2, _, _ = _cache_with_tail(np.random.default_rng(83), Hkv, g, T, n_new, mixed)
    # a zero budget evicts the whole tail: what is left is the prefix alone
    prefix_only = {k: v for k, v in cache2.items() if k != "tail"}
    want, lse_want = O.decode(prefix_only, q)
    O.rebudget_tail(cache2, Qobs, [np.float32(0.0)])
    got, lse_got = O.decode(cache2, q)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse_got, lse_want, rtol=0, atol=1e-12)


def test_rebudget_is_the_compression_pass_on_the_tail_and_decode_merges_the_generations():
    rng = np.random.default_rng(82)
    Hkv, g, T, n_new, S_w = 2, 2, 150, 96, 16
    q = rand_bf16(rng, (1, Hkv * g, 128))
    Qobs = [rand_bf16(rng, (Hkv * g, S_w, 128))]
    cache, kn, vn = _cache_with_tail(rng, Hkv, g, T, n_new)
    prefix_only = {k: v for k, v in cache.items() if k != "tail"}
    out_p, lse_p = O.decode(prefix_only, q)
    child = O.rebudget_tail(cache, Qobs, [np.float32(3.0)])
    # the child is what the one-shot pass makes of the appended rows taken as a sequence of their own
    K_tail = np.ascontiguousarray(kn[:, 0].transpose(1, 0, 2))
    V_tail = np.ascontiguousarray(vn[:, 0].transpose(1, 0, 2))
    alone = O.compress_tokenwise([K_tail], [V_tail], Qobs, [np.float32(3.0)])
    assert np.array_equal(child["arena"], alone["arena"]) and np.array_equal(child["tier_idx"], alone["tier_idx"])
    for h in range(Hkv):
        assert int(child["bits"][0][h].astype(np.int64).sum()) <= math.floor(3.0 * n_new)      # its own budget (Eq. 6)
        assert 0 < int((child["bits"][0][h] > 0).sum()) <= n_new
    # three more tokens arrive; the output is the log-sum-exp merge of prefix, absorbed generation and new tail
    k3, v3 = rand_bf16(rng, (3, 1, Hkv, 128)), rand_bf16(rng, (3, 1, Hkv, 128))
    for i in range(3):
        O.append_tokens(cache, k3[i], v3[i])
    out, lse = O.decode(cache, q)
    out_c, lse_c = O.decode(alone, q)
    for j in range(Hkv * g):
        h = j // g
        o_t, l_t = _bruteforce_attention(q[0, j], k3[:, 0, h], v3[:, 0, h])
        ls = np.array([lse_p[0, j], lse_c[0, j], l_t])
        m = ls.max()
        w = np.exp(ls - m)
        want = (w[0] * out_p[0, j] + w[1] * out_c[0, j] + w[2] * np.asarray(o_t)) / w.sum()
        np.testing.assert_allclose(out[0, j], want, rtol=1e-11, atol=1e-12)
        assert abs(lse[0, j] - (m + np.log(w.sum()))) < 1e-11


def test_rebudget_of_a_mixed_cache_is_the_mixed_pass_on_the_tail():
    rng = np.random.default_rng(84)
    Hkv, g, T, n_new, S_w = 2, 2, 150, 96, 16
    q = rand_bf16(rng, (1, Hkv * g, 128))
    Qobs = [rand_bf16(rng, (Hkv * g, S_w, 128))]
    cache, kn, vn = _cache_with_tail(rng, Hkv, g, T, n_new, mixed=True)
    out_p, lse_p = O.decode({k: v for k, v in cache.items() if k != "tail"}, q)
    child = O.rebudget_tail(cache, Qobs, [np.float32(2.0)])
    # the same maps as the stages called one by one on the appended rows (Alg. 1, Sec. 3.2)
    K_tail = np.ascontiguousarray(kn[:, 0].transpose(1, 0, 2))
    V_tail = np.ascontiguousarray(vn[:, 0].transpose(1, 0, 2))
    w_tok = O.avg_pool(O.token_weights(K_tail, Qobs[0]), 5).astype(np.float32)
    w_ch = O.channel_weights(K_tail, Qobs[0]).astype(np.float32)
    for h in range(Hkv):
        bt, bc = O.allocate_mixed(w_tok[h], w_ch[h], np.float32(2.0))
        assert np.array_equal(child["bits"][0][h], bt) and np.array_equal(child["bits_ch"][h], bc)
        n_kept = int((bt > 0).sum())
        assert 0 < n_kept < n_new and 0 < int((bc > 0).sum())
    alone = O.build_cache_mixed([K_tail], [V_tail], child["bits"], [child["bits_ch"].reshape(Hkv, 128)])
    assert np.array_equal(child["arena"], alone["arena"])
    out, lse = O.decode(cache, q)
    out_c, lse_c = O.decode(alone, q)
    for j in range(Hkv * g):
        ls = np.array([lse_p[0, j], lse_c[0, j]])
        m = ls.max()
        w = np.exp(ls - m)
        np.testing.assert_allclose(out[0, j], (w[0] * out_p[0, j] + w[1] * out_c[0, j]) / w.sum(), rtol=1e-11, atol=1e-12)
        assert abs(lse[0, j] - (m + np.log(w.sum()))) < 1e-11


# ---- one scale per token row (the per-token format of App. B; Table 9's "per-token" errors) ------------------------
def test_row_wide_scale_obeys_the_half_step_bound_over_the_whole_row():
    rng = np.random.default_rng(101)
    X = rand_bf16(rng, (200, 128))
    X[:, 5] *= np.float32(8.0)                                   # one outlier channel stretches every row's range
    for b in (2, 4, 8):
        c, s, m = O.quantize_rows(X, b, group=128)
        assert c.shape == (200, 128) and s.shape == m.shape == (200, 4)
        assert np.array_equal(s, np.repeat(s[:, :1], 4, axis=1)) and np.array_equal(m, np.repeat(m[:, :1], 4, axis=1))
        Q = (1 << b) - 1
        assert c.max() <= Q
        # the scale is the row's range over Q, the offset its minimum (both rounded to fp16)
        rng_row = X.max(axis=1) - X.min(axis=1)
        np.testing.assert_array_equal(s[:, 0], (rng_row / np.float32(Q)).astype(np.float32).astype(np.float16))
        np.testing.assert_array_equal(m[:, 0], X.min(axis=1).astype(np.float16))
        xh = O.dequantize_groups(c.reshape(200, 4, 32), s, m).reshape(200, 128)
        step = s[:, 0].astype(np.float64)[:, None]
        assert np.all(np.abs(xh - X.astype(np.float64)) <= step * (0.5 + 2.0 ** -10 + Q * 2.0 ** -11))
        # coarser than groups of 32: the error cannot be smaller on average
        c32, s32, m32 = O.quantize_rows(X, b, group=32)
        xh32 = O.dequantize_groups(c32.reshape(200, 4, 32), s32, m32).reshape(200, 128)
        assert ((xh - X) ** 2).sum() >= ((xh32 - X) ** 2).sum()


def test_row_wide_scale_equals_groups_of_32_when_the_groups_share_their_range():
    """If every group of 32 channels of a row has the row's minimum and maximum, the four group quantizers and the
    row quantizer are the same function: codes, scales, offsets and the packed cache must be identical."""
    rng = np.random.default_rng(102)
    n = 150
    X = rand_bf16(rng, (2, n, 128))
    V = rand_bf16(rng, (2, n, 128))
    for A in (X, V):
        lo, hi = A.min(axis=2, keepdims=True), A.max(axis=2, keepdims=True)
        for g in range(4):                                      # plant the row's extremes in every group
            A[:, :, 32 * g + 3] = lo[:, :, 0]
            A[:, :, 32 * g + 17] = hi[:, :, 0]
    bits = rng.choice(np.array([0, 2, 4, 8, 16], np.uint8), size=(2, n))
    a = O.build_cache_tokenwise([X], [V], [bits], group=32)
    b = O.build_cache_tokenwise([X], [V], [bits], group=128)
    assert np.array_equal(a["arena"], b["arena"]) and np.array_equal(a["seg_off"], b["seg_off"])
    # on ordinary rows the two formats differ
    X2, V2 = rand_bf16(rng, (2, n, 128)), rand_bf16(rng, (2, n, 128))
    a = O.build_cache_tokenwise([X2], [V2], [bits], group=32)
    b = O.build_cache_tokenwise([X2], [V2], [bits], group=128)
    assert a["arena"].shape == b["arena"].shape and not np.array_equal(a["arena"], b["arena"])


@pytest.mark.parametrize("mixed", [False, True])
def test_decode_of_a_row_wide_cache_is_attention_over_its_dequantized_rows(mixed):
    rng = np.random.default_rng(103)
    Hkv, g, T, d = 2, 2, 90, 128
    K, V = rand_bf16(rng, (Hkv, T, d)), rand_bf16(rng, (Hkv, T, d))
    q = rand_bf16(rng, (1, Hkv * g, d))
    bt = rng.choice(np.array([0, 2, 4, 8, 16], np.uint8), size=(Hkv, T))
    if mixed:
        bc = rng.choice(np.array([0, 2, 4, 8, 16], np.uint8), size=(Hkv, d), p=[.1, .3, .3, .2, .1])
        cache = O.build_cache_mixed([K], [V], [bt], [bc], k_per_channel_scale=True, group=128)   # the paper's own format
    else:
        cache = O.build_cache_tokenwise([K], [V], [bt], group=128)
    out, lse = O.decode(cache, q)
    for h in range(Hkv):
        Kh, Vh = [], []
        kept = np.concatenate([np.nonzero(bt[h] == b)[0] for b in (16, 8, 4, 2)])
        for b in (16, 8, 4, 2):
            idx = np.nonzero(bt[h] == b)[0]
            for X, dst, is_k in ((K[h][idx], Kh, True), (V[h][idx], Vh, False)):
                if mixed and is_k:
                    continue
                if b == 16:
                    dst.append(X.astype(np.float64))
                else:                                            # one scale per row, written out by hand
                    Q = np.float32((1 << b) - 1)
                    mn = X.min(axis=1, keepdims=True) + np.float32(0)
                    sc = ((X.max(axis=1, keepdims=True) - mn) / Q).astype(np.float32).astype(np.float16).astype(np.float32)
                    m16 = mn.astype(np.float16).astype(np.float32)
                    with np.errstate(divide="ignore", invalid="ignore"):
                        code = np.clip(np.rint(((X - m16).astype(np.float32) / sc).astype(np.float32)), 0, Q)
                    code = np.where(sc == 0, 0, code)
                    dst.append(sc.astype(np.float64) * code + m16.astype(np.float64))
        if mixed:
            codes, sc, of = O.quantize_channelwise(K[h][kept], bc[h], None)
            Kh = [O.dequantize_channelwise(codes, sc, of, bc[h], None)]
        Kh, Vh = np.concatenate(Kh), np.concatenate(Vh)
        for j in range(g):
            o, l = _bruteforce_attention(q[0, h * g + j], Kh, Vh)
            np.testing.assert_allclose(out[0, h * g + j], o, rtol=1e-11, atol=1e-12)
            assert abs(lse[0, h * g + j] - l) < 1e-10


def test_calibration_with_row_wide_groups_is_coarser_and_matches_a_hand_count():
    rng = np.random.default_rng(104)
    K, V = rand_bf16(rng, (1, 300, 128)), rand_bf16(rng, (1, 300, 128))
    ek32, ev32 = O.calibrate_eps([K], [V])
    ek, ev = O.calibrate_eps([K], [V], group=128)
    assert np.all(ev > ev32) and np.all(ek > ek32)              # a wider range, a coarser step
    # by hand for 2 bits: sum of squared errors over sum of squares
    c, s, m = O.quantize_rows(V[0], 2, group=128)
    xh = s[:, :1].astype(np.float64) * c + m[:, :1].astype(np.float64)
    assert abs(ev[0, 0] - ((xh - V[0]) ** 2).sum() / (V[0].astype(np.float64) ** 2).sum()) < 1e-15
    # Gaussian rows: the range of 128 samples is about 5.3 sigma against 4.1 sigma for 32, (5.3 / 4.1)^2 = 1.7
    assert 1.3 < ev[0, 1] / ev32[0, 1] < 2.2
