"""Pins for the oracle's code construction: values printed in the paper, closed
forms of Thm 1/2 and Tables I/III, and the two special cases (Polynomial / MatDot)."""
import itertools
import os

import numpy as np
import pytest

from oracle import gpd_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def load_gold():
    vals = {}
    for line in open(GOLD):
        line = line.split("#")[0].strip()
        if not line:
            continue
        k, v = [t.strip() for t in line.split("=")]
        nums = [int(t) for t in v.split()]
        vals[k] = nums if len(nums) > 1 else nums[0]
    return vals


G = load_gold()


def test_worked_example_2x2x2():
    # Sec. III: substitution u=v^2, w=v^4 gives degree 8, threshold 9, S_ik at v^(2i+4k+1)
    pl = O.make_plan(2, 2, 2, 10)
    assert pl.K == G["gpd_threshold_m2n2d2"]
    assert pl.K - 1 == G["gpd_degree_m2n2d2"]
    assert sorted(pl.eC.ravel().tolist()) == G["gpd_useful_exponents_m2n2d2"]
    tab = O.product_exponent_table(pl)
    assert len(set(tab.values())) == G["gpd_threshold_m2n2d2"]
    # the bijective substitution would keep u^i v^(1+j-j') w^k distinct: 2*3*2 unknowns
    distinct_multivariate = {(i, 1 + j - jp, k) for (i, j, jp, k) in tab}
    assert len(distinct_multivariate) == G["polydot_bijective_unknowns_2x2"]
    # garbage alignment named in the text: u v^2 (i=1, j-j'=1, k=0) and w (i=0, j-j'=-1, k=1)
    assert tab[(1, 1, 0, 0)] == tab[(0, 0, 1, 1)] == G["gpd_aligned_exponent_m2n2d2"]


def test_worked_example_matvec_2x2():
    pl = O.make_plan(2, 2, 1, 6)
    assert pl.K == G["gpd_matvec_threshold_m2n2"]
    assert pl.K - 1 == G["gpd_matvec_degree_formula_m2n2"]
    assert sorted(pl.eC.ravel().tolist()) == G["gpd_matvec_useful_exponents_m2n2"]
    # Eq. for s~(u,v) with m=n=2: s_0 at v, s_1 at u v; garbage u and v^2 align under u=v^2
    assert pl.eA[1, 0] + pl.eB[1, 0] == pl.eA[0, 1] + pl.eB[0, 0] == 2


@pytest.mark.parametrize("m,n,d", [(1, 1, 1), (2, 2, 2), (4, 2, 1), (2, 4, 1), (3, 2, 2), (2, 3, 4), (6, 6, 6)])
def test_threshold_closed_forms(m, n, d):
    # Thm 2: mnd + n - 1 under u=v^n;  error-tolerance appendix: mnd + mn - m under v=u^m
    assert O.make_plan(m, n, d, 1000).K == m * n * d + n - 1
    assert O.make_plan(m, n, d, 1000, "v=u^m").K == m * n * d + m * n - m


@pytest.mark.parametrize("subst", ["u=v^n", "v=u^m"])
@pytest.mark.parametrize("m,n,d", [(2, 2, 2), (4, 2, 1), (2, 4, 1), (3, 2, 2), (2, 3, 3), (1, 4, 1), (4, 1, 4)])
def test_useful_exponents_only_hit_by_matching_terms(m, n, d, subst):
    # proof of Thm 2: the coefficient of the useful exponent is exactly sum_j W_ij X_jk
    pl = O.make_plan(m, n, d, 1000, subst)
    tab = O.product_exponent_table(pl)
    assert len(set(pl.eC.ravel().tolist())) == m * d
    for i in range(m):
        for k in range(d):
            hits = sorted(key for key, e in tab.items() if e == pl.eC[i, k])
            assert hits == [(i, j, j, k) for j in range(n)]
    assert max(tab.values()) == pl.K - 1


def test_special_case_polynomial_codes():
    # Sec. III/IV: n=1, m=K, d=K' is the Polynomial code: exponents i and jK, threshold K K'
    K = 4
    pl = O.make_plan(K, 1, K, 100)
    assert pl.K == G["polynomial_code_threshold_K4"]
    assert pl.eA[:, 0].tolist() == [0, 1, 2, 3]
    assert pl.eB[0].tolist() == [0, 4, 8, 12]
    assert sorted(pl.eC.ravel().tolist()) == list(range(16))
    assert O.make_plan(36, 1, 36, 2000).K == G["polynomial_code_threshold_K36"]


def test_special_case_matdot():
    # Sec. III/IV: m=d=1, n=K is MatDot: W exponents j, X exponents K-1-j, answer at v^(K-1)
    K = 4
    pl = O.make_plan(1, K, 1, 100)
    assert pl.K == G["matdot_threshold_K4"]
    assert pl.eA[0].tolist() == [0, 1, 2, 3]
    assert pl.eB[:, 0].tolist() == [3, 2, 1, 0]
    assert pl.eC.ravel().tolist() == [G["matdot_useful_exponent_K4"]]
    assert O.make_plan(1, 36, 1, 100).K == G["matdot_threshold_K36"]


@pytest.mark.parametrize("m,n,d1,d2,P", [(4, 2, 1, 1, 24), (2, 4, 1, 1, 32), (3, 3, 2, 2, 60), (2, 2, 1, 2, 20)])
def test_dnn_error_tolerances_tables_I_and_III(m, n, d1, d2, P):
    # Table III (Table I is d1=d2=1), probabilistic model: t = P - (#coefficients) - 1
    lp = O.make_layer_plan(m * 8, n * 8, d1 * d2 * 2, m, n, d1, d2, P, "u=v^n")
    assert (P - lp.Kf - 1, P - lp.Kb - 1) == (P - d1 * m * n - n, P - (d2 + 1) * m * n + n - 1)
    lp = O.make_layer_plan(m * 8, n * 8, d1 * d2 * 2, m, n, d1, d2, P, "v=u^m")
    assert (P - lp.Kf - 1, P - lp.Kb - 1) == (P - (d1 + 1) * m * n + m - 1, P - d2 * m * n - m)


@pytest.mark.parametrize("subst", ["u=v^n", "v=u^m"])
@pytest.mark.parametrize("m,n,d2", [(4, 2, 1), (2, 4, 1), (3, 2, 2), (2, 3, 3)])
def test_backward_useful_exponents(m, n, d2, subst):
    # Sec. IX backprop: C^T_{k,j} is the coefficient of w^k u^(m-1) v^j: only i == i' terms
    lp = O.make_layer_plan(m * 2, n * 2, d2 * 2, m, n, 1, d2, 200, subst)
    tab = {}
    for k in range(d2):
        for ip in range(m):
            for i in range(m):
                for j in range(n):
                    tab[(k, ip, i, j)] = int(lp.eD[k, ip] + lp.fwd.eA[i, j])
    for k in range(d2):
        for j in range(n):
            hits = sorted(key for key, e in tab.items() if e == lp.eCb[k, j])
            assert hits == [(k, i, i, j) for i in range(m)]
    assert max(tab.values()) == lp.Kb - 1
    if subst == "u=v^n":
        # appendix: none of the n(2m-1) coefficients align under u=v^n (d2 = 1)
        if d2 == 1:
            assert len(set(tab.values())) == n * (2 * m - 1) == lp.Kb
    # weight polynomial: exponents are a bijection onto 0..mn-1 (regeneration footnote: degree mn-1)
    assert sorted(lp.fwd.eA.ravel().tolist()) == list(range(m * n))


def test_chebyshev_points():
    P = 16
    b = O.chebyshev_points(P)
    assert len(np.unique(b)) == P and np.all(np.abs(b) < 1)
    # roots of T_P: cos(P arccos b) = 0
    assert np.allclose(np.cos(P * np.arccos(b)), 0, atol=1e-12)
    assert np.allclose(b, -b[::-1])


def test_plan_rejects_bad_input():
    with pytest.raises(ValueError):
        O.make_plan(2, 2, 2, 8)            # K = 9 > P
    with pytest.raises(ValueError):
        O.make_plan(2, 2, 2, 10, points=[0.1] * 10)
    with pytest.raises(ValueError):
        O.make_plan(0, 2, 2, 10)


def test_parity_check_matches_closed_form_dual():
    # textbook dual of a Vandermonde (generalised Reed-Solomon) code:
    # H'[r,p] = b_p^r / prod_{q != p} (b_p - b_q), r = 0..P-K-1, annihilates all monomials of degree < K
    P, K = 12, 7
    b = O.chebyshev_points(P)
    H = O.parity_check(b, K)
    assert H.shape == (P - K, P)
    assert np.allclose(H @ H.T, np.eye(P - K), atol=1e-12)
    V = O.vandermonde(b, K)
    assert np.abs(H @ V).max() < 1e-12
    w = np.array([1.0 / np.prod([b[p] - b[q] for q in range(P) if q != p]) for p in range(P)])
    Hd = np.array([b ** r * w for r in range(P - K)])
    assert np.abs(Hd @ V).max() < 1e-9 * np.abs(Hd).max()
    # same row space: projecting Hd's rows onto span(H) loses nothing
    resid = Hd - (Hd @ H.T) @ H
    assert np.abs(resid).max() < 1e-9 * np.abs(Hd).max()
    # MDS property of the dual: every (P-K) columns of H are independent
    for cols in itertools.combinations(range(P), P - K):
        assert abs(np.linalg.det(H[:, cols])) > 1e-12


def test_vandermonde_layout():
    V = O.vandermonde(np.array([2.0, 3.0]), 4)
    assert V.tolist() == [[1, 2, 4, 8], [1, 3, 9, 27]]
    assert O.int_power(np.array(3.0), 5) == 243.0
