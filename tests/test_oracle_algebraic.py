"""Pins of the oracle's algebraic (locator-polynomial) error locator: the polynomial-time decoder
inside the adversarial radius floor((P-Q)/2) of Sec. V.  Checked against what the mathematics
fixes (annihilation of codewords, the closed form for one error, uniqueness of the explaining
support) and against the exhaustive search of Algorithm 1 where that is feasible."""
import itertools

import numpy as np
import pytest

from oracle import gpd_oracle as O


def codeword(pts, K, rng):
    return O.vandermonde(pts, K) @ rng.uniform(-1, 1, K)


def plant(z, t, rng, scale=None):
    A = np.sort(rng.choice(len(z), t, replace=False))
    s = 10.0 ** rng.uniform(-1, 1) if scale is None else scale
    e = rng.choice([-1.0, 1.0], t) * rng.uniform(0.5, 2.0, t) * s
    z2 = z.copy()
    z2[A] += e
    return z2, tuple(int(a) for a in A), e


@pytest.mark.parametrize("P,K,pts_kind", [(16, 9, "cheb"), (24, 9, "cheb"), (20, 7, "random"), (12, 5, "shifted")])
def test_dual_syndromes_annihilate_codewords(P, K, pts_kind):
    rng = np.random.default_rng(P + K)
    pts = {"cheb": O.chebyshev_points(P), "random": np.sort(rng.uniform(-1, 1, P)),
           "shifted": np.linspace(2.0, 5.0, P)}[pts_kind]
    r = P - K
    for _ in range(5):
        z = codeword(pts, K, rng)
        S = O.dual_syndromes(z, pts, r)
        assert np.abs(S).max() <= 1e-10 * np.linalg.norm(z)
    # and not one syndrome more: a polynomial with K + 1 coefficients is seen by the last one
    z = O.vandermonde(pts, K + 1)[:, K]
    S = O.dual_syndromes(z, pts, r)
    assert abs(S[r - 1]) > 1e-6 * np.abs(z).max() / 2.0 ** P and np.abs(S[:r - 1]).max() <= 1e-9 * abs(S[r - 1]) + 1e-13


def test_one_error_closed_form():
    # S_j = a T_j(x_i): the locator is T_1(x) - x_i, the error value is recovered exactly
    P, K = 16, 9
    rng = np.random.default_rng(1)
    pts = O.chebyshev_points(P)
    H = O.parity_check(pts, K)
    z = codeword(pts, K, rng)
    for i in (0, 5, 15):
        z2 = z.copy()
        z2[i] += 0.75
        S = O.dual_syndromes(z2, pts, P - K)
        x = (2 * pts - (pts.min() + pts.max())) / (pts.max() - pts.min())
        ratio = S[1] / S[0]
        assert abs(ratio - x[i]) < 1e-9                       # T_1(x_i) / T_0(x_i)
        st, supp, e = O.algebraic_locate(z2, H, pts, 2.0 ** -12 * np.linalg.norm(z2))
        assert st == "located" and supp == (i,) and abs(e[0] - 0.75) < 1e-9


@pytest.mark.parametrize("P,K", [(16, 9), (14, 6), (24, 9)])
def test_agrees_with_exhaustive_search_inside_radius(P, K):
    rng = np.random.default_rng(100 + P)
    pts = O.chebyshev_points(P)
    H = O.parity_check(pts, K)
    r = P - K
    for t in range(0, min(r // 2, 4) + 1):
        for _ in range(6):
            z = O.round_to_f32(codeword(pts, K, rng))
            z2, A, e = plant(z, t, rng) if t else (z, (), np.zeros(0))
            z2 = O.round_to_f32(z2)
            tau = 2.0 ** -12 * np.linalg.norm(z2)
            a = O.algebraic_locate(z2, H, pts, tau)
            b = O.algorithm1(z2, H, tau)
            assert a[0] == b[0] and a[1] == b[1] == A
            assert np.allclose(a[2], b[2], rtol=1e-9, atol=1e-12)
            if t:
                assert np.allclose(a[2], z2[list(A)] - z[list(A)], atol=1e-5)


def test_never_accepts_a_wrong_support_beyond_the_radius():
    # t > floor(r / 2): the locator may fail, but what it accepts passes Algorithm 1's criterion,
    # and by Thm 3 the explaining support of at most r - 1 nodes is unique
    P, K = 16, 9
    rng = np.random.default_rng(7)
    pts = O.chebyshev_points(P)
    H = O.parity_check(pts, K)
    located = failed = 0
    for t in (4, 5, 6):
        for _ in range(15):
            z = codeword(pts, K, rng)
            z2, A, e = plant(z, t, rng)
            tau = 2.0 ** -12 * np.linalg.norm(z2)
            st, supp, eh = O.algebraic_locate(z2, H, pts, tau)
            if st == "located":
                located += 1
                assert supp == A
            else:
                failed += 1
                assert st == "failed"
    assert failed > 0                                          # the radius is real


def test_forced_nodes_are_erasures():
    P, K = 20, 8
    rng = np.random.default_rng(11)
    pts = O.chebyshev_points(P)
    H = O.parity_check(pts, K)
    for nforced, t in ((1, 0), (2, 3), (3, 4), (4, 4)):
        z = codeword(pts, K, rng)
        z2, A, e = plant(z, nforced + t, rng)
        forced = tuple(A[:nforced]) if nforced else ()
        zs = z2.copy()
        zs[list(forced)] = 0.0                                # sanitised like a non-finite response
        tau = 2.0 ** -12 * np.linalg.norm(zs)
        st, supp, eh = O.algebraic_locate(zs, H, pts, tau, forced)
        assert st == "located" and supp == A
        st1, supp1, eh1 = O.algorithm1(zs, H, tau, forced)
        assert supp1 == supp and np.allclose(eh, eh1, rtol=1e-8, atol=1e-10)


def test_large_code_where_the_search_is_out_of_reach():
    # P = 64, K = 40: C(64, 10) > 10^11 supports for the exhaustive search; the locator needs
    # a 14 x 10 least-squares problem
    P, K = 64, 40
    rng = np.random.default_rng(5)
    pts = O.chebyshev_points(P)
    H = O.parity_check(pts, K)
    ok = 0
    for _ in range(10):
        z = O.round_to_f32(codeword(pts, K, rng))
        z2, A, e = plant(z, 8, rng)
        z2 = O.round_to_f32(z2)
        st, supp, eh = O.algebraic_locate(z2, H, pts, 2.0 ** -12 * np.linalg.norm(z2))
        if st == "located":
            assert supp == A
            assert np.allclose(eh, z2[list(A)] - z[list(A)], atol=1e-4)
            ok += 1
    assert ok >= 8


def test_decode_with_algebraic_locator_matches_search():
    plan = O.make_plan(2, 2, 2, 16)
    rng = np.random.default_rng(3)
    A = rng.uniform(-1, 1, (32, 32))
    B = rng.uniform(-1, 1, (32, 32))
    Ct = O.round_to_f32(O.worker_products(O.encode_A(A, plan), O.encode_B(B, plan)))
    bad = Ct.copy()
    bad[3, 1, 2] += 50.0
    bad[9, 1, 2] -= 7.0
    bad[12, 1, 2] += 3.0
    bad[5, 10, 11] = np.inf
    bad[0, 4, 4] *= -3.0
    C1, r1 = O.decode(bad, plan, None, "lsq_all", True, locator="search")
    C2, r2 = O.decode(bad, plan, None, "lsq_all", True, locator="algebraic")
    assert r1.status == r2.status == "ok"
    assert [l[:3] for l in r1.located] == [l[:3] for l in r2.located]
    assert np.allclose(C1, C2, rtol=1e-10, atol=1e-12)
    assert np.abs(C2 - A @ B).max() < 1e-4


@pytest.mark.parametrize("P,K", [(16, 9), (24, 9), (32, 12), (48, 9)])
def test_guard_nodes_change_nothing_in_exact_arithmetic(P, K):
    # Inside the radius floor((P-Q)/2) (Sec. V, adversarial model) the locator polynomial vanishes
    # on the erroneous nodes and nowhere else, so the textbook form (the t nodes of smallest |L|,
    # guard_nodes = 0) and the form with two guard nodes must accept the same support, the planted
    # one, on exact fp64 words with a tiny threshold.
    rng = np.random.default_rng(3 * P + K)
    pts = O.chebyshev_points(P)
    H = O.parity_check(pts, K)
    r = P - K
    for t in range(1, min(r // 2, 8) + 1):
        for _ in range(4):
            z = codeword(pts, K, rng)
            z2, A, e = plant(z, t, rng, scale=1.0)
            tau = 1e-9 * np.linalg.norm(z2)
            plain = O.algebraic_locate(z2, H, pts, tau, guard_nodes=0)
            guarded = O.algebraic_locate(z2, H, pts, tau)
            assert plain[0] == guarded[0] == "located"
            assert plain[1] == guarded[1] == A
            assert np.allclose(plain[2], guarded[2], rtol=1e-9, atol=1e-12)
            assert np.allclose(guarded[2], e, atol=1e-6)


def test_the_case_that_needs_the_guard_nodes():
    # fp32-rounded responses of a (24, 9) code with 7 errors (the radius): the t nodes of smallest
    # |L| are not the erroneous ones (a neighbour on the Chebyshev grid comes out ahead), the textbook
    # form reports a failure; with two guard nodes the fitted error values single out the right 7.
    # Either way nothing wrong is ever accepted: acceptance is Algorithm 1's criterion.
    P, K = 24, 9
    rng = np.random.default_rng(0)
    pts = O.chebyshev_points(P)
    H = O.parity_check(pts, K)
    found = None
    for _ in range(2000):
        t = int(rng.integers(1, (P - K) // 2 + 1))
        z = O.round_to_f32(O.vandermonde(pts, K) @ rng.standard_normal(K))
        nodes = np.sort(rng.choice(P, t, replace=False))
        z2 = z.copy()
        z2[nodes] += rng.choice([-1, 1], t) * rng.uniform(0.5, 2, t) * np.abs(z).max()
        tau = 2.0 ** -12 * np.linalg.norm(z2)
        plain = O.algebraic_locate(z2, H, pts, tau, guard_nodes=0)
        guarded = O.algebraic_locate(z2, H, pts, tau)
        want = tuple(int(q) for q in nodes)
        for res in (plain, guarded):
            assert res[0] == "failed" or res[1] == want          # never a wrong support
        if guarded[0] == "located" and plain[0] == "failed" and found is None:
            found = (t, want)
    assert found is not None and found[0] >= 5
