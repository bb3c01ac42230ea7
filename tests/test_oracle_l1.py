"""Pins for the oracle's L1-relaxation locator (remark after Thm 3): the linear program against
brute force over its vertices, a closed form, an optimality certificate from LP duality that uses
no solver, and the locator's decisions against Algorithm 1's exhaustive search."""
import itertools

import numpy as np
import pytest

from oracle import gpd_oracle as O


def _code(P, K):
    pts = O.chebyshev_points(P)
    return pts, O.parity_check(pts, K), O.vandermonde(pts, K)


def _brute_force_lad(z, V, cost):
    """min_c sum_i cost_i |z_i - (V c)_i| by enumeration: a least-absolute-deviations fit with K
    coefficients interpolates at least K points exactly (a vertex of the linear program), so the
    minimum is attained at the interpolant of some K-subset of the nodes."""
    n, K = V.shape
    best = (np.inf, None)
    for B in itertools.combinations(range(n), K):
        c = np.linalg.solve(V[list(B)], z[list(B)])
        e = z - V @ c
        e[list(B)] = 0.0
        f = float(np.sum(cost * np.abs(e)))
        if f < best[0]:
            best = (f, e)
    return best


@pytest.mark.parametrize("P,K", [(6, 2), (7, 3), (8, 4), (8, 2)])
def test_l1_minimiser_equals_brute_force_over_vertices(P, K):
    rng = np.random.default_rng(P * 100 + K)
    for trial in range(6):
        # Chebyshev points, and points in general position: symmetric point sets give linear
        # programs with several optimal vertices (like the median of an even number of values),
        # where only the optimal value is unique
        generic = trial % 3 != 2
        pts = np.sort(rng.uniform(-1, 1, P)) if generic else O.chebyshev_points(P)
        H, V = O.parity_check(pts, K), O.vandermonde(pts, K)
        z = rng.standard_normal(P)
        # the locator's costs (1 up to a tie-breaking 1e-6) where the points are symmetric, else ones
        cost = np.ones(P) if generic else O.l1_costs(P)
        if trial >= 3:
            cost[rng.choice(P, 1)] = 0.0                   # a known-bad entry costs nothing
        e = O.l1_minimiser(H, H @ z, cost)
        f_ref, e_ref = _brute_force_lad(z, V, cost)
        assert np.abs(H @ e - H @ z).max() < 1e-10         # feasible: e differs from z by a codeword
        assert abs(np.sum(cost * np.abs(e)) - f_ref) < 1e-9 * max(1.0, f_ref)
        # (the optimum is unique for generic data, and on Chebyshev points with the tie-breaking costs)
        assert np.abs(e - e_ref).max() < 1e-8


def test_l1_minimiser_one_parity_row_closed_form():
    # r = 1: min ||e||_1 subject to h^T e = y puts everything on the entry where |h| is largest
    P, K = 7, 6
    pts, H, V = _code(P, K)
    assert H.shape == (1, P)
    h = H[0]
    rng = np.random.default_rng(3)
    z = rng.standard_normal(P)
    y = H @ z
    e = O.l1_minimiser(H, y)
    i = int(np.argmax(np.abs(h)))
    want = np.zeros(P)
    want[i] = y[0] / h[i]
    assert np.abs(e - want).max() < 1e-10


@pytest.mark.parametrize("P,K,t", [(16, 9, 1), (16, 9, 3), (24, 9, 5), (32, 12, 4), (48, 9, 8)])
def test_l1_minimiser_carries_a_dual_certificate(P, K, t):
    """LP duality without a solver: e* is optimal iff there is a lambda with |H^T lambda| <= 1
    everywhere and (H^T lambda)_i = sign(e*_i) on the support; then y^T lambda = ||e*||_1.  The
    support of a vertex has r = P - K entries (generic data), so lambda solves an r x r system."""
    pts, H, V = _code(P, K)
    r = P - K
    rng = np.random.default_rng(P + 7 * t)
    for trial in range(4):
        z = (V @ rng.standard_normal(K)).astype(np.float32).astype(np.float64)
        A = rng.choice(P, t, replace=False)
        z[A] += rng.standard_normal(t) * 2.0
        y = H @ z
        e = O.l1_minimiser(H, y)
        assert np.abs(H @ e - y).max() < 1e-9
        order = np.argsort(-np.abs(e))
        B = np.sort(order[:r])
        assert np.abs(e[order[r:]]).max() <= 1e-9 * np.abs(e).max()
        lam = np.linalg.solve(H[:, B].T, np.sign(e[B]))
        assert np.abs(H.T @ lam).max() <= 1.0 + 1e-7
        assert abs(y @ lam - np.abs(e).sum()) <= 1e-8 * np.abs(e).sum()
        # the planted error vector is feasible too, so it cannot have a smaller L1 norm
        e_true = z - V @ np.linalg.lstsq(np.delete(V, A, axis=0), np.delete(z, A), rcond=None)[0]
        assert np.abs(e).sum() <= np.abs(e_true).sum() * (1 + 1e-9)


def test_l1_locate_against_the_exhaustive_search():
    """Whatever the relaxation returns passes Algorithm 1's criterion; where it returns a support
    of the planted size it is the planted support with the search's error values; it recovers
    fewer errors than the search (which finds all of these), most single errors.  A wrong ranking
    can make it return a larger support that also explains the syndrome within tau (seen once in
    this sweep: five nodes for three planted errors, one of them missed): rare, and counted."""
    P, K = 16, 9
    pts, H, V = _code(P, K)
    rng = np.random.default_rng(11)
    found = {t: 0 for t in range(1, 5)}
    other = 0
    N = 30
    for t in found:
        for trial in range(N):
            z = (V @ rng.standard_normal(K)).astype(np.float32).astype(np.float64)
            A = tuple(sorted(int(a) for a in rng.choice(P, t, replace=False)))
            z[list(A)] += rng.uniform(1.0, 3.0, t) * rng.choice([-1.0, 1.0], t)
            tau = 2.0 ** -12 * np.linalg.norm(z)
            st, supp, e = O.l1_locate(z, H, tau)
            st1, supp1, e1 = O.algorithm1(z, H, tau)
            assert st1 == "located" and supp1 == A
            if st == "located":
                res, _ = O.support_residual(H, H @ z, supp)
                assert res <= tau and len(supp) <= P - K - 1
                if len(supp) == t:
                    assert supp == A and np.abs(e - e1).max() <= 1e-9 * np.abs(e1).max()
                    found[t] += 1
                else:
                    assert len(supp) > t
                    other += 1
            else:
                assert st == "failed"
    assert found[1] >= 0.8 * N and found[2] >= 0.6 * N
    assert found[4] < found[1]                             # the relaxation is the weaker decoder
    assert other <= 0.05 * 4 * N


def test_l1_locate_clean_word_and_forced_entries():
    P, K = 16, 9
    pts, H, V = _code(P, K)
    rng = np.random.default_rng(5)
    z = V @ rng.standard_normal(K)
    tau = 1e-9 * np.linalg.norm(z)
    assert O.l1_locate(z, H, tau) == ("clean", (), pytest.approx(np.zeros(0)))
    # a known-bad entry (zeroed by the caller) alone: the forced support explains the syndrome
    zf = z.copy()
    zf[4] = 0.0
    st, supp, e = O.l1_locate(zf, H, tau, forced=(4,))
    assert st == "located" and supp == (4,) and abs(e[0] + z[4]) < 1e-8 * abs(z).max()
    # a known-bad entry plus one unknown error
    zf[11] += 2.5
    st, supp, e = O.l1_locate(zf, H, tau, forced=(4,))
    assert st == "located" and supp == (4, 11) and abs(e[1] - 2.5) < 1e-8


def test_decode_with_the_l1_locator_corrects_what_it_locates():
    plan = O.make_plan(2, 2, 2, 16)
    rng = np.random.default_rng(2)
    A = rng.uniform(-1, 1, (8, 8))
    B = rng.uniform(-1, 1, (8, 8))
    Ct = O.worker_products(O.encode_A(A, plan), O.encode_B(B, plan))
    Ct[3, 1, 2] += 5.0
    Ct[12, 3, 0] = np.inf
    C, rep = O.decode(Ct, plan, mode="lsq_all", correct=True, rho=1e-9, locator="l1")
    assert rep.n_failed == 0 and [(n, r, c) for n, r, c, _ in rep.located] == [(3, 1, 2), (12, 3, 0)]
    assert np.abs(C - A @ B).max() < 1e-8


def test_tie_breaking_costs_leave_one_optimum_on_chebyshev_points():
    """On the (12, 9) Chebyshev code about every third word with one or two errors has several
    optimal vertices under equal costs (equal objective, different e); with the locator's costs the
    brute-force minimum over all vertices is attained once, and it is the solver's answer."""
    P, K = 12, 9
    pts, H, V = _code(P, K)
    cost = O.l1_costs(P)
    assert np.all(cost >= 1.0) and np.all(cost < 1.0 + 1e-6) and len(set(cost.tolist())) == P
    rng = np.random.default_rng(1)
    ties = 0
    for trial in range(12):
        z = (V @ rng.standard_normal(K)).astype(np.float32).astype(np.float64)
        A = rng.choice(P, 1 + trial % 2, replace=False)
        z[A] += rng.uniform(1, 3, len(A)) * rng.choice([-1.0, 1.0], len(A))
        vals = []
        import itertools as it_
        for B in it_.combinations(range(P), K):
            e = z - V @ np.linalg.solve(V[list(B)], z[list(B)])
            e[list(B)] = 0.0
            vals.append((float(np.sum(cost * np.abs(e))), float(np.sum(np.abs(e))), e))
        vals.sort(key=lambda v: v[0])
        best = vals[0]
        # no other vertex within 1e-9 of the weighted optimum unless it is the same point up to entries
        # at the level of the responses' rounding (1e-7 of the largest)
        for v in vals[1:6]:
            assert v[0] - best[0] > 1e-9 * best[0] or np.abs(v[2] - best[2]).max() < 1e-7 * np.abs(best[2]).max()
        plain = sorted(vals, key=lambda v: v[1])
        ties += any(abs(v[1] - plain[0][1]) < 1e-12 and np.abs(v[2] - plain[0][2]).max() > 1e-6 for v in plain[1:4])
        e_lp = O.l1_minimiser(H, H @ z, cost)
        assert np.abs(e_lp - best[2]).max() < 1e-7 * np.abs(best[2]).max()
    assert ties >= 2                                        # (equal costs: the ties are really there)
