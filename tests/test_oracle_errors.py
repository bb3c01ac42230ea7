"""Pins for the oracle's real-number error correction (Sec. V, Thm 3 and Algorithm 1):
detection always, correction up to P-K-1 errors under the probabilistic model, failure
declared beyond, unique decoding up to floor((P-K)/2), and the replication special case."""
import itertools

import numpy as np
import pytest

import gpd_workloads as WL
from oracle import gpd_oracle as O


def coded_outputs(N1, N0, Nc, m, n, d, P, seed, round_outputs="f32"):
    A, B = WL.matmul_inputs(N1, N0, Nc, seed)
    pl = O.make_plan(m, n, d, P)
    Ct = O.worker_products(O.encode_A(A, pl), O.encode_B(B, pl), round_outputs=round_outputs)
    return A, B, pl, Ct


def test_no_errors_means_no_flags():
    A, B, pl, Ct = coded_outputs(8, 8, 8, 2, 2, 2, 14, 0)
    C, rep = O.decode(Ct, pl, correct=True)
    assert rep.status == "ok" and rep.n_flagged == 0 and not rep.located
    assert rep.max_syndrome_ratio < 1.0 / 16          # fp32 rounding noise is far below tau
    assert np.abs(C - O.uncoded_matmul(A, B)).max() < 1e-3


@pytest.mark.parametrize("t", [1, 2, 3, 4])
def test_whole_node_gaussian_errors_are_located_and_corrected(t):
    # Thm 3 item 2 with (P, Q) = (14, 9): up to P-Q-1 = 4 erroneous nodes, every element corrupted
    A, B, pl, Ct = coded_outputs(4, 8, 4, 2, 2, 2, 14, 1)
    bad, noise = WL.gaussian_node_errors(40 + t, pl.P, t, Ct.shape[1:])
    Cbad = Ct.copy()
    Cbad[bad] += noise
    C, rep = O.decode(Cbad, pl, correct=True)
    n_cw = Ct.shape[1] * Ct.shape[2]
    assert rep.status == "ok" and rep.n_flagged == n_cw and rep.n_failed == 0
    want = sorted((int(p), r, c) for p in bad for r in range(Ct.shape[1]) for c in range(Ct.shape[2]))
    assert [x[:3] for x in rep.located] == want
    assert rep.node_err_count.tolist() == [n_cw if p in bad else 0 for p in range(pl.P)]
    # estimated error values equal the injected noise
    got = np.array([x[3] for x in rep.located]).reshape(t, -1)
    assert np.abs(got - noise.reshape(t, -1)).max() < 1e-2
    assert np.abs(C - O.uncoded_matmul(A, B)).max() < 2e-2
    # ... and equal the erasure decode from the good nodes only (definition of correction)
    present = np.ones(pl.P, dtype=np.uint8)
    present[bad] = 0
    C_er, _ = O.decode(Ct, pl, present, "lsq_all")
    assert np.abs(C - C_er).max() < 1e-9


def test_too_many_errors_declare_failure():
    # Thm 3 item 3: P-Q errors (or more) are detected but not correctable
    # The statement is for exact reals: with a tolerance tau, one of the C(P, P-K-1) candidate
    # supports passes by chance with probability of order C(P, P-K-1) * tau / ||Hz||, so this pin
    # uses unrounded fp64 products and a tolerance near fp64 rounding.
    A, B, pl, Ct = coded_outputs(4, 8, 4, 2, 2, 2, 14, 2, round_outputs=None)
    for t in (5, 6):
        bad, noise = WL.gaussian_node_errors(70 + t, pl.P, t, Ct.shape[1:])
        Cbad = Ct.copy()
        Cbad[bad] += noise
        C, rep = O.decode(Cbad, pl, correct=True, rho=1e-11)
        assert rep.status == "decode_fail"
        assert rep.n_failed == rep.n_flagged == Ct.shape[1] * Ct.shape[2]
        assert not rep.located


def test_detection_with_no_correction_capacity():
    # P = K + 1: one parity row: errors are detected (Thm 3 item 1) but P-K-1 = 0 can be corrected
    A, B, pl, Ct = coded_outputs(4, 4, 4, 2, 2, 2, 10, 3)
    C, rep = O.decode(Ct, pl, correct=True)
    assert rep.status == "ok" and rep.n_flagged == 0
    Cbad = Ct.copy()
    Cbad[4, 1, 1] += 0.5
    C, rep = O.decode(Cbad, pl, correct=True)
    assert rep.status == "decode_fail" and rep.failed == [(1, 1)] and rep.n_flagged == 1


def test_replication_special_case_two_equal_values_win():
    # Sec. V: replication is a (P,1) code; P-2 errors are corrected as long as two values agree
    P = 6
    z = np.full((P, 1, 1), 3.25)
    z[[0, 1, 3, 5], 0, 0] = [7.0, -2.0, 100.0, 3.3]           # 4 = P-2 errors, nodes 2 and 4 agree
    coeffs, rep = O.decode_coefficients(z, O.chebyshev_points(P), 1, [0], correct=True)
    assert rep.status == "ok" and [x[0] for x in rep.located] == [0, 1, 3, 5]
    assert abs(coeffs[0][0, 0] - 3.25) < 1e-12
    z[2, 0, 0] = 9.0                                           # no two agree any more
    coeffs, rep = O.decode_coefficients(z, O.chebyshev_points(P), 1, [0], correct=True)
    assert rep.status == "decode_fail"


def test_adversarial_radius_gives_unique_solutions():
    # Lemma (adversarial model): with |A| <= floor((P-Q)/2) the sparsest solution of He = Hz is unique.
    # Brute force: for a fixed error pattern of size 2 (P-Q = 5), no other support of size <= 2 fits.
    P, K = 12, 7
    b = O.chebyshev_points(P)
    H = O.parity_check(b, K)
    rng = np.random.default_rng(5)
    e = np.zeros(P)
    e[[3, 8]] = rng.standard_normal(2)
    y = H @ e
    fits = [s for s in itertools.combinations(range(P), 2) if O.support_residual(H, y, s)[0] < 1e-9]
    assert fits == [(3, 8)]
    status, supp, e_hat = O.algorithm1(e + O.vandermonde(b, K) @ rng.standard_normal(K), H, 1e-9)
    assert status == "located" and supp == (3, 8) and np.allclose(e_hat, e[[3, 8]], atol=1e-8)


def test_algorithm1_prefers_the_smallest_support():
    P, K = 10, 5
    b = O.chebyshev_points(P)
    H = O.parity_check(b, K)
    e = np.zeros(P)
    e[6] = 2.0
    status, supp, e_hat = O.algorithm1(e, H, 1e-9)
    assert (status, supp) == ("located", (6,)) and abs(e_hat[0] - 2.0) < 1e-9
    assert O.algorithm1(np.zeros(P), H, 0.0)[0] == "clean"


def test_erasures_and_errors_together():
    # MDS: after dropping erased nodes the code is (|S|, K) and corrects |S|-K-1 errors
    A, B, pl, Ct = coded_outputs(4, 8, 4, 2, 2, 2, 16, 4)
    present = np.ones(16, dtype=np.uint8)
    present[[2, 9, 15]] = 0                                    # |S| = 13, capacity 13-9-1 = 3
    Cbad = Ct.copy()
    Cbad[5] += 1.0
    Cbad[11, 0, 1] -= 3.0
    Cbad[2] = 1e9                                              # erased node's garbage must not matter
    C, rep = O.decode(Cbad, pl, present, correct=True)
    assert rep.status == "ok" and rep.n_present == 13
    assert set(x[0] for x in rep.located) == {5, 11}
    assert rep.node_err_count[5] == 4 and rep.node_err_count[11] == 1
    assert np.abs(C - O.uncoded_matmul(A, B)).max() < 1e-2


def test_bit_flips_decisions_follow_the_injected_magnitude():
    # One flipped bit in one fp32 element of one node: located iff its effect on the syndrome
    # is above tau, invisible (and harmless) if far below; non-finite results are always located.
    A, B, pl, Ct = coded_outputs(16, 32, 16, 2, 2, 2, 16, 6)
    C_ref = O.uncoded_matmul(A, B)
    H = O.parity_check(pl.points, pl.K)
    rho = 2.0 ** -12
    cols = Ct.shape[2]
    n_loc = n_clean = n_nonfinite = 0
    for bit in range(32):
        node, elem = (bit * 5) % 16, (bit * 7) % (Ct.shape[1] * cols)
        flipped = WL.apply_bitflips(Ct.astype(np.float32), [(node, elem, bit)]).astype(np.float64)
        r, c = divmod(elem, cols)
        dv = flipped[node, r, c] - Ct[node, r, c]
        C, rep = O.decode(flipped, pl, correct=True, rho=rho)
        z = np.where(np.isfinite(flipped[:, r, c]), flipped[:, r, c], 0.0)
        tau = rho * np.linalg.norm(z)
        if not np.isfinite(dv):
            n_nonfinite += 1
            assert [x[:3] for x in rep.located] == [(node, r, c)] and np.isnan(rep.located[0][3])
        else:
            effect = abs(dv) * np.linalg.norm(H[:, node])
            if effect > 8 * tau:
                n_loc += 1
                assert [x[:3] for x in rep.located] == [(node, r, c)], (bit, effect, tau)
                assert abs(rep.located[0][3] - dv) <= 1e-3 * abs(dv) + 1e-4
            elif effect < tau / 8:
                n_clean += 1
                assert rep.n_flagged == 0
        assert rep.status == "ok"
        # a flip that stays below tau is not corrected; it can move the result by at most its own
        # size times the amplification of the all-node least-squares decoder
        slack = 0.0 if rep.located else abs(dv) * O.amplification(pl, mode="lsq_all")
        assert np.linalg.norm(C - C_ref) <= 1e-4 * np.linalg.norm(C_ref) + slack
    assert n_loc >= 8 and n_clean >= 8 and n_nonfinite >= 0


def test_non_finite_responses_are_forced_locations():
    A, B, pl, Ct = coded_outputs(4, 8, 4, 2, 2, 2, 14, 7)
    Cbad = Ct.copy()
    Cbad[3, 0, 0] = np.inf
    Cbad[7, 0, 0] = np.nan
    Cbad[9, 1, 1] = -np.inf
    C, rep = O.decode(Cbad, pl, correct=True)
    assert rep.status == "ok"
    assert [x[:3] for x in rep.located] == [(3, 0, 0), (7, 0, 0), (9, 1, 1)]
    assert np.all(np.isfinite(C)) and np.abs(C - O.uncoded_matmul(A, B)).max() < 1e-2
