"""Pins for the oracle's node-level fault handling: location of erroneous nodes once for a
whole stack (Sec. V Algorithm 1 applied to the whole-node error models of Sec. III),
regeneration of a node's coded weights from good nodes (Sec. VII) and the projection of a
coded stack back onto the code."""
import itertools

import numpy as np
import pytest

import gpd_workloads as WL
from oracle import gpd_oracle as O


def coded_outputs(N1, N0, Nc, m, n, d, P, seed, round_outputs=None):
    A, B = WL.matmul_inputs(N1, N0, Nc, seed)
    pl = O.make_plan(m, n, d, P)
    Ct = O.worker_products(O.encode_A(A, pl), O.encode_B(B, pl), round_outputs=round_outputs)
    return A, B, pl, Ct


# ----------------------------------------------------------------------------- location


def test_clean_stack_has_no_syndrome_energy():
    A, B, pl, Ct = coded_outputs(8, 8, 8, 2, 2, 2, 14, 0)
    rep = O.locate_nodes(Ct, pl.points, pl.K)
    assert rep.status == "clean" and rep.bad == ()
    assert rep.syndrome_energy <= 1e-24 * rep.energy
    # fp32-rounded responses: rounding noise stays far below the default threshold
    rep32 = O.locate_nodes(O.round_to_f32(Ct), pl.points, pl.K)
    assert rep32.status == "clean" and rep32.syndrome_energy < rep32.threshold / 256


def test_gram_sees_only_the_errors():
    # H annihilates every codeword, so the Gram matrix of (clean + E) is that of E alone
    A, B, pl, Ct = coded_outputs(8, 8, 8, 2, 2, 2, 14, 3)
    rng = np.random.default_rng(3)
    E = np.zeros_like(Ct)
    E[[2, 9]] = rng.standard_normal((2,) + Ct.shape[1:])
    g1 = O.locate_nodes(Ct + E, pl.points, pl.K).gram
    g2 = O.locate_nodes(E, pl.points, pl.K).gram
    assert np.abs(g1 - g2).max() <= 1e-10 * np.abs(g2).max()


def test_single_bad_node_closed_form():
    # one bad node p with errors e_c: Gram = (sum e_c^2) h_p h_p^T, of rank one, and
    # ||h_p||^2 = 1 - (V V^+)_pp because H^T H = I - V V^+ for orthonormal H
    A, B, pl, Ct = coded_outputs(4, 8, 4, 2, 2, 2, 13, 5)
    rng = np.random.default_rng(5)
    p = 6
    e = rng.standard_normal(Ct.shape[1:])
    bad = Ct.copy()
    bad[p] += e
    rep = O.locate_nodes(bad, pl.points, pl.K)
    V = O.vandermonde(pl.points, pl.K)
    lev = (V @ np.linalg.pinv(V))[p, p]
    assert np.isclose(np.trace(rep.gram), (e * e).sum() * (1.0 - lev), rtol=1e-9)
    ev = np.linalg.eigvalsh(rep.gram)
    assert ev[-2] <= 1e-12 * ev[-1]
    assert rep.status == "located" and rep.bad == (p,)
    assert rep.residual <= 1e-20 * rep.syndrome_energy


@pytest.mark.parametrize("t", [0, 1, 2, 3, 4])
def test_planted_bad_nodes_are_found(t):
    # (P, K) = (14, 9): up to P-K-1 = 4 bad nodes, every element of their output corrupted
    A, B, pl, Ct = coded_outputs(4, 8, 4, 2, 2, 2, 14, 1, round_outputs="f32")
    bad, noise = WL.gaussian_node_errors(70 + t, pl.P, t, Ct.shape[1:])
    Cbad = Ct.copy()
    if t:
        Cbad[bad] += noise
    C, rep = O.decode_nodes(Cbad, pl)
    assert rep.bad == tuple(sorted(int(b) for b in bad))
    assert rep.status == ("located" if t else "clean")
    assert np.abs(C - O.uncoded_matmul(A, B)).max() < 1e-3


def test_too_many_bad_nodes_is_a_failure_not_a_wrong_answer():
    # exact-arithmetic regime (unrounded responses, tiny rho): P-K = 5 bad nodes cannot be
    # explained by any 4 columns of H, so failure is declared; detection still happens
    A, B, pl, Ct = coded_outputs(4, 8, 4, 2, 2, 2, 14, 1)
    bad, noise = WL.gaussian_node_errors(99, pl.P, 5, Ct.shape[1:])
    Cbad = Ct.copy()
    Cbad[bad] += noise
    C, rep = O.decode_nodes(Cbad, pl, rho=1e-11)
    assert rep.status == "failed" and C is None
    assert rep.syndrome_energy > rep.threshold


def test_one_codeword_reduces_to_algorithm_1():
    # a stack with a single element codeword: the node search is Algorithm 1 on that word
    rng = np.random.default_rng(11)
    P, K = 12, 7
    pts = O.chebyshev_points(P)
    H = O.parity_check(pts, K)
    V = O.vandermonde(pts, K)
    for trial in range(20):
        z = V @ rng.standard_normal(K)
        supp = sorted(rng.choice(P, rng.integers(1, 4), replace=False).tolist())
        z[supp] += rng.standard_normal(len(supp)) * 3
        tau = 2.0 ** -12 * np.linalg.norm(z)
        status, s1, _ = O.algorithm1(z, H, tau)
        rep = O.locate_nodes(z.reshape(P, 1, 1), pts, K)
        assert status == "located" and rep.status == "located"
        assert rep.bad == tuple(s1) == tuple(supp)


def test_node_search_agrees_with_the_per_codeword_search():
    A, B, pl, Ct = coded_outputs(4, 8, 4, 2, 2, 2, 14, 2, round_outputs="f32")
    bad, noise = WL.gaussian_node_errors(7, pl.P, 3, Ct.shape[1:])
    Cbad = Ct.copy()
    Cbad[bad] += noise
    rep = O.locate_nodes(Cbad, pl.points, pl.K)
    _, rep_cw = O.decode(Cbad, pl, correct=True)
    assert rep.bad == tuple(p for p in range(pl.P) if rep_cw.node_err_count[p] > 0)
    assert np.isclose(rep.syndrome_energy, (rep_cw.syndrome ** 2).sum(), rtol=1e-9)


def test_correlated_errors_on_two_nodes_need_both_nodes():
    # errors of two nodes proportional to each other: the syndromes span one direction
    # (h_p + c h_q) that no single column of H matches, so the smallest set is the pair
    A, B, pl, Ct = coded_outputs(4, 8, 4, 2, 2, 2, 14, 4)
    rng = np.random.default_rng(4)
    e = rng.standard_normal(Ct.shape[1:])
    Cbad = Ct.copy()
    Cbad[3] += e
    Cbad[10] += -0.7 * e
    rep = O.locate_nodes(Cbad, pl.points, pl.K)
    ev = np.linalg.eigvalsh(rep.gram)
    assert ev[-2] <= 1e-12 * ev[-1]                      # rank one
    assert rep.status == "located" and rep.bad == (3, 10)


def test_wild_and_non_finite_values_force_their_node():
    A, B, pl, Ct = coded_outputs(4, 8, 4, 2, 2, 2, 14, 6, round_outputs="f32")
    Cbad = Ct.copy()
    Cbad[1, 0, 0] = np.inf
    Cbad[5, 1, 1] = np.nan
    Cbad[8, 0, 1] = -3e13                                # >= 2^40: handled like non-finite
    noise = np.random.default_rng(6).standard_normal(Ct.shape[1:])
    Cbad[12] += noise
    C, rep = O.decode_nodes(Cbad, pl)
    assert rep.status == "located" and rep.bad == (1, 5, 8, 12)
    assert np.isfinite(rep.energy) and np.abs(C - O.uncoded_matmul(A, B)).max() < 1e-3
    # one forced node beyond the capacity: failure
    Cbad[2, 0, 0] = np.nan
    C2, rep2 = O.decode_nodes(Cbad, pl, rho=1e-11)
    assert rep2.status == "failed" and C2 is None and set((1, 2, 5, 8)) <= set(rep2.bad)


def test_erasures_and_bad_nodes_together():
    A, B, pl, Ct = coded_outputs(4, 8, 4, 2, 2, 2, 16, 8, round_outputs="f32")
    present = np.ones(16, dtype=bool)
    present[[0, 7, 15]] = False                          # 13 present: capacity 13-9-1 = 3
    Cbad = Ct.copy()
    Cbad[[0, 7, 15]] = 1e6                               # stragglers' buffers hold garbage
    rng = np.random.default_rng(8)
    for p in (4, 11, 12):
        Cbad[p] += rng.standard_normal(Ct.shape[1:])
    C, rep = O.decode_nodes(Cbad, pl, present)
    assert rep.status == "located" and rep.bad == (4, 11, 12)
    assert np.abs(C - O.uncoded_matmul(A, B)).max() < 1e-3
    with pytest.raises(O.TooFewResponses):
        O.locate_nodes(Cbad, pl.points, pl.K, np.arange(16) < 8)


def test_errors_below_the_threshold_are_not_reported():
    A, B, pl, Ct = coded_outputs(4, 8, 4, 2, 2, 2, 14, 9)
    Cbad = Ct.copy()
    Cbad[5] += 1e-6 * np.random.default_rng(9).standard_normal(Ct.shape[1:])
    rep = O.locate_nodes(Cbad, pl.points, pl.K)
    assert rep.status == "clean" and 0 < rep.syndrome_energy < rep.threshold


# ----------------------------------------------------------------------------- regeneration


def layer_case(N_out=24, N_in=20, m=4, n=2, P=14, seed=0, subst="auto"):
    lp = O.make_layer_plan(N_out, N_in, 1, m, n, 1, 1, P, subst)
    W = np.random.default_rng(seed).standard_normal((N_out, N_in))
    return lp, W, O.layer_encode_weights(W, lp)


@pytest.mark.parametrize("subst", ["u=v^n", "v=u^m"])
@pytest.mark.parametrize("mode", ["first_k", "lsq_all"])
def test_regeneration_restores_the_encoding_of_W(subst, mode):
    lp, W, Wt = layer_case(subst=subst)
    assert O.weight_polynomial_terms(lp) == lp.m * lp.n
    bad = [2, 5, 13]
    broken = Wt.copy()
    broken[bad] = np.random.default_rng(1).standard_normal((3,) + Wt.shape[1:]) * 100
    fixed = O.layer_regenerate(broken, lp, bad, mode)
    assert np.abs(fixed - Wt).max() <= 1e-9 * np.abs(Wt).max()       # equals the encoding of W
    good = [p for p in range(lp.P) if p not in bad]
    assert np.array_equal(fixed[good], broken[good])                # good nodes untouched


def test_regeneration_from_mn_nodes_is_lagrange_interpolation():
    lp, W, Wt = layer_case(m=2, n=2, P=9, N_out=8, N_in=6)
    bad = [1, 4]
    good = [p for p in range(lp.P) if p not in bad][:4]              # first mn good nodes
    rng = np.random.default_rng(2)
    stack = rng.standard_normal(Wt.shape)                            # not even a codeword
    fixed = O.layer_regenerate(stack, lp, bad, "first_k")
    b = lp.points
    for p in bad:
        want = np.zeros(Wt.shape[1:])
        for q in good:
            L = np.prod([(b[p] - b[r]) / (b[q] - b[r]) for r in good if r != q])
            want += L * stack[q]
        assert np.abs(fixed[p] - want).max() <= 1e-10 * max(1.0, np.abs(want).max())


def test_regeneration_needs_mn_good_nodes():
    lp, W, Wt = layer_case(m=2, n=2, P=6, N_out=8, N_in=6)
    O.layer_regenerate(Wt, lp, [0, 1])                               # 4 good: enough
    with pytest.raises(O.TooFewResponses):
        O.layer_regenerate(Wt, lp, [0, 1, 2])


def test_locate_then_regenerate_a_corrupted_weight_stack():
    # the coded weights at rest are themselves a code word stack with K = mn
    lp, W, Wt = layer_case()
    broken = O.round_to_f32(Wt)
    broken[9] += np.random.default_rng(3).standard_normal(Wt.shape[1:])
    rep = O.locate_nodes(broken, lp.points, O.weight_polynomial_terms(lp))
    assert rep.status == "located" and rep.bad == (9,)
    fixed = O.layer_regenerate(broken, lp, rep.bad)
    assert np.abs(fixed - Wt).max() <= 1e-6 * np.abs(Wt).max()
    # fp32 rounding of the stored blocks (2^-24) times the amplification of the weight decoder
    assert np.abs(O.layer_decode_weights(fixed, lp) - W).max() <= 1e-4 * np.abs(W).max()


# ----------------------------------------------------------------------------- projection


def test_projection_is_the_orthogonal_projector_onto_the_code():
    lp, W, Wt = layer_case()
    Kw = O.weight_polynomial_terms(lp)
    V = O.vandermonde(lp.points, Kw)
    H = O.parity_check(lp.points, Kw)
    rng = np.random.default_rng(4)
    # code words are fixed points
    assert np.abs(O.layer_project(Wt, lp) - Wt).max() <= 1e-12 * np.abs(Wt).max()
    # a component in the row space of H (orthogonal to the code) is removed exactly
    off = np.einsum("rp,rxy->pxy", H, rng.standard_normal((H.shape[0],) + Wt.shape[1:]))
    assert np.abs(O.layer_project(Wt + off, lp) - Wt).max() <= 1e-11 * np.abs(Wt).max()
    # for any stack: idempotent, and what is removed is orthogonal to the code
    stack = rng.standard_normal(Wt.shape)
    proj = O.layer_project(stack, lp)
    assert np.abs(O.layer_project(proj, lp) - proj).max() <= 1e-10
    removed = (stack - proj).reshape(lp.P, -1)
    assert np.abs(V.T @ removed).max() <= 1e-10
    # the least-squares decoder does not see the removed part
    assert np.abs(O.layer_decode_weights(proj, lp) - O.layer_decode_weights(stack, lp)).max() <= 1e-10


def test_projection_from_a_subset_of_nodes():
    lp, W, Wt = layer_case()
    present = np.ones(lp.P, dtype=bool)
    present[[0, 6]] = False
    stack = Wt.copy()
    stack[[0, 6]] = 123.0
    assert np.abs(O.layer_project(stack, lp, present) - Wt).max() <= 1e-9 * np.abs(Wt).max()


# ----------------------------------------------------------------------------- verification step


def test_check_positions_are_spread_evenly():
    assert O.check_positions(100, 10).tolist() == [0, 10, 20, 30, 40, 50, 60, 70, 80, 90]
    assert O.check_positions(7, 3).tolist() == [0, 2, 4]
    assert O.check_positions(4, 16).tolist() == [0, 1, 2, 3]


def test_verification_passes_on_a_correct_decode_and_catches_a_wrong_one():
    A, B, pl, Ct = coded_outputs(8, 8, 8, 2, 2, 2, 14, 12, round_outputs="f32")
    present = np.ones(14, dtype=bool)
    present[[2, 11]] = False
    C, _ = O.decode(Ct, pl, present, "first_k")
    rep = O.verify_decode(Ct, pl, C, present, "first_k")
    assert rep.status == "ok" and rep.n_checked == 14 and rep.max_ratio < 1.0 and rep.bad == ()
    pos = O.check_positions(16, 14)
    rows = cols = 4
    # a decoding error at a checked position is caught ...
    Cbad = C.copy()
    r_, c_ = divmod(int(pos[5]), cols)
    Cbad[rows + r_, c_] += 1e-2                                     # block (1, 0)
    rep = O.verify_decode(Ct, pl, Cbad, present, "first_k")
    assert rep.status == "mismatch" and rep.n_value_mismatch == 1
    # ... one at an unchecked position is not (the step looks at P values only)
    unchecked = [e for e in range(16) if e not in pos.tolist()][0]
    Cbad = C.copy()
    Cbad[unchecked // cols, unchecked % cols] += 1.0
    assert O.verify_decode(Ct, pl, Cbad, present, "first_k").status == "ok"
    # a decode from the wrong nodes (an erased node's garbage used) is caught
    Cgar = Ct.copy()
    Cgar[2] = 5.0
    Cwrong, _ = O.decode(Cgar, pl, np.ones(14, dtype=bool), "first_k")
    assert O.verify_decode(Cgar, pl, Cwrong, present, "first_k").status == "mismatch"


def test_verification_crosschecks_the_located_nodes():
    A, B, pl, Ct = coded_outputs(8, 8, 8, 2, 2, 2, 14, 13, round_outputs="f32")
    bad, noise = WL.gaussian_node_errors(5, 14, 2, Ct.shape[1:])
    Cb = Ct.copy()
    Cb[bad] += noise
    C, nrep = O.decode_nodes(Cb, pl)
    assert nrep.bad == tuple(int(b) for b in bad)
    rep = O.verify_decode(Cb, pl, C, None, "lsq_all", bad=nrep.bad)
    assert rep.status == "ok" and rep.locations_agree and rep.bad == nrep.bad
    # claiming a different set of erroneous nodes fails the crosscheck
    other = (int(bad[0]),)
    rep = O.verify_decode(Cb, pl, C, None, "lsq_all", bad=other)
    assert rep.status == "mismatch" and not rep.locations_agree
    # a decode that did not leave the erroneous nodes out has wrong values
    Cnaive, _ = O.decode(Cb, pl, None, "lsq_all")
    rep = O.verify_decode(Cb, pl, Cnaive, None, "lsq_all", bad=nrep.bad)
    assert rep.status == "mismatch" and rep.n_value_mismatch > 0
