"""Pins for the oracle's coded DNN layer step (Sec. VII, IX): the coded forward/backward
products equal W x and W^T delta, the coded update keeps W~_p a codeword of the updated W,
and the whole coded trajectory equals plain SGD, whose gradients are pinned by finite
differences."""
import numpy as np
import pytest

import gpd_workloads as WL
from oracle import gpd_oracle as O


CASES = [
    # N_out, N_in, batch, m, n, d1, d2, P, subst
    (8, 12, 1, 4, 2, 1, 1, 16, "u=v^n"),
    (8, 12, 1, 4, 2, 1, 1, 16, "v=u^m"),
    (6, 8, 4, 2, 4, 1, 1, 14, "u=v^n"),
    (6, 8, 4, 2, 4, 2, 2, 24, "u=v^n"),
    (6, 9, 6, 3, 3, 2, 3, 40, "v=u^m"),
    (10, 8, 2, 4, 2, 1, 1, 16, "auto"),          # 10 rows with m=4: padded to 12
]


@pytest.mark.parametrize("N_out,N_in,batch,m,n,d1,d2,P,subst", CASES)
def test_forward_backward_update_match_the_plain_layer(N_out, N_in, batch, m, n, d1, d2, P, subst):
    rng = np.random.default_rng(N_out * 1000 + N_in * 10 + batch)
    W = rng.standard_normal((N_out, N_in))
    X = rng.standard_normal((N_in, batch))
    D = rng.standard_normal((N_out, batch))
    lp = O.make_layer_plan(N_out, N_in, batch, m, n, d1, d2, P, subst)
    Wt = O.layer_encode_weights(W, lp)
    assert Wt.shape == (P, lp.N_out_pad // m, lp.N_in_pad // n)
    # monomial-basis interpolation with ~30 coefficients is ill-conditioned even in fp64
    tol = 1e-7 if max(lp.Kf, lp.Kb) <= 16 else 1e-4
    # O1: S = W X
    S, _ = O.layer_forward(Wt, X, lp)
    assert np.abs(S - W @ X).max() < tol
    # O2: C^T = Delta^T W, i.e. C = W^T Delta
    C, _ = O.layer_backward(Wt, D, lp)
    assert np.abs(C - W.T @ D).max() < tol
    # O3 in coded form: the updated blocks are the encoding of the updated W (Eq. coded update)
    eta, decay = 0.05, 0.01
    Wt2 = O.layer_update(Wt, D, X, lp, eta, decay)
    W2 = (1 - decay) * W + eta * D @ X.T
    assert np.abs(Wt2 - O.layer_encode_weights(W2, lp)).max() < 1e-12
    assert np.abs(O.layer_decode_weights(Wt2, lp) - W2).max() < 1e-8
    # regeneration footnote: any mn nodes determine W~ (degree mn-1)
    present = np.zeros(P, dtype=np.uint8)
    present[rng.choice(P, m * n, replace=False)] = 1
    assert np.abs(O.layer_decode_weights(Wt2, lp, present) - W2).max() < 1e-6
    # erasures within tolerance, forward and backward
    pf = np.ones(P, dtype=np.uint8)
    pf[rng.choice(P, P - lp.Kf, replace=False)] = 0
    S2, _ = O.layer_forward(Wt, X, lp, pf)
    assert np.abs(S2 - W @ X).max() < 1e3 * tol
    pb = np.ones(P, dtype=np.uint8)
    pb[rng.choice(P, P - lp.Kb, replace=False)] = 0
    C2, _ = O.layer_backward(Wt, D, lp, pb)
    assert np.abs(C2 - W.T @ D).max() < 1e3 * tol


def test_uncoded_step_is_gradient_descent_on_the_l2_loss():
    # delta = -d(eps^2)/ds and W += eta delta x^T (App. on DNN background): the update
    # direction must equal minus the finite-difference gradient of the mini-batch L2 loss.
    rng = np.random.default_rng(0)
    sizes = (5, 4, 3)
    Ws = [rng.standard_normal((sizes[l + 1], sizes[l])) * 0.5 for l in range(2)]
    X = rng.uniform(-1, 1, (5, 3))
    Y = np.zeros((3, 3))
    Y[[0, 2, 1], [0, 1, 2]] = 1
    eta = 1.0
    new_Ws, _, deltas = O.mlp_uncoded_step(Ws, X, Y, eta)
    h = 1e-6
    for l in range(2):
        G = np.zeros_like(Ws[l])
        for i in range(G.shape[0]):
            for j in range(G.shape[1]):
                Wp = [w.copy() for w in Ws]
                Wm = [w.copy() for w in Ws]
                Wp[l][i, j] += h
                Wm[l][i, j] -= h
                G[i, j] = (O.mlp_loss(Wp, X, Y) - O.mlp_loss(Wm, X, Y)) / (2 * h)
        assert np.abs((new_Ws[l] - Ws[l]) + eta * G).max() < 1e-8
    # g(f(u)) = f'(u) for the logistic function
    u = np.linspace(-3, 3, 7)
    fd = (O.sigmoid(u + h) - O.sigmoid(u - h)) / (2 * h)
    assert np.abs(O.sigmoid_grad_from_output(O.sigmoid(u)) - fd).max() < 1e-9


@pytest.mark.parametrize("batch,m,n,P,subst", [(1, 4, 2, 16, "auto"), (4, 2, 4, 16, "u=v^n")])
def test_coded_training_trajectory_equals_plain_sgd(batch, m, n, P, subst):
    sizes = (16, 16, 16, 10)
    Ws = [w.astype(np.float64) * 8 for w in WL.mlp_init(sizes, seed=2)]
    lps = [O.make_layer_plan(sizes[l + 1], sizes[l], batch, m, n, 1, 1, P, subst) for l in range(3)]
    Wts = [O.layer_encode_weights(W, lp) for W, lp in zip(Ws, lps)]
    eta = 0.5
    for step in range(5):
        X, Y = WL.mlp_batch(2, step, sizes[0], sizes[-1], batch)
        Ws, yhat, deltas = O.mlp_uncoded_step(Ws, X, Y, eta, decay=0.001)
        Wts, yhat_c, trace = O.mlp_coded_step(Wts, lps, X, Y, eta, decay=0.001)
        assert np.abs(yhat - yhat_c).max() < 1e-9
        for l in range(3):
            assert np.abs(trace[l]["delta"] - deltas[l]).max() < 1e-9
            assert np.abs(O.layer_decode_weights(Wts[l], lps[l]) - Ws[l]).max() < 1e-8
            assert np.abs(Wts[l] - O.layer_encode_weights(Ws[l], lps[l])).max() < 1e-10


def test_forward_corrects_a_corrupted_weight_block():
    # Sec. VII "errors during update stage": a corrupted W~_p shows up in step O1 of the next
    # iteration as an erroneous node output and is located there.
    rng = np.random.default_rng(9)
    lp = O.make_layer_plan(8, 8, 1, 2, 2, 1, 1, 12)
    W = rng.standard_normal((8, 8))
    x = rng.standard_normal((8, 1))
    Wt = O.layer_encode_weights(W, lp)
    Wt[7] += 0.1 * rng.standard_normal(Wt[7].shape)
    S, rep = O.layer_forward(Wt, x, lp, correct=True, rho=1e-9)
    assert rep.status == "ok" and set(t[0] for t in rep.located) == {7}
    assert np.abs(S - W @ x).max() < 1e-8


def test_substitution_choice():
    assert O.choose_substitution(4, 2) == "v=u^m" and O.choose_substitution(2, 4) == "u=v^n"
    a = O.make_layer_plan(16, 16, 1, 4, 2, 1, 1, 24, "u=v^n")
    b = O.make_layer_plan(16, 16, 1, 4, 2, 1, 1, 24, "v=u^m")
    assert (a.Kf, a.Kb) == (9, 14) and (b.Kf, b.Kb) == (12, 11)
    c = O.make_layer_plan(16, 16, 4, 2, 4, 1, 1, 32, "auto")
    assert (c.Kf, c.Kb) == (11, 12)


# ----------------------------------------------------------------------------- sparse autoencoder (Sec. X)


def test_autoencoder_step_is_minus_the_gradient_of_its_loss():
    # finite differences of the printed loss (data term + beta KL term) against the update direction
    rng = np.random.default_rng(0)
    N0, N1, B = 7, 5, 4
    W1 = rng.standard_normal((N1, N0)) * 0.5
    W2 = rng.standard_normal((N0, N1)) * 0.5
    X = rng.uniform(0.1, 0.9, (N0, B))
    rho, beta, eta = 0.2, 0.7, 1.0
    n1, n2, _ = O.autoencoder_uncoded_step(W1, W2, X, eta, rho, beta)
    g1, g2 = (n1 - W1) / eta, (n2 - W2) / eta                   # claimed minus-gradients
    h = 1e-6
    for (W, g, which) in ((W1, g1, 1), (W2, g2, 2)):
        for _ in range(12):
            i, j = rng.integers(0, W.shape[0]), rng.integers(0, W.shape[1])
            Wp, Wm = W.copy(), W.copy()
            Wp[i, j] += h
            Wm[i, j] -= h
            if which == 1:
                fd = (O.autoencoder_loss(Wp, W2, X, rho, beta) - O.autoencoder_loss(Wm, W2, X, rho, beta)) / (2 * h)
            else:
                fd = (O.autoencoder_loss(W1, Wp, X, rho, beta) - O.autoencoder_loss(W1, Wm, X, rho, beta)) / (2 * h)
            assert abs(-fd - g[i, j]) <= 1e-6 * max(1.0, abs(fd))


def test_autoencoder_sparsity_term_vanishes_at_the_target_and_reduces_to_the_mlp():
    assert np.allclose(O.kl_slope(0.3, np.array([0.3, 0.3])), 0.0)
    assert O.kl_slope(0.3, np.array([0.5]))[0] > 0 > O.kl_slope(0.3, np.array([0.1]))[0]
    rng = np.random.default_rng(1)
    W1, W2 = rng.standard_normal((6, 8)) * 0.3, rng.standard_normal((8, 6)) * 0.3
    X = rng.uniform(0, 1, (8, 3))
    # beta = 0: an ordinary two-layer network trained to reproduce its input
    a1, a2, _ = O.autoencoder_uncoded_step(W1, W2, X, 0.1, 0.2, 0.0)
    (m1, m2), _, _ = O.mlp_uncoded_step([W1, W2], X, X, 0.1)
    assert np.allclose(a1, m1) and np.allclose(a2, m2)


def test_coded_autoencoder_step_equals_the_plain_one():
    rng = np.random.default_rng(2)
    N0, N1, B, m, n, P = 12, 8, 4, 2, 2, 12
    lp1 = O.make_layer_plan(N1, N0, B, m, n, 1, 1, P)
    lp2 = O.make_layer_plan(N0, N1, B, m, n, 1, 1, P)
    W1, W2 = rng.standard_normal((N1, N0)) * 0.4, rng.standard_normal((N0, N1)) * 0.4
    Wt1, Wt2 = O.layer_encode_weights(W1, lp1), O.layer_encode_weights(W2, lp2)
    for step in range(3):
        X = rng.uniform(0.05, 0.95, (N0, B))
        Wt1, Wt2, xh_c = O.autoencoder_coded_step(Wt1, Wt2, lp1, lp2, X, 0.3, 0.15, 0.5, decay=0.01)
        W1, W2, xh_p = O.autoencoder_uncoded_step(W1, W2, X, 0.3, 0.15, 0.5, decay=0.01)
        assert np.abs(xh_c - xh_p).max() < 1e-9
    assert np.abs(O.layer_decode_weights(Wt1, lp1) - W1).max() < 1e-9
    assert np.abs(O.layer_decode_weights(Wt2, lp2) - W2).max() < 1e-9
