"""GPU parity of the coded DNN layer step (forward O1, backward O2, coded update O3) against
the oracle, fp32 workers: small shapes with padding and both substitutions, a few training
iterations of a small MLP, and the B=1 benchmark MLP (4096-4096-4096-10) at full size."""
import numpy as np
import pytest
import torch

import gpd_workloads as WL
import paper_1811_10751_amd as G
from paper_1811_10751_amd.mlp import CodedMLP
from oracle import gpd_oracle as O
from gpu_util import DEV, rel_fro, say, to_dev, to_np

pytestmark = pytest.mark.gpu

SUB = {"u=v^n": G.GPD_SUB_U_VN, "v=u^m": G.GPD_SUB_V_UM, "auto": G.GPD_SUB_AUTO}

CASES = [
    # N_out, N_in, batch, m, n, d1, d2, P, subst
    (64, 96, 1, 4, 2, 1, 1, 24, "auto"),          # cfg2's code at a small size (skinny kernels)
    (64, 96, 1, 4, 2, 1, 1, 24, "u=v^n"),
    (10, 96, 1, 4, 2, 1, 1, 24, "auto"),          # 10 rows, m = 4: padded to 12
    (70, 50, 2, 2, 4, 1, 1, 20, "u=v^n"),         # batch 2, N_in padded to 52: encodes inside the product kernels
    (66, 54, 2, 2, 2, 2, 2, 16, "auto"),          # batch 2 split over d1 = d2 = 2 (per-node batch 1)
    (70, 50, 4, 2, 4, 1, 1, 20, "u=v^n"),         # N_in = 50, n = 4: padded to 52; batch 4 skinny
    (130, 260, 8, 2, 2, 2, 2, 16, "u=v^n"),       # d1 = d2 = 2, skinny kernels
    (66, 36, 8, 2, 2, 1, 4, 24, "u=v^n"),         # d2 = 4: K_b = 18, ill-conditioned (amp ~1e5)
    (300, 200, 24, 2, 4, 1, 1, 32, "auto"),       # cfg3's code, MFMA GEMM path, ragged tiles
    (256, 384, 48, 2, 2, 2, 3, 20, "v=u^m"),      # GEMM path with d1, d2 > 1
]


@pytest.mark.parametrize("N_out,N_in,batch,m,n,d1,d2,P,subst", CASES)
def test_layer_forward_backward_update(N_out, N_in, batch, m, n, d1, d2, P, subst):
    say("layer case", N_out, N_in, batch, m, n, d1, d2, P, subst)
    rng = np.random.default_rng(N_out + 7 * N_in + batch)
    W = (rng.standard_normal((N_out, N_in)) / np.sqrt(N_in)).astype(np.float32)
    X = rng.uniform(-1, 1, (N_in, batch)).astype(np.float32)
    D = rng.standard_normal((N_out, batch)).astype(np.float32)
    olp = O.make_layer_plan(N_out, N_in, batch, m, n, d1, d2, P, subst)
    L = G.gpd_layer_create(N_out, N_in, batch, m, n, d1, d2, P, subst=SUB[subst])
    assert (L.Kf, L.Kb) == (olp.Kf, olp.Kb)
    assert (L.wt_rows, L.wt_cols) == (olp.N_out_pad // m, olp.N_in_pad // n)

    Wt = G.gpd_layer_encode_weights(L, to_dev(W))
    torch.cuda.synchronize()
    Wt_o = O.layer_encode_weights(W, olp)
    assert np.abs(to_np(Wt) - Wt_o).max() <= 4e-7 * m * n * np.abs(W).max()
    Wt_h = to_np(Wt).copy()

    # weights back from the coded blocks (all nodes, then exactly mn of them)
    W_back = G.gpd_layer_decode_weights(L, Wt)
    assert rel_fro(to_np(W_back), W) < 1e-5
    present = np.zeros(P, dtype=np.uint8)
    present[rng.choice(P, m * n, replace=False)] = 1
    W_back = G.gpd_layer_decode_weights(L, Wt, present=present)
    W_back_o = O.layer_decode_weights(Wt_h, olp, present)
    amp_w = np.linalg.norm(np.linalg.pinv(O.vandermonde(olp.points[present.astype(bool)], m * n)), axis=1).max()
    say("  weight decode from mn nodes: err %.3g (amp %.3g)" % (rel_fro(to_np(W_back), W_back_o), amp_w))
    assert rel_fro(to_np(W_back), W_back_o) <= 2e-6 * max(amp_w, 1.0)

    # forward: oracle works from the GPU's own coded weights (fp32 words)
    S, _ = G.gpd_coded_layer_step(L, G.GPD_STEP_FORWARD, Wt, to_dev(X))
    S_o, _ = O.layer_forward(Wt_h, X, olp)
    ampf = O.amplification(olp.fwd, None, "lsq_all")
    say("  forward err %.3g (amp %.3g)" % (rel_fro(to_np(S), S_o), ampf))
    assert rel_fro(to_np(S), S_o) <= 2e-6 * max(ampf, 1.0)
    assert rel_fro(to_np(S), W.astype(np.float64) @ X) <= max(1e-3, 4e-6 * ampf)

    # the element-wise step C1 done by the decode itself: the same values as the separate kernel
    # on the plain output, whichever decode path runs (plain, element correction, node search)
    for corr in (G.GPD_CORRECT_NONE, G.GPD_CORRECT_ELEMENTS, G.GPD_CORRECT_NODES):
        S_c, _ = G.gpd_coded_layer_step(L, G.GPD_STEP_FORWARD, Wt, to_dev(X), correct_errors=corr)
        Y_f, _ = G.gpd_coded_layer_step(L, G.GPD_STEP_FORWARD, Wt, to_dev(X), correct_errors=corr,
                                        fuse_sigmoid=True)
        assert torch.equal(Y_f, G.gpd_sigmoid_fwd(S_c)), corr
        assert np.abs(to_np(Y_f) - 1 / (1 + np.exp(-S_o))).max() < 1e-5 * max(ampf, 1.0)
    # step C2 likewise: C o Xs (1 - Xs) for an input Xs in (0, 1); eta = 0 leaves the weights alone
    Xs = to_dev((0.5 * (X + 1)).astype(np.float32).clip(0.01, 0.99))
    for corr in (G.GPD_CORRECT_NONE, G.GPD_CORRECT_ELEMENTS, G.GPD_CORRECT_NODES):
        C_c, _ = G.gpd_coded_layer_step(L, G.GPD_STEP_BACKWARD_UPDATE, Wt, Xs, Dlt=to_dev(D), eta=0.0,
                                        decay=0.0, correct_errors=corr)
        D_f, _ = G.gpd_coded_layer_step(L, G.GPD_STEP_BACKWARD_UPDATE, Wt, Xs, Dlt=to_dev(D), eta=0.0,
                                        decay=0.0, correct_errors=corr, fuse_sigmoid=True)
        assert torch.equal(D_f, G.gpd_sigmoid_bwd(C_c, Xs)), corr
    assert np.array_equal(to_np(Wt), Wt_h)

    # backward + update in one call; backward uses the pre-update weights
    eta, decay = 0.05, 0.01
    C, _ = G.gpd_coded_layer_step(L, G.GPD_STEP_BACKWARD_UPDATE, Wt, to_dev(X), Dlt=to_dev(D), eta=eta, decay=decay)
    torch.cuda.synchronize()
    C_o, _ = O.layer_backward(Wt_h, D, olp)
    Db = np.linalg.pinv(O.vandermonde(olp.points, olp.Kb))
    ampb = max(np.linalg.norm(Db[int(e)]) for e in olp.eCb.ravel())
    say("  backward err %.3g (amp %.3g)" % (rel_fro(to_np(C), C_o), ampb))
    assert rel_fro(to_np(C), C_o) <= 2e-6 * max(ampb, 1.0)
    assert rel_fro(to_np(C), W.astype(np.float64).T @ D) <= max(2e-3, 4e-6 * ampb)
    Wt2_o = O.layer_update(Wt_h, D, X, olp, eta, np.float32(decay))
    scale = np.abs(Wt2_o).max()
    assert np.abs(to_np(Wt) - Wt2_o).max() <= 1e-5 * scale
    # the updated blocks are still a codeword: decoding them gives the updated W
    W2 = (1 - decay) * W.astype(np.float64) + eta * D.astype(np.float64) @ X.astype(np.float64).T
    assert rel_fro(to_np(G.gpd_layer_decode_weights(L, Wt)), W2) < 1e-4

    # update only (out skipped)
    Wt_before = to_np(Wt).copy()
    out, _ = G.gpd_coded_layer_step(L, G.GPD_STEP_BACKWARD_UPDATE, Wt, to_dev(X), Dlt=to_dev(D), eta=eta,
                                    decay=0.0, skip_output=True)
    assert out is None
    Wt3_o = O.layer_update(Wt_before, D, X, olp, eta, 0.0)
    assert np.abs(to_np(Wt) - Wt3_o).max() <= 1e-5 * scale


def test_forward_with_erasures_and_a_corrupted_node():
    # stragglers among the nodes + one node whose stored W~_p was corrupted (shows up as an
    # erroneous response in step O1 and is located there)
    N_out, N_in, P = 64, 96, 24
    rng = np.random.default_rng(3)
    W = (rng.standard_normal((N_out, N_in)) / 8).astype(np.float32)
    X = rng.uniform(-1, 1, (N_in, 1)).astype(np.float32)
    olp = O.make_layer_plan(N_out, N_in, 1, 4, 2, 1, 1, P, "auto")
    L = G.gpd_layer_create(N_out, N_in, 1, 4, 2, 1, 1, P)
    Wt = G.gpd_layer_encode_weights(L, to_dev(W))
    noise = np.random.default_rng(11).standard_normal(tuple(Wt[7].shape)).astype(np.float32)
    Wt[7] += 0.05 * to_dev(noise)
    present = np.ones(P, dtype=np.uint8)
    present[[1, 20]] = 0
    S, rep = G.gpd_coded_layer_step(L, G.GPD_STEP_FORWARD, Wt, to_dev(X), present=present, correct_errors=True,
                                    want_report=True)
    S_o, orep = O.layer_forward(to_np(Wt), X, olp, present, correct=True)
    assert rep.status == G.GPD_OK and rep.n_present == 22
    assert [x[:3] for x in rep.located] == [x[:3] for x in orep.located]
    assert set(x[0] for x in rep.located) == {7}
    assert rel_fro(to_np(S), S_o) < 1e-4
    # a corrupted response whose error is below tau is not corrected; it moves the result by at
    # most tau times the amplification
    assert rel_fro(to_np(S), W.astype(np.float64) @ X) < 1e-3 + O.amplification(olp.fwd, present, "lsq_all") * 2.0 ** -12


@pytest.mark.parametrize("batch,m,n,P", [(1, 4, 2, 24), (4, 2, 4, 32), (24, 2, 4, 32)])
def test_small_mlp_training_tracks_the_oracle(batch, m, n, P):
    sizes = (96, 128, 64, 10)
    Ws = WL.mlp_init(sizes, seed=2)
    Ws = [(w * 8).astype(np.float32) for w in Ws]
    olps = [O.make_layer_plan(sizes[l + 1], sizes[l], batch, m, n, 1, 1, P, "auto") for l in range(3)]
    mlp = CodedMLP(sizes, batch, m, n, 1, 1, P)
    mlp.encode_weights([to_dev(w) for w in Ws])
    Wts_o = [to_np(wt).astype(np.float64) for wt in mlp.Wts]
    Ws_plain = [w.astype(np.float64) for w in Ws]
    eta = 0.5
    for step in range(6):
        X, Y = WL.mlp_batch(2, step, sizes[0], sizes[-1], batch)
        yhat, _ = mlp.step(to_dev(X), to_dev(Y), eta)
        Wts_o, yhat_o, _ = O.mlp_coded_step(Wts_o, olps, X, Y, np.float32(eta))
        Ws_plain, yhat_p, _ = O.mlp_uncoded_step(Ws_plain, X, Y, np.float32(eta))
        e1, e2 = rel_fro(to_np(yhat), yhat_o), rel_fro(to_np(yhat), yhat_p)
        say("  step", step, "yhat err vs coded oracle %.3g, vs plain SGD %.3g" % (e1, e2))
        assert e1 < 1e-3 and e2 < 1e-3
    for l in range(3):
        assert rel_fro(to_np(mlp.Wts[l]), Wts_o[l]) < 1e-3
    for W_dec, W_ref in zip(mlp.decode_weights(), Ws_plain):
        assert rel_fro(to_np(W_dec), W_ref) < 1e-3


def test_hip_graph_replay_matches_eager():
    # a whole training iteration captured once as a HIP graph and replayed must leave exactly
    # the coded weights the same calls leave when made one by one (the kernels are deterministic;
    # tables are uploaded on first use, so every distinct call is made before the capture)
    sizes, batch, m, n, P = (96, 128, 64, 10), 1, 4, 2, 24
    Ws = [to_dev((w * 8).astype(np.float32)) for w in WL.mlp_init(sizes, seed=5)]
    data = [WL.mlp_batch(5, t, sizes[0], sizes[-1], batch) for t in range(5)]
    eager = CodedMLP(sizes, batch, m, n, 1, 1, P)
    eager.encode_weights(Ws)
    for X, Y in data:
        eager.step(to_dev(X), to_dev(Y), 0.5)
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        gm = CodedMLP(sizes, batch, m, n, 1, 1, P, stream=side)
        gm.encode_weights(Ws)
        Xs, Ys = to_dev(data[0][0]).clone(), to_dev(data[0][1]).clone()
        snapshot = [w.clone() for w in gm.Wts]
        gm.step(Xs, Ys, 0.5)                       # warm-up call: fills the table cache
        for w, s0 in zip(gm.Wts, snapshot):
            w.copy_(s0)                            # undo its update
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        yhat, _ = gm.step(Xs, Ys, 0.5)
    for X, Y in data:
        Xs.copy_(to_dev(X))
        Ys.copy_(to_dev(Y))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
    for a, b in zip(eager.Wts, gm.Wts):
        assert torch.equal(a, b)


@pytest.mark.parametrize("N0,N1,batch,m,n,P", [(96, 160, 8, 2, 2, 12), (130, 70, 1, 4, 2, 24), (256, 512, 64, 2, 4, 32)])
def test_sparse_autoencoder_training_tracks_the_oracle(N0, N1, batch, m, n, P):
    from paper_1811_10751_amd.mlp import CodedAutoencoder
    rng = np.random.default_rng(N0)
    W1 = (rng.standard_normal((N1, N0)) / np.sqrt(N0)).astype(np.float32)
    W2 = (rng.standard_normal((N0, N1)) / np.sqrt(N1)).astype(np.float32)
    ae = CodedAutoencoder(N0, N1, batch, m, n, P)
    ae.encode_weights(to_dev(W1), to_dev(W2))
    P1, P2 = W1.astype(np.float64), W2.astype(np.float64)
    eta, rho, beta, decay = 0.5, 0.2, 0.3, 0.001
    for step in range(5):
        X = rng.uniform(0.05, 0.95, (N0, batch)).astype(np.float32)
        xh = ae.step(to_dev(X), eta, rho, beta, decay)
        P1, P2, xh_o = O.autoencoder_uncoded_step(P1, P2, X, np.float32(eta), np.float32(rho), np.float32(beta),
                                                  np.float32(decay))
        err = rel_fro(to_np(xh), xh_o)
        say("  autoencoder step", step, "reconstruction err vs plain SGD %.3g" % err)
        assert err < 1e-3
    D1, D2 = ae.decode_weights()
    assert rel_fro(to_np(D1), P1) < 1e-3 and rel_fro(to_np(D2), P2) < 1e-3
    # the two extra element-wise steps alone
    Y = torch.rand((37, 19), device=DEV) * 0.9 + 0.05
    Cm = torch.randn((37, 19), device=DEV)
    rh = G.gpd_row_mean(Y)
    assert np.abs(to_np(rh) - to_np(Y).astype(np.float64).mean(axis=1)).max() < 1e-6
    d = G.gpd_sigmoid_bwd_sparse(Cm, Y, rh, 0.2, 0.3 / 19)
    want = O.autoencoder_delta1(to_np(Cm), to_np(Y), 0.2, 0.3)
    assert np.abs(to_np(d) - want).max() <= 1e-5 * np.abs(want).max()
