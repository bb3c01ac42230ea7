"""GPU parity of the node-level fault path against the oracle: the Gram matrix of the
syndromes element by element (in a basis-free form), the set of nodes found erroneous, the
decode that leaves them out, regeneration of coded weights and the projection onto the code.
The oracle always works on the GPU's own fp32 stacks."""
import numpy as np
import pytest
import torch

import gpd_workloads as WL
import paper_1811_10751_amd as G
from oracle import gpd_oracle as O
from gpu_util import DEV, rel_fro, say, to_dev, to_np

pytestmark = pytest.mark.gpu


def random_stack(P, K, rows, cols, seed, bad=(), scale=1.0):
    """fp32 stack [P, rows, cols] whose element codewords are evaluations of random polynomials
    with K coefficients (rounded to fp32), plus dense Gaussian noise on the nodes in `bad`."""
    rng = np.random.default_rng(seed)
    pts = O.chebyshev_points(P)
    Z = (O.vandermonde(pts, K) @ rng.standard_normal((K, rows * cols))).reshape(P, rows, cols)
    for p in bad:
        Z[p] += scale * rng.standard_normal((rows, cols))
    return Z.astype(np.float32)


def basis_free(gram, H):
    """H^T G H = sum_c (P_perp z_c)(P_perp z_c)^T: the same whatever orthonormal H is used."""
    return H.T @ gram @ H


def plan_for(P, K, rows, cols):
    """A matmul plan whose response stack is [P, rows, cols] with threshold K = 4d + 1 (m=n=2)
    or K = d (m=n=1)."""
    if (K - 1) % 4 == 0 and K >= 5:
        d = (K - 1) // 4
        return G.gpd_plan(2 * rows, 2, d * cols, 2, 2, d, P)
    return G.gpd_plan(rows, 1, K * cols, 1, 1, K, P)


GRAM_CASES = [
    # P, K, rows, cols, bad nodes, present mask zeros
    (16, 9, 64, 64, (3, 11), ()),            # 4096 codewords, float4 path, one tile
    (14, 9, 33, 20, (5,), ()),               # 660 codewords: float4 path with a ragged last chunk
    (12, 5, 17, 13, (0, 7), (2,)),           # odd count: scalar path, an erasure
    (32, 9, 40, 24, (1, 20, 31), (4, 9)),    # 30 present, 21 syndromes: two tiles of 16
    (64, 13, 24, 16, (2, 40), ()),           # 51 syndromes: four tiles, 16 node steps
    (48, 21, 9, 7, (47,), (0, 1, 2)),        # 45 present, 24 syndromes, scalar path
    (9, 9, 8, 8, (), ()),                    # no parity at all
]


@pytest.mark.parametrize("P,K,rows,cols,bad,absent", GRAM_CASES)
def test_gram_matrix_and_node_search(P, K, rows, cols, bad, absent):
    say("gram", P, K, rows, cols, bad, absent)
    plan = plan_for(P, K, rows, cols)
    assert plan.K == K
    Z = random_stack(P, K, rows, cols, seed=P * 100 + K, bad=bad)
    present = np.ones(P, dtype=np.uint8)
    present[list(absent)] = 0
    Z[list(absent)] = 777.0                                    # absent nodes hold garbage
    rep, gram = G.gpd_locate_nodes(plan, to_dev(Z), present=present, want_gram=True)
    want = O.locate_nodes(Z, O.chebyshev_points(P), K, present)
    assert rep.bad == want.bad == tuple(sorted(bad))
    assert rep.status == G.GPD_OK and rep.wild == ()
    assert np.isclose(rep.energy, want.energy, rtol=1e-12)
    assert np.isclose(rep.threshold, want.threshold, rtol=1e-12)
    S = np.flatnonzero(present)
    if len(S) > K:
        H = G.gpd_host_parity_check(P, K, present=present)
        Ho = O.parity_check(O.chebyshev_points(P)[S], K)
        got, ref = basis_free(gram, H), basis_free(want.gram, Ho)
        # fp32 syndromes: each carries a rounding error of about 2^-24 ||z||
        tol = 1e-6 * np.abs(ref).max() + 1e-12 * want.energy
        assert np.abs(got - ref).max() <= tol
        assert np.isclose(rep.syndrome_energy, want.syndrome_energy, rtol=1e-5, atol=1e-9 * want.energy)


@pytest.mark.parametrize("t", [0, 1, 2, 3, 4, 5, 6, 7])
def test_decode_with_node_correction(t):
    # (P, K) = (16, 9): up to 6 erroneous nodes are located and left out; 7 is a failure
    N = 96
    A, B = WL.matmul_inputs(N, N, N, seed=t)
    plan = G.gpd_plan(N, N, N, 2, 2, 2, 16)
    At, Bt = G.gpd_encode(plan, to_dev(A), to_dev(B))
    Ct = G.gpd_worker_products(plan, At, Bt)
    bad, noise = WL.gaussian_node_errors(300 + t, 16, t, tuple(Ct.shape[1:]))
    if t:
        Ct[torch.from_numpy(np.asarray(bad)).to(DEV)] += to_dev(noise.astype(np.float32))
    torch.cuda.synchronize()
    Ct_h = to_np(Ct)
    opl = O.make_plan(2, 2, 2, 16)
    C, rep = G.gpd_decode(plan, Ct, mode=G.GPD_DEC_LSQ_ALL, correct_errors=G.GPD_CORRECT_NODES)
    C_o, orep = O.decode_nodes(Ct_h, opl, rho=2.0 ** -12)
    ncw = Ct.shape[1] * Ct.shape[2]
    if t <= 6:
        assert orep.status == ("located" if t else "clean") and rep.status == G.GPD_OK
        found = tuple(p for p in range(16) if rep.node_err_count[p] > 0)
        assert found == orep.bad
        assert rep.n_located == len(found) * ncw and rep.n_failed == 0
        assert rep.n_flagged == (ncw if t else 0)
        present = np.ones(16, dtype=bool)
        present[list(orep.bad)] = False
        assert rel_fro(to_np(C), C_o) <= 1e-6 * max(O.amplification(opl, present, "lsq_all"), 1.0)
        planted = tuple(sorted(int(b) for b in bad))
        if t <= 5:
            assert found == planted
        if found == planted:
            assert rel_fro(to_np(C), O.uncoded_matmul(A, B)) <= max(1e-3, 1e-6 * O.amplification(opl, present, "lsq_all"))
        else:
            # with a finite threshold a smaller node set can explain the syndromes when the planted
            # nodes' columns of H are nearly dependent (here nodes 0, 1, 2 sit close together at the
            # end of the Chebyshev grid): both sides take the same, smaller, set
            say("  t = %d: planted %s, both sides found %s" % (t, planted, found))
    else:
        assert orep.status == "failed" and rep.status == G.GPD_E_DECODE_FAIL
        assert rep.n_failed == ncw and rep.n_located == 0


def test_wild_values_erasures_and_first_k_mode():
    N = 64
    A, B = WL.matmul_inputs(N, N, N, seed=5)
    plan = G.gpd_plan(N, N, N, 2, 2, 2, 16)
    At, Bt = G.gpd_encode(plan, to_dev(A), to_dev(B))
    Ct = G.gpd_worker_products(plan, At, Bt)
    present = np.ones(16, dtype=np.uint8)
    present[[0, 9]] = 0                                        # 14 present: capacity 4
    Ct[0] = float("nan")                                       # absent nodes hold garbage
    Ct[9] = 1e30
    Ct[3, 5, 7] = float("inf")
    Ct[6, 0, 0] = -4e12                                        # >= 2^40
    Ct[12] += 0.5 * torch.randn(Ct.shape[1:], generator=torch.Generator(device=DEV).manual_seed(1), device=DEV)
    torch.cuda.synchronize()
    opl = O.make_plan(2, 2, 2, 16)
    nrep = G.gpd_locate_nodes(plan, Ct, present=present)
    want = O.locate_nodes(to_np(Ct), opl.points, opl.K, present)
    assert nrep.bad == want.bad == (3, 6, 12) and nrep.wild == (3, 6)
    assert np.isfinite(nrep.energy) and np.isclose(nrep.energy, want.energy, rtol=1e-12)
    for mode, oname in ((G.GPD_DEC_FIRST_K, "first_k"), (G.GPD_DEC_LSQ_ALL, "lsq_all")):
        C, rep = G.gpd_decode(plan, Ct, present=present, mode=mode, correct_errors=G.GPD_CORRECT_NODES)
        C_o, _ = O.decode_nodes(to_np(Ct), opl, present, oname)
        keep = present.astype(bool).copy()
        keep[[3, 6, 12]] = False
        assert rep.status == G.GPD_OK
        assert rel_fro(to_np(C), C_o) <= 1e-6 * max(O.amplification(opl, keep, oname), 1.0)
        assert np.isfinite(to_np(C)).all()


def test_small_errors_stay_below_the_threshold_and_rho_is_honoured():
    N = 64
    A, B = WL.matmul_inputs(N, N, N, seed=6)
    opl = O.make_plan(2, 2, 2, 14)
    for rho in (0.0, 1e-5):                                    # 0 = default 2^-12
        plan = G.gpd_plan(N, N, N, 2, 2, 2, 14, rho_detect=rho)
        At, Bt = G.gpd_encode(plan, to_dev(A), to_dev(B))
        Ct = G.gpd_worker_products(plan, At, Bt)
        Ct[4] *= 1.0 + 2e-4                                    # relative error 2e-4 on node 4
        torch.cuda.synchronize()
        rep = G.gpd_locate_nodes(plan, Ct)
        want = O.locate_nodes(to_np(Ct), opl.points, opl.K, rho=rho or 2.0 ** -12)
        assert rep.bad == want.bad == (() if rho == 0.0 else (4,))


def test_bad_arguments():
    plan = G.gpd_plan(32, 32, 32, 2, 2, 2, 12)
    Ct = torch.zeros((12, 16, 16), device=DEV)
    with pytest.raises(G.GpdError) as e:
        G.gpd_locate_nodes(plan, Ct, present=np.arange(12) < 8)
    assert e.value.status == G.GPD_E_TOO_FEW
    with pytest.raises(G.GpdError) as e:
        G.gpd_locate_nodes(plan, Ct, workspace=torch.zeros(256, dtype=torch.uint8, device=DEV))
    assert e.value.status == G.GPD_E_WORKSPACE
    with pytest.raises(G.GpdError) as e:
        G.gpd_decode(plan, Ct, correct_errors=7)
    assert e.value.status == G.GPD_E_INVALID
    rep = G.gpd_locate_nodes(plan, Ct)                         # all zero: clean, nothing to divide by
    assert rep.bad == () and rep.energy == 0.0


# ----------------------------------------------------------------------------- coded layer


LAYERS = [
    (96, 80, 1, 4, 2, 1, 1, 14),          # batch 1 (vectors), v = u^m
    (301, 204, 3, 2, 3, 1, 1, 20),        # rows padded to 302
    (256, 384, 32, 2, 4, 1, 1, 32),       # the cfg3 code (projection on the matrix cores, 32 nodes)
    (128, 64, 1, 4, 2, 1, 1, 24),         # the cfg2 code, 1024-element blocks (the same, 24 nodes)
]


def layer_setup(N_out, N_in, batch, m, n, d1, d2, P, seed=0):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((N_out, N_in)) / np.sqrt(N_in)).astype(np.float32)
    X = rng.uniform(-1, 1, (N_in, batch)).astype(np.float32)
    D = rng.standard_normal((N_out, batch)).astype(np.float32)
    olp = O.make_layer_plan(N_out, N_in, batch, m, n, d1, d2, P, "auto")
    L = G.gpd_layer_create(N_out, N_in, batch, m, n, d1, d2, P)
    Wt = G.gpd_layer_encode_weights(L, to_dev(W))
    return W, X, D, olp, L, Wt


@pytest.mark.parametrize("N_out,N_in,batch,m,n,d1,d2,P", LAYERS)
def test_regenerate_and_project(N_out, N_in, batch, m, n, d1, d2, P):
    say("regenerate", N_out, N_in, batch, m, n, P)
    W, X, D, olp, L, Wt = layer_setup(N_out, N_in, batch, m, n, d1, d2, P)
    clean = to_np(Wt).copy()
    bad = [1, P - 2] if P - m * n >= 3 else [1]
    g = torch.Generator(device=DEV).manual_seed(3)
    for p in bad:
        Wt[p] = torch.randn(Wt.shape[1:], generator=g, device=DEV) * 10
    torch.cuda.synchronize()
    broken = to_np(Wt).copy()
    # the stored stack is itself a code: the node search finds the overwritten blocks
    rep = G.gpd_layer_locate_nodes(L, G.GPD_STACK_WEIGHTS, Wt)
    want = O.locate_nodes(broken, olp.points, m * n)
    assert rep.bad == want.bad == tuple(bad)
    for mode, oname in ((G.GPD_DEC_LSQ_ALL, "lsq_all"), (G.GPD_DEC_FIRST_K, "first_k")):
        Wt.copy_(to_dev(broken))
        G.gpd_layer_regenerate(L, Wt, bad, mode)
        torch.cuda.synchronize()
        ref = O.layer_regenerate(broken, olp, bad, oname)
        got = to_np(Wt)
        good = [p for p in range(P) if p not in bad]
        assert np.array_equal(got[good], broken[good])                 # good nodes untouched
        # fp32 combination of up to P blocks; the interpolation weights can be large for first_k
        V = O.vandermonde(olp.points[good if oname == "lsq_all" else good[:m * n]], m * n)
        amp = max(np.abs(O.vandermonde(olp.points[bad], m * n) @ np.linalg.pinv(V)).sum(axis=1).max(), 1.0)
        assert np.abs(got - ref).max() <= 4e-7 * amp * np.abs(clean).max()
        if oname == "lsq_all":
            assert np.abs(got - clean).max() <= 1e-5 * np.abs(clean).max()   # the encoding of W is back
    # projection: drift added to every node is reduced to its component inside the code
    Wt.copy_(to_dev(clean))
    drift = (np.random.default_rng(4).standard_normal(clean.shape) * 1e-3).astype(np.float32)
    Wt += to_dev(drift)
    torch.cuda.synchronize()
    before = to_np(Wt).copy()
    G.gpd_layer_project(L, Wt)
    torch.cuda.synchronize()
    ref = O.layer_project(before, olp)
    assert np.abs(to_np(Wt) - ref).max() <= 4e-6 * np.abs(clean).max()
    rep2 = G.gpd_layer_locate_nodes(L, G.GPD_STACK_WEIGHTS, Wt)
    assert rep2.bad == () and rep2.syndrome_energy <= 1e-10 * rep2.energy   # on the code again
    # projection from a subset regenerates the absent nodes
    present = np.ones(P, dtype=np.uint8)
    present[bad] = 0
    Wt.copy_(to_dev(broken))
    G.gpd_layer_project(L, Wt, present)
    torch.cuda.synchronize()
    assert np.abs(to_np(Wt) - O.layer_project(broken, olp, present)).max() <= 4e-6 * np.abs(clean).max()
    with pytest.raises(G.GpdError) as e:
        G.gpd_layer_regenerate(L, Wt, list(range(P - m * n + 1)))
    assert e.value.status == G.GPD_E_TOO_FEW


@pytest.mark.parametrize("N_out,N_in,batch,m,n,d1,d2,P", LAYERS)
def test_layer_step_with_a_corrupted_node(N_out, N_in, batch, m, n, d1, d2, P):
    # a node whose stored W~_p was overwritten gives a wrong output in both products: the node
    # search names it, the decode leaves it out, regeneration repairs it after the update
    say("layer node fault", N_out, N_in, batch, m, n, P)
    W, X, D, olp, L, Wt = layer_setup(N_out, N_in, batch, m, n, d1, d2, P, seed=1)
    badp = 2
    Wt[badp] += 0.3 * torch.randn(Wt.shape[1:], generator=torch.Generator(device=DEV).manual_seed(9), device=DEV)
    torch.cuda.synchronize()
    Wt_before = to_np(Wt).copy()
    S, rep = G.gpd_coded_layer_step(L, G.GPD_STEP_FORWARD, Wt, to_dev(X), correct_errors=G.GPD_CORRECT_NODES,
                                    want_report=True)
    St = to_np(L.view(1, DEV))
    want = O.locate_nodes(St, olp.points, olp.Kf)
    found = tuple(p for p in range(P) if rep.node_err_count[p] > 0)
    assert found == want.bad == (badp,) and rep.status == G.GPD_OK
    keep = np.ones(P, dtype=bool)
    keep[badp] = False
    Sref = W.astype(np.float64) @ X
    assert rel_fro(to_np(S), Sref) <= 1e-6 * max(O.amplification(olp.fwd, keep, "lsq_all"), 100.0)
    # the same responses seen through the layer's own locate call
    nrep = G.gpd_layer_locate_nodes(L, G.GPD_STACK_FORWARD, L.view(1, DEV))
    assert nrep.bad == (badp,)
    eta = 0.05
    C, rep_b = G.gpd_coded_layer_step(L, G.GPD_STEP_BACKWARD_UPDATE, Wt, to_dev(X), Dlt=to_dev(D), eta=eta,
                                      correct_errors=G.GPD_CORRECT_NODES, want_report=True)
    found_b = tuple(p for p in range(P) if rep_b.node_err_count[p] > 0)
    assert found_b == (badp,) and rep_b.status == G.GPD_OK
    Db = np.linalg.pinv(O.vandermonde(olp.points[keep], olp.Kb))
    ampb = max(np.linalg.norm(Db[int(e)]) for e in olp.eCb.ravel())
    assert rel_fro(to_np(C), W.astype(np.float64).T @ D) <= 1e-6 * max(ampb, 100.0)
    G.gpd_layer_regenerate(L, Wt, found_b)
    torch.cuda.synchronize()
    # after regeneration the stack encodes exactly the uncoded update W + eta D X^T
    W2 = W.astype(np.float64) + eta * D.astype(np.float64) @ X.astype(np.float64).T
    Wd = G.gpd_layer_decode_weights(L, Wt)
    assert rel_fro(to_np(Wd), W2) <= 1e-4
    ref = O.layer_regenerate(O.layer_update(Wt_before, D, X, olp, eta), olp, [badp])
    assert np.abs(to_np(Wt) - ref).max() <= 1e-5 * np.abs(ref).max()


def test_cfg4_size_stack_node_search():
    # full-size launch configuration: 16 blocks of 2048 x 2048 (4.2 M codewords); three nodes get
    # dense noise.  Checked against the closed form: H annihilates the clean part, so
    # H^T G H = P_perp[:, bad] (E E^T) P_perp[bad, :] with E the planted noise, up to the fp32
    # rounding of the clean responses.
    c = WL.CONFIGS[4]
    N, P = c["N1"], c["P"]
    plan = G.gpd_plan(N, N, N, c["m"], c["n"], c["d"], P)
    K = plan.K
    rows = cols = N // 2
    g = torch.Generator(device=DEV).manual_seed(44)
    coef = torch.randn((K, rows * cols), generator=g, device=DEV)
    V = torch.from_numpy(O.vandermonde(O.chebyshev_points(P), K).astype(np.float32)).to(DEV)
    Ct = (V @ coef).reshape(P, rows, cols).contiguous()
    del coef
    bad = (2, 7, 13)
    E = torch.randn((3, rows, cols), generator=g, device=DEV)
    for i, p in enumerate(bad):
        Ct[p] += E[i]
    torch.cuda.synchronize()
    rep, gram = G.gpd_locate_nodes(plan, Ct, want_gram=True)
    assert rep.bad == bad and rep.status == G.GPD_OK
    H = G.gpd_host_parity_check(P, K)
    Ef = E.reshape(3, -1).double()
    EEt = (Ef @ Ef.T).cpu().numpy()
    Pp = H.T @ H
    ref = Pp[:, list(bad)] @ EEt @ Pp[list(bad), :]
    got = basis_free(gram, H)
    say("  cfg4-size gram: max rel dev %.3g" % (np.abs(got - ref).max() / np.abs(ref).max()))
    assert np.abs(got - ref).max() <= 1e-5 * np.abs(ref).max()
    energy = float((Ct.double() ** 2).sum().item())
    assert np.isclose(rep.energy, energy, rtol=1e-9)
    C, drep = G.gpd_decode(plan, Ct, mode=G.GPD_DEC_LSQ_ALL, correct_errors=G.GPD_CORRECT_NODES)
    assert drep.status == G.GPD_OK and tuple(p for p in range(P) if drep.node_err_count[p]) == bad


@pytest.mark.parametrize("batch,m,n,P", [(1, 4, 2, 24), (8, 2, 4, 32)])
def test_training_with_node_faults_and_regeneration(batch, m, n, P):
    # the paper's strategy end to end (Sec. VII): stored coded weights of a node are overwritten
    # between iterations; the next product exposes the node, the decode leaves it out, its
    # weights are regenerated, and training stays on the trajectory of plain SGD
    from paper_1811_10751_amd.mlp import CodedMLP
    sizes = (96, 128, 64, 10)
    Ws = [(w * 8).astype(np.float32) for w in WL.mlp_init(sizes, seed=2)]
    mlp = CodedMLP(sizes, batch, m, n, 1, 1, P)
    mlp.encode_weights([to_dev(w) for w in Ws])
    Ws_plain = [w.astype(np.float64) for w in Ws]
    eta = 0.5
    faults = {2: (1, 5), 4: (0, P - 1), 5: (2, 3)}           # step -> (layer, node)
    g = torch.Generator(device=DEV).manual_seed(8)
    for step in range(7):
        if step in faults:
            l, p = faults[step]
            mlp.Wts[l][p] += 0.5 * torch.randn(mlp.Wts[l].shape[1:], generator=g, device=DEV)
        X, Y = WL.mlp_batch(2, step, sizes[0], sizes[-1], batch)
        yhat, reps = mlp.step(to_dev(X), to_dev(Y), eta, correct_errors=G.GPD_CORRECT_NODES, regenerate=True)
        Ws_plain, yhat_p, _ = O.mlp_uncoded_step(Ws_plain, X, Y, np.float32(eta))
        err = rel_fro(to_np(yhat), yhat_p)
        say("  step", step, "repaired", mlp.repaired, "yhat err vs plain SGD %.3g" % err)
        if step in faults:
            l, p = faults[step]
            assert mlp.repaired == [(l, "forward", p)]
        else:
            assert mlp.repaired == []
        assert all(r[0].status == G.GPD_OK for r in reps)
        assert err < 1e-3
    for L, Wt, W_ref in zip(mlp.layers, mlp.Wts, Ws_plain):
        assert rel_fro(to_np(G.gpd_layer_decode_weights(L, Wt)), W_ref) < 1e-3
        rep = G.gpd_layer_locate_nodes(L, G.GPD_STACK_WEIGHTS, Wt)
        assert rep.bad == ()


# ----------------------------------------------------------------------------- verification step


def test_verification_step_against_the_oracle():
    N = 128
    A, B = WL.matmul_inputs(N, N, N, seed=21)
    plan = G.gpd_plan(N, N, N, 2, 2, 2, 16)
    opl = O.make_plan(2, 2, 2, 16)
    At, Bt = G.gpd_encode(plan, to_dev(A), to_dev(B))
    Ct = G.gpd_worker_products(plan, At, Bt)
    rows = cols = N // 2
    pos = O.check_positions(rows * cols, 16)
    # (1) erasures, both modes: a correct decode passes, with the oracle's ratio
    present = WL.erasure_trial(4, 16, 5)
    for mode, oname in ((G.GPD_DEC_FIRST_K, "first_k"), (G.GPD_DEC_LSQ_ALL, "lsq_all")):
        C, _ = G.gpd_decode(plan, Ct, present=present, mode=mode)
        rep = G.gpd_verify_decode(plan, Ct, C, present=present, mode=mode)
        want = O.verify_decode(to_np(Ct), opl, to_np(C), present, oname)
        assert rep.status == G.GPD_OK and want.status == "ok"
        assert rep.n_checked == want.n_checked == 16 and rep.locations_agree and rep.bad == ()
        assert abs(rep.max_ratio - want.max_ratio) <= 1e-6 + 1e-3 * want.max_ratio and rep.max_ratio < 1.0
    # (2) a wrong value at a checked position is caught, one elsewhere is not
    C, _ = G.gpd_decode(plan, Ct, present=present, mode=G.GPD_DEC_FIRST_K)
    r_, c_ = divmod(int(pos[7]), cols)
    Cbad = C.clone()
    Cbad[rows + r_, cols + c_] += 100.0                           # block (1, 1); far above the tolerance
    rep = G.gpd_verify_decode(plan, Ct, Cbad, present=present, mode=G.GPD_DEC_FIRST_K)
    want = O.verify_decode(to_np(Ct), opl, to_np(Cbad), present, "first_k")
    assert rep.status == G.GPD_E_VERIFY and rep.n_value_mismatch == want.n_value_mismatch == 1
    unchecked = [e for e in range(rows * cols) if e not in set(pos.tolist())][0]
    Cbad = C.clone()
    Cbad[unchecked // cols, unchecked % cols] += 1.0
    assert G.gpd_verify_decode(plan, Ct, Cbad, present=present, mode=G.GPD_DEC_FIRST_K).status == G.GPD_OK
    # (3) erroneous nodes: the decode in node mode passes when it reports its nodes, a naive decode fails,
    #     a wrong claim about the nodes fails the crosscheck
    bad, noise = WL.gaussian_node_errors(9, 16, 2, (rows, cols))
    Cb = Ct.clone()
    Cb[torch.from_numpy(np.asarray(bad)).to(DEV)] += to_dev(noise)
    Cd, drep = G.gpd_decode(plan, Cb, mode=G.GPD_DEC_LSQ_ALL, correct_errors=G.GPD_CORRECT_NODES)
    found = tuple(p for p in range(16) if drep.node_err_count[p] > 0)
    assert found == tuple(int(b) for b in bad)
    rep = G.gpd_verify_decode(plan, Cb, Cd, mode=G.GPD_DEC_LSQ_ALL, bad=found)
    want = O.verify_decode(to_np(Cb), opl, to_np(Cd), None, "lsq_all", bad=found)
    assert rep.status == G.GPD_OK and want.status == "ok" and rep.bad == want.bad == found
    Cnaive, _ = G.gpd_decode(plan, Cb, mode=G.GPD_DEC_LSQ_ALL)
    rep = G.gpd_verify_decode(plan, Cb, Cnaive, mode=G.GPD_DEC_LSQ_ALL, bad=found)
    assert rep.status == G.GPD_E_VERIFY and rep.n_value_mismatch > 0 and rep.locations_agree
    rep = G.gpd_verify_decode(plan, Cb, Cd, mode=G.GPD_DEC_LSQ_ALL, bad=found[:1])
    assert rep.status == G.GPD_E_VERIFY and not rep.locations_agree
    # (4) more values than codewords, and a non-finite decoded value
    rep = G.gpd_verify_decode(plan, Ct, C, present=present, mode=G.GPD_DEC_FIRST_K, n_check=4096)
    assert rep.status == G.GPD_OK and rep.n_checked == 4096
    Cnan = C.clone()
    Cnan[0, 0] = float("nan")
    assert G.gpd_verify_decode(plan, Ct, Cnan, present=present, mode=G.GPD_DEC_FIRST_K).status == G.GPD_E_VERIFY


def test_decoding_failure_restores_the_checkpoint():
    # more erroneous nodes than the code can locate: the failure is reported, the iteration is
    # abandoned and the coded weights go back to the last checkpoint (Sec. VII, error model 2)
    from paper_1811_10751_amd.mlp import CodedMLP
    sizes, batch, m, n, P = (96, 128, 64, 10), 4, 2, 4, 16          # K_f = 11, K_b = 12: capacity 4 / 3
    Ws = [(w * 8).astype(np.float32) for w in WL.mlp_init(sizes, seed=2)]
    mlp = CodedMLP(sizes, batch, m, n, 1, 1, P, rho_detect=1e-6)
    mlp.encode_weights([to_dev(w) for w in Ws])
    X, Y = WL.mlp_batch(2, 0, sizes[0], sizes[-1], batch)
    mlp.step(to_dev(X), to_dev(Y), 0.5, correct_errors=G.GPD_CORRECT_NODES, regenerate=True)
    mlp.checkpoint()
    saved = [to_np(w).copy() for w in mlp.Wts]
    X, Y = WL.mlp_batch(2, 1, sizes[0], sizes[-1], batch)
    mlp.step(to_dev(X), to_dev(Y), 0.5, correct_errors=G.GPD_CORRECT_NODES, regenerate=True)
    assert not mlp.restored and any(not np.array_equal(to_np(w), s0) for w, s0 in zip(mlp.Wts, saved))
    g = torch.Generator(device=DEV).manual_seed(2)
    for p in (0, 3, 5, 8, 9, 12):                                    # six bad nodes in layer 1
        mlp.Wts[1][p] += torch.randn(mlp.Wts[1].shape[1:], generator=g, device=DEV)
    X, Y = WL.mlp_batch(2, 2, sizes[0], sizes[-1], batch)
    yhat, reps = mlp.step(to_dev(X), to_dev(Y), 0.5, correct_errors=G.GPD_CORRECT_NODES, regenerate=True,
                          restore_on_failure=True)
    assert yhat is None and mlp.restored
    assert reps[1][0].status == G.GPD_E_DECODE_FAIL and reps[0][0].status == G.GPD_OK
    for w, s0 in zip(mlp.Wts, saved):
        assert np.array_equal(to_np(w), s0)
    # training goes on from the checkpoint
    yhat, reps = mlp.step(to_dev(X), to_dev(Y), 0.5, correct_errors=G.GPD_CORRECT_NODES, regenerate=True,
                          restore_on_failure=True)
    assert yhat is not None and not mlp.restored and mlp.repaired == []
