"""GPU parity of the bf16 worker products (bf16 MFMA, fp32 accumulation), stage by stage:
encode (fp32 -> bf16 round-to-nearest-even), products (the oracle multiplies the GPU's own
bf16 operands in fp64), decode (the oracle decodes the GPU's own responses).  End-to-end
figures against the exact product are printed and bounded by the rounding of the operands
times the amplification of the decoder."""
import numpy as np
import pytest
import torch

import gpd_workloads as WL
import paper_1811_10751_amd as G
from paper_1811_10751_amd.mlp import CodedMLP
from oracle import gpd_oracle as O
from gpu_util import DEV, rel_fro, say, to_dev, to_np

pytestmark = pytest.mark.gpu


def bf16_to_f64(t):
    return t.to(torch.float32).cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("N1,N0,Nc,m,n,d,P", [(256, 256, 256, 2, 2, 2, 12), (512, 320, 384, 2, 2, 2, 16),
                                              (300, 204, 140, 2, 2, 2, 11), (264, 520, 136, 1, 4, 1, 9)])
def test_bf16_matmul_stagewise(N1, N0, Nc, m, n, d, P):
    say("bf16 matmul", N1, N0, Nc, m, n, d, P)
    A, B = WL.matmul_inputs(N1, N0, Nc, seed=N1)
    opl = O.make_plan(m, n, d, P)
    plan = G.gpd_plan(N1, N0, Nc, m, n, d, P, worker_dtype=G.GPD_BF16)
    At, Bt = G.gpd_encode(plan, to_dev(A), to_dev(B))
    assert At.dtype == torch.bfloat16 and Bt.dtype == torch.bfloat16
    # encode: equal to the oracle's bf16 rounding except where fp32 summation order moves a value
    # across a bf16 rounding boundary (then off by one bf16 step)
    for got, want in ((bf16_to_f64(At), O.round_to_bf16(O.encode_A(A, opl))),
                      (bf16_to_f64(Bt), O.round_to_bf16(O.encode_B(B, opl)))):
        diff = np.abs(got - want)
        assert (diff > 0).mean() < 1e-3
        # one bf16 step, or (for sums that cancel to almost nothing) the fp32 rounding of the sum
        assert np.all(diff <= 2.0 ** -7 * np.abs(want) + 4e-7 * 4)
    # products
    Ct = G.gpd_worker_products(plan, At, Bt)
    torch.cuda.synchronize()
    Ct_o = O.worker_products(bf16_to_f64(At), bf16_to_f64(Bt))
    assert rel_fro(to_np(Ct), Ct_o) < 2e-6
    # decode of the GPU's responses
    for present in (None, WL.erasure_trial(3, P, P - opl.K)):
        C, _ = G.gpd_decode(plan, Ct, present=present, mode=G.GPD_DEC_LSQ_ALL)
        C_o, _ = O.decode(to_np(Ct), opl, present, "lsq_all")
        amp = O.amplification(opl, present, "lsq_all")
        assert rel_fro(to_np(C), C_o) <= 1e-6 * max(amp, 1.0)
    # end to end vs the exact product: bf16 operand rounding (2^-9 each) amplified by the decoder
    C, _ = G.gpd_decode(plan, Ct, mode=G.GPD_DEC_LSQ_ALL)
    e2e = rel_fro(to_np(C), O.uncoded_matmul(A, B))
    amp = O.amplification(opl, None, "lsq_all")
    say("  bf16 end-to-end vs exact A.B: %.3g (amp %.3g)" % (e2e, amp))
    assert e2e <= 4 * amp * 2.0 ** -9


LAYER_CASES = [
    (256, 384, 128, 2, 4, 1, 1, 32),      # cfg3's code, full tiles
    (300, 200, 24, 2, 4, 1, 1, 32),       # ragged tiles
    (130, 260, 48, 2, 2, 2, 3, 20),       # d1, d2 > 1
    (300, 200, 64, 2, 4, 1, 1, 32),       # update operands as bf16 planes, ragged tiles, one ring of stages
    (512, 1024, 192, 2, 4, 1, 1, 32),     # planes, full tiles, steady-state loop and tail
    (1024, 1024, 128, 2, 4, 1, 1, 32),    # planes, 256 full tiles
    (10, 1000, 64, 2, 4, 1, 1, 32),       # output layer: 5 rows per node (few-row forward kernel)
    (7, 520, 24, 1, 4, 1, 1, 20),         # 7 rows, batch 24 (ragged 64-column groups)
    (10, 1024, 64, 2, 4, 1, 1, 32),       # output layer whose backward product takes the few-row kernel too
    (16, 512, 128, 2, 2, 2, 2, 20),       # 8 rows per node, d1 = d2 = 2
]


@pytest.mark.parametrize("N_out,N_in,batch,m,n,d1,d2,P", LAYER_CASES)
def test_bf16_layer_stagewise(N_out, N_in, batch, m, n, d1, d2, P):
    say("bf16 layer", N_out, N_in, batch, m, n, d1, d2, P)
    rng = np.random.default_rng(N_out + N_in)
    W = (rng.standard_normal((N_out, N_in)) / np.sqrt(N_in)).astype(np.float32)
    X = rng.uniform(-1, 1, (N_in, batch)).astype(np.float32)
    D = rng.standard_normal((N_out, batch)).astype(np.float32)
    olp = O.make_layer_plan(N_out, N_in, batch, m, n, d1, d2, P, "auto")
    L = G.gpd_layer_create(N_out, N_in, batch, m, n, d1, d2, P, worker_dtype=G.GPD_BF16)
    Wt = G.gpd_layer_encode_weights(L, to_dev(W))
    Wt_h = to_np(Wt).copy()

    # ---- forward
    S, _ = G.gpd_coded_layer_step(L, G.GPD_STEP_FORWARD, Wt, to_dev(X))
    torch.cuda.synchronize()
    Xt = to_np(L.view(0, DEV).float())             # stored in bf16 (the product's operand type)
    St = to_np(L.view(1, DEV))
    Xt_o = O.layer_encode_x(X, olp)                # fp32 encode, then one rounding to bf16
    assert np.abs(Xt - Xt_o).max() <= (2.0 ** -8 + 4e-7 * n * d1) * np.abs(Xt_o).max()
    assert np.array_equal(Xt, O.round_to_bf16(Xt))
    St_o = O.worker_products(Wt_h, Xt, operands="bf16")                          # bf16 products
    assert rel_fro(St, St_o) < 2e-6
    S_o, _ = O.decode(St, olp.fwd, None, "lsq_all")                              # fp32 decode
    ampf = O.amplification(olp.fwd, None, "lsq_all")
    assert rel_fro(to_np(S), S_o[:N_out]) <= 1e-6 * max(ampf, 1.0)
    e2e = rel_fro(to_np(S), W.astype(np.float64) @ X)
    say("  forward vs exact W X: %.3g (amp %.3g)" % (e2e, ampf))
    assert e2e <= 4 * ampf * 2.0 ** -9

    # ---- backward + update
    eta, decay = 0.05, 0.01
    C, _ = G.gpd_coded_layer_step(L, G.GPD_STEP_BACKWARD_UPDATE, Wt, to_dev(X), Dlt=to_dev(D), eta=eta, decay=decay)
    torch.cuda.synchronize()
    Dt = to_np(L.view(2, DEV).float())              # [P][N_out/m][batch/d2], stored in bf16
    Ct = to_np(L.view(3, DEV))                      # [P][N_in/n][batch/d2]
    Dt_o = np.transpose(O.layer_encode_delta(D, olp), (0, 2, 1))
    assert np.abs(Dt - Dt_o).max() <= (2.0 ** -8 + 4e-7 * m * d2) * np.abs(Dt_o).max()
    Ct_o = np.matmul(np.transpose(O.round_to_bf16(Wt_h), (0, 2, 1)), O.round_to_bf16(Dt))
    assert rel_fro(Ct, Ct_o) < 2e-6
    useful = sorted(set(int(e) for e in olp.eCb.ravel()))
    coeffs, _ = O.decode_coefficients(Ct, olp.points, olp.Kb, useful, mode="lsq_all")
    rows, cols = Ct.shape[1], Ct.shape[2]
    C_o = np.zeros((n * rows, d2 * cols))
    for j in range(n):
        for k in range(d2):
            C_o[j * rows:(j + 1) * rows, k * cols:(k + 1) * cols] = coeffs[int(olp.eCb[k, j])]
    Db = np.linalg.pinv(O.vandermonde(olp.points, olp.Kb))
    ampb = max(np.linalg.norm(Db[int(e)]) for e in olp.eCb.ravel())
    assert rel_fro(to_np(C), C_o[:N_in]) <= 1e-6 * max(ampb, 1.0)
    say("  backward vs exact W^T D: %.3g (amp %.3g)" % (rel_fro(to_np(C), W.astype(np.float64).T @ D), ampb))
    # the update stays fp32
    Wt2_o = O.layer_update(Wt_h, D, X, olp, eta, np.float32(decay))
    assert np.abs(to_np(Wt) - Wt2_o).max() <= 1e-5 * np.abs(Wt2_o).max()


def test_cfg3_full_size_one_layer_step():
    # cfg3's middle layer (8192 x 8192, batch 256, m=2, n=4, P=32), bf16 products: stage-wise
    # parity on the full-size launch configuration, with the oracle checking sampled node outputs
    c = WL.CONFIGS[3]
    N, batch, m, n, P = 8192, c["batch"], c["m"], c["n"], c["P"]
    rng = np.random.default_rng(c["seed"])
    W = (rng.standard_normal((N, N)) / 64).astype(np.float32)
    X = rng.uniform(-1, 1, (N, batch)).astype(np.float32)
    D = (rng.standard_normal((N, batch)) / 16).astype(np.float32)
    olp = O.make_layer_plan(N, N, batch, m, n, 1, 1, P, "auto")
    L = G.gpd_layer_create(N, N, batch, m, n, 1, 1, P, worker_dtype=G.GPD_BF16)
    assert (L.Kf, L.Kb) == (11, 12)
    Wd = to_dev(W)
    Wt = G.gpd_layer_encode_weights(L, Wd)
    S, _ = G.gpd_coded_layer_step(L, G.GPD_STEP_FORWARD, Wt, to_dev(X))
    torch.cuda.synchronize()
    Xt, St = to_np(L.view(0, DEV).float()), to_np(L.view(1, DEV))
    sample_p = [0, 13, 31]
    rows_s = rng.choice(N // m, 64, replace=False)
    for p in sample_p:
        ref = O.round_to_bf16(to_np(Wt[p][torch.from_numpy(rows_s).to(DEV)])) @ O.round_to_bf16(Xt[p])
        assert rel_fro(St[p][rows_s], ref) < 2e-6
    S_o, _ = O.decode(St, olp.fwd, None, "lsq_all")
    assert rel_fro(to_np(S), S_o) <= 1e-6 * O.amplification(olp.fwd, None, "lsq_all")
    say("  cfg3 L2 forward vs exact: %.3g" % rel_fro(to_np(S), W.astype(np.float64) @ X))
    Wt_rows_before = {p: to_np(Wt[p][torch.from_numpy(rows_s).to(DEV)]).copy() for p in sample_p}
    C, _ = G.gpd_coded_layer_step(L, G.GPD_STEP_BACKWARD_UPDATE, Wt, to_dev(X), Dlt=to_dev(D), eta=0.01, decay=0.0)
    torch.cuda.synchronize()
    Dt, Ct = to_np(L.view(2, DEV).float()), to_np(L.view(3, DEV))
    # update operands as the kernel holds them: two fp16 planes (hi, lo) of the operand / 2^E,
    # [P][batch/16][rows][16] each, E per operand
    def planes(v, e):
        s = v.double().sum(0).permute(0, 2, 1, 3) * 2.0 ** e   # [P][rows][batch/16][16]
        return s.reshape(s.shape[0], s.shape[1], -1).cpu().numpy()
    exps = L.view(6, DEV).cpu().numpy()
    Dh, Xh = planes(L.view(4, DEV), int(exps[0])), planes(L.view(5, DEV), int(exps[1]))
    # the scale leaves headroom: every fp16 value is finite and below 2^15, and uses at most the
    # bits the bound on the encode's row sums gives away (2 terms for Dhat, 4 for Xhat)
    for v, lo_bits in ((L.view(4, DEV), 1), (L.view(5, DEV), 2)):
        top = float(v[0].abs().max())
        assert 2.0 ** (13 - lo_bits) <= top < 2.0 ** 15, top
    for p in sample_p:
        # the planes add up to the encoded operands Dhat_p = sum_i Delta_i a_p^i, Xhat_p = sum_j X_j b_p^j
        Dh_o = sum(D[i * (N // m):(i + 1) * (N // m)].astype(np.float64) * O.int_power(olp.points[p], olp.eUd[i])
                   for i in range(m))
        Xh_o = sum(X[j * (N // n):(j + 1) * (N // n)].astype(np.float64) * O.int_power(olp.points[p], olp.eUx[j])
                   for j in range(n))
        # hi + lo carries 22 significand bits, the fp32 encode in front of it 24
        assert np.abs(Dh[p] - Dh_o).max() <= 2.0 ** -21 * np.abs(Dh_o).max()
        assert np.abs(Xh[p] - Xh_o).max() <= 2.0 ** -21 * np.abs(Xh_o).max()
    for p in sample_p:
        # update on sampled rows: W~_p[r,:] + eta * Dh_p[r,:] Xh_p^T
        ref = Wt_rows_before[p] + np.float32(0.01) * (Dh[p][rows_s].astype(np.float64) @ Xh[p].astype(np.float64).T)
        got = to_np(Wt[p][torch.from_numpy(rows_s).to(DEV)])
        assert np.abs(got - ref).max() <= 1e-5 * np.abs(ref).max()
    say("  cfg3 L2 backward vs exact: %.3g" % rel_fro(to_np(C), W.astype(np.float64).T @ D))


@pytest.mark.parametrize("regime", ["unit", "tiny", "huge", "spread", "zero", "nonfinite"])
def test_bf16_layer_update_scale_regimes(regime):
    # The update operands of a bf16 layer are two fp16 planes of Dhat_p / 2^E and Xhat_p / 2^E with
    # E taken from the largest finite |Delta| and |X| of the call: the update must keep fp32-level
    # accuracy whatever the magnitude of Delta, and a non-finite entry must stay in its own row.
    say("bf16 update, Delta regime", regime)
    N_out, N_in, batch, m, n, P = 256, 384, 128, 2, 4, 32
    rng = np.random.default_rng(17)
    W = (rng.standard_normal((N_out, N_in)) / 16).astype(np.float32)
    X = rng.uniform(0, 1, (N_in, batch)).astype(np.float32)
    D = rng.standard_normal((N_out, batch)).astype(np.float32)
    if regime == "tiny":
        D = (D * 1e-30).astype(np.float32)
    elif regime == "huge":
        D = (D * 1e25).astype(np.float32)
    elif regime == "spread":
        D = (D * np.exp(rng.uniform(-40, 0, D.shape))).astype(np.float32)
    elif regime == "zero":
        D[:] = 0
    elif regime == "nonfinite":
        D[5, 7] = np.inf
        D[130, 0] = np.nan
    olp = O.make_layer_plan(N_out, N_in, batch, m, n, 1, 1, P, "auto")
    L = G.gpd_layer_create(N_out, N_in, batch, m, n, 1, 1, P, worker_dtype=G.GPD_BF16)
    Wt = G.gpd_layer_encode_weights(L, to_dev(W))
    Wt0 = to_np(Wt).copy()
    # eta such that the update is of the order of the weights (the sum's own fp32 rounding then
    # stays below the bound)
    finite = np.abs(D[np.isfinite(D)])
    eta = np.float32(1.0 if finite.max() == 0 else 2.0 ** -np.ceil(np.log2(finite.max() * 8)))
    G.gpd_coded_layer_step(L, G.GPD_STEP_BACKWARD_UPDATE, Wt, to_dev(X), Dlt=to_dev(D), eta=float(eta), decay=0.0,
                           skip_output=True)
    torch.cuda.synchronize()
    got = to_np(Wt)
    if regime == "nonfinite":
        # Dhat_p rows 5 and 130 - 128 = 2 of every node carry the non-finite entries (m = 2 blocks of
        # 128 rows); every other row is what the same call gives with those two entries at zero
        bad_rows = {5, 2}
        D0 = D.copy()
        D0[5, 7] = 0
        D0[130, 0] = 0
        ref = O.layer_update(Wt0, D0, X, olp, eta, 0.0)
        keep = np.array([r not in bad_rows for r in range(got.shape[1])])
        assert np.isfinite(got[:, keep]).all()
        assert not np.isfinite(got[:, ~keep]).any()
        upd = np.abs(ref - Wt0)[:, keep].max()
        assert np.abs(got[:, keep] - ref[:, keep]).max() <= 2e-6 * upd
        return
    ref = O.layer_update(Wt0, D, X, olp, eta, 0.0)
    if regime == "zero":
        assert np.array_equal(got, Wt0)
        return
    upd = np.abs(ref - Wt0).max()
    err = np.abs(got - ref).max()
    say("  max|err| / max|update| = %.3g (update / weights = %.3g)" % (err / upd, upd / np.abs(Wt0).max()))
    assert err <= 2e-6 * upd


def test_bf16_layer_update_with_points_outside_the_unit_interval():
    # Evaluation points of magnitude up to 1.3 (m = 2, n = 4: Xhat_p sums |b_p|^j up to the cube):
    # the bound on the encode's row sums grows and the exponent leaves more headroom.  Points far
    # outside [-1, 1] (bound above 2^16) make the layer fall back to the three-way bf16 split;
    # both give the oracle's update.
    N_out, N_in, batch, m, n, P = 128, 256, 64, 2, 4, 16
    rng = np.random.default_rng(23)
    W = (rng.standard_normal((N_out, N_in)) / 16).astype(np.float32)
    X = rng.uniform(0, 1, (N_in, batch)).astype(np.float32)
    D = rng.standard_normal((N_out, batch)).astype(np.float32)
    for stretch, fp16 in ((1.3, True), (40.0, False)):
        pts = O.chebyshev_points(P) * stretch
        olp = O.make_layer_plan(N_out, N_in, batch, m, n, 1, 1, P, "auto", points=pts)
        L = G.gpd_layer_create(N_out, N_in, batch, m, n, 1, 1, P, points=pts, worker_dtype=G.GPD_BF16)
        Wt = G.gpd_layer_encode_weights(L, to_dev(W))
        Wt0 = to_np(Wt).copy()
        G.gpd_coded_layer_step(L, G.GPD_STEP_BACKWARD_UPDATE, Wt, to_dev(X), Dlt=to_dev(D), eta=0.01, decay=0.0,
                               skip_output=True)
        torch.cuda.synchronize()
        assert (L.view(4, DEV).dtype == torch.float16) == fp16
        ref = O.layer_update(Wt0, D, X, olp, np.float32(0.01), 0.0)
        upd = np.abs(ref - Wt0).max()
        err = np.abs(to_np(Wt) - ref).max()
        say("  points x %.1f: fp16 planes %s, max|err| / max|update| = %.3g" % (stretch, fp16, err / upd))
        assert err <= 2e-6 * upd + 2.0 ** -23 * np.abs(ref).max()
