"""GPU parity of the three-way bf16 split of fp32 products (GPD_F32_SPLIT): the same bars as the
fp32 MFMA path (the oracle multiplies the GPU's own fp32 operands in fp64), and a side-by-side
of the two paths' errors on the same operands."""
import numpy as np
import pytest
import torch

import gpd_workloads as WL
import paper_1811_10751_amd as G
from oracle import gpd_oracle as O
from gpu_util import DEV, rel_fro, say, to_dev, to_np

pytestmark = pytest.mark.gpu

SHAPES = [
    (256, 256, 256, 2, 2, 2, 12),       # 128-tiles, full
    (1024, 2048, 1024, 2, 2, 2, 16),    # 16 x 4 tiles of 256: the large shape, K = 1024
    (300, 204, 140, 2, 2, 2, 11),       # ragged
    (264, 520, 136, 1, 4, 1, 9),        # long contraction, n = 4
    (256, 96, 256, 2, 2, 2, 12),        # full tiles, 3 stages of 16 k (odd: bounds-checked kernel)
    (2048, 2048, 2048, 2, 2, 2, 16),    # 256 tiles of 256 x 256: the 8-wavefront shape, 64 stages
    (2048, 2080, 2048, 2, 2, 2, 16),    # the same with 65 stages (odd: small shape)
]


@pytest.mark.parametrize("N1,N0,Nc,m,n,d,P", SHAPES)
def test_split_products_are_fp32_accurate(N1, N0, Nc, m, n, d, P):
    say("split matmul", N1, N0, Nc, m, n, d, P)
    A, B = WL.matmul_inputs(N1, N0, Nc, seed=N1 + 1)
    opl = O.make_plan(m, n, d, P)
    plan_s = G.gpd_plan(N1, N0, Nc, m, n, d, P, worker_dtype=G.GPD_F32_SPLIT)
    plan_f = G.gpd_plan(N1, N0, Nc, m, n, d, P)
    At, Bt = G.gpd_encode(plan_s, to_dev(A), to_dev(B))
    assert At.dtype == torch.float32 and Bt.dtype == torch.float32
    Ct_s = G.gpd_worker_products(plan_s, At, Bt)
    Ct_f = G.gpd_worker_products(plan_f, At, Bt)
    torch.cuda.synchronize()
    Ct_o = O.worker_products(to_np(At), to_np(Bt))
    kdim = N0 // n
    bound = 2.0 ** -23 * np.sqrt(kdim) * 4 * np.sqrt((to_np(At).astype(np.float64) ** 2).sum(axis=2).max() *
                                                   (to_np(Bt).astype(np.float64) ** 2).sum(axis=1).max() / kdim)
    err_s, err_f = np.abs(to_np(Ct_s) - Ct_o).max(), np.abs(to_np(Ct_f) - Ct_o).max()
    rf_s, rf_f = rel_fro(to_np(Ct_s), Ct_o), rel_fro(to_np(Ct_f), Ct_o)
    say("  max abs err split %.3g fp32 MFMA %.3g (bound %.3g); rel Frobenius split %.3g fp32 MFMA %.3g"
        % (err_s, err_f, bound, rf_s, rf_f))
    assert err_s <= max(bound, 1e-6)                     # the bar of the fp32 path
    assert rf_s < 2e-6
    assert rf_s <= 2.0 * rf_f + 1e-8                     # and no worse than the fp32 MFMA path
    # end to end through the decoder
    C, _ = G.gpd_decode(plan_s, Ct_s, mode=G.GPD_DEC_LSQ_ALL)
    C_o, _ = O.decode(to_np(Ct_s), opl, None, "lsq_all")
    assert rel_fro(to_np(C), C_o) <= 1e-6 * max(O.amplification(opl, None, "lsq_all"), 1.0)
    assert rel_fro(to_np(C), O.uncoded_matmul(A, B)) < 1e-3


def test_split_handles_wide_dynamic_range():
    # entries over 60 binades, both signs: the low planes must keep their bits through bf16
    rng = np.random.default_rng(3)
    N = 256
    A = (rng.standard_normal((N, N)) * 2.0 ** rng.integers(-30, 30, (N, N))).astype(np.float32)
    B = (rng.standard_normal((N, N)) * 2.0 ** rng.integers(-30, 30, (N, N))).astype(np.float32)
    ref = A.astype(np.float64) @ B.astype(np.float64)
    mag = np.abs(A.astype(np.float64)) @ np.abs(B.astype(np.float64))
    worst = {}
    for name, dt in (("split", G.GPD_F32_SPLIT), ("fp32 MFMA", G.GPD_F32)):
        plan = G.gpd_plan(N, N, N, 1, 1, 1, 1, worker_dtype=dt)                 # one node: C~_0 = A B
        Ct = G.gpd_worker_products(plan, to_dev(A).reshape(1, N, N), to_dev(B).reshape(1, N, N))
        torch.cuda.synchronize()
        worst[name] = float((np.abs(to_np(Ct)[0] - ref) / mag).max())
    say("  worst |error| / (|A| |B|): split 2^%.1f, fp32 MFMA 2^%.1f"
        % (np.log2(worst["split"]), np.log2(worst["fp32 MFMA"])))
    # the matrix cores align the 16 products of a step to the largest one and truncate, so the
    # error is relative to |A| |B|, a few units in the 24th bit per step of the contraction
    assert worst["split"] <= 2.0 ** -19
    assert worst["split"] <= 4.0 * worst["fp32 MFMA"]


LAYERS = [(256, 384, 128, 2, 4, 1, 1, 32), (300, 200, 24, 2, 4, 1, 1, 32), (130, 260, 48, 2, 2, 2, 3, 20),
          (300, 200, 64, 2, 4, 1, 1, 32), (512, 1024, 192, 2, 4, 1, 1, 32)]


@pytest.mark.parametrize("N_out,N_in,batch,m,n,d1,d2,P", LAYERS)
def test_split_layer_step(N_out, N_in, batch, m, n, d1, d2, P):
    # forward, backward and update of a GPD_F32_SPLIT layer against the fp64 oracle, with the
    # tolerances of the fp32 layer tests
    say("split layer", N_out, N_in, batch, m, n, d1, d2, P)
    rng = np.random.default_rng(N_out + N_in)
    W = (rng.standard_normal((N_out, N_in)) / np.sqrt(N_in)).astype(np.float32)
    X = rng.uniform(-1, 1, (N_in, batch)).astype(np.float32)
    D = rng.standard_normal((N_out, batch)).astype(np.float32)
    olp = O.make_layer_plan(N_out, N_in, batch, m, n, d1, d2, P, "auto")
    L = G.gpd_layer_create(N_out, N_in, batch, m, n, d1, d2, P, worker_dtype=G.GPD_F32_SPLIT)
    Wt = G.gpd_layer_encode_weights(L, to_dev(W))
    Wt_h = to_np(Wt).copy()
    S, _ = G.gpd_coded_layer_step(L, G.GPD_STEP_FORWARD, Wt, to_dev(X))
    torch.cuda.synchronize()
    St_o = O.worker_products(Wt_h, to_np(L.view(0, DEV)))
    assert rel_fro(to_np(L.view(1, DEV)), St_o) < 2e-6
    ampf = O.amplification(olp.fwd, None, "lsq_all")
    assert rel_fro(to_np(S), W.astype(np.float64) @ X) <= 1e-6 * max(ampf, 100.0)
    eta, decay = 0.05, 0.01
    C, _ = G.gpd_coded_layer_step(L, G.GPD_STEP_BACKWARD_UPDATE, Wt, to_dev(X), Dlt=to_dev(D), eta=eta, decay=decay)
    torch.cuda.synchronize()
    Dt, Ct = to_np(L.view(2, DEV)), to_np(L.view(3, DEV))
    Ct_o = np.matmul(np.transpose(Wt_h.astype(np.float64), (0, 2, 1)), Dt.astype(np.float64))
    assert rel_fro(Ct, Ct_o) < 2e-6
    Db = np.linalg.pinv(O.vandermonde(olp.points, olp.Kb))
    ampb = max(np.linalg.norm(Db[int(e)]) for e in olp.eCb.ravel())
    assert rel_fro(to_np(C), W.astype(np.float64).T @ D) <= 1e-6 * max(ampb, 100.0)
    Wt2_o = O.layer_update(Wt_h, D, X, olp, eta, np.float32(decay))
    assert np.abs(to_np(Wt) - Wt2_o).max() <= 2e-6 * np.abs(Wt2_o).max()
