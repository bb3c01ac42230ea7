"""GPU parity of encode / worker products / erasure decode against the oracle, element by
element, at sizes that span several tiles and ragged tails (all calls go through the C ABI)."""
import numpy as np
import pytest
import torch

import gpd_workloads as WL
import paper_1811_10751_amd as G
from oracle import gpd_oracle as O
from gpu_util import DEV, rel_fro, say, to_dev, to_np

pytestmark = pytest.mark.gpu

SUB = {"u=v^n": G.GPD_SUB_U_VN, "v=u^m": G.GPD_SUB_V_UM}

SHAPES = [
    # N1, N0, Nc, m, n, d, P, subst
    (256, 256, 256, 2, 2, 2, 10, "u=v^n"),        # cfg0
    (512, 384, 640, 2, 2, 2, 12, "u=v^n"),        # several 128-tiles, K not a multiple of 16*... (192)
    (300, 204, 140, 2, 2, 2, 11, "u=v^n"),        # ragged everywhere: blocks 150 x 102 x 70
    (96, 90, 66, 3, 2, 2, 16, "v=u^m"),           # blocks 32 x 45 x 33: odd widths (scalar path)
    (520, 136, 264, 4, 1, 3, 14, "u=v^n"),        # polynomial-code special case (n = 1)
    (136, 1040, 264, 1, 5, 1, 10, "u=v^n"),       # MatDot special case (m = d = 1)
    (64, 64, 96, 2, 2, 4, 64, "u=v^n"),           # the largest number of nodes (64), K = 17
]


@pytest.mark.parametrize("N1,N0,Nc,m,n,d,P,subst", SHAPES)
def test_encode_products_decode_stagewise(N1, N0, Nc, m, n, d, P, subst):
    say("case", N1, N0, Nc, m, n, d, P, subst)
    A, B = WL.matmul_inputs(N1, N0, Nc, seed=N1 + N0)
    opl = O.make_plan(m, n, d, P, subst)
    plan = G.gpd_plan(N1, N0, Nc, m, n, d, P, subst=SUB[subst])
    assert plan.K == opl.K and plan.t_max == max(0, P - opl.K - 1)
    pts, eA, eB, eC = plan.tables()
    assert np.array_equal(eA, opl.eA) and np.array_equal(eB, opl.eB) and np.array_equal(eC, opl.eC)

    # ---- encode: fp32 linear combinations of <= mn blocks with |coef| <= 1
    At, Bt = G.gpd_encode(plan, to_dev(A), to_dev(B))
    torch.cuda.synchronize()
    At_o, Bt_o = O.encode_A(A, opl), O.encode_B(B, opl)
    assert np.abs(to_np(At) - At_o).max() <= 4e-7 * m * n
    assert np.abs(to_np(Bt) - Bt_o).max() <= 4e-7 * n * d

    # ---- products: oracle multiplies the GPU's own fp32 operands (data shared, code not)
    Ct = G.gpd_worker_products(plan, At, Bt)
    torch.cuda.synchronize()
    Ct_o = O.worker_products(to_np(At), to_np(Bt))
    kdim = N0 // n
    bound = 2.0 ** -23 * np.sqrt(kdim) * 4 * np.sqrt((to_np(At).astype(np.float64) ** 2).sum(axis=2).max() *
                                                   (to_np(Bt).astype(np.float64) ** 2).sum(axis=1).max() / kdim)
    assert np.abs(to_np(Ct) - Ct_o).max() <= max(bound, 1e-6), (np.abs(to_np(Ct) - Ct_o).max(), bound)
    assert rel_fro(to_np(Ct), Ct_o) < 2e-6

    # ---- decode: oracle decodes the GPU's own responses
    rng = np.random.default_rng(7)
    masks = [None]
    if P > opl.K:
        pm = np.ones(P, dtype=np.uint8)
        pm[rng.choice(P, P - opl.K, replace=False)] = 0
        masks.append(pm)
    for present in masks:
        for mode, oname in ((G.GPD_DEC_FIRST_K, "first_k"), (G.GPD_DEC_LSQ_ALL, "lsq_all")):
            C, rep = G.gpd_decode(plan, Ct, present=present, mode=mode)
            C_o, _ = O.decode(to_np(Ct), opl, present, oname)
            amp = O.amplification(opl, present, oname)
            err = rel_fro(to_np(C), C_o)
            say("  decode", "all" if present is None else "erasures", oname, "amp %.3g err %.3g" % (amp, err))
            assert err <= 1e-6 * max(amp, 1.0)
            assert rep.n_present == (P if present is None else int(present.sum()))
    # end to end against the definition A.B (first K, as cfg0 asks), 1e-3 where the erasure set allows
    C, _ = G.gpd_decode(plan, Ct, mode=G.GPD_DEC_FIRST_K)
    e2e = rel_fro(to_np(C), O.uncoded_matmul(A, B))
    amp = O.amplification(opl, None, "first_k")
    say("  end-to-end vs A.B: %.3g (amp %.3g)" % (e2e, amp))
    if amp < 1e6:
        assert e2e <= max(1e-3, 4 * amp * 2.0 ** -21)
    else:
        # the first K of 64 Chebyshev points sit in a corner of the interval: nothing can be decoded
        # from them in fp32; least squares over all nodes still gives the product
        C, _ = G.gpd_decode(plan, Ct, mode=G.GPD_DEC_LSQ_ALL)
        amp_all = O.amplification(opl, None, "lsq_all")
        assert rel_fro(to_np(C), O.uncoded_matmul(A, B)) <= max(1e-3, 4 * amp_all * 2.0 ** -21)


def test_too_few_responses_and_bad_arguments():
    plan = G.gpd_plan(64, 64, 64, 2, 2, 2, 12)
    Ct = torch.zeros((12, 32, 32), device=DEV)
    present = np.zeros(12, dtype=np.uint8)
    present[:8] = 1
    with pytest.raises(G.GpdError) as e:
        G.gpd_decode(plan, Ct, present=present)
    assert e.value.status == G.GPD_E_TOO_FEW
    with pytest.raises(G.GpdError) as e:
        G.gpd_plan(65, 64, 64, 2, 2, 2, 12)
    assert e.value.status == G.GPD_E_SHAPE
    with pytest.raises(G.GpdError) as e:
        G.gpd_plan(64, 64, 64, 2, 2, 2, 8)
    assert e.value.status == G.GPD_E_SHAPE
    with pytest.raises(G.GpdError) as e:
        G.gpd_decode(plan, Ct, correct_errors=True, workspace=torch.zeros(16, dtype=torch.uint8, device=DEV))
    assert e.value.status == G.GPD_E_WORKSPACE


def test_empty_matrices():
    plan = G.gpd_plan(0, 64, 64, 2, 2, 2, 12)
    A = torch.zeros((0, 64), device=DEV)
    B = torch.rand((64, 64), device=DEV)
    At, Bt = G.gpd_encode(plan, A, B)
    Ct = G.gpd_worker_products(plan, At, Bt)
    C, _ = G.gpd_decode(plan, Ct)
    torch.cuda.synchronize()
    assert C.shape == (0, 64)


def test_strided_inputs_and_outputs():
    # A, B and C are windows of larger buffers (leading dimension > row length)
    N1, N0, Nc = 128, 96, 160
    A, B = WL.matmul_inputs(N1, N0, Nc, seed=5)
    bigA = torch.zeros((N1, N0 + 8), device=DEV)
    bigB = torch.zeros((N0, Nc + 4), device=DEV)
    bigA[:, :N0] = to_dev(A)
    bigB[:, :Nc] = to_dev(B)
    plan = G.gpd_plan(N1, N0, Nc, 2, 2, 2, 12)
    At, Bt = G.gpd_encode(plan, bigA[:, :N0], bigB[:, :Nc])
    Ct = G.gpd_worker_products(plan, At, Bt)
    bigC = torch.full((N1, Nc + 12), 7.0, device=DEV)
    G.gpd_decode(plan, Ct, mode=G.GPD_DEC_LSQ_ALL, C_out=bigC[:, :Nc])
    torch.cuda.synchronize()
    assert rel_fro(to_np(bigC[:, :Nc]), O.uncoded_matmul(A, B)) < 1e-4
    assert torch.all(bigC[:, Nc:] == 7.0)
