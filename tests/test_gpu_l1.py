"""GPU parity of error location by L1-norm relaxation (GPD_CORRECT_ELEMENTS_L1; remark after
Thm 3): the kernel solves the linear program min ||e||_1 s.t. H e = H z by simplex steps on the
equivalent least-absolute-deviations fit, the oracle hands it to a general LP solver; both rank
the nodes by |e*| and accept the first prefix of the ranking that meets Algorithm 1's criterion.
Decisions (flagged, located, failed: per codeword) must agree, outputs within tolerance."""
import numpy as np
import pytest
import torch

import gpd_workloads as WL
import paper_1811_10751_amd as G
from oracle import gpd_oracle as O
from gpu_util import DEV, rel_fro, say, to_dev, to_np
from test_gpu_errors import check_outputs, compare_reports, flip_on_gpu, gpu_responses
from test_gpu_algebraic import plant

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("P", [12, 16, 24, 48])
def test_l1_locator_matches_the_oracle(P):
    m = n = d = 2
    N1, N0, Nc = 64, 32, 32
    A, B, plan, Ct = gpu_responses(N1, N0, Nc, m, n, d, P, seed=100 + P)
    K, r = plan.K, P - plan.K
    rows, cols = N1 // m, Nc // d
    rng = np.random.default_rng(P)
    t_list = [1 + (i % min(r - 1, 6)) for i in range(48)]
    flat = rng.choice(rows * cols, len(t_list), replace=False)
    positions = [(int(f) // cols, int(f) % cols) for f in flat]
    bad, planted = plant(Ct, rng, positions, t_list, scale_lo=-0.5, scale_hi=1.0)
    C, rep = G.gpd_decode(plan, bad, mode=G.GPD_DEC_LSQ_ALL, correct_errors=G.GPD_CORRECT_ELEMENTS_L1,
                          located_cap=4096)
    opl = O.make_plan(m, n, d, P)
    C_o, orep = O.decode(to_np(bad), opl, None, "lsq_all", True, locator="l1")
    say("  P=%d K=%d r=%d: flagged %d located %d failed %d (oracle: located %d failed %d)"
        % (P, K, r, rep.n_flagged, rep.n_located, rep.n_failed, len(orep.located), orep.n_failed))
    compare_reports(rep, orep, P)
    check_outputs(C, C_o, orep, plan, tol=1e-6 * max(O.amplification(opl, None, "lsq_all"), 20.0))
    # how much of what was planted the relaxation finds, by number of errors in the codeword
    got = {}
    for (node, rr_, cc_, mag) in rep.located:
        got.setdefault((rr_, cc_), []).append(node)
    hits = {}
    for pos, t in zip(positions, t_list):
        ok = pos in got and tuple(sorted(got[pos])) == planted[pos]
        hits.setdefault(t, [0, 0])
        hits[t][0] += ok
        hits[t][1] += 1
    say("  recovered / planted by errors per codeword:", {t: tuple(v) for t, v in sorted(hits.items())})
    assert rep.n_flagged == len(t_list)
    assert hits[1][0] >= 0.6 * hits[1][1]                 # single errors: most are found
    # the search locates all of these where the relaxation gives up on some
    C_s, rep_s = G.gpd_decode(plan, bad, mode=G.GPD_DEC_LSQ_ALL, correct_errors=True, located_cap=4096)
    assert rep_s.n_failed == 0 and rep_s.n_located == sum(t_list)
    assert rep.n_failed + rep.n_located >= 1 and rep.n_located <= rep_s.n_located + 2 * len(t_list)


def test_l1_locator_with_non_finite_entries_and_erasures():
    P, m, n, d = 24, 2, 2, 2
    N1, N0, Nc = 64, 32, 32
    A, B, plan, Ct = gpu_responses(N1, N0, Nc, m, n, d, P, seed=7)
    rng = np.random.default_rng(8)
    positions = [(3, 4), (10, 11), (20, 2), (31, 15), (0, 0)]
    present = np.ones(P, dtype=np.uint8)
    present[[2, 17]] = 0
    bad = Ct.clone()
    for k, (r_, c_) in enumerate(positions):
        nodes = [q for q in rng.permutation(P) if present[q]][:k + 2]
        bad[int(nodes[0]), r_, c_] = float("inf") if k % 2 else float("nan")
        for q in nodes[1:1 + (k % 3)]:
            bad[int(q), r_, c_] += 25.0
        if k == 4:
            for q in nodes[1:]:
                bad[int(q), r_, c_] = float("nan")         # 6 non-finite entries: all the code can take but one
    # (values on absent nodes are never read)
    bad[2] = float("nan")
    C, rep = G.gpd_decode(plan, bad, present=present, mode=G.GPD_DEC_LSQ_ALL,
                          correct_errors=G.GPD_CORRECT_ELEMENTS_L1, located_cap=1000)
    opl = O.make_plan(m, n, d, P)
    bad_h = to_np(bad)
    bad_h[2] = 0.0
    C_o, orep = O.decode(bad_h, opl, present, "lsq_all", True, locator="l1")
    say("  flagged %d located %d failed %d" % (rep.n_flagged, rep.n_located, rep.n_failed))
    compare_reports(rep, orep, P)
    check_outputs(C, C_o, orep, plan, tol=1e-6 * max(O.amplification(opl, present, "lsq_all"), 20.0))
    assert rep.n_flagged == 5 and rep.n_failed == 0


def test_l1_locator_full_size_bit_flips():
    # the soft-error workload at full size (4096^2, P = 16, 2048^2 codewords per trial), 150 of its
    # seeded trials in L1 mode: per trial the oracle decodes exactly the touched codewords
    c = WL.CONFIGS[4]
    A, B, plan, Ct = gpu_responses(c["N1"], c["N0"], c["Nc"], c["m"], c["n"], c["d"], c["P"], c["seed"])
    opl = O.make_plan(c["m"], c["n"], c["d"], c["P"])
    rows = cols = 2048
    ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device=DEV)
    C0, rep0 = G.gpd_decode(plan, Ct, mode=G.GPD_DEC_LSQ_ALL, correct_errors=G.GPD_CORRECT_ELEMENTS_L1, workspace=ws)
    assert rep0.n_flagged == 0 and rep0.status == G.GPD_OK
    Cf = Ct.clone()
    C = torch.empty_like(C0)
    Ct_flat = Ct.view(16, -1)
    useful = sorted(int(e) for e in opl.eC.ravel())
    n_flips = n_loc = n_fail = 0
    for t in range(150):
        flips = WL.bitflip_trial(c["trial_seed0"] + t, c["P"], rows * cols, c["P"] - plan.K - 1, c["flip_prob"])
        flip_on_gpu(Cf, flips, cols)
        _, rep = G.gpd_decode(plan, Cf, mode=G.GPD_DEC_LSQ_ALL, correct_errors=G.GPD_CORRECT_ELEMENTS_L1,
                              workspace=ws, C_out=C)
        elems = sorted(set(e for (_, e, _) in flips))
        if elems:
            sub = to_np(Ct_flat[:, torch.tensor(elems, device=DEV)]).reshape(16, 1, len(elems)).copy()
            sub_f = WL.apply_bitflips(sub, [(p, elems.index(e), b) for (p, e, b) in flips])
            coeffs, orep = O.decode_coefficients(sub_f, opl.points, opl.K, useful, correct=True, locator="l1")
            want = [(node, elems[cc] // cols, elems[cc] % cols) for (node, _, cc, _) in orep.located]
            assert sorted(want) == [x[:3] for x in rep.located], (t, flips)
            assert rep.n_flagged == orep.n_flagged and rep.n_failed == orep.n_failed
            failed = set(cc for (_, cc) in orep.failed)
            for cc, e in enumerate(elems):
                if cc in failed:
                    continue
                r_, c_ = divmod(e, cols)
                for i in range(2):
                    for k in range(2):
                        o = coeffs[int(opl.eC[i, k])][0, cc]
                        g = float(C[i * rows + r_, k * cols + c_])
                        assert np.isfinite(g) and abs(g - o) <= 1e-3 * max(1.0, abs(o)), (t, e, g, o)
            n_fail += rep.n_failed
        else:
            assert rep.n_flagged == 0 and rep.n_located == 0
        n_flips += len(flips)
        n_loc += rep.n_located
        flip_on_gpu(Cf, flips, cols)             # undo
    say("L1, full size: 150 trials,", n_flips, "flips,", n_loc, "located,", n_fail, "codewords given up")
    assert torch.equal(Cf, Ct)
    assert n_loc > 30


def test_layer_forward_with_l1_correction_and_static_decode():
    # the same locator behind the two other entry points that take a correction mode: the coded
    # layer step (stragglers + one node whose stored W~_p was corrupted: one error in every
    # codeword) and the decode that allocates nothing
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
    S, rep = G.gpd_coded_layer_step(L, G.GPD_STEP_FORWARD, Wt, to_dev(X), present=present,
                                    correct_errors=G.GPD_CORRECT_ELEMENTS_L1, want_report=True)
    St_o = O.worker_products(to_np(Wt), O.layer_encode_x(X, olp))
    S_o, orep = O.decode(St_o, olp.fwd, present, "lsq_all", True, locator="l1")
    say("  layer: flagged %d located %d failed %d (oracle %d %d)"
        % (rep.n_flagged, rep.n_located, rep.n_failed, len(orep.located), orep.n_failed))
    assert rep.n_flagged == orep.n_flagged and rep.n_failed == orep.n_failed
    assert [x[:3] for x in rep.located] == [x[:3] for x in orep.located]
    assert rep.n_located > 0 and set(x[0] for x in rep.located) == {7}
    assert orep.n_failed == 0                              # (node 7 is one the relaxation finds in every codeword)
    assert rel_fro(to_np(S), S_o[:N_out]) < 1e-4

    # gpd_decode_static in L1 mode against gpd_decode in L1 mode
    m = n = d = 2
    A, B, plan, Ct = gpu_responses(64, 32, 32, m, n, d, 16, seed=5)
    bad_ct, planted = plant(Ct, np.random.default_rng(6), [(1, 2), (7, 3), (30, 15)], [1, 2, 1], 0.0, 1.0)
    C1, rep1 = G.gpd_decode(plan, bad_ct, mode=G.GPD_DEC_LSQ_ALL, correct_errors=G.GPD_CORRECT_ELEMENTS_L1)
    C2 = torch.empty_like(C1)
    _, rep2 = G.gpd_decode_static(plan, bad_ct, C2, mode=G.GPD_DEC_LSQ_ALL, correct_errors=G.GPD_CORRECT_ELEMENTS_L1)
    assert rep1.n_flagged == rep2.n_flagged == 3 and rep1.n_failed == rep2.n_failed
    assert [x[:3] for x in rep1.located] == [x[:3] for x in rep2.located]
    assert torch.equal(C1, C2)
