"""Seeded sweep over random valid shapes: the stage-wise parity tests of the matmul path and of the
layer step (fp32, bf16 and split workers) called with shapes nobody picked by hand: block grids
from 1 x 1 to 4 x 4, ragged sizes, per-node batches on and off the streaming path, codes from
P = K (no redundancy) to P = K + 8."""
import numpy as np
import pytest

from oracle import gpd_oracle as O
import test_gpu_bf16 as TB
import test_gpu_layer as TL
import test_gpu_matmul as TM
import test_gpu_split as TS
from gpu_util import say

pytestmark = pytest.mark.gpu


def cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    it = 0
    while len(out) < count:
        kind = it % 6
        it += 1
        if kind in (0, 3, 4):
            m, n, d = (int(rng.integers(1, 4)) for _ in range(3))
            K = m * n * d + n - 1
            if K > 14:
                continue
            P = K + int(rng.integers(0, 7))
            hi = 520 if (kind != 0 and rng.random() < 0.5) else 200
            N1, N0, Nc = (q * int(rng.integers(1, hi // q + 1)) for q in (m, n, d))
            out.append((kind, (N1, N0, Nc, m, n, d, P)))
        else:
            m, n = int(rng.integers(1, 5)), int(rng.integers(1, 5))
            d1, d2 = int(rng.integers(1, 3)), int(rng.integers(1, 3))
            pool = [1, 2, 4, 8, 16, 24, 48] if kind == 1 else [1, 2, 4, 8, 6, 12, 24, 64, 128, 192]
            batch = int(rng.choice(pool))
            if batch % d1 or batch % d2:
                d1 = d2 = 1
            N_out, N_in = int(rng.integers(3, 400)), int(rng.integers(3, 400))
            lp = O.make_layer_plan(N_out, N_in, batch, m, n, d1, d2, 64, "auto")
            K = max(lp.Kf, lp.Kb)
            if K > 14:
                continue
            out.append((kind, (N_out, N_in, batch, m, n, d1, d2, K + int(rng.integers(0, 9)))))
    return out


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_shapes(seed):
    for kind, a in cases(seed, 36):
        say("sweep", seed, kind, a)
        if kind == 0:
            TM.test_encode_products_decode_stagewise(*a, "u=v^n")
        elif kind == 3:
            TB.test_bf16_matmul_stagewise(*a)
        elif kind == 4:
            TS.test_split_products_are_fp32_accurate(*a)
        elif kind == 1:
            TL.test_layer_forward_backward_update(*a, "auto")
        elif kind == 2:
            TB.test_bf16_layer_stagewise(*a)
        else:
            TS.test_split_layer_step(*a)


@pytest.mark.parametrize("seed,locator", [(21, "search"), (22, "search"), (23, "l1"), (24, "l1")])
def test_random_soft_errors(seed, locator):
    """Random codes (K <= 12, P - K from 2 to 8), random erasures, and in up to a quarter of the
    codewords between 0 and one more error than Algorithm 1 can correct: offsets, huge values,
    non-finite values and single bit flips.  The GPU must take the oracle's decisions exactly, with
    Algorithm 1's search and with the L1 relaxation in its place."""
    import test_gpu_errors as TE
    import paper_1811_10751_amd as G
    from gpu_util import to_dev, to_np
    rng = np.random.default_rng(seed)
    done = 0
    mode = G.GPD_CORRECT_ELEMENTS_L1 if locator == "l1" else G.GPD_CORRECT_ELEMENTS
    while done < (16 if locator == "l1" else 30):
        m, n, d = (int(rng.integers(1, 4)) for _ in range(3))
        K = m * n * d + n - 1
        if K > 12:
            continue
        r = int(rng.integers(2, 9))
        P = K + r
        N1, N0, Nc = (q * int(rng.integers(2, 20)) for q in (m, n, d))
        A, B, plan, Ct = TE.gpu_responses(N1, N0, Nc, m, n, d, P, seed * 1000 + done)
        Ct_h = to_np(Ct).copy()
        n_er = int(rng.integers(0, max(1, r - 1)))
        present = np.ones(P, dtype=np.uint8)
        if n_er:
            present[rng.choice(P, n_er, replace=False)] = 0
        room = r - n_er - 1                       # errors Algorithm 1 can correct per codeword
        rows, cols = Ct_h.shape[1:]
        ncw = rows * cols
        nbad = int(rng.integers(0, max(2, ncw // 4)))
        for cw in rng.choice(ncw, nbad, replace=False):
            t = int(rng.integers(0, room + 2))
            for p in rng.choice(np.flatnonzero(present), min(t, int(present.sum())), replace=False):
                i, j = cw // cols, cw % cols
                v = Ct_h[p, i, j]
                how = rng.integers(0, 4)
                if how == 0:
                    Ct_h[p, i, j] = v + np.float32(rng.standard_normal() * 10 * (abs(v) + 1))
                elif how == 1:
                    Ct_h[p, i, j] = np.float32(rng.standard_normal() * 1e20)
                elif how == 2:
                    Ct_h[p, i, j] = np.float32(np.inf if rng.random() < .5 else np.nan)
                else:
                    w = np.array([v], dtype=np.float32).view(np.uint32)
                    w ^= np.uint32(1 << int(rng.integers(0, 32)))
                    Ct_h[p, i, j] = w.view(np.float32)[0]
        say("soft-error sweep", seed, (N1, N0, Nc, m, n, d, P), "erasures", n_er, "codewords hit", nbad)
        opl = O.make_plan(m, n, d, P)
        C_o, orep = O.decode(Ct_h, opl, present, correct=True, locator=locator)
        C, rep = G.gpd_decode(plan, to_dev(Ct_h), present=present, mode=G.GPD_DEC_LSQ_ALL, correct_errors=mode,
                              located_cap=100000)
        TE.compare_reports(rep, orep, P)
        TE.check_outputs(C, C_o, orep, plan, tol=max(2e-5, 1e-6 * O.amplification(opl, present, "lsq_all")))
        done += 1


@pytest.mark.parametrize("seed", [31])
def test_random_node_searches(seed):
    """Random codes up to P = 64 nodes with absent nodes and up to four erroneous ones (kept small
    enough for the oracle's exhaustive search): Gram matrix, threshold and located set."""
    from math import comb
    import test_gpu_nodes as TN
    rng = np.random.default_rng(seed)
    for _ in range(40):
        K = int(rng.integers(1, 25))
        P = K + int(rng.integers(0, min(40, 64 - K) + 1))
        n_abs = int(rng.integers(0, min(4, P - K) + 1))
        present_n = P - n_abs
        t = int(rng.integers(0, max(0, min(present_n - K - 1, 4)) + 1))
        while t > 0 and comb(present_n, t) > 1000:
            t -= 1
        nodes = rng.permutation(P)
        absent = tuple(sorted(int(x) for x in nodes[:n_abs]))
        bad = tuple(sorted(int(x) for x in nodes[n_abs:n_abs + t]))
        rows, cols = int(rng.integers(1, 70)), int(rng.integers(1, 70))
        if rows * cols < 8 * max(1, t):
            rows, cols = 16, 16                  # enough codewords to tell the nodes apart
        TN.test_gram_matrix_and_node_search(P, K, rows, cols, bad, absent)


@pytest.mark.parametrize("seed", [41])
def test_random_projections(seed):
    """Projection of a drifted weight stack onto the code for random block grids, node counts on
    both sides of 32 (matrix-core kernel / vector-unit kernel), block sizes on and off a multiple of
    128 elements, and absent nodes whose blocks hold garbage."""
    import torch
    import paper_1811_10751_amd as G
    from gpu_util import to_dev, to_np
    rng = np.random.default_rng(seed)
    done = 0
    while done < 40:
        m, n = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        K = m * n
        P = min(K + int(rng.integers(1, 33)), 40 if rng.random() < 0.2 else 32)
        if P <= K:
            continue
        wr, wc = int(rng.choice([4, 8, 16, 32, 48, 64])), int(rng.choice([8, 16, 32, 64, 96, 128]))
        if rng.random() < 0.2:
            wc += 3
        N_out, N_in = wr * m, wc * n
        try:
            olp = O.make_layer_plan(N_out, N_in, 1, m, n, 1, 1, P, "auto")
        except ValueError:                       # too few nodes for the layer's backward product
            continue
        L = G.gpd_layer_create(N_out, N_in, 1, m, n, 1, 1, P)
        W = (rng.standard_normal((N_out, N_in)) / 8).astype(np.float32)
        Wt = G.gpd_layer_encode_weights(L, to_dev(W))
        clean = to_np(Wt).copy()
        n_abs = int(rng.integers(0, P - K + 1)) if rng.random() < 0.6 else 0
        present = np.ones(P, dtype=np.uint8)
        if n_abs:
            present[rng.choice(P, n_abs, replace=False)] = 0
        noisy = clean + (rng.standard_normal(clean.shape) * 1e-3).astype(np.float32)
        noisy[present == 0] = 777.0
        say("projection sweep", (N_out, N_in, m, n, P), "absent", n_abs, "block", wr * wc)
        Wt.copy_(to_dev(noisy))
        G.gpd_layer_project(L, Wt, present if n_abs else None)
        torch.cuda.synchronize()
        ref = O.layer_project(noisy, olp, present if n_abs else None)
        V = O.vandermonde(olp.points[present.astype(bool)], K)
        amp = max(np.abs(O.vandermonde(olp.points, K) @ np.linalg.pinv(V)).sum(axis=1).max(), 1.0)
        assert np.abs(to_np(Wt) - ref).max() <= 4e-6 * amp * np.abs(clean).max()
        L.close()
        done += 1
