"""Pins for the oracle's encode -> products -> decode path: the method must reproduce the
plain product A B (the definition) from any K of the P node outputs."""
import itertools

import numpy as np
import pytest
import torch

import gpd_workloads as WL
from oracle import gpd_oracle as O


def triple_loop_matmul(A, B):
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    C = np.zeros((A.shape[0], B.shape[1]))
    for i in range(A.shape[0]):
        for k in range(B.shape[1]):
            s = 0.0
            for j in range(A.shape[1]):
                s += A[i, j] * B[j, k]
            C[i, k] = s
    return C


@pytest.mark.parametrize("subst", ["u=v^n", "v=u^m"])
def test_every_K_subset_recovers_the_product(subst):
    # Thm 2: any mnd+n-1 of the P evaluations interpolate the product polynomial
    A, B = WL.matmul_inputs(8, 12, 6, seed=11)       # non-square on purpose: catches transposes
    pl = O.make_plan(2, 2, 2, 12 if subst == "u=v^n" else 13, subst)
    C_ref = triple_loop_matmul(A, B)
    Ct = O.worker_products(O.encode_A(A, pl), O.encode_B(B, pl))
    n_sub = 0
    for S in itertools.combinations(range(pl.P), pl.K):
        present = np.zeros(pl.P, dtype=np.uint8)
        present[list(S)] = 1
        C, _ = O.decode(Ct, pl, present, "first_k")
        amp = O.amplification(pl, present)
        assert np.abs(C - C_ref).max() <= 1e-13 * amp * 64, (S, amp)
        n_sub += 1
    assert pl.K == (9 if subst == "u=v^n" else 10)
    assert n_sub == (220 if subst == "u=v^n" else 286)   # C(12,9), C(13,10)


@pytest.mark.parametrize("m,n,d", [(1, 1, 1), (4, 1, 3), (1, 5, 1), (3, 2, 1), (2, 3, 2)])
def test_shapes_and_special_cases(m, n, d):
    # includes the Polynomial-code (n=1) and MatDot (m=d=1) special cases of Sec. IV
    A, B = WL.matmul_inputs(m * 3, n * 4, d * 5, seed=m * 100 + n * 10 + d)
    pl = O.make_plan(m, n, d, m * n * d + n + 2)
    C_ref = O.uncoded_matmul(A, B)
    for mode in ("first_k", "lsq_all"):
        C, rep = O.coded_matmul(A, B, pl, mode=mode)
        assert np.abs(C - C_ref).max() < 1e-8
    present = np.ones(pl.P, dtype=np.uint8)
    present[[0, 2, pl.P - 1]] = 0                          # exactly P-K = 3 erasures (the tolerated number)
    C, rep = O.coded_matmul(A, B, pl, present=present)
    assert rep.n_present == pl.K and np.abs(C - C_ref).max() < 1e-8
    present[1] = 0
    with pytest.raises(O.TooFewResponses):
        O.coded_matmul(A, B, pl, present=present)


def test_matdot_answer_is_the_middle_coefficient():
    # Sec. III MatDot: S is the coefficient of v^(K-1); every other coefficient is garbage
    A, B = WL.matmul_inputs(5, 8, 7, seed=3)
    pl = O.make_plan(1, 4, 1, 9)
    Ct = O.worker_products(O.encode_A(A, pl), O.encode_B(B, pl))
    coeffs, _ = O.decode_coefficients(Ct, pl.points, pl.K, range(pl.K), mode="lsq_all")
    assert np.abs(coeffs[3] - O.uncoded_matmul(A, B)).max() < 1e-10
    # garbage coefficient of v^0 is W_{:,0} X_{3,:}
    assert np.abs(coeffs[0] - A[:, 0:2].astype(float) @ B[6:8, :].astype(float)).max() < 1e-10


def test_encode_is_polynomial_evaluation():
    # A~ at a point b equals sum of blocks times explicit powers: check one entry by hand
    A, B = WL.matmul_inputs(4, 6, 4, seed=5)
    pl = O.make_plan(2, 3, 2, 20)
    At, Bt = O.encode_A(A, pl), O.encode_B(B, pl)
    b = pl.points[7]
    # u = v^3: W~ = sum W_ij b^(3i+j); X~ = sum X_jk b^((2-j) + 6k)
    a00 = sum(float(A[i * 2 + 0, j * 2 + 1]) * b ** (3 * i + j) for i in range(2) for j in range(3))
    assert abs(At[7, 0, 1] - a00) < 1e-14
    x01 = sum(float(B[j * 2 + 1, k * 2 + 0]) * b ** ((2 - j) + 6 * k) for j in range(3) for k in range(2))
    assert abs(Bt[7, 1, 0] - x01) < 1e-14
    assert At.shape == (20, 2, 2) and Bt.shape == (20, 2, 2)


def test_cfg0_tiny_coded_matmul_matches_definition():
    c = WL.CONFIGS[0]
    A, B = WL.matmul_inputs(c["N1"], c["N0"], c["Nc"], c["seed"])
    pl = O.make_plan(c["m"], c["n"], c["d"], c["P"])
    present = np.zeros(c["P"], dtype=np.uint8)
    present[:pl.K] = 1
    C, rep = O.coded_matmul(A, B, pl, present=present, mode="first_k")
    C_ref = O.uncoded_matmul(A, B)
    rel = np.linalg.norm(C - C_ref) / np.linalg.norm(C_ref)
    assert rel < 1e-11
    # with fp32-rounded worker outputs the error is the rounding noise times the amplification
    C32, _ = O.coded_matmul(A, B, pl, present=present, mode="first_k", round_outputs="f32")
    rel32 = np.linalg.norm(C32 - C_ref) / np.linalg.norm(C_ref)
    assert 1e-9 < rel32 < 1e-3


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4096) * 10.0 ** rng.integers(-20, 20, 4096),
                        [0.0, -0.0, np.inf, -np.inf, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -9,
                         3.3895314e38, 1e-40]])
    want = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    got = O.round_to_bf16(x)
    assert np.array_equal(got, want)
    assert np.isnan(O.round_to_bf16(np.array([np.nan]))[0])


def test_workload_generators_are_seeded():
    A1, B1 = WL.matmul_inputs(16, 16, 16, 0)
    A2, B2 = WL.matmul_inputs(16, 16, 16, 0)
    assert np.array_equal(A1, A2) and np.array_equal(B1, B2) and A1.dtype == np.float32
    assert np.abs(A1).max() <= 1
    m = WL.erasure_trial(1000, 16, 7)
    assert m.sum() == 9 and np.array_equal(m, WL.erasure_trial(1000, 16, 7))
    f = WL.bitflip_trial(5001, 16, 2048 * 2048, 6)
    assert f == WL.bitflip_trial(5001, 16, 2048 * 2048, 6) and len(f) <= 6
    x = np.ones((2, 2, 2), dtype=np.float32)
    y = WL.apply_bitflips(x, [(1, 3, 31)])
    assert y[1, 1, 1] == -1.0 and x[1, 1, 1] == 1.0 and (y != x).sum() == 1


def test_amplification_closed_forms():
    # the decoder's noise amplification is pinned by cases that can be inverted by hand
    # (a) m = n = d = 1: K = 1, replication; the single coefficient is the mean of the present
    #     responses (lsq_all: row (1/|S|, ..., 1/|S|), norm 1/sqrt|S|) or the first one (first_k: 1)
    pl = O.make_plan(1, 1, 1, 7)
    assert pl.K == 1
    assert abs(O.amplification(pl, None, "lsq_all") - 1 / np.sqrt(7)) < 1e-14
    assert abs(O.amplification(pl, None, "first_k") - 1.0) < 1e-14
    present = np.array([0, 1, 1, 0, 1, 1, 0], dtype=np.uint8)
    assert abs(O.amplification(pl, present, "lsq_all") - 0.5) < 1e-14
    # (b) m = 2, n = d = 1: K = 2, both coefficients useful; two points a, b:
    #     [[1, a], [1, b]]^-1 = [[b, -a], [-1, 1]] / (b - a); the larger row norm is sqrt 2 / |b - a|
    #     when a^2 + b^2 <= 2
    a, b = 0.5, -0.25
    pl = O.make_plan(2, 1, 1, 2, points=[a, b])
    assert pl.K == 2 and sorted(pl.eC.ravel().tolist()) == [0, 1]
    assert abs(O.amplification(pl, None, "first_k") - np.sqrt(2.0) / 0.75) < 1e-13
    # (c) the useful row only, and nodes that first_k must ignore: m = d = 1, n = 2 (MatDot) has
    #     K = 3 and the single useful exponent 1.  Points -2, -1, 1, 2: by symmetry the least-squares
    #     coefficient of b is sum b z / sum b^2 = (-2 z_0 - z_1 + z_2 + 2 z_3) / 10, norm 1 / sqrt 10
    #     (the other two rows have norms 0.97 and 1/3); the parabola through the first three points
    #     has the linear coefficient (z_2 - z_1) / 2 (Lagrange basis), norm 1 / sqrt 2
    pl = O.make_plan(1, 2, 1, 4, points=[-2.0, -1.0, 1.0, 2.0])
    assert pl.K == 3 and pl.eC.ravel().tolist() == [1]
    assert abs(O.amplification(pl, None, "lsq_all") - 1 / np.sqrt(10.0)) < 1e-14
    assert abs(O.amplification(pl, None, "first_k") - 1 / np.sqrt(2.0)) < 1e-14


@pytest.mark.parametrize("mode", ["first_k", "lsq_all"])
def test_amplification_is_the_noise_gain_of_the_decoder(mode):
    # independent unit-variance noise in the responses comes out of O.decode with a standard
    # deviation, in the worst useful block, equal to the amplification: measured through the decoder
    # itself on 40 000 noise codewords, not through the decoding matrix
    pl = O.make_plan(2, 2, 2, 16)
    present = WL.erasure_trial(1003, 16, 4)
    rng = np.random.default_rng(8)
    noise = rng.standard_normal((16, 200, 200))
    C, _ = O.decode(noise, pl, present, mode)
    stds = [C[i * 200:(i + 1) * 200, k * 200:(k + 1) * 200].std() for i in range(2) for k in range(2)]
    amp = O.amplification(pl, present, mode)
    assert abs(max(stds) / amp - 1.0) < 0.03, (max(stds), amp)
    # and it is no bound on anything else: the dropped nodes' values are never read
    noise[present == 0] = 1e30
    C2, _ = O.decode(noise, pl, present, mode)
    assert np.array_equal(C, C2)
