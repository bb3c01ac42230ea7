"""GPU test of gpd_decode_static, the decode entry point that allocates nothing and keeps its
scratch memory (counters, the screen's bit map, the located list) in a fixed array inside the
library: it must give bit for bit what gpd_decode gives with a caller's workspace, on two calls in
a row, the second on a smaller problem (what the first call left in the array must not leak into
the second).  Runs last: a failure here must not hide the parity tests."""
import numpy as np
import pytest
import torch

import gpd_workloads as WL
import paper_1811_10751_amd as G
from oracle import gpd_oracle as O
from gpu_util import DEV, rel_fro, say, to_dev, to_np

pytestmark = pytest.mark.gpu


def responses(N1, N0, Nc, P, seed):
    A, B = WL.matmul_inputs(N1, N0, Nc, seed)
    plan = G.gpd_plan(N1, N0, Nc, 2, 2, 2, P)
    At, Bt = G.gpd_encode(plan, to_dev(A), to_dev(B))
    Ct = G.gpd_worker_products(plan, At, Bt)
    torch.cuda.synchronize()
    return A, B, plan, Ct


def corrupt(Ct, rng, n_single, n_double, burst):
    P, rows, cols = Ct.shape
    bad = Ct.clone()
    flat = bad.view(P, -1)
    cws = rng.choice(rows * cols, n_single + n_double, replace=False)
    for i, cw in enumerate(cws):
        for p in rng.choice(P, 1 if i < n_single else 2, replace=False):
            flat[int(p), int(cw)] += float(rng.choice([-1.0, 1.0]) * rng.uniform(20.0, 90.0))
    for cw in range(burst[0], burst[1]):
        flat[5, cw] -= 33.0
    flat[2, 7] = float("inf")
    flat[9, rows * cols - 1] = float("nan")
    return bad


def same_report(a, b):
    assert (a.status, a.n_present, a.n_screened, a.n_flagged, a.n_located, a.n_failed) == \
           (b.status, b.n_present, b.n_screened, b.n_flagged, b.n_located, b.n_failed)
    assert a.node_err_count.tolist() == b.node_err_count.tolist()
    assert a.max_syndrome_ratio == b.max_syndrome_ratio
    assert len(a.located) == len(b.located)
    for x, y in zip(a.located, b.located):
        assert x[:3] == y[:3] and (x[3] == y[3] or (np.isnan(x[3]) and np.isnan(y[3])))


def test_static_decode_equals_workspace_decode_on_two_calls_in_a_row():
    rng = np.random.default_rng(5)
    # first call: 256 x 320 blocks (81 920 codewords), hundreds of flagged codewords, erasures
    A1, B1, plan1, Ct1 = responses(512, 64, 640, 16, 31)
    bad1 = corrupt(Ct1, rng, 300, 60, (4000, 4200))
    present1 = np.ones(16, dtype=np.uint8)
    present1[[3, 12]] = 0
    # second call: a smaller problem (48 x 40 blocks), few errors, all nodes present
    A2, B2, plan2, Ct2 = responses(96, 32, 80, 14, 32)
    bad2 = corrupt(Ct2, rng, 5, 2, (100, 103))
    C1s = torch.empty((512, 640), dtype=torch.float32, device=DEV)
    C2s = torch.empty((96, 80), dtype=torch.float32, device=DEV)

    want1, rep1 = G.gpd_decode(plan1, bad1, present=present1, mode=G.GPD_DEC_LSQ_ALL,
                               correct_errors=G.GPD_CORRECT_ELEMENTS, located_cap=100000)
    want2, rep2 = G.gpd_decode(plan2, bad2, mode=G.GPD_DEC_LSQ_ALL, correct_errors=G.GPD_CORRECT_ELEMENTS,
                               located_cap=100000)
    # (single errors on the two erased nodes of the first problem are not seen)
    assert rep1.n_flagged >= 450 and rep1.n_located > rep1.n_flagged and 9 <= rep2.n_flagged <= 12

    say("static decode, first call")
    _, got1 = G.gpd_decode_static(plan1, bad1, C1s, present=present1, mode=G.GPD_DEC_LSQ_ALL,
                                  correct_errors=G.GPD_CORRECT_ELEMENTS, located_cap=100000)
    say("static decode, second call (smaller)")
    _, got2 = G.gpd_decode_static(plan2, bad2, C2s, mode=G.GPD_DEC_LSQ_ALL,
                                  correct_errors=G.GPD_CORRECT_ELEMENTS, located_cap=100000)
    torch.cuda.synchronize()
    same_report(got1, rep1)
    same_report(got2, rep2)
    assert torch.equal(C1s, want1) and torch.equal(C2s, want2)
    # and what both return is the oracle's decision and value on the second problem
    C_o, orep = O.decode(to_np(bad2), O.make_plan(2, 2, 2, 14), None, "lsq_all", True)
    assert [x[:3] for x in got2.located] == [x[:3] for x in orep.located] and got2.n_failed == orep.n_failed == 0
    assert rel_fro(to_np(C2s), C_o) < 2e-5

    # the first problem again, then without a report (asynchronous) and without correction
    _, got1b = G.gpd_decode_static(plan1, bad1, C1s.zero_(), present=present1, mode=G.GPD_DEC_LSQ_ALL,
                                   correct_errors=G.GPD_CORRECT_ELEMENTS, located_cap=100000)
    same_report(got1b, rep1)
    assert torch.equal(C1s, want1)
    G.gpd_decode_static(plan2, bad2, C2s.zero_(), mode=G.GPD_DEC_LSQ_ALL, correct_errors=G.GPD_CORRECT_ELEMENTS,
                        want_report=False)
    torch.cuda.synchronize()
    assert torch.equal(C2s, want2)
    plain, _ = G.gpd_decode(plan1, Ct1, present=present1, mode=G.GPD_DEC_FIRST_K)
    G.gpd_decode_static(plan1, Ct1, C1s.zero_(), present=present1, mode=G.GPD_DEC_FIRST_K, want_report=False)
    torch.cuda.synchronize()
    assert torch.equal(C1s, plain)


def test_static_decode_allocates_no_device_memory_and_rejects_what_does_not_fit():
    A, B, plan, Ct = responses(256, 32, 256, 12, 33)
    Cs = torch.empty((256, 256), dtype=torch.float32, device=DEV)
    for _ in range(2):                                     # first calls load code and fill the table cache
        G.gpd_decode_static(plan, Ct, Cs, mode=G.GPD_DEC_LSQ_ALL, correct_errors=G.GPD_CORRECT_ELEMENTS)
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    for _ in range(3):
        _, rep = G.gpd_decode_static(plan, Ct, Cs, mode=G.GPD_DEC_LSQ_ALL, correct_errors=G.GPD_CORRECT_ELEMENTS)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free0
    assert rep.status == G.GPD_OK and rep.n_flagged == 0
    assert rel_fro(to_np(Cs), O.uncoded_matmul(A, B)) < 1e-3
    with pytest.raises(G.GpdError) as e:
        G.gpd_decode_static(plan, Ct, Cs, mode=G.GPD_DEC_LSQ_ALL, correct_errors=G.GPD_CORRECT_NODES)
    assert e.value.status == G.GPD_E_UNSUPPORTED
    # blocks beyond the limit (4096 x 2048 > 2^22 codewords) are refused before anything is read
    big = G.gpd_plan(8192, 2, 4096, 2, 2, 2, 12)
    lib = G.load_library()
    st = lib.gpd_decode_static(big.handle, Ct.data_ptr(), None, G.GPD_DEC_LSQ_ALL, G.GPD_CORRECT_ELEMENTS,
                               Cs.data_ptr(), 4096, None)
    assert st == G.GPD_E_WORKSPACE and b"exceed" in lib.gpd_last_error()
