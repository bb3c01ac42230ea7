"""CPU-only checks of the built C-ABI library: it loads, exports every symbol the header
declares, and its host-side code construction and fp64 decoding matrices agree with the
oracle (compute entry points are not called here: they need a GPU)."""
import os
import re

import numpy as np
import pytest

import paper_1811_10751_amd as G
from oracle import gpd_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = G.load_library()
    header = open(os.path.join(ROOT, "include", "gpd.h")).read()
    declared = set(re.findall(r"\b(gpd_[a-z0-9_]+)\s*\(", header))
    declared -= {"gpd_decmode_t"}
    assert {"gpd_plan", "gpd_encode", "gpd_worker_products", "gpd_decode", "gpd_coded_layer_step"} <= declared
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert set(G.binding.EXPORTS) == declared
    assert "gfx950" in G.gpd_version()


@pytest.mark.parametrize("m,n,d,P", [(2, 2, 2, 16), (4, 2, 1, 24), (2, 4, 1, 32), (3, 2, 2, 20), (1, 4, 1, 9)])
@pytest.mark.parametrize("subst", [G.GPD_SUB_U_VN, G.GPD_SUB_V_UM])
def test_host_code_matches_oracle(m, n, d, P, subst):
    name = {G.GPD_SUB_U_VN: "u=v^n", G.GPD_SUB_V_UM: "v=u^m"}[subst]
    try:
        pl = O.make_plan(m, n, d, P, name)
    except ValueError:
        with pytest.raises(G.GpdError):
            G.gpd_host_code(m, n, d, P, subst)
        return
    K, eA, eB, eC, pts = G.gpd_host_code(m, n, d, P, subst)
    assert K == pl.K
    assert np.array_equal(eA, pl.eA) and np.array_equal(eB, pl.eB) and np.array_equal(eC, pl.eC)
    assert np.abs(pts - pl.points).max() < 1e-15


def test_host_decode_matrices_match_oracle():
    m, n, d, P = 2, 2, 2, 16
    pl = O.make_plan(m, n, d, P)
    rng = np.random.default_rng(0)
    for trial in range(20):
        present = np.ones(P, dtype=np.uint8)
        present[rng.choice(P, rng.integers(0, P - pl.K + 1), replace=False)] = 0
        S = np.flatnonzero(present)
        useful = [int(e) for e in pl.eC.ravel()]
        # least squares over all present nodes
        D, H = G.gpd_host_decode_matrices(m, n, d, P, present=present, first_k=False)
        Dref = np.linalg.pinv(O.vandermonde(pl.points[S], pl.K))[useful]
        assert np.abs(D - Dref).max() <= 1e-9 * np.abs(Dref).max()
        Href = O.parity_check(pl.points[S], pl.K)
        assert H.shape == Href.shape
        if H.shape[0]:
            assert np.abs(H @ H.T - np.eye(H.shape[0])).max() < 1e-12
            assert np.abs(H @ O.vandermonde(pl.points[S], pl.K)).max() < 1e-11
            # same row space as the oracle's parity check
            assert np.abs(H - (H @ Href.T) @ Href).max() < 1e-10
        # first K present nodes
        D1, _ = G.gpd_host_decode_matrices(m, n, d, P, present=present, first_k=True, want_H=False)
        inv = np.linalg.inv(O.vandermonde(pl.points[S[:pl.K]], pl.K))[useful]
        assert np.abs(D1[:, :pl.K] - inv).max() <= 1e-8 * np.abs(inv).max()
        assert np.all(D1[:, pl.K:] == 0)


def test_host_rejects_bad_requests():
    with pytest.raises(G.GpdError) as e:
        G.gpd_host_code(2, 2, 2, 8)
    assert e.value.status == G.GPD_E_SHAPE
    with pytest.raises(G.GpdError) as e:
        G.gpd_host_code(2, 2, 2, 10, points=[0.5] * 10)
    assert e.value.status == G.GPD_E_POINTS
    with pytest.raises(G.GpdError) as e:
        G.gpd_host_code(2, 2, 2, 10, points=[float("nan")] + list(range(9)))
    assert e.value.status == G.GPD_E_POINTS
    with pytest.raises(G.GpdError) as e:
        G.gpd_host_code(0, 2, 2, 10)
    assert e.value.status == G.GPD_E_INVALID
    with pytest.raises(G.GpdError) as e:
        G.gpd_host_code(2, 2, 2, 100)
    assert e.value.status == G.GPD_E_INVALID
    present = np.zeros(16, dtype=np.uint8)
    present[:8] = 1
    with pytest.raises(G.GpdError) as e:
        G.gpd_host_decode_matrices(2, 2, 2, 16, present=present)
    assert e.value.status == G.GPD_E_TOO_FEW


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1811_10751_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                for needle in ("gpd_oracle", "from oracle", "import oracle", "oracle/"):
                    assert needle not in text, (f, needle)
