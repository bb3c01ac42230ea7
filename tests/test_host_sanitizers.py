"""The host half of the library (csrc/gpd_host.cpp: code construction, fp64 linear algebra of
the decoding matrices, combinatorial node search, table packing) under AddressSanitizer and
UndefinedBehaviorSanitizer on the CPU: tests/host_sanitize_driver.cpp is compiled together with
that source, run, and what it prints is compared with the oracle.  A sanitizer report fails the
run (no recovery); no GPU and no built library is needed."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import gpd_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SUB = {1: "u=v^n", 2: "v=u^m"}


@pytest.fixture(scope="module")
def records(tmp_path_factory):
    cxx = shutil.which("g++")
    if cxx is None or not os.path.isdir("/opt/rocm/include"):
        pytest.skip("g++ or the ROCm headers are missing")
    out = tmp_path_factory.mktemp("san") / "host_san"
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_1811_10751_amd", "csrc"),
           os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"),
           os.path.join(ROOT, "paper_1811_10751_amd", "csrc", "gpd_host.cpp"), "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(out)], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "runtime error" not in r.stderr and "Sanitizer" not in r.stderr, r.stderr[-4000:]
    assert r.stdout.rstrip().endswith("done")
    recs, cur = [], None
    for ln in r.stdout.splitlines():
        tok = ln.split()
        if tok[0] in ("code", "decode", "locate", "pack", "points_same", "points_nan", "too_few", "last_error", "done"):
            cur = {"kind": tok[0], "head": tok[1:], "raw": ln}
            recs.append(cur)
        else:
            cur[tok[0]] = np.array([float(x) for x in tok[1:]])
    return recs


def test_code_construction_under_sanitizers(records):
    n = 0
    for rec in (r for r in records if r["kind"] == "code"):
        m, nn, d, P, subst = (int(x) for x in rec["head"][:5])
        status, K = int(rec["head"][6]), int(rec["head"][8])
        try:
            pl = O.make_plan(m, nn, d, P, SUB[subst]) if P <= 64 else None
        except ValueError:
            pl = None
        if pl is None:
            assert status != 0, rec["raw"]
            continue
        assert status == 0 and K == pl.K, rec["raw"]
        assert np.array_equal(rec["eA"], pl.eA.ravel()) and np.array_equal(rec["eB"], pl.eB.ravel())
        assert np.array_equal(rec["eC"], pl.eC.ravel())
        assert np.abs(rec["pts"] - pl.points).max() < 1e-15
        n += 1
    assert n >= 14
    by = {r["kind"]: r for r in records}
    assert by["points_same"]["head"][1] == "3" and by["points_nan"]["head"][1] == "3" and by["too_few"]["head"][1] == "4"
    assert "needed" in by["last_error"]["raw"]


def test_decoding_matrices_under_sanitizers(records):
    n = 0
    for rec in (r for r in records if r["kind"] == "decode"):
        m, nn, d, P, subst = (int(x) for x in rec["head"][:5])
        first_k, ns = int(rec["head"][6]), int(rec["head"][10])
        pl = O.make_plan(m, nn, d, P, SUB[subst])
        S = np.flatnonzero(rec["present"])
        assert len(S) == ns
        useful = [int(e) for e in pl.eC.ravel()]
        D = rec["D"].reshape(m * d, ns)
        if first_k:
            # rows of the inverse of the first K present nodes' Vandermonde matrix (by its residual: the
            # first K of many Chebyshev points make an ill-conditioned system, entries up to 1e9)
            VK = O.vandermonde(pl.points[S[:pl.K]], pl.K)
            assert np.abs(D[:, :pl.K] @ VK - np.eye(pl.K)[useful]).max() <= 1e-10 * max(1.0, np.abs(D).max()), rec["raw"]
            assert np.all(D[:, pl.K:] == 0)
        else:
            V = O.vandermonde(pl.points[S], pl.K)
            # rows of a left inverse of V with minimal norm: D V = the useful rows of the identity, D H^T = 0
            assert np.abs(D @ V - np.eye(pl.K)[useful]).max() <= 1e-6 * max(1.0, np.abs(D).max()), rec["raw"]
            if ns > pl.K:
                H = rec["H"].reshape(ns - pl.K, ns)
                assert np.abs(H @ H.T - np.eye(ns - pl.K)).max() < 1e-11
                assert np.abs(H @ V).max() < 1e-9
                assert np.abs(D @ H.T).max() <= 1e-8 * np.abs(D).max()
        n += 1
    assert n >= 40


def test_node_search_and_packing_under_sanitizers(records):
    seen = 0
    for rec in (r for r in records if r["kind"] == "locate"):
        P, K, ncw, t = (int(x) for x in rec["head"][:4])
        status, n_bad, exhaustive = int(rec["head"][5]), int(rec["head"][7]), int(rec["head"][9])
        present = rec["present"].astype(bool)
        r_ = int(present.sum()) - K
        want = (rec["planted"] + rec["forced"]) > 0
        if want.sum() <= max(r_ - 1, 0) and not (r_ == 0 and want.any()):
            # Thm 3: up to |S| - K - 1 erroneous nodes are found, and only those
            assert status == 0 and np.array_equal(rec["found"] > 0, want), rec["raw"]
            assert n_bad == want.sum()
            energy, syn, res, thr = rec["stats"]
            assert res <= thr or n_bad == 0
        else:
            assert status == 5, rec["raw"]                       # decoding failure
        if (P, K) == (48, 12):
            assert exhaustive == 0
        seen += 1
    assert seen >= 12
    packs = [r for r in records if r["kind"] == "pack"]
    assert len(packs) == 4 and all(int(r["head"][4]) % 256 == 0 for r in packs)
