"""CPU oracle for Generalized PolyDot coded matrix multiplication and coded DNN steps.

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow, fp64 numpy
statement of what the method in arXiv 1811.10751 computes, written from the
paper and independent of the GPU library (no shared code, tables or helpers).
Only tests, the smoke check and the benchmark's cpu_baseline leg may import it.

Every function names the passage of the paper it follows.  Library primitives
used as single steps: numpy matmul, numpy.linalg.solve / lstsq / qr, and
scipy.optimize.linprog for the one linear program (l1_locate).

Notation (paper -> here): W -> A (N1 x N0, split m x n), X -> B (N0 x Nc, split
n x d), S -> C (split m x d); b_p are the P distinct evaluation points; the
"recovery threshold" K is the number of coefficients of the product polynomial.

Readings taken where the paper is silent (all restated in the design notes):
  * evaluation points default to Chebyshev points of the first kind on [-1,1];
  * "Hz = 0" (Algorithm 1, step 1) is tested as ||Hz||_2 <= tau(z) with H
    orthonormal and tau(z) = rho * max(||z||_2, abs_floor);
  * Algorithm 1's arg-min ||e||_0 is an exhaustive search by increasing support
    size; inside one size the support with the smallest residual wins (ties: the
    lexicographically first); a support is admissible if its least-squares
    residual is <= tau(z);
  * non-finite responses are treated as located errors (forced members of the
    support) and replaced by zero before any arithmetic;
  * after location the coefficients are interpolated by least squares from all
    remaining (clean, present) nodes;
  * whole-node errors (Sec. III error models) are located once for a whole stack
    by the same search run on the aggregate of all element codewords (locate_nodes);
  * the polynomial-time locator the remark after Thm 3 asks for is the classical
    algebraic one (locator polynomial from the syndromes, in the Chebyshev basis),
    valid inside the adversarial radius floor((P-Q)/2) and accepted by Algorithm 1's
    own criterion (algebraic_locate);
  * the L1-norm relaxation the same remark names is the linear program min ||e||_1 subject to
    H e = H z; its solution only proposes supports (its largest entries), Algorithm 1's
    criterion accepts (l1_locate).
Parity pins: see tests/test_oracle_*.py.  Unpinned: the numeric value of rho
(this build's choice).
"""
from __future__ import annotations

import itertools
from dataclasses import dataclass, field

import numpy as np

# --------------------------------------------------------------------------- points


def chebyshev_points(P: int) -> np.ndarray:
    """b_p = cos((2p+1)pi/(2P)), p = 0..P-1.  The paper only asks for distinct reals
    (Sec. IV, proof of Thm 1); first-kind Chebyshev points are this build's choice."""
    p = np.arange(P, dtype=np.float64)
    return np.cos((2.0 * p + 1.0) * np.pi / (2.0 * P))


def int_power(b: np.ndarray, e: int) -> np.ndarray:
    """b**e by repeated multiplication (e >= 0), fp64."""
    out = np.ones_like(np.asarray(b, dtype=np.float64))
    for _ in range(int(e)):
        out = out * b
    return out


# --------------------------------------------------------------------------- plan


@dataclass
class Plan:
    """Exponent tables of one coded product W~(u,v) X~(v,w) after substitution.

    Sec. IV (Thm 2 and its proof): W~(u,v) = sum W_ij u^i v^j,
    X~(v,w) = sum X_jk v^(n-1-j) w^k, and S_ik is the coefficient of
    u^i v^(n-1) w^k.  With u = b^eu, v = b^ev, w = b^ew the three become
    polynomials in the single variable b.
      'u=v^n' : (eu, ev, ew) = (n, 1, mn)     (Thm 2)
      'v=u^m' : (eu, ev, ew) = (1, m, mn)     (App. on error tolerance, second case)
    """
    m: int
    n: int
    d: int
    P: int
    subst: str
    eu: int
    ev: int
    ew: int
    eA: np.ndarray          # [m, n]  exponent of W_ij
    eB: np.ndarray          # [n, d]  exponent of X_jk
    eC: np.ndarray          # [m, d]  exponent whose coefficient is S_ik
    K: int                  # number of coefficients of the product polynomial
    points: np.ndarray      # [P] fp64


def substitution_exponents(m: int, n: int, subst: str):
    if subst == "u=v^n":
        return n, 1, m * n
    if subst == "v=u^m":
        return 1, m, m * n
    raise ValueError(f"unknown substitution {subst!r}")


def make_plan(m: int, n: int, d: int, P: int, subst: str = "u=v^n", points=None) -> Plan:
    """Sec. IV, Thm 2: exponent tables and recovery threshold.

    K is computed as 1 + degree of the product polynomial (largest exponent of
    W~ plus largest exponent of X~), not from the closed form, so that the
    closed form mnd+n-1 is a test pin rather than an input.
    """
    if min(m, n, d, P) < 1:
        raise ValueError("m, n, d, P must be >= 1")
    eu, ev, ew = substitution_exponents(m, n, subst)
    eA = np.array([[eu * i + ev * j for j in range(n)] for i in range(m)], dtype=np.int64)
    eB = np.array([[ev * (n - 1 - j) + ew * k for k in range(d)] for j in range(n)], dtype=np.int64)
    eC = np.array([[eu * i + ev * (n - 1) + ew * k for k in range(d)] for i in range(m)], dtype=np.int64)
    K = int(eA.max() + eB.max() + 1)
    pts = chebyshev_points(P) if points is None else np.asarray(points, dtype=np.float64).copy()
    if pts.shape != (P,) or not np.all(np.isfinite(pts)) or len(np.unique(pts)) != P:
        raise ValueError("evaluation points must be P distinct finite reals")
    if K > P:
        raise ValueError(f"recovery threshold K={K} exceeds P={P}")
    return Plan(m, n, d, P, subst, eu, ev, ew, eA, eB, eC, K, pts)


def product_exponent_table(plan: Plan):
    """All (i, j, j', k) -> exponent of the product polynomial (proof of Thm 2).
    Used by tests to check that only j == j' terms land on the useful exponents."""
    out = {}
    for i in range(plan.m):
        for j in range(plan.n):
            for jp in range(plan.n):
                for k in range(plan.d):
                    out[(i, j, jp, k)] = int(plan.eA[i, j] + plan.eB[jp, k])
    return out


# --------------------------------------------------------------------------- encode


def split_blocks(M: np.ndarray, r: int, c: int):
    """M -> grid[r][c] of equal blocks (matrix partitioning notation, Sec. II)."""
    R, Cc = M.shape
    if R % r or Cc % c:
        raise ValueError("matrix does not split into equal blocks")
    br, bc = R // r, Cc // c
    return [[M[i * br:(i + 1) * br, j * bc:(j + 1) * bc] for j in range(c)] for i in range(r)]


def encode_A(A: np.ndarray, plan: Plan) -> np.ndarray:
    """A~_p = sum_ij A_ij b_p^eA(i,j)  (Eq. for W~(u,v) in Thm 1/2).  -> [P, N1/m, N0/n]."""
    A = np.asarray(A, dtype=np.float64)
    blk = split_blocks(A, plan.m, plan.n)
    out = np.zeros((plan.P,) + blk[0][0].shape)
    for p in range(plan.P):
        for i in range(plan.m):
            for j in range(plan.n):
                out[p] += blk[i][j] * int_power(plan.points[p], plan.eA[i, j])
    return out


def encode_B(B: np.ndarray, plan: Plan) -> np.ndarray:
    """B~_p = sum_jk B_jk b_p^eB(j,k)  (Eq. for X~(v,w), proof of Thm 2; the upper
    limit of k is d-1).  -> [P, N0/n, Nc/d]."""
    B = np.asarray(B, dtype=np.float64)
    blk = split_blocks(B, plan.n, plan.d)
    out = np.zeros((plan.P,) + blk[0][0].shape)
    for p in range(plan.P):
        for j in range(plan.n):
            for k in range(plan.d):
                out[p] += blk[j][k] * int_power(plan.points[p], plan.eB[j, k])
    return out


# --------------------------------------------------------------------------- rounding helpers


def round_to_f32(x: np.ndarray) -> np.ndarray:
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp64 -> fp32 (RNE) -> bfloat16 (RNE on the upper 16 bits) -> fp64.
    NaN stays NaN; Inf stays Inf."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    rounded = ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)) << np.uint64(16)
    rounded = np.where(np.isnan(f), u | np.uint64(0x00400000), rounded)
    out = (rounded & np.uint64(0xFFFF0000)).astype(np.uint32).view(np.float32)
    return out.astype(np.float64).reshape(np.shape(x))


# --------------------------------------------------------------------------- worker products


def worker_products(At: np.ndarray, Bt: np.ndarray, operands: str = "f64",
                    round_outputs: str | None = None) -> np.ndarray:
    """C~_p = A~_p B~_p for every node p (proof of Thm 2: each node multiplies its
    two coded blocks).

    operands: 'f64' exact inputs; 'f32' inputs rounded to fp32 first; 'bf16' inputs
    rounded to fp32 then bfloat16 (what a bf16 worker holds).  The product itself is
    always accumulated in fp64.  round_outputs='f32' rounds C~_p to fp32, which is
    what a worker would send and what a bit flip is defined on.
    """
    if operands == "f32":
        At, Bt = round_to_f32(At), round_to_f32(Bt)
    elif operands == "bf16":
        At, Bt = round_to_bf16(At), round_to_bf16(Bt)
    elif operands != "f64":
        raise ValueError(operands)
    Ct = np.matmul(np.asarray(At, dtype=np.float64), np.asarray(Bt, dtype=np.float64))
    if round_outputs == "f32":
        Ct = round_to_f32(Ct)
    elif round_outputs is not None:
        raise ValueError(round_outputs)
    return Ct


# --------------------------------------------------------------------------- code matrices


def vandermonde(points: np.ndarray, K: int) -> np.ndarray:
    """G^T: rows (1, b, b^2, ..., b^(K-1)) (App. on decoding, polynomial-interpolation case)."""
    pts = np.asarray(points, dtype=np.float64)
    V = np.ones((len(pts), K))
    for k in range(1, K):
        V[:, k] = V[:, k - 1] * pts
    return V


def parity_check(points: np.ndarray, K: int) -> np.ndarray:
    """Orthonormal H of shape (len(points)-K, len(points)) with H G^T = 0 (Sec. V,
    paragraph before Algorithm 1).  Taken as the trailing columns of the full QR of
    the Vandermonde matrix; any orthonormal basis of that null space gives the same
    norms and the same span tests."""
    V = vandermonde(points, K)
    Q, _ = np.linalg.qr(V, mode="complete")
    return Q[:, K:].T.copy()


# --------------------------------------------------------------------------- Algorithm 1


def support_residual(H: np.ndarray, y: np.ndarray, support):
    """min_e ||y - H[:,support] e||_2 and the minimiser (least squares)."""
    if len(support) == 0:
        return float(np.linalg.norm(y)), np.zeros(0)
    Hs = H[:, list(support)]
    e, *_ = np.linalg.lstsq(Hs, y, rcond=None)
    return float(np.linalg.norm(y - Hs @ e)), e


def algorithm1(z: np.ndarray, H: np.ndarray, tau: float, forced=()):
    """Algorithm 1 (Sec. V) for one received word z (already sanitised: finite).

    Returns (status, support, e_hat) with status in {'clean','located','failed'}.
      step 1: ||Hz|| <= tau and no forced locations -> no errors.
      step 2: smallest support A (containing the forced locations) such that
              Hz lies in span(H_A) up to tau; e_hat is the least-squares solution
              of H_A e = Hz.
      step 3: accept only if |A| <= P - Q - 1, where P - Q is the number of rows
              of H; otherwise decoding failure.
    """
    r, Pn = H.shape
    y = H @ z
    forced = tuple(sorted(int(f) for f in forced))
    if not forced and np.linalg.norm(y) <= tau:
        return "clean", (), np.zeros(0)
    max_size = r - 1
    free = [p for p in range(Pn) if p not in forced]
    start = max(len(forced), 1)
    for size in range(start, max_size + 1):
        best = None
        for extra in itertools.combinations(free, size - len(forced)):
            supp = tuple(sorted(forced + extra))
            res, e = support_residual(H, y, supp)
            if res <= tau and (best is None or res < best[0]):
                best = (res, supp, e)
        if best is not None:
            return "located", best[1], best[2]
    return "failed", forced, np.zeros(len(forced))


# --------------------------------------------------------------------------- algebraic locator


def dual_syndromes(z: np.ndarray, pts: np.ndarray, count: int) -> np.ndarray:
    """S_j = sum_s w_s T_j(x_s) z_s for j < count, with the barycentric weights
    w_s = 1 / prod_{q != s} (x_s - x_q) (scaled to max |w| = 1) and T_j the Chebyshev
    polynomials in the variable mapped affinely so that the points span [-1, 1].
    sum_s w_s q(x_s) is the (len(pts)-1)-th divided difference of q: zero for every
    polynomial q of degree <= len(pts) - 2, so S_j vanishes on the evaluations of a
    polynomial with K coefficients as long as j <= len(pts) - K - 1: these are the
    syndromes of the same (P, Q) MDS code (Sec. V) in another basis of the parity space."""
    x = _unit_interval(pts)
    n = len(x)
    w = np.ones(n)
    for s_ in range(n):
        for q in range(n):
            if q != s_:
                w[s_] /= (x[s_] - x[q])
    w /= np.abs(w).max()
    T = _chebyshev_table(x, count)
    return T @ (w * np.asarray(z, dtype=np.float64))


def _unit_interval(pts: np.ndarray) -> np.ndarray:
    pts = np.asarray(pts, dtype=np.float64)
    lo, hi = pts.min(), pts.max()
    return (2.0 * pts - (lo + hi)) / (hi - lo) if hi > lo else np.zeros_like(pts)


def _chebyshev_table(x: np.ndarray, count: int) -> np.ndarray:
    T = np.ones((max(count, 1), len(x)))
    if count > 1:
        T[1] = x
    for j in range(2, count):
        T[j] = 2.0 * x * T[j - 1] - T[j - 2]
    return T[:count]


def algebraic_locate(z: np.ndarray, H: np.ndarray, pts: np.ndarray, tau: float, forced=(), guard_nodes: int = 2):
    """Polynomial-time error location inside the adversarial radius |A| <= floor((P-Q)/2)
    (Sec. V, definition of the adversarial error model; the remark after Thm 3 asks for a
    polynomial-time reconstruction in place of the exhaustive search of Algorithm 1).
    This is the classical decoder of a real-number Reed-Solomon / MDS code:

      errors e at the nodes A turn the syndromes into S_j = sum_{i in A} a_i T_j(x_i)
      (a_i = w_i e_i).  For the locator polynomial L(x) = T_t(x) + sum_{k<t} c_k T_k(x),
      zero exactly at the x_i, sum_i a_i T_j(x_i) L(x_i) = 0 for every j, and with
      T_j T_k = (T_{j+k} + T_{|j-k|}) / 2 this is the linear system
          sum_{k<t} c_k (S_{j+k} + S_{|j-k|}) = -(S_{j+t} + S_{|j-t|}),  j = 0 .. r - t - 1,
      with r syndromes: solvable for t <= r / 2.

    For t = 1, 2, ... the system is solved in the least-squares sense; of the t + 2 nodes
    where |L| is smallest the t with the largest fitted error values are the candidate, and
    the candidate is accepted by the criterion of Algorithm 1 (residual of H z on the span of
    those columns of H <= tau), so a wrong candidate is never accepted silently.  Known-bad
    (forced) nodes are erasures: they are left out of the syndromes, which costs one syndrome each.
    guard_nodes = 0 is the textbook form (the t nodes where |L| is smallest, nothing fitted);
    in exact arithmetic both forms return the same support, since L vanishes on the erroneous
    nodes only.
    Returns (status, support, e_hat) like algorithm1."""
    r_full, ns = H.shape
    y = H @ z
    forced = tuple(sorted(int(f) for f in forced))
    if not forced and np.linalg.norm(y) <= tau:
        return "clean", (), np.zeros(0)
    free = np.array([q for q in range(ns) if q not in forced], dtype=np.int64)
    r = r_full - len(forced)
    if forced:
        res, e = support_residual(H, y, forced)
        if res <= tau and len(forced) <= r_full - 1:
            return "located", forced, e
    if r < 2:
        return "failed", forced, np.zeros(len(forced))
    S = dual_syndromes(np.asarray(z, dtype=np.float64)[free], np.asarray(pts, dtype=np.float64)[free], r)
    x = _unit_interval(np.asarray(pts, dtype=np.float64)[free])
    for t in range(1, r // 2 + 1):
        if len(forced) + t > r_full - 1:
            break
        rows = r - t
        M = np.empty((rows, t))
        b = np.empty(rows)
        for j in range(rows):
            for k in range(t):
                M[j, k] = S[j + k] + S[abs(j - k)]
            b[j] = -(S[j + t] + S[abs(j - t)])
        c, *_ = np.linalg.lstsq(M, b, rcond=None)
        T = _chebyshev_table(x, t + 1)
        L = T[t] + c @ T[:t]
        # two guard nodes: with rounding, a neighbour of an erroneous node can have a smaller
        # |L| than the node itself; the error values fitted on the t + 2 best nodes tell them apart
        guard = max(0, min(int(guard_nodes), r_full - 1 - len(forced) - t, len(free) - t))
        order = np.argsort(np.abs(L), kind="stable")[:t + guard]
        wide = tuple(sorted(forced + tuple(int(free[q]) for q in order)))
        _, e_wide = support_residual(H, y, wide)
        mag = {node: abs(v) for node, v in zip(wide, e_wide) if node not in forced}
        picked = sorted(mag, key=lambda node: (-mag[node], node))[:t]
        supp = tuple(sorted(forced + tuple(picked)))
        res, e = support_residual(H, y, supp)
        if res <= tau:
            return "located", supp, e
    return "failed", forced, np.zeros(len(forced))


# --------------------------------------------------------------------------- L1 relaxation


def l1_minimiser(H: np.ndarray, y: np.ndarray, free_cost=None) -> np.ndarray:
    """argmin sum_i cost_i |e_i| subject to H e = y (cost_i = 1, or 0 for entries that
    may take any value at no cost), as the linear program in e = e+ - e-, e+, e- >= 0:
    the L1-norm relaxation of arg-min ||e||_0 (remark after Thm 3, "decoding by linear
    programming").  Equivalently the least-absolute-deviations fit of a codeword to z:
    e = z - V c with c = argmin ||z - V c||_1, since H e = H z fixes e up to a codeword."""
    from scipy.optimize import linprog

    r, n = H.shape
    cost = np.ones(n) if free_cost is None else np.asarray(free_cost, dtype=np.float64)
    scale = float(np.abs(y).max())
    if scale == 0.0:
        return np.zeros(n)
    # (solved for y / max|y| with the solver's tightest tolerances, so that entries at the level of
    # the responses' rounding noise are not cut off as infeasibilities)
    res = linprog(np.concatenate([cost, cost]), A_eq=np.hstack([H, -H]), b_eq=y / scale,
                  bounds=[(0, None)] * (2 * n), method="highs-ds",
                  options={"primal_feasibility_tolerance": 1e-10, "dual_feasibility_tolerance": 1e-10})
    if res.status != 0:
        raise RuntimeError(f"linear program not solved: {res.message}")
    return scale * (res.x[:n] - res.x[n:])


def l1_costs(ns: int) -> np.ndarray:
    """Costs 1 + 1e-6 frac((s + 1)^2 phi), phi = (sqrt(5) - 1) / 2, of an error at node s of ns.
    With equal costs the linear program of l1_locate often has several optimal vertices on
    symmetric point sets such as the Chebyshev points (two vertices can differ by a codeword
    whose few non-zero values cancel in the sum of magnitudes), and which of them a solver
    returns is the solver's affair; slightly unequal costs in no regular pattern leave one
    (a rotation frac(s phi) does not: its differences between neighbours are all equal and
    cancel in exactly those sums).  This build's choice; the paper only names the relaxation."""
    s = np.arange(1, ns + 1, dtype=np.float64)
    return 1.0 + 1e-6 * ((s * s * 0.6180339887498949) % 1.0)


def l1_locate(z: np.ndarray, H: np.ndarray, tau: float, forced=()):
    """Error location by L1-norm relaxation (remark after Thm 3: the arg-min ||e||_0 of
    Algorithm 1 is NP-hard in general; an L1-norm relaxation is one of the polynomial-time
    sparse reconstructions it suggests).

      e* = argmin sum_s c_s |e_s| subject to H e = H z, with c_s = 1 up to a tie-breaking 1e-6
      (l1_costs) and c_s = 0 at known-bad (forced) nodes;
      the nodes are ranked by |e*| (largest first, ties: the lowest node); for sizes 1, 2, ...
      the forced nodes plus the first nodes of that ranking are the candidate support, and the
      first candidate that meets the criterion of Algorithm 1 (residual of H z on the span of
      those columns of H <= tau, at most P - Q - 1 nodes) is returned with its least-squares
      error values.

    The linear program only proposes: what is accepted passes Algorithm 1's own test.  In exact
    arithmetic (tau -> 0) a wrong support of at most P - Q - 1 nodes passes it with probability
    zero (Thm 3), so what is accepted is the support the exhaustive search would return; with a
    finite tau a larger support can pass where the ranking went wrong, which the search, trying
    small supports first, would not return.  Where no prefix of the ranking passes, the word is a
    decoding failure although the search might still succeed: the relaxation recovers fewer
    errors than P - Q - 1 (how many depends on H; measured in the tests).
    Returns (status, support, e_hat) like algorithm1."""
    r, ns = H.shape
    y = H @ z
    forced = tuple(sorted(int(f) for f in forced))
    if not forced and np.linalg.norm(y) <= tau:
        return "clean", (), np.zeros(0)
    cost = l1_costs(ns)
    cost[list(forced)] = 0.0
    e_star = l1_minimiser(H, y, cost)
    free = [q for q in range(ns) if q not in forced]
    ranking = sorted(free, key=lambda q: (-abs(e_star[q]), q))
    for size in range(max(len(forced), 1), r):
        supp = tuple(sorted(forced + tuple(ranking[:size - len(forced)])))
        res, e = support_residual(H, y, supp)
        if res <= tau:
            return "located", supp, e
    return "failed", forced, np.zeros(len(forced))


# --------------------------------------------------------------------------- decode


@dataclass
class DecodeReport:
    status: str = "ok"                       # 'ok' | 'decode_fail'
    n_present: int = 0
    n_flagged: int = 0                       # codewords with ||Hz|| > tau or a non-finite entry
    n_failed: int = 0
    located: list = field(default_factory=list)   # sorted (node, row, col, e_hat)
    failed: list = field(default_factory=list)    # sorted (row, col)
    node_err_count: np.ndarray | None = None
    max_syndrome_ratio: float = 0.0          # max over clean codewords of ||Hz|| / tau
    syndrome: np.ndarray | None = None       # ||Hz|| per codeword (rows x cols)
    tau: np.ndarray | None = None


class TooFewResponses(Exception):
    pass


def default_rho(worker: str) -> float:
    return 2.0 ** -12 if worker != "bf16" else 2.0 ** -3


def interpolate(Z: np.ndarray, pts: np.ndarray, K: int, mode: str) -> np.ndarray:
    """Coefficients [K, ...] of the degree-(K-1) polynomial through (pts, Z).
    'first_k': exact solve on the first K points (Remark after Thm 2: the master
    waits for K nodes and solves a linear system).  'lsq_all': least squares over
    all given points (G^T q = z - e of Sec. V restricted to the rows kept)."""
    if mode == "first_k":
        V = vandermonde(pts[:K], K)
        return np.linalg.solve(V, Z[:K])
    if mode == "lsq_all":
        V = vandermonde(pts, K)
        G, *_ = np.linalg.lstsq(V, Z, rcond=None)
        return G
    raise ValueError(mode)


def decode_coefficients(Zt: np.ndarray, points: np.ndarray, K: int, useful,
                        present=None, mode: str = "first_k", correct: bool = False,
                        rho: float = 2.0 ** -12, abs_floor: float = 0.0, locator: str = "search"):
    """Generic decoder: Zt[P, rows, cols] are evaluations at `points` of a matrix
    polynomial with K coefficients; returns {e: coefficient block} for e in `useful`
    and a DecodeReport.  (Remark after Thm 2; Sec. V Algorithm 1; App. 'Decoding
    Methods'.)"""
    Zt = np.asarray(Zt, dtype=np.float64)
    P = Zt.shape[0]
    rows, cols = Zt.shape[1], Zt.shape[2]
    pres = np.ones(P, dtype=bool) if present is None else np.asarray(present).astype(bool)
    S = np.flatnonzero(pres)
    rep = DecodeReport(n_present=len(S), node_err_count=np.zeros(P, dtype=np.int64))
    if len(S) < K:
        raise TooFewResponses(f"{len(S)} responses present, {K} needed")
    pts = np.asarray(points, dtype=np.float64)[S]
    Z = Zt[S].reshape(len(S), rows * cols)
    useful = [int(e) for e in useful]

    if not correct:
        G = interpolate(Z, pts, K, mode)
        return {e: G[e].reshape(rows, cols) for e in useful}, rep

    # ---- error detection on every codeword (Algorithm 1, step 1)
    finite = np.isfinite(Z)
    Zs = np.where(finite, Z, 0.0)
    H = parity_check(pts, K)                         # (|S|-K) x |S|
    Y = H @ Zs
    sigma = np.linalg.norm(Y, axis=0)
    tau = rho * np.maximum(np.linalg.norm(Zs, axis=0), abs_floor)
    flagged = (sigma > tau) | (~finite.all(axis=0))
    rep.n_flagged = int(flagged.sum())
    rep.syndrome = sigma.reshape(rows, cols)
    rep.tau = tau.reshape(rows, cols)
    clean_ratio = np.where(flagged | (tau == 0), 0.0, sigma / np.where(tau == 0, 1.0, tau))
    rep.max_syndrome_ratio = float(clean_ratio.max()) if clean_ratio.size else 0.0

    # ---- unflagged codewords: least squares over all present nodes
    G = interpolate(Zs, pts, K, "lsq_all")
    out = {e: G[e].copy() for e in useful}

    # ---- flagged codewords: locate (steps 2-3), then solve from the clean nodes
    for idx in np.flatnonzero(flagged):
        r_, c_ = divmod(int(idx), cols)
        forced = tuple(np.flatnonzero(~finite[:, idx]))
        if locator == "algebraic":
            status, supp, e_hat = algebraic_locate(Zs[:, idx], H, pts, float(tau[idx]), forced)
        elif locator == "l1":
            status, supp, e_hat = l1_locate(Zs[:, idx], H, float(tau[idx]), forced)
        else:
            status, supp, e_hat = algorithm1(Zs[:, idx], H, float(tau[idx]), forced)
        if status == "failed":
            rep.n_failed += 1
            rep.failed.append((r_, c_))
            continue
        keep = np.array([q for q in range(len(S)) if q not in supp], dtype=np.int64)
        g = interpolate(Zs[keep, idx], pts[keep], K, "lsq_all")
        for e in useful:
            out[e][idx] = g[e]
        for q, ev in zip(supp, e_hat):
            node = int(S[q])
            mag = float(ev) if finite[q, idx] else float("nan")
            rep.located.append((node, r_, c_, mag))
            rep.node_err_count[node] += 1
    rep.located.sort(key=lambda t: t[:3])
    rep.failed.sort()
    if rep.n_failed:
        rep.status = "decode_fail"
    return {e: out[e].reshape(rows, cols) for e in useful}, rep


def decode(Ct: np.ndarray, plan: Plan, present=None, mode: str = "first_k",
           correct: bool = False, rho: float = 2.0 ** -12, abs_floor: float = 0.0, locator: str = "search"):
    """C (N1 x Nc) from the node outputs Ct[P, N1/m, Nc/d]: block (i,k) of C is the
    coefficient of b^eC(i,k) (proof of Thm 2)."""
    useful = sorted(set(int(e) for e in plan.eC.ravel()))
    coeffs, rep = decode_coefficients(Ct, plan.points, plan.K, useful, present, mode,
                                      correct, rho, abs_floor, locator)
    rows, cols = Ct.shape[1], Ct.shape[2]
    C = np.zeros((plan.m * rows, plan.d * cols))
    for i in range(plan.m):
        for k in range(plan.d):
            C[i * rows:(i + 1) * rows, k * cols:(k + 1) * cols] = coeffs[int(plan.eC[i, k])]
    return C, rep


def coded_matmul(A, B, plan: Plan, present=None, mode="first_k", correct=False,
                 operands="f64", round_outputs=None, rho=2.0 ** -12):
    """encode -> P products -> decode, end to end (Sec. IV)."""
    At, Bt = encode_A(A, plan), encode_B(B, plan)
    Ct = worker_products(At, Bt, operands, round_outputs)
    return decode(Ct, plan, present, mode, correct, rho)


def uncoded_matmul(A, B):
    """The definition the method must reproduce: C = A B in fp64."""
    return np.asarray(A, dtype=np.float64) @ np.asarray(B, dtype=np.float64)


def amplification(plan: Plan, present=None, mode="first_k") -> float:
    """Largest 2-norm of a useful row of the decoding matrix: how much independent
    per-node rounding noise in the responses is amplified into C."""
    pres = np.ones(plan.P, dtype=bool) if present is None else np.asarray(present).astype(bool)
    S = np.flatnonzero(pres)
    if mode == "first_k":
        S = S[:plan.K]
    V = vandermonde(plan.points[S], plan.K)
    D = np.linalg.pinv(V)
    return float(max(np.linalg.norm(D[int(e)]) for e in plan.eC.ravel()))


# --------------------------------------------------------------------------- coded DNN layer


@dataclass
class LayerPlan:
    """One coded layer (Sec. VII for B=1, Sec. IX for B>1): weight W (N_out x N_in)
    split m x n; X (N_in x batch) split n x d1; Delta^T (batch x N_out) split d2 x m."""
    N_out: int
    N_in: int
    batch: int
    m: int
    n: int
    d1: int
    d2: int
    P: int
    subst: str
    fwd: Plan                 # plan of W~ X~ (feedforward, step O1)
    eD: np.ndarray            # [d2, m] exponent of Delta^T_{k,i}
    eCb: np.ndarray           # [d2, n] exponent whose coefficient is C^T_{k,j}
    Kb: int                   # coefficients of the backward product polynomial
    eUd: np.ndarray           # [m] update exponent of delta_i  (u^i)
    eUx: np.ndarray           # [n] update exponent of x_j      (v^j)
    N_out_pad: int
    N_in_pad: int

    @property
    def Kf(self):
        return self.fwd.K

    @property
    def points(self):
        return self.fwd.points


def choose_substitution(m: int, n: int) -> str:
    """This build's default: the substitution with the smaller max(K_f, K_b);
    for m > n that is v = u^m, otherwise u = v^n (Table I gives both)."""
    return "v=u^m" if m > n else "u=v^n"


def make_layer_plan(N_out, N_in, batch, m, n, d1, d2, P, subst="auto", points=None) -> LayerPlan:
    if subst == "auto":
        subst = choose_substitution(m, n)
    if batch % d1 or batch % d2:
        raise ValueError("d1 and d2 must divide the batch")
    eu, ev, ew = substitution_exponents(m, n, subst)
    fwd = make_plan(m, n, d1, P, subst, points)
    # Sec. IX backpropagation stage: Delta~^T(w,u) = sum_{k,i} Delta^T_{k,i} w^k u^(m-1-i);
    # C^T_{k,j} is the coefficient of w^k u^(m-1) v^j.
    eD = np.array([[ew * k + eu * (m - 1 - i) for i in range(m)] for k in range(d2)], dtype=np.int64)
    eCb = np.array([[ew * k + eu * (m - 1) + ev * j for j in range(n)] for k in range(d2)], dtype=np.int64)
    Kb = int(eD.max() + fwd.eA.max() + 1)
    if Kb > P:
        raise ValueError(f"backward threshold {Kb} exceeds P={P}")
    eUd = np.array([eu * i for i in range(m)], dtype=np.int64)
    eUx = np.array([ev * j for j in range(n)], dtype=np.int64)
    N_out_pad = -(-N_out // m) * m
    N_in_pad = -(-N_in // n) * n
    return LayerPlan(N_out, N_in, batch, m, n, d1, d2, P, subst, fwd, eD, eCb, Kb, eUd, eUx,
                     N_out_pad, N_in_pad)


def _pad_rows(M: np.ndarray, rows: int) -> np.ndarray:
    M = np.asarray(M, dtype=np.float64)
    if M.shape[0] == rows:
        return M
    out = np.zeros((rows,) + M.shape[1:])
    out[:M.shape[0]] = M
    return out


def layer_encode_weights(W: np.ndarray, lp: LayerPlan) -> np.ndarray:
    """Initial encoding of W (Sec. VII, pre-processing step).  Rows/columns are
    zero-padded up to multiples of m / n first (this build's rule for m not dividing
    N_out)."""
    Wp = np.zeros((lp.N_out_pad, lp.N_in_pad))
    Wp[:lp.N_out, :lp.N_in] = np.asarray(W, dtype=np.float64)
    return encode_A(Wp, lp.fwd)


def layer_decode_weights(Wt: np.ndarray, lp: LayerPlan, present=None) -> np.ndarray:
    """W from the coded blocks: W~(b) has mn coefficients W_ij at exponents eA(i,j)
    (footnote on regeneration, Sec. VII); least squares over the present nodes."""
    useful = sorted(int(e) for e in lp.fwd.eA.ravel())
    Kw = int(lp.fwd.eA.max()) + 1
    coeffs, _ = decode_coefficients(Wt, lp.points, Kw, useful, present, "lsq_all")
    rows, cols = Wt.shape[1], Wt.shape[2]
    W = np.zeros((lp.N_out_pad, lp.N_in_pad))
    for i in range(lp.m):
        for j in range(lp.n):
            W[i * rows:(i + 1) * rows, j * cols:(j + 1) * cols] = coeffs[int(lp.fwd.eA[i, j])]
    return W[:lp.N_out, :lp.N_in]


def layer_encode_x(X: np.ndarray, lp: LayerPlan) -> np.ndarray:
    """X~_p (Sec. VII feedforward stage / Sec. IX): [P, N_in/n, batch/d1]."""
    return encode_B(_pad_rows(X, lp.N_in_pad), lp.fwd)


def layer_forward(Wt, X, lp: LayerPlan, present=None, mode="lsq_all", correct=False,
                  operands="f64", round_outputs=None, rho=2.0 ** -12, corrupt=None):
    """Step O1 in coded form: S = W X decoded from S~_p = W~_p X~_p.
    `corrupt`, if given, maps the fp64 response stack to a corrupted one (tests)."""
    Xt = layer_encode_x(X, lp)
    St = worker_products(Wt, Xt, operands, round_outputs)
    if corrupt is not None:
        St = corrupt(St)
    S, rep = decode(St, lp.fwd, present, mode, correct, rho)
    return S[:lp.N_out], rep


def layer_encode_delta(Dlt: np.ndarray, lp: LayerPlan) -> np.ndarray:
    """Delta~^T_p = sum_{k,i} Delta^T_{k,i} b_p^eD(k,i)  (Sec. IX backpropagation stage).
    Dlt is N_out x batch; returns [P, batch/d2, N_out/m]."""
    DT = _pad_rows(Dlt, lp.N_out_pad).T                       # batch x N_out_pad
    blk = split_blocks(DT, lp.d2, lp.m)
    out = np.zeros((lp.P,) + blk[0][0].shape)
    for p in range(lp.P):
        for k in range(lp.d2):
            for i in range(lp.m):
                out[p] += blk[k][i] * int_power(lp.points[p], lp.eD[k, i])
    return out


def layer_backward(Wt, Dlt, lp: LayerPlan, present=None, mode="lsq_all", correct=False,
                   operands="f64", round_outputs=None, rho=2.0 ** -12, corrupt=None):
    """Step O2 in coded form: C^T = Delta^T W decoded from C~^T_p = Delta~^T_p W~_p.
    Returns C as N_in x batch."""
    Dt = layer_encode_delta(Dlt, lp)
    if operands == "f32":
        Dt, Wt_ = round_to_f32(Dt), round_to_f32(Wt)
    elif operands == "bf16":
        Dt, Wt_ = round_to_bf16(Dt), round_to_bf16(Wt)
    else:
        Wt_ = np.asarray(Wt, dtype=np.float64)
    CtT = np.matmul(Dt, Wt_)                                  # [P, batch/d2, N_in/n]
    if round_outputs == "f32":
        CtT = round_to_f32(CtT)
    if corrupt is not None:
        CtT = corrupt(CtT)
    useful = sorted(set(int(e) for e in lp.eCb.ravel()))
    coeffs, rep = decode_coefficients(CtT, lp.points, lp.Kb, useful, present, mode, correct, rho)
    rows, cols = CtT.shape[1], CtT.shape[2]
    CT = np.zeros((lp.d2 * rows, lp.n * cols))
    for k in range(lp.d2):
        for j in range(lp.n):
            CT[k * rows:(k + 1) * rows, j * cols:(j + 1) * cols] = coeffs[int(lp.eCb[k, j])]
    return CT.T[:lp.N_in], rep


def layer_update(Wt, Dlt, X, lp: LayerPlan, eta: float, decay: float = 0.0) -> np.ndarray:
    """Coded update (Eq. 'coded update', Sec. VII; rank-B form and the L2-regularised
    form in Sec. IX): W~_p <- (1-decay) W~_p + eta * Dhat_p Xhat_p^T with
    Dhat_p = sum_i Delta_i a_p^i and Xhat_p = sum_j X_j b_p^j; decay = eta*lambda."""
    Dp = _pad_rows(Dlt, lp.N_out_pad)
    Xp = _pad_rows(X, lp.N_in_pad)
    dblk = [Dp[i * (lp.N_out_pad // lp.m):(i + 1) * (lp.N_out_pad // lp.m)] for i in range(lp.m)]
    xblk = [Xp[j * (lp.N_in_pad // lp.n):(j + 1) * (lp.N_in_pad // lp.n)] for j in range(lp.n)]
    out = np.empty_like(np.asarray(Wt, dtype=np.float64))
    for p in range(lp.P):
        Dh = sum(dblk[i] * int_power(lp.points[p], lp.eUd[i]) for i in range(lp.m))
        Xh = sum(xblk[j] * int_power(lp.points[p], lp.eUx[j]) for j in range(lp.n))
        out[p] = (1.0 - decay) * Wt[p] + eta * (Dh @ Xh.T)
    return out


# --------------------------------------------------------------------------- node-level faults


WILD = 2.0 ** 40      # responses of this magnitude or more are handled like non-finite ones


@dataclass
class NodeReport:
    status: str = "clean"                    # 'clean' | 'located' | 'failed'
    bad: tuple = ()                          # sorted global node indices found erroneous
    energy: float = 0.0                      # sum over codewords of ||z||^2 (sanitised)
    syndrome_energy: float = 0.0             # sum over codewords of ||Hz||^2
    residual: float = 0.0                    # syndrome energy left outside span(H_bad)
    threshold: float = 0.0                   # tau^2 of the aggregate test
    gram: np.ndarray | None = None           # sum over codewords of (Hz)(Hz)^T


def locate_nodes(Zt: np.ndarray, points: np.ndarray, K: int, present=None,
                 rho: float = 2.0 ** -12, abs_floor: float = 0.0) -> NodeReport:
    """Algorithm 1 (Sec. V) under the error models of Sec. III, where an erroneous node's
    whole output is wrong: every element codeword z_c of the stack Zt[P, rows, cols] has
    its errors on the same set of nodes, so the set is searched once for all codewords.

      step 1: no errors if sum_c ||H z_c||^2 <= tau^2,
              tau^2 = rho^2 * max(sum_c ||z_c||^2, n_codewords * abs_floor^2);
      step 2: the smallest node set A such that every H z_c lies in span(H_A), tested in
              aggregate: sum_c min_e ||H z_c - H_A e||^2 <= tau^2; inside one size the
              set with the smallest residual wins;
      step 3: accept only if |A| <= (number of rows of H) - 1, else decoding failure.
    Nodes holding a non-finite value, or one of magnitude >= 2^40, are forced members of
    A and those values are replaced by zero before any arithmetic."""
    Zt = np.asarray(Zt, dtype=np.float64)
    P = Zt.shape[0]
    pres = np.ones(P, dtype=bool) if present is None else np.asarray(present).astype(bool)
    S = np.flatnonzero(pres)
    if len(S) < K:
        raise TooFewResponses(f"{len(S)} responses present, {K} needed")
    Z = Zt[S].reshape(len(S), -1)
    ncw = Z.shape[1]
    wild = ~np.isfinite(Z) | (np.abs(np.where(np.isfinite(Z), Z, 0.0)) >= WILD)
    forced = tuple(int(q) for q in np.flatnonzero(wild.any(axis=1)))
    Zs = np.where(wild, 0.0, Z)
    rep = NodeReport()
    r = len(S) - K
    rep.energy = float((Zs * Zs).sum())
    rep.threshold = rho * rho * max(rep.energy, ncw * abs_floor * abs_floor)
    if r == 0:
        rep.gram = np.zeros((0, 0))
        if forced:
            rep.status, rep.bad = "failed", tuple(int(S[q]) for q in forced)
        return rep
    H = parity_check(np.asarray(points, dtype=np.float64)[S], K)
    Y = H @ Zs
    rep.gram = Y @ Y.T
    rep.syndrome_energy = float((Y * Y).sum())
    rep.residual = rep.syndrome_energy
    if not forced and rep.syndrome_energy <= rep.threshold:
        return rep
    free = [q for q in range(len(S)) if q not in forced]
    for size in range(max(len(forced), 1), r):
        best = None
        for extra in itertools.combinations(free, size - len(forced)):
            supp = tuple(sorted(forced + extra))
            Hs = H[:, list(supp)]
            E, *_ = np.linalg.lstsq(Hs, Y, rcond=None)
            R = Y - Hs @ E
            res = float((R * R).sum())
            if res <= rep.threshold and (best is None or res < best[0]):
                best = (res, supp)
        if best is not None:
            rep.status, rep.residual = "located", best[0]
            rep.bad = tuple(int(S[q]) for q in best[1])
            return rep
    rep.status, rep.bad = "failed", tuple(int(S[q]) for q in forced)
    return rep


def decode_nodes(Ct: np.ndarray, plan: Plan, present=None, mode: str = "lsq_all",
                 rho: float = 2.0 ** -12, abs_floor: float = 0.0):
    """Locate the erroneous nodes once for the whole response stack, then decode with
    those nodes left out like stragglers (Sec. V: errors whose locations are known are
    erasures).  Returns (C or None on failure, NodeReport)."""
    rep = locate_nodes(Ct, plan.points, plan.K, present, rho, abs_floor)
    if rep.status == "failed":
        return None, rep
    pres = np.ones(plan.P, dtype=bool) if present is None else np.asarray(present).astype(bool).copy()
    pres[list(rep.bad)] = False
    C, _ = decode(Ct, plan, pres, mode)
    return C, rep


def check_positions(n_codewords: int, n_check: int) -> np.ndarray:
    """The pre-decided element positions of the verification step: n_check positions spread
    evenly over the block, position t = floor(t * n_codewords / n_check)."""
    n_check = min(n_check, n_codewords)
    return (np.arange(n_check, dtype=np.int64) * n_codewords) // max(n_check, 1)


@dataclass
class VerifyReport:
    status: str = "ok"                       # 'ok' | 'mismatch'
    n_checked: int = 0
    n_value_mismatch: int = 0
    locations_agree: bool = True
    bad: tuple = ()                          # nodes the independent search found erroneous
    max_ratio: float = 0.0                   # max |difference| / tolerance


def verify_decode(Ct: np.ndarray, plan: Plan, C: np.ndarray, present=None, mode: str = "first_k",
                  bad=(), n_check: int = 0, rho: float = 2.0 ** -12, abs_floor: float = 0.0) -> VerifyReport:
    """Verification step for decoding errors (Sec. VII, Error Model 2, and the crosscheck item of
    the complexity appendix): P pre-decided values of the decoded result are recomputed by a
    second, independent decoder and compared, and the vector saying which nodes were found
    erroneous is compared as well.  Here the second decoder works in fp64 on the P sampled
    element codewords only: node search on those codewords (locate_nodes), then least squares
    over the present nodes it leaves.  A decoded value disagrees if it differs by more than
    2^-20 (a_main + a_check) ||z||, a_* the norms of the decoding rows used by the two decoders
    (`mode` over `present` without `bad` for the main one)."""
    Ct = np.asarray(Ct, dtype=np.float64)
    P, rows, cols = Ct.shape
    ncw = rows * cols
    n_check = P if n_check <= 0 else n_check
    pos = check_positions(ncw, n_check)
    rep = VerifyReport(n_checked=len(pos))
    pres = np.ones(P, dtype=bool) if present is None else np.asarray(present).astype(bool)
    Z = Ct.reshape(P, ncw)[:, pos]                               # [P, n_check]
    nrep = locate_nodes(Z.reshape(P, len(pos), 1), plan.points, plan.K, pres, rho, abs_floor)
    rep.bad = nrep.bad
    rep.locations_agree = nrep.status != "failed" and tuple(sorted(int(b) for b in bad)) == nrep.bad
    main = pres.copy()
    main[list(bad)] = False
    check = pres.copy()
    check[list(nrep.bad)] = False
    S_main = np.flatnonzero(main)
    if mode == "first_k":
        S_main = S_main[:plan.K]
    S_chk = np.flatnonzero(check)
    D_main = np.linalg.pinv(vandermonde(plan.points[S_main], plan.K))
    D_chk = np.linalg.pinv(vandermonde(plan.points[S_chk], plan.K))
    C = np.asarray(C, dtype=np.float64)
    for t, e in enumerate(pos):
        r_, c_ = divmod(int(e), cols)
        z = np.where(np.isfinite(Z[:, t]), Z[:, t], 0.0)
        znorm = float(np.linalg.norm(z[S_chk]))
        worst = 0.0
        for i in range(plan.m):
            for k in range(plan.d):
                ex = int(plan.eC[i, k])
                want = float(D_chk[ex] @ z[S_chk])
                tol = 2.0 ** -20 * (np.linalg.norm(D_main[ex]) + np.linalg.norm(D_chk[ex])) * znorm
                got = C[i * rows + r_, k * cols + c_]
                ratio = abs(got - want) / tol if tol > 0 else (0.0 if got == want else np.inf)
                if not np.isfinite(got):
                    ratio = np.inf
                worst = max(worst, ratio)
        rep.max_ratio = max(rep.max_ratio, worst)
        if worst > 1.0:
            rep.n_value_mismatch += 1
    if rep.n_value_mismatch or not rep.locations_agree:
        rep.status = "mismatch"
    return rep


def weight_polynomial_terms(lp: LayerPlan) -> int:
    """Number of coefficients of W~(b) after the substitution: max exponent + 1 = mn
    (footnote on regeneration, Sec. VII)."""
    return int(lp.fwd.eA.max()) + 1


def layer_regenerate(Wt: np.ndarray, lp: LayerPlan, bad, mode: str = "lsq_all") -> np.ndarray:
    """Regeneration (Sec. VII): the coded block of every node in `bad` is re-evaluated from
    the polynomial W~(b) (mn coefficients) interpolated through nodes known to be correct:
    'first_k' takes the first mn good nodes by index, 'lsq_all' all good nodes."""
    Wt = np.asarray(Wt, dtype=np.float64)
    P = Wt.shape[0]
    Kw = weight_polynomial_terms(lp)
    isbad = np.zeros(P, dtype=bool)
    isbad[list(bad)] = True
    good = np.flatnonzero(~isbad)
    if len(good) < Kw:
        raise TooFewResponses(f"{len(good)} good nodes, {Kw} needed")
    coef = interpolate(Wt[good].reshape(len(good), -1), lp.points[good], Kw, mode)
    out = Wt.copy()
    for p in np.flatnonzero(isbad):
        acc = np.zeros(coef.shape[1])
        for e in range(Kw):
            acc += coef[e] * int_power(lp.points[p], e)
        out[p] = acc.reshape(Wt.shape[1:])
    return out


def layer_project(Wt: np.ndarray, lp: LayerPlan, present=None) -> np.ndarray:
    """Nearest stack (least squares, node by node) whose element codewords are exact
    evaluations of a polynomial with mn coefficients: interpolate from the present nodes,
    re-evaluate at every node.  (Regeneration applied to all nodes at once; this build
    uses it to remove the rounding drift of many coded updates.)"""
    Wt = np.asarray(Wt, dtype=np.float64)
    P = Wt.shape[0]
    Kw = weight_polynomial_terms(lp)
    pres = np.ones(P, dtype=bool) if present is None else np.asarray(present).astype(bool)
    S = np.flatnonzero(pres)
    if len(S) < Kw:
        raise TooFewResponses(f"{len(S)} nodes present, {Kw} needed")
    coef = interpolate(Wt[S].reshape(len(S), -1), lp.points[S], Kw, "lsq_all")
    out = np.empty_like(Wt)
    for p in range(P):
        acc = np.zeros(coef.shape[1])
        for e in range(Kw):
            acc += coef[e] * int_power(lp.points[p], e)
        out[p] = acc.reshape(Wt.shape[1:])
    return out


# --------------------------------------------------------------------------- MLP (uncoded definition + coded method)


def sigmoid(s):
    return 1.0 / (1.0 + np.exp(-np.asarray(s, dtype=np.float64)))


def sigmoid_grad_from_output(y):
    """g with g(f(u)) = f'(u) for the logistic f (step C2)."""
    return y * (1.0 - y)


def last_layer_delta(Y, Yhat):
    """delta^L = 2 (y - yhat) f'(s^L) for the L2 loss, with the mini-batch mean 1/B
    folded in (App. on DNN background, Eq. for the last layer; mini-batch section)."""
    B = Y.shape[1]
    return (2.0 / B) * (Y - Yhat) * sigmoid_grad_from_output(Yhat)


def mlp_uncoded_step(Ws, X, Y, eta, decay=0.0):
    """One SGD iteration of the plain MLP: steps O1, C1 forward; O2, C2 backward; O3
    update (Sec. II background).  Returns (new weights, last-layer output, deltas)."""
    Ws = [np.asarray(W, dtype=np.float64) for W in Ws]
    acts = [np.asarray(X, dtype=np.float64)]
    for W in Ws:
        acts.append(sigmoid(W @ acts[-1]))
    delta = last_layer_delta(np.asarray(Y, dtype=np.float64), acts[-1])
    new_Ws = [None] * len(Ws)
    deltas = [None] * len(Ws)
    for l in range(len(Ws) - 1, -1, -1):
        deltas[l] = delta
        c = Ws[l].T @ delta                                    # O2 with the pre-update W
        new_Ws[l] = (1.0 - decay) * Ws[l] + eta * delta @ acts[l].T   # O3
        if l > 0:
            delta = c * sigmoid_grad_from_output(acts[l])      # C2
    return new_Ws, acts[-1], deltas


def mlp_loss(Ws, X, Y):
    """(1/B) sum_b ||yhat_b - y_b||^2 (mini-batch L2 loss)."""
    a = np.asarray(X, dtype=np.float64)
    for W in Ws:
        a = sigmoid(np.asarray(W, dtype=np.float64) @ a)
    return float(np.sum((a - Y) ** 2) / Y.shape[1])


def mlp_coded_step(Wts, lps, X, Y, eta, decay=0.0, operands="f64", round_outputs=None,
                   correct=False, rho=2.0 ** -12, mode="lsq_all"):
    """One iteration of the coded strategy over all layers (Sec. VII / IX): the weights
    stay encoded; only X and Delta are encoded and decoded.  Returns (new coded weights,
    last-layer output, per-layer dict of intermediate values)."""
    acts = [np.asarray(X, dtype=np.float64)]
    trace = []
    for Wt, lp in zip(Wts, lps):
        S, _ = layer_forward(Wt, acts[-1], lp, None, mode, correct, operands, round_outputs, rho)
        acts.append(sigmoid(S))
    delta = last_layer_delta(np.asarray(Y, dtype=np.float64), acts[-1])
    new_Wts = [None] * len(Wts)
    for l in range(len(Wts) - 1, -1, -1):
        C, _ = layer_backward(Wts[l], delta, lps[l], None, mode, correct, operands, round_outputs, rho)
        new_Wts[l] = layer_update(Wts[l], delta, acts[l], lps[l], eta, decay)
        trace.append(dict(layer=l, delta=delta, C=C, X=acts[l]))
        if l > 0:
            delta = C * sigmoid_grad_from_output(acts[l])
    return new_Wts, acts[-1], trace[::-1]


# --------------------------------------------------------------------------- sparse autoencoder


def kl_slope(rho: float, rho_hat: np.ndarray) -> np.ndarray:
    """Q(rho_hat) = d KL(rho || rho_hat) / d rho_hat = -rho / rho_hat + (1 - rho) / (1 - rho_hat)
    (Sec. X, definition under Eq. for Delta_auto)."""
    rho_hat = np.asarray(rho_hat, dtype=np.float64)
    return -rho / rho_hat + (1.0 - rho) / (1.0 - rho_hat)


def autoencoder_loss(W1, W2, X, rho: float, beta: float) -> float:
    """Mini-batch loss of the sparse autoencoder without the weight-decay term (Sec. X):
    (1/B) sum_b ||x_b - xhat_b||^2 + beta sum_i KL(rho || rho_hat_i)."""
    X = np.asarray(X, dtype=np.float64)
    Y1 = sigmoid(np.asarray(W1, dtype=np.float64) @ X)
    Y2 = sigmoid(np.asarray(W2, dtype=np.float64) @ Y1)
    rh = Y1.mean(axis=1)
    kl = rho * np.log(rho / rh) + (1.0 - rho) * np.log((1.0 - rho) / (1.0 - rh))
    return float(((X - Y2) ** 2).sum() / X.shape[1] + beta * kl.sum())


def autoencoder_delta1(C2, Y1, rho: float, beta: float) -> np.ndarray:
    """Delta_auto^1 = (C^2 - (beta / B) Q_rhohat) o f'(S^1) (Lemma on autoencoder
    backpropagation; the factor beta / B, dropped in the printed lemma, is what makes
    W^1 + eta Delta_auto^1 X^T a step along minus the gradient of the loss above, in the same
    units as Delta^2 = (2 / B)(X - Xhat) o f'(S^2))."""
    Y1 = np.asarray(Y1, dtype=np.float64)
    B = Y1.shape[1]
    q = kl_slope(rho, Y1.mean(axis=1))
    return (np.asarray(C2, dtype=np.float64) - (beta / B) * q[:, None]) * sigmoid_grad_from_output(Y1)


def autoencoder_uncoded_step(W1, W2, X, eta, rho: float, beta: float, decay=0.0):
    """One SGD iteration of the plain sparse autoencoder (Sec. X, Eqs. for the update of
    W^1 and for Delta_auto^1; W^2 is updated as in any network).  Returns (W1', W2', Xhat)."""
    W1 = np.asarray(W1, dtype=np.float64)
    W2 = np.asarray(W2, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    Y1 = sigmoid(W1 @ X)
    Y2 = sigmoid(W2 @ Y1)
    d2 = last_layer_delta(X, Y2)
    C2 = W2.T @ d2
    d1 = autoencoder_delta1(C2, Y1, rho, beta)
    return ((1.0 - decay) * W1 + eta * d1 @ X.T, (1.0 - decay) * W2 + eta * d2 @ Y1.T, Y2)


def autoencoder_coded_step(Wt1, Wt2, lp1: LayerPlan, lp2: LayerPlan, X, eta, rho: float, beta: float,
                           decay=0.0, mode="lsq_all"):
    """The same iteration with both weight matrices kept encoded (Sec. X, list of key steps):
    coded feedforward twice, coded backpropagation at layer 2, Delta_auto^1 from the decoded
    C^2 and rho_hat, coded updates of both layers."""
    X = np.asarray(X, dtype=np.float64)
    S1, _ = layer_forward(Wt1, X, lp1, None, mode)
    Y1 = sigmoid(S1)
    S2, _ = layer_forward(Wt2, Y1, lp2, None, mode)
    Y2 = sigmoid(S2)
    d2 = last_layer_delta(X, Y2)
    C2, _ = layer_backward(Wt2, d2, lp2, None, mode)
    new2 = layer_update(Wt2, d2, Y1, lp2, eta, decay)
    d1 = autoencoder_delta1(C2, Y1, rho, beta)
    new1 = layer_update(Wt1, d1, X, lp1, eta, decay)
    return new1, new2, Y2
