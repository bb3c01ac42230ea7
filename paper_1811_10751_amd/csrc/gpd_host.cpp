// Host-side mathematics of the code construction: exponent tables, evaluation points and the
// fp64 decoding matrices.  No device code here.
#include <algorithm>
#include <cmath>
#include <cstring>

#include "gpd_internal.hpp"

namespace gpd {

static thread_local std::string g_last_error;

void set_error(const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  g_last_error = buf;
}

gpd_status_t fail(gpd_status_t st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return st;
}

const char* last_error_cstr() { return g_last_error.c_str(); }

double ipow(double b, int e) {
  double r = 1.0;
  for (int i = 0; i < e; ++i) r *= b;
  return r;
}

// Sec. IV proof of Thm 2 (u = v^n, w = v^mn) and the second case of the error-tolerance
// appendix (v = u^m, w = u^mn), written as powers of the single evaluation variable b.
gpd_status_t substitution(int m, int n, int subst, int* eu, int* ev, int* ew) {
  if (subst == GPD_SUB_U_VN) {
    *eu = n; *ev = 1; *ew = m * n;
  } else if (subst == GPD_SUB_V_UM) {
    *eu = 1; *ev = m; *ew = m * n;
  } else {
    return fail(GPD_E_INVALID, "unknown substitution %d", subst);
  }
  return GPD_OK;
}

gpd_status_t make_points(int P, const double* user, std::vector<double>* out) {
  out->resize(P);
  if (user) {
    for (int p = 0; p < P; ++p) {
      if (!std::isfinite(user[p])) return fail(GPD_E_POINTS, "evaluation point %d is not finite", p);
      (*out)[p] = user[p];
    }
    std::vector<double> s(*out);
    std::sort(s.begin(), s.end());
    for (int p = 1; p < P; ++p)
      if (s[p] == s[p - 1]) return fail(GPD_E_POINTS, "evaluation points are not distinct");
  } else {
    // Chebyshev points of the first kind on [-1, 1]
    const double pi = 3.14159265358979323846;
    for (int p = 0; p < P; ++p) (*out)[p] = std::cos((2.0 * p + 1.0) * pi / (2.0 * P));
  }
  return GPD_OK;
}

gpd_status_t make_code(int m, int n, int d, int P, int subst, const double* points, Code* c) {
  if (m < 1 || n < 1 || d < 1 || P < 1) return fail(GPD_E_INVALID, "m, n, d, P must be >= 1");
  if (P > GPD_MAX_P) return fail(GPD_E_INVALID, "P = %d exceeds GPD_MAX_P = %d", P, GPD_MAX_P);
  if (m * n > GPD_MAX_BLOCKS || n * d > GPD_MAX_BLOCKS || m * d > GPD_MAX_BLOCKS)
    return fail(GPD_E_INVALID, "block grid larger than GPD_MAX_BLOCKS = %d", GPD_MAX_BLOCKS);
  if (subst == GPD_SUB_AUTO) subst = GPD_SUB_U_VN;
  c->m = m; c->n = n; c->d = d; c->P = P;
  gpd_status_t st = substitution(m, n, subst, &c->eu, &c->ev, &c->ew);
  if (st != GPD_OK) return st;
  c->eA.resize(m * n); c->eB.resize(n * d); c->eC.resize(m * d);
  int maxA = 0, maxB = 0;
  for (int i = 0; i < m; ++i)
    for (int j = 0; j < n; ++j) {
      c->eA[i * n + j] = c->eu * i + c->ev * j;                 // W_ij u^i v^j
      maxA = std::max(maxA, c->eA[i * n + j]);
    }
  for (int j = 0; j < n; ++j)
    for (int k = 0; k < d; ++k) {
      c->eB[j * d + k] = c->ev * (n - 1 - j) + c->ew * k;       // X_jk v^(n-1-j) w^k
      maxB = std::max(maxB, c->eB[j * d + k]);
    }
  for (int i = 0; i < m; ++i)
    for (int k = 0; k < d; ++k)
      c->eC[i * d + k] = c->eu * i + c->ev * (n - 1) + c->ew * k;   // S_ik at u^i v^(n-1) w^k
  c->K = maxA + maxB + 1;
  if (c->K > P) return fail(GPD_E_SHAPE, "recovery threshold K = %d exceeds P = %d", c->K, P);
  return make_points(P, points, &c->pts);
}

// ---------------------------------------------------------------- small dense fp64 algebra

namespace {

// Householder QR of the rows x cols matrix a (row-major, rows >= cols).  On return `q` is the
// full rows x rows orthogonal factor (row-major) and `r` the cols x cols upper triangle.
void householder_qr(const std::vector<double>& a_in, int rows, int cols, std::vector<double>* q,
                    std::vector<double>* r) {
  std::vector<double> a(a_in);
  q->assign((size_t)rows * rows, 0.0);
  for (int i = 0; i < rows; ++i) (*q)[(size_t)i * rows + i] = 1.0;
  std::vector<double> v(rows);
  for (int k = 0; k < cols; ++k) {
    double norm = 0.0;
    for (int i = k; i < rows; ++i) norm += a[(size_t)i * cols + k] * a[(size_t)i * cols + k];
    norm = std::sqrt(norm);
    if (norm == 0.0) continue;
    double alpha = a[(size_t)k * cols + k] > 0 ? -norm : norm;
    double vnorm2 = 0.0;
    for (int i = k; i < rows; ++i) {
      v[i] = a[(size_t)i * cols + k] - (i == k ? alpha : 0.0);
      vnorm2 += v[i] * v[i];
    }
    if (vnorm2 == 0.0) continue;
    // a <- (I - 2 v v^T / v^T v) a
    for (int j = k; j < cols; ++j) {
      double s = 0.0;
      for (int i = k; i < rows; ++i) s += v[i] * a[(size_t)i * cols + j];
      s = 2.0 * s / vnorm2;
      for (int i = k; i < rows; ++i) a[(size_t)i * cols + j] -= s * v[i];
    }
    // q <- q (I - 2 v v^T / v^T v)
    for (int i = 0; i < rows; ++i) {
      double s = 0.0;
      for (int l = k; l < rows; ++l) s += (*q)[(size_t)i * rows + l] * v[l];
      s = 2.0 * s / vnorm2;
      for (int l = k; l < rows; ++l) (*q)[(size_t)i * rows + l] -= s * v[l];
    }
  }
  r->assign((size_t)cols * cols, 0.0);
  for (int i = 0; i < cols; ++i)
    for (int j = i; j < cols; ++j) (*r)[(size_t)i * cols + j] = a[(size_t)i * cols + j];
}

}  // namespace

gpd_status_t decode_matrices(const std::vector<double>& pts, const std::vector<int>& S, int K,
                             const std::vector<int>& useful, bool first_k,
                             std::vector<double>* D, std::vector<double>* H) {
  const int ns = (int)S.size();
  if (ns < K) return fail(GPD_E_TOO_FEW, "%d responses present, %d needed", ns, K);
  const int nu = first_k ? K : ns;        // nodes the interpolation uses
  // Vandermonde rows (1, b, ..., b^(K-1)) of the nodes used (appendix on decoding)
  std::vector<double> V((size_t)nu * K);
  for (int s = 0; s < nu; ++s) {
    double x = 1.0;
    for (int k = 0; k < K; ++k) {
      V[(size_t)s * K + k] = x;
      x *= pts[S[s]];
    }
  }
  std::vector<double> Q, R;
  householder_qr(V, nu, K, &Q, &R);
  for (int k = 0; k < K; ++k)
    if (R[(size_t)k * K + k] == 0.0) return fail(GPD_E_POINTS, "singular Vandermonde matrix");
  // pinv(V) = R^-1 Q1^T; row e: solve R x = Q1^T column by column, keep row e
  D->assign(useful.size() * (size_t)ns, 0.0);
  std::vector<double> x(K);
  for (int s = 0; s < nu; ++s) {
    for (int k = K - 1; k >= 0; --k) {
      double acc = Q[(size_t)s * nu + k];          // (Q1^T)[k][s] = Q[s][k]
      for (int l = k + 1; l < K; ++l) acc -= R[(size_t)k * K + l] * x[l];
      x[k] = acc / R[(size_t)k * K + k];
    }
    for (size_t u = 0; u < useful.size(); ++u) {
      if (useful[u] < 0 || useful[u] >= K) return fail(GPD_E_INVALID, "useful exponent out of range");
      (*D)[u * ns + s] = x[useful[u]];
    }
  }
  if (H) {
    // orthonormal basis of the left null space of the Vandermonde matrix of ALL present nodes
    std::vector<double> Vall((size_t)ns * K), Qa, Ra;
    for (int s = 0; s < ns; ++s) {
      double xx = 1.0;
      for (int k = 0; k < K; ++k) {
        Vall[(size_t)s * K + k] = xx;
        xx *= pts[S[s]];
      }
    }
    householder_qr(Vall, ns, K, &Qa, &Ra);
    const int r = ns - K;
    H->assign((size_t)r * ns, 0.0);
    for (int i = 0; i < r; ++i)
      for (int s = 0; s < ns; ++s) (*H)[(size_t)i * ns + s] = Qa[(size_t)s * ns + K + i];
  }
  return GPD_OK;
}

// ---------------------------------------------------------------- node-level error location

namespace {

// Eigenvalues (descending) and eigenvectors (columns of `vec`, row-major n x n) of the symmetric
// n x n matrix a: cyclic Jacobi rotations.
void jacobi_eigen(std::vector<double> a, int n, std::vector<double>* val, std::vector<double>* vec) {
  std::vector<double>& v = *vec;
  v.assign((size_t)n * n, 0.0);
  for (int i = 0; i < n; ++i) v[(size_t)i * n + i] = 1.0;
  for (int sweep = 0; sweep < 60; ++sweep) {
    double off = 0.0, diag = 0.0;
    for (int i = 0; i < n; ++i)
      for (int j = 0; j < n; ++j) (i == j ? diag : off) += a[(size_t)i * n + j] * a[(size_t)i * n + j];
    if (off <= 1e-30 * diag || off == 0.0) break;
    for (int p = 0; p < n - 1; ++p)
      for (int q = p + 1; q < n; ++q) {
        const double apq = a[(size_t)p * n + q];
        if (apq == 0.0) continue;
        const double theta = (a[(size_t)q * n + q] - a[(size_t)p * n + p]) / (2.0 * apq);
        const double t = (theta >= 0 ? 1.0 : -1.0) / (std::fabs(theta) + std::sqrt(theta * theta + 1.0));
        const double c = 1.0 / std::sqrt(t * t + 1.0), sn = t * c;
        for (int k = 0; k < n; ++k) {          // columns p, q of a
          const double akp = a[(size_t)k * n + p], akq = a[(size_t)k * n + q];
          a[(size_t)k * n + p] = c * akp - sn * akq;
          a[(size_t)k * n + q] = sn * akp + c * akq;
        }
        for (int k = 0; k < n; ++k) {          // rows p, q of a
          const double apk = a[(size_t)p * n + k], aqk = a[(size_t)q * n + k];
          a[(size_t)p * n + k] = c * apk - sn * aqk;
          a[(size_t)q * n + k] = sn * apk + c * aqk;
        }
        for (int k = 0; k < n; ++k) {
          const double vkp = v[(size_t)k * n + p], vkq = v[(size_t)k * n + q];
          v[(size_t)k * n + p] = c * vkp - sn * vkq;
          v[(size_t)k * n + q] = sn * vkp + c * vkq;
        }
      }
  }
  std::vector<int> order(n);
  for (int i = 0; i < n; ++i) order[i] = i;
  std::sort(order.begin(), order.end(), [&](int x, int y) { return a[(size_t)x * n + x] > a[(size_t)y * n + y]; });
  val->resize(n);
  std::vector<double> sorted((size_t)n * n);
  for (int c = 0; c < n; ++c) {
    (*val)[c] = a[(size_t)order[c] * n + order[c]];
    for (int k = 0; k < n; ++k) sorted[(size_t)k * n + c] = v[(size_t)k * n + order[c]];
  }
  v.swap(sorted);
}

// Depth-first enumeration of the node sets of one size, in lexicographic order, with the
// orthonormal basis of span(H_A) grown one column at a time: the syndrome energy left
// outside span(H_A) is trace(G) - sum_k q_k^T G q_k.
struct SupportSearch {
  int r = 0, ns = 0, size = 0;
  const double* H = nullptr;       // r x ns
  const double* G = nullptr;       // r x r
  std::vector<int> free_nodes;
  double threshold = 0;
  std::vector<double> Q;           // size x r
  std::vector<int> cur, best;
  double best_res = 0;
  bool found = false;

  // appends column `node` at depth k; returns the energy it explains
  double push(int k, int node) {
    double* q = &Q[(size_t)k * r];
    double n0 = 0.0;
    for (int i = 0; i < r; ++i) { q[i] = H[(size_t)i * ns + node]; n0 += q[i] * q[i]; }
    for (int pass = 0; pass < 2; ++pass)
      for (int l = 0; l < k; ++l) {
        const double* ql = &Q[(size_t)l * r];
        double dot = 0.0;
        for (int i = 0; i < r; ++i) dot += ql[i] * q[i];
        for (int i = 0; i < r; ++i) q[i] -= dot * ql[i];
      }
    double n1 = 0.0;
    for (int i = 0; i < r; ++i) n1 += q[i] * q[i];
    if (!(n1 > 1e-24 * n0)) {                  // numerically inside the span already
      for (int i = 0; i < r; ++i) q[i] = 0.0;
      return 0.0;
    }
    const double inv = 1.0 / std::sqrt(n1);
    for (int i = 0; i < r; ++i) q[i] *= inv;
    double gain = 0.0;
    for (int i = 0; i < r; ++i) {
      double gi = 0.0;
      for (int j = 0; j < r; ++j) gi += G[(size_t)i * r + j] * q[j];
      gain += q[i] * gi;
    }
    return gain;
  }

  void go(int depth, int first_free, double res) {
    if (depth == size) {
      if (res <= threshold && (!found || res < best_res)) { found = true; best_res = res; best = cur; }
      return;
    }
    const int need = size - depth;
    for (int f = first_free; f + need <= (int)free_nodes.size(); ++f) {
      cur[depth] = free_nodes[f];
      const double gain = push(depth, free_nodes[f]);
      go(depth + 1, f + 1, res - gain);
    }
  }
};

double binomial(int n, int k) {
  double b = 1.0;
  for (int i = 1; i <= k; ++i) b = b * (n - k + i) / i;
  return b;
}

}  // namespace

gpd_status_t locate_nodes_host(const std::vector<double>& H, int r, int ns, const std::vector<double>& G,
                               double energy, int64_t n_codewords, double rho, double abs_floor,
                               const std::vector<int>& forced, NodeSearchResult* out) {
  NodeSearchResult& o = *out;
  o = NodeSearchResult();
  o.energy = energy;
  o.threshold = rho * rho * std::max(energy, (double)n_codewords * abs_floor * abs_floor);
  double trace = 0.0;
  for (int i = 0; i < r; ++i) trace += G[(size_t)i * r + i];
  o.syndrome_energy = trace;
  o.residual = trace;
  if (r == 0) {
    o.status = forced.empty() ? 0 : 2;
    o.bad = forced;
    return GPD_OK;
  }
  if (forced.empty() && trace <= o.threshold) return GPD_OK;          // step 1: no errors

  std::vector<double> lam, vec;
  jacobi_eigen(G, r, &lam, &vec);
  std::vector<char> is_forced(ns, 0);
  for (int f : forced) is_forced[f] = 1;
  SupportSearch ss;
  ss.r = r; ss.ns = ns; ss.H = H.data(); ss.G = G.data(); ss.threshold = o.threshold;
  for (int q = 0; q < ns; ++q)
    if (!is_forced[q]) ss.free_nodes.push_back(q);
  const int nf = (int)forced.size();
  for (int size = std::max(nf, 1); size <= r - 1; ++size) {
    // no set of `size` nodes can leave less than the sum of the r - size smallest
    // eigenvalues of G outside its span: skip sizes that cannot reach the threshold
    double tail = 0.0;
    for (int i = size; i < r; ++i) tail += std::max(lam[i], 0.0);
    if (tail > o.threshold * (1.0 + 1e-6) + 1e-12 * trace) continue;
    ss.size = size;
    ss.Q.assign((size_t)size * r, 0.0);
    ss.cur.assign(size, 0);
    ss.found = false;
    double res = trace;
    for (int k = 0; k < nf; ++k) { ss.cur[k] = forced[k]; res -= ss.push(k, forced[k]); }
    if (binomial((int)ss.free_nodes.size(), size - nf) <= kNodeSearchBudget) {
      ss.go(nf, 0, res);
    } else {
      // too many sets of this size to try them all: test the one set made of the nodes whose
      // columns of H lie closest to the span of the `size` dominant eigenvectors of G
      o.exhaustive = false;
      std::vector<std::pair<double, int>> dist;
      for (int q : ss.free_nodes) {
        double n0 = 0.0, inside = 0.0;
        for (int i = 0; i < r; ++i) n0 += H[(size_t)i * ns + q] * H[(size_t)i * ns + q];
        for (int c = 0; c < size; ++c) {
          double dot = 0.0;
          for (int i = 0; i < r; ++i) dot += vec[(size_t)i * r + c] * H[(size_t)i * ns + q];
          inside += dot * dot;
        }
        dist.push_back({1.0 - inside / n0, q});
      }
      std::sort(dist.begin(), dist.end());
      std::vector<int> pick;
      for (int k = 0; k < size - nf; ++k) pick.push_back(dist[k].second);
      std::sort(pick.begin(), pick.end());
      for (int k = 0; k < size - nf; ++k) { ss.cur[nf + k] = pick[k]; res -= ss.push(nf + k, pick[k]); }
      if (res <= o.threshold) { ss.found = true; ss.best_res = res; ss.best = ss.cur; }
    }
    if (ss.found) {
      o.status = 1;
      o.residual = std::max(ss.best_res, 0.0);
      o.bad = ss.best;
      std::sort(o.bad.begin(), o.bad.end());
      return GPD_OK;
    }
  }
  o.status = 2;                                                      // decoding failure
  o.bad = forced;
  return GPD_OK;
}

gpd_status_t parity_check_host(const std::vector<double>& pts, const std::vector<int>& S, int K,
                               std::vector<double>* H) {
  std::vector<double> D;
  return decode_matrices(pts, S, K, std::vector<int>(), false, &D, H);
}

void fill_node_report(const NodeSearchResult& res, const std::vector<int>& S, gpd_node_report_t* rep) {
  rep->n_bad = (int32_t)res.bad.size();
  for (int q : res.bad) rep->bad[S[q]] = 1;
  rep->exhaustive = res.exhaustive ? 1 : 0;
  rep->energy = res.energy;
  rep->syndrome_energy = res.syndrome_energy;
  rep->residual = res.residual;
  rep->threshold = res.threshold;
  rep->status = res.status == 2 ? GPD_E_DECODE_FAIL : GPD_OK;
}

// ---------------------------------------------------------------- table packing

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

size_t HostCombineTable::bytes() const {
  size_t b = 0;
  b += align_up(sizeof(int64_t) * nin, 16);
  b += align_up(sizeof(int64_t) * nout, 16);
  b += align_up(sizeof(float) * nout * nin, 16);
  b += align_up(sizeof(float) * r * nin, 16);
  b += align_up(sizeof(double) * nout * nin, 16);
  b += align_up(sizeof(double) * r * nin, 16);
  b += align_up(sizeof(int32_t) * nin, 16);
  b += align_up(sizeof(double) * nin, 16);
  b += 2 * align_up(sizeof(int32_t) * nin, 16) + 2 * align_up(sizeof(int32_t) * nout, 16);
  return align_up(b, 256);
}

CombineTable HostCombineTable::pack(void* dst, const void* dev_base) const {
  CombineTable t;
  t.nin = nin; t.nout = nout; t.r = r;
  t.off_align = 4;
  for (int64_t o : in_off) while (o % t.off_align) t.off_align /= 2;
  for (int64_t o : out_off) while (o % t.off_align) t.off_align /= 2;
  char* h = (char*)dst;
  const char* dv = (const char*)dev_base;
  size_t off = 0;
  auto put = [&](const void* src, size_t n) -> const void* {
    if (n) std::memcpy(h + off, src, n);
    const void* p = dv + off;
    off += align_up(n, 16);
    return p;
  };
  t.in_off = (const int64_t*)put(in_off.data(), sizeof(int64_t) * nin);
  t.out_off = (const int64_t*)put(out_off.data(), sizeof(int64_t) * nout);
  std::vector<float> c32(coef.begin(), coef.end()), h32(H.begin(), H.end());
  t.coef = (const float*)put(c32.data(), sizeof(float) * nout * nin);
  t.H = (const float*)put(h32.data(), sizeof(float) * r * nin);
  t.coef64 = (const double*)put(coef.data(), sizeof(double) * nout * nin);
  t.H64 = (const double*)put(H.data(), sizeof(double) * r * nin);
  t.node = (const int32_t*)put(node.data(), sizeof(int32_t) * nin);
  if (nin <= 64 && nout <= 64) {
    t.k_offsets = true;
    for (int i = 0; i < nin; ++i) t.k_in_off[i] = in_off[i];
    for (int i = 0; i < nout; ++i) t.k_out_off[i] = out_off[i];
    if (nout * nin <= 256 && r * nin <= 256) {
      t.k_coefs = true;
      for (int i = 0; i < nout * nin; ++i) t.k_coef[i] = c32[i];
      for (int i = 0; i < r * nin; ++i) t.k_H[i] = h32[i];
    }
  }
  if (!pts.empty()) t.pts64 = (const double*)put(pts.data(), sizeof(double) * nin);
  if (!in_rows.empty() || !out_rows.empty()) {
    // limits given for one side only mean "no limit" on the other
    std::vector<int32_t> ir(in_rows), ic(in_cols), orow(out_rows), oc(out_cols);
    if (ir.empty()) { ir.assign(nin, 0x7fffffff); ic.assign(nin, 0x7fffffff); }
    if (orow.empty()) { orow.assign(nout, 0x7fffffff); oc.assign(nout, 0x7fffffff); }
    t.in_rows = (const int32_t*)put(ir.data(), sizeof(int32_t) * nin);
    t.in_cols = (const int32_t*)put(ic.data(), sizeof(int32_t) * nin);
    t.out_rows = (const int32_t*)put(orow.data(), sizeof(int32_t) * nout);
    t.out_cols = (const int32_t*)put(oc.data(), sizeof(int32_t) * nout);
    t.limit_align = 4;
    for (int32_t c : ic) if (c != 0x7fffffff) while (c % t.limit_align) t.limit_align /= 2;
    for (int32_t c : oc) if (c != 0x7fffffff) while (c % t.limit_align) t.limit_align /= 2;
  }
  return t;
}

}  // namespace gpd

// Host-only entry points: the code construction and the fp64 decoding matrices, without a GPU.
extern "C" gpd_status_t gpd_host_code(int32_t m, int32_t n, int32_t d, int32_t P, int32_t subst,
                                      const double* points, int32_t* K, int32_t* eA, int32_t* eB,
                                      int32_t* eC, double* points_out) {
  gpd::Code c;
  gpd_status_t st = gpd::make_code(m, n, d, P, subst, points, &c);
  if (st != GPD_OK) return st;
  if (K) *K = c.K;
  if (eA) std::copy(c.eA.begin(), c.eA.end(), eA);
  if (eB) std::copy(c.eB.begin(), c.eB.end(), eB);
  if (eC) std::copy(c.eC.begin(), c.eC.end(), eC);
  if (points_out) std::copy(c.pts.begin(), c.pts.end(), points_out);
  return GPD_OK;
}

extern "C" gpd_status_t gpd_host_decode_matrices(int32_t m, int32_t n, int32_t d, int32_t P,
                                                 int32_t subst, const double* points,
                                                 const uint8_t* present, int32_t first_k, double* D,
                                                 double* H, int32_t* n_present) {
  gpd::Code c;
  gpd_status_t st = gpd::make_code(m, n, d, P, subst, points, &c);
  if (st != GPD_OK) return st;
  std::vector<int> S;
  for (int p = 0; p < P; ++p)
    if (!present || present[p]) S.push_back(p);
  if (n_present) *n_present = (int32_t)S.size();
  std::vector<double> Dv, Hv;
  st = gpd::decode_matrices(c.pts, S, c.K, c.eC, first_k != 0, &Dv, H ? &Hv : nullptr);
  if (st != GPD_OK) return st;
  if (D) std::copy(Dv.begin(), Dv.end(), D);
  if (H) std::copy(Hv.begin(), Hv.end(), H);
  return GPD_OK;
}

extern "C" gpd_status_t gpd_host_parity_check(int32_t P, int32_t K, const double* points,
                                              const uint8_t* present, double* H, int32_t* n_present) {
  if (P < 1 || P > GPD_MAX_P || K < 1) return gpd::fail(GPD_E_INVALID, "gpd_host_parity_check: bad P or K");
  std::vector<double> pts;
  gpd_status_t st = gpd::make_points(P, points, &pts);
  if (st != GPD_OK) return st;
  std::vector<int> S;
  for (int p = 0; p < P; ++p)
    if (!present || present[p]) S.push_back(p);
  if (n_present) *n_present = (int32_t)S.size();
  std::vector<double> Hv;
  st = gpd::parity_check_host(pts, S, K, &Hv);
  if (st != GPD_OK) return st;
  if (H) std::copy(Hv.begin(), Hv.end(), H);
  return GPD_OK;
}

extern "C" gpd_status_t gpd_host_locate_nodes(int32_t P, int32_t K, const double* points,
                                              const uint8_t* present, const double* gram,
                                              double energy, int64_t n_codewords, double rho,
                                              double abs_floor, const uint8_t* forced,
                                              gpd_node_report_t* report) {
  if (P < 1 || P > GPD_MAX_P || K < 1 || !report || n_codewords < 0)
    return gpd::fail(GPD_E_INVALID, "gpd_host_locate_nodes: bad argument");
  std::vector<double> pts;
  gpd_status_t st = gpd::make_points(P, points, &pts);
  if (st != GPD_OK) return st;
  std::vector<int> S;
  for (int p = 0; p < P; ++p)
    if (!present || present[p]) S.push_back(p);
  std::memset(report, 0, sizeof(*report));
  report->n_present = (int32_t)S.size();
  std::vector<double> H;
  st = gpd::parity_check_host(pts, S, K, &H);
  if (st != GPD_OK) { report->status = st; return st; }
  const int ns = (int)S.size(), r = ns - K;
  if (r > 0 && !gram) return gpd::fail(GPD_E_INVALID, "gpd_host_locate_nodes: null Gram matrix");
  std::vector<double> G(gram, gram + (size_t)r * r);
  std::vector<int> f;
  for (int q = 0; q < ns; ++q)
    if (forced && forced[S[q]]) { f.push_back(q); report->wild[S[q]] = 1; }
  gpd::NodeSearchResult res;
  st = gpd::locate_nodes_host(H, r, ns, G, energy, n_codewords, rho, abs_floor, f, &res);
  if (st != GPD_OK) { report->status = st; return st; }
  gpd::fill_node_report(res, S, report);
  if (res.status == 2) return gpd::fail(GPD_E_DECODE_FAIL, "more erroneous nodes than can be located");
  return GPD_OK;
}

extern "C" const char* gpd_last_error(void) {
  const char* s = gpd::last_error_cstr();
  return s ? s : "";
}

extern "C" const char* gpd_version(void) { return "gpd 0.1 (gfx950)"; }
