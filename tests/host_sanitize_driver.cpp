// CPU-only driver for the host half of the library (csrc/gpd_host.cpp: code construction,
// fp64 decoding matrices, orthonormal parity check, node search on a Gram matrix, table
// packing), meant to be built with -fsanitize=address,undefined and run by
// tests/test_host_sanitizers.py.  It calls the host entry points of include/gpd.h over a sweep
// of codes, erasure patterns and planted node errors and prints what they return as text lines
//   <tag> <numbers ...>
// which the test compares with the oracle; any sanitizer report ends the run with an error.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "gpd_internal.hpp"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t next_u32() {                       // xorshift64*
  rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
  return (uint32_t)((rng_state * 0x2545F4914F6CDD1Dull) >> 32);
}
static double next_unit() { return (next_u32() + 0.5) / 4294967296.0; }          // (0, 1)
static double next_normal() { return std::sqrt(-2.0 * std::log(next_unit())) * std::cos(6.283185307179586 * next_unit()); }

template <typename T>
static void line(const char* tag, const std::vector<T>& v) {
  std::printf("%s", tag);
  for (const T& x : v) std::printf(" %.17g", (double)x);
  std::printf("\n");
}

static void code_case(int m, int n, int d, int P, int subst) {
  int32_t K = -1;
  std::vector<int32_t> eA(m * n), eB(n * d), eC(m * d);
  std::vector<double> pts(P);
  const gpd_status_t st = gpd_host_code(m, n, d, P, subst, nullptr, &K, eA.data(), eB.data(), eC.data(), pts.data());
  std::printf("code %d %d %d %d %d status %d K %d\n", m, n, d, P, subst, (int)st, (int)K);
  if (st != GPD_OK) return;
  line("eA", eA); line("eB", eB); line("eC", eC); line("pts", pts);
}

static void decode_case(int m, int n, int d, int P, int subst, int n_masks) {
  int32_t K = 0;
  if (gpd_host_code(m, n, d, P, subst, nullptr, &K, nullptr, nullptr, nullptr, nullptr) != GPD_OK) std::exit(3);
  for (int t = 0; t < n_masks; ++t) {
    std::vector<uint8_t> present(P, 1);
    const int drop = (int)(next_u32() % (uint32_t)(P - K + 1));
    for (int k = 0; k < drop;) {
      const int p = (int)(next_u32() % (uint32_t)P);
      if (present[p]) { present[p] = 0; ++k; }
    }
    const int ns = P - drop;
    for (int first_k = 0; first_k < 2; ++first_k) {
      std::vector<double> D((size_t)m * d * ns), H((size_t)(ns - K) * ns);
      int32_t nsv = 0;
      const gpd_status_t st = gpd_host_decode_matrices(m, n, d, P, subst, nullptr, present.data(), first_k, D.data(),
                                                       first_k ? nullptr : H.data(), &nsv);
      std::printf("decode %d %d %d %d %d first_k %d status %d ns %d\n", m, n, d, P, subst, first_k, (int)st, (int)nsv);
      if (st != GPD_OK || nsv != ns) std::exit(4);
      line("present", present);
      line("D", D);
      if (!first_k) line("H", H);
    }
  }
}

// planted whole-node errors: Z = evaluations of random polynomials with K coefficients, plus noise on
// `bad`; the Gram matrix of the syndromes in the library's own basis goes to the host search
static void locate_case(int P, int K, int ncw, int t, double rho, int n_erased, bool force_one) {
  std::vector<double> pts(P);
  if (gpd_host_code(1, 1, 1, P, GPD_SUB_U_VN, nullptr, nullptr, nullptr, nullptr, nullptr, pts.data()) != GPD_OK) std::exit(5);
  std::vector<uint8_t> present(P, 1);
  for (int k = 0; k < n_erased;) {
    const int p = (int)(next_u32() % (uint32_t)P);
    if (present[p]) { present[p] = 0; ++k; }
  }
  std::vector<int> S;
  for (int p = 0; p < P; ++p) if (present[p]) S.push_back(p);
  const int ns = (int)S.size(), r = ns - K;
  std::vector<uint8_t> bad(P, 0), forced(P, 0);
  for (int k = 0; k < t;) {
    const int p = S[next_u32() % (uint32_t)ns];
    if (!bad[p]) { bad[p] = 1; ++k; }
  }
  std::vector<double> Z((size_t)ns * ncw, 0.0);
  for (int c = 0; c < ncw; ++c) {
    std::vector<double> coef(K);
    for (double& x : coef) x = next_normal();
    for (int q = 0; q < ns; ++q) {
      double acc = 0.0, pw = 1.0;
      for (int k = 0; k < K; ++k) { acc += coef[k] * pw; pw *= pts[S[q]]; }
      Z[(size_t)q * ncw + c] = acc + (bad[S[q]] ? next_normal() : 0.0);
    }
  }
  if (force_one) {
    // one more node counted as erroneous at sight: its values are taken as zero, as the kernel does
    for (int q = 0; q < ns; ++q)
      if (!bad[S[q]]) { forced[S[q]] = 1; for (int c = 0; c < ncw; ++c) Z[(size_t)q * ncw + c] = 0.0; break; }
  }
  std::vector<double> H((size_t)r * ns);
  int32_t nsv = 0;
  if (gpd_host_parity_check(P, K, nullptr, present.data(), H.data(), &nsv) != GPD_OK || nsv != ns) std::exit(6);
  std::vector<double> Y((size_t)r * ncw, 0.0), G((size_t)r * r, 0.0);
  double energy = 0.0;
  for (double z : Z) energy += z * z;
  for (int i = 0; i < r; ++i)
    for (int q = 0; q < ns; ++q)
      for (int c = 0; c < ncw; ++c) Y[(size_t)i * ncw + c] += H[(size_t)i * ns + q] * Z[(size_t)q * ncw + c];
  for (int i = 0; i < r; ++i)
    for (int j = 0; j < r; ++j)
      for (int c = 0; c < ncw; ++c) G[(size_t)i * r + j] += Y[(size_t)i * ncw + c] * Y[(size_t)j * ncw + c];
  gpd_node_report_t rep;
  const gpd_status_t st = gpd_host_locate_nodes(P, K, nullptr, present.data(), G.data(), energy, ncw, rho, 0.0,
                                                force_one ? forced.data() : nullptr, &rep);
  std::printf("locate %d %d %d %d status %d n_bad %d exhaustive %d\n", P, K, ncw, t, (int)st, rep.n_bad, rep.exhaustive);
  line("present", present);
  line("planted", bad);
  line("forced", forced);
  line("found", std::vector<uint8_t>(rep.bad, rep.bad + P));
  line("stats", std::vector<double>{rep.energy, rep.syndrome_energy, rep.residual, rep.threshold});
}

static void pack_case(int nin, int nout, int r, bool with_pts, bool with_limits) {
  gpd::HostCombineTable t;
  t.nin = nin; t.nout = nout; t.r = r;
  t.in_off.assign(nin, 4); t.out_off.assign(nout, 8);
  t.coef.assign((size_t)nout * nin, 0.5); t.H.assign((size_t)r * nin, 0.25);
  t.node.assign(nin, 1);
  if (with_pts) t.pts.assign(nin, 0.1);
  if (with_limits) { t.in_rows.assign(nin, 3); t.in_cols.assign(nin, 8); t.out_rows.assign(nout, 3); t.out_cols.assign(nout, 8); }
  gpd::HostCombineTable probe;                      // what the library sizes its staging slots with
  probe.nin = nin; probe.nout = nout; probe.r = r;
  const size_t need = probe.bytes();
  char* buf = (char*)std::malloc(need);             // exactly that many bytes: an overrun is a sanitizer report
  const gpd::CombineTable v = t.pack(buf, buf);
  std::printf("pack %d %d %d bytes %zu karg %d %d align %d\n", nin, nout, r, need, (int)v.k_offsets, (int)v.k_coefs, v.off_align);
  std::free(buf);
}

int main() {
  const int subs[2] = {GPD_SUB_U_VN, GPD_SUB_V_UM};
  const int codes[][4] = {{2, 2, 2, 16}, {4, 2, 1, 24}, {2, 4, 1, 32}, {3, 2, 2, 20}, {1, 4, 1, 9}, {1, 1, 1, 1},
                          {2, 2, 4, 64}, {8, 8, 1, 64}, {2, 2, 2, 8}, {0, 2, 2, 10}, {2, 2, 2, 100}, {64, 1, 1, 64}};
  for (const auto& c : codes)
    for (int s : subs) code_case(c[0], c[1], c[2], c[3], s);
  {
    // evaluation points given by the caller: repeated and non-finite ones are refused
    std::vector<double> same(10, 0.5), nan_first(10, 0.0);
    for (int i = 0; i < 10; ++i) nan_first[i] = i;
    nan_first[0] = std::nan("");
    int32_t K = 0;
    std::printf("points_same status %d\n", (int)gpd_host_code(2, 2, 2, 10, 0, same.data(), &K, nullptr, nullptr, nullptr, nullptr));
    std::printf("points_nan status %d\n", (int)gpd_host_code(2, 2, 2, 10, 0, nan_first.data(), &K, nullptr, nullptr, nullptr, nullptr));
    std::vector<uint8_t> few(16, 0);
    for (int i = 0; i < 8; ++i) few[i] = 1;
    std::vector<double> D(4 * 16), H(16 * 16);
    int32_t ns = 0;
    std::printf("too_few status %d\n", (int)gpd_host_decode_matrices(2, 2, 2, 16, 0, nullptr, few.data(), 0, D.data(), H.data(), &ns));
    std::printf("last_error %s\n", gpd_last_error());
  }
  decode_case(2, 2, 2, 16, GPD_SUB_U_VN, 12);
  decode_case(4, 2, 1, 24, GPD_SUB_V_UM, 4);
  decode_case(2, 4, 1, 32, GPD_SUB_U_VN, 4);
  decode_case(2, 2, 4, 64, GPD_SUB_U_VN, 2);
  for (int t = 0; t <= 7; ++t) locate_case(16, 9, 40, t, t == 7 ? 1e-11 : 1.0 / 4096.0, 0, false);
  locate_case(16, 9, 24, 1, 1.0 / 4096.0, 2, true);
  locate_case(48, 12, 64, 14, 1.0 / 4096.0, 0, false);      // beyond the exhaustive budget
  locate_case(64, 40, 32, 5, 1.0 / 4096.0, 3, true);
  locate_case(12, 12, 8, 0, 1.0 / 4096.0, 0, false);         // no parity rows at all
  pack_case(64, 64, 64, true, true);
  pack_case(16, 4, 7, true, false);
  pack_case(4, 16, 0, false, true);
  pack_case(1, 1, 0, false, false);
  std::printf("done\n");
  return 0;
}
