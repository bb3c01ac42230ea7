// Error location and correction for the codewords the fp32 screen passed on
// (Sec. V, Algorithm 1 steps 1-3; appendix "Decoding Methods"), in fp64.
//
// One wavefront handles one codeword z (the values one element position takes over the
// present nodes):
//   step 1   y = H z, sigma = ||y||, tau = rho * max(||z||, floor); clean if sigma <= tau
//            and every entry is finite (this fp64 test is the decision; the fp32 screen only
//            preselects).
//   step 2   supports of increasing size (always containing the non-finite entries, which
//            are set to zero first); inside one size the lanes share out the supports, each
//            computes the least-squares residual of y against the support's columns of H by
//            modified Gram-Schmidt, and the smallest residual <= tau wins (ties: the first
//            support in lexicographic order).
//   step 3   supports larger than |S| - K - 1 are never tried: decoding failure.
// Correction: e_hat solves H_A e = y in the least-squares sense; the outputs are the rows of
// the all-node least-squares decoding matrix applied to z - e_hat, which equals least squares
// over the nodes outside the support.
// Latency-bound plain-ALU work on a handful of codewords; not on the bandwidth path.
#include "gpd_internal.hpp"

namespace gpd {

namespace {

constexpr int S_MAX = 8;                       // largest support size searched
constexpr int R_MAX = 64;                      // largest number of parity rows
constexpr unsigned long long kBudget = 1ull << 22;   // supports tried per size, at most

struct LocateParams {
  CombineTable t;
  const float* in; int64_t in_ld;
  float* out; int64_t out_ld;
  int64_t cols;
  double rho, abs_floor;
  uint32_t* counters;         // [0] screened, [2] flagged, [3] failed, [4] located
  const int32_t* list; int32_t cap;
  gpd_located_t* located; int64_t located_cap;
  int32_t* node_err;
};

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// Residual of y against the columns `supp[0..size)` of H (r x ns, row-major) by modified
// Gram-Schmidt; optionally returns the least-squares coefficients.
__device__ double support_residual(const double* __restrict__ H, int r, int ns,
                                   const double* __restrict__ y, const int* supp, int size,
                                   double* e_out) {
  double Q[S_MAX][R_MAX];
  double R[S_MAX][S_MAX];
  double qty[S_MAX];
  for (int j = 0; j < size; ++j) {
    for (int i = 0; i < r; ++i) Q[j][i] = H[(int64_t)i * ns + supp[j]];
    for (int l = 0; l < j; ++l) {
      double dot = 0.0;
      for (int i = 0; i < r; ++i) dot += Q[l][i] * Q[j][i];
      R[l][j] = dot;
      for (int i = 0; i < r; ++i) Q[j][i] -= dot * Q[l][i];
    }
    double nrm = 0.0;
    for (int i = 0; i < r; ++i) nrm += Q[j][i] * Q[j][i];
    nrm = sqrt(nrm);
    R[j][j] = nrm;
    const double inv = nrm > 0.0 ? 1.0 / nrm : 0.0;
    for (int i = 0; i < r; ++i) Q[j][i] *= inv;
  }
  double w[R_MAX];
  for (int i = 0; i < r; ++i) w[i] = y[i];
  for (int j = 0; j < size; ++j) {
    double dot = 0.0;
    for (int i = 0; i < r; ++i) dot += Q[j][i] * w[i];
    qty[j] = dot;
    for (int i = 0; i < r; ++i) w[i] -= dot * Q[j][i];
  }
  double res = 0.0;
  for (int i = 0; i < r; ++i) res += w[i] * w[i];
  if (e_out) {
    for (int j = size - 1; j >= 0; --j) {
      double acc = qty[j];
      for (int l = j + 1; l < size; ++l) acc -= R[j][l] * e_out[l];
      e_out[j] = R[j][j] > 0.0 ? acc / R[j][j] : 0.0;
    }
  }
  return sqrt(res);
}

__global__ __launch_bounds__(64) void locate_kernel(LocateParams p) {
  __shared__ double zs[64];
  __shared__ double ys[R_MAX];
  __shared__ unsigned long long binom[65][S_MAX + 1];
  __shared__ int freelist[64];
  __shared__ int forcedlist[64];

  const int lane = threadIdx.x;
  const int ns = p.t.nin, r = p.t.r, nout = p.t.nout;

  uint32_t n_list = p.counters[0];
  if (n_list > (uint32_t)p.cap) n_list = (uint32_t)p.cap;
  if (blockIdx.x >= n_list) return;                        // nothing screened for this wavefront

  // Pascal's triangle for the unranking of supports: row a is built by lane b from row a - 1
  if (lane <= S_MAX) binom[0][lane] = lane == 0 ? 1ull : 0ull;
  __syncthreads();
  for (int a = 1; a <= 64; ++a) {
    if (lane <= S_MAX) binom[a][lane] = lane == 0 ? 1ull : binom[a - 1][lane - 1] + binom[a - 1][lane];
    __syncthreads();
  }

  for (uint32_t w = blockIdx.x; w < n_list; w += gridDim.x) {
    const int32_t cw = p.list[w];
    const int64_t row = cw / p.cols, col = cw % p.cols;

    // ---- step 1 in fp64
    double z = 0.0;
    bool bad = false;
    if (lane < ns) {
      const float zf = p.in[p.t.in_off[lane] + row * p.in_ld + col];
      bad = !(fabsf(zf) <= 3.4028234664e38f);
      z = bad ? 0.0 : (double)zf;
    }
    zs[lane] = z;
    const unsigned long long forced_mask = __ballot(bad);
    const int nforced = __popcll(forced_mask);
    __syncthreads();
    double y = 0.0;
    if (lane < r) {
      const double* __restrict__ hrow = p.t.H64 + (int64_t)lane * ns;
      for (int s = 0; s < ns; ++s) y += hrow[s] * zs[s];
    }
    if (lane < R_MAX) ys[lane] = y;
    const double sigma = sqrt(wave_sum(y * y));
    const double znorm = sqrt(wave_sum(z * z));
    const double tau = p.rho * fmax(znorm, p.abs_floor);
    __syncthreads();
    if (nforced == 0 && sigma <= tau) continue;            // clean (wave-uniform)
    if (lane == 0) atomicAdd(&p.counters[2], 1u);

    // ---- step 2: free / forced node lists (positions inside the present set)
    if (lane == 0) {
      int nf = 0, nfo = 0;
      for (int s = 0; s < ns; ++s) {
        if ((forced_mask >> s) & 1ull) forcedlist[nfo++] = s; else freelist[nf++] = s;
      }
    }
    __syncthreads();
    const int nfree = ns - nforced;
    int max_size = r - 1;                                  // step 3: |A| <= |S| - K - 1
    if (max_size > S_MAX) max_size = S_MAX;

    bool found = false;
    int best_size = 0;
    unsigned long long best_c = 0;
    int supp[S_MAX];
    for (int size = nforced > 1 ? nforced : 1; size <= max_size && !found; ++size) {
      const int tpick = size - nforced;
      const unsigned long long total = binom[nfree][tpick];
      if (total > kBudget) break;
      double my_res = 1.0e300;
      unsigned long long my_c = ~0ull;
      for (unsigned long long c = lane; c < total; c += 64) {
        // unrank c among the tpick-subsets of the free nodes, lexicographic order
        for (int f = 0; f < nforced; ++f) supp[f] = forcedlist[f];
        unsigned long long rest = c;
        int x = 0;
        for (int i = 0; i < tpick; ++i) {
          for (;; ++x) {
            const unsigned long long cnt = binom[nfree - x - 1][tpick - i - 1];
            if (rest < cnt) break;
            rest -= cnt;
          }
          supp[nforced + i] = freelist[x];
          ++x;
        }
        const double res = support_residual(p.t.H64, r, ns, ys, supp, size, nullptr);
        if (res <= tau && res < my_res) { my_res = res; my_c = c; }
      }
      // wave-wide arg-min (smallest residual, then smallest index)
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        const double o_res = __shfl_xor(my_res, off);
        const unsigned long long o_c = __shfl_xor(my_c, off);
        if (o_res < my_res || (o_res == my_res && o_c < my_c)) { my_res = o_res; my_c = o_c; }
      }
      if (my_c != ~0ull) { found = true; best_size = size; best_c = my_c; }
    }

    if (!found) {
      if (lane == 0) atomicAdd(&p.counters[3], 1u);
      continue;
    }

    // ---- correction: every lane rebuilds the winning support and its e_hat
    const int tpick = best_size - nforced;
    for (int f = 0; f < nforced; ++f) supp[f] = forcedlist[f];
    {
      unsigned long long rest = best_c;
      int x = 0;
      for (int i = 0; i < tpick; ++i) {
        for (;; ++x) {
          const unsigned long long cnt = binom[nfree - x - 1][tpick - i - 1];
          if (rest < cnt) break;
          rest -= cnt;
        }
        supp[nforced + i] = freelist[x];
        ++x;
      }
    }
    // The located entries are now treated as erasures: set them to zero, recompute the
    // syndrome and solve H_A e' = H z' for the values the code predicts there (-e').  This
    // keeps all arithmetic at the scale of the clean responses however large the error was.
    double z_orig[S_MAX];
    for (int j = 0; j < best_size; ++j) z_orig[j] = zs[supp[j]];
    __syncthreads();
    if (lane == 0)
      for (int j = 0; j < best_size; ++j) zs[supp[j]] = 0.0;
    __syncthreads();
    double y2 = 0.0;
    if (lane < r) {
      const double* __restrict__ hrow = p.t.H64 + (int64_t)lane * ns;
      for (int s = 0; s < ns; ++s) y2 += hrow[s] * zs[s];
    }
    __syncthreads();
    ys[lane] = y2;
    __syncthreads();
    double e_hat[S_MAX];
    support_residual(p.t.H64, r, ns, ys, supp, best_size, e_hat);
    __syncthreads();
    if (lane == 0)
      for (int j = 0; j < best_size; ++j) zs[supp[j]] = -e_hat[j];
    __syncthreads();
    // estimated error value = received - predicted
    for (int j = 0; j < best_size; ++j) e_hat[j] = z_orig[j] + e_hat[j];
    bool write = lane < nout;
    if (write && p.t.out_rows) write = row < p.t.out_rows[lane] && col < p.t.out_cols[lane];
    if (write) {
      const double* __restrict__ drow = p.t.coef64 + (int64_t)lane * ns;
      double acc = 0.0;
      for (int s = 0; s < ns; ++s) acc += drow[s] * zs[s];
      p.out[p.t.out_off[lane] + row * p.out_ld + col] = (float)acc;
    }
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(&p.counters[4], (uint32_t)best_size);
    base = __shfl(base, 0);
    if (lane < best_size) {
      const int s = supp[lane];
      const int node = p.t.node[s];
      atomicAdd(&p.node_err[node], 1);
      if ((int64_t)base + lane < p.located_cap) {
        gpd_located_t rec;
        rec.node = node; rec.row = (int32_t)row; rec.col = (int32_t)col;
        rec.magnitude = ((forced_mask >> s) & 1ull) ? __uint_as_float(0x7fc00000u) : (float)e_hat[lane];
        p.located[base + lane] = rec;
      }
    }
    __syncthreads();
  }
}

__global__ void zero_words_kernel(uint32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

}  // namespace

gpd_status_t launch_zero_words(hipStream_t stream, void* p, int n_words) {
  if (n_words <= 0) return GPD_OK;
  hipLaunchKernelGGL(zero_words_kernel, dim3((n_words + 255) / 256), dim3(256), 0, stream,
                     (uint32_t*)p, n_words);
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}

gpd_status_t launch_locate(hipStream_t stream, const LocateArgs& a) {
  if (a.t.nin > 64 || a.t.r > R_MAX || a.t.nout > 64)
    return fail(GPD_E_UNSUPPORTED, "locate: more than 64 nodes, parity rows or outputs");
  LocateParams p;
  p.t = a.t; p.in = a.in; p.in_ld = a.in_ld; p.out = a.out; p.out_ld = a.out_ld;
  p.cols = a.cols; p.rho = a.rho; p.abs_floor = a.abs_floor;
  p.counters = a.counters; p.list = a.list; p.cap = a.n_list;
  p.located = a.located; p.located_cap = a.located_cap; p.node_err = a.node_err;
  // every wavefront strides over the screened list and leaves when it runs out
  const int blocks = a.n_list < 2048 ? (a.n_list > 0 ? a.n_list : 1) : 2048;
  hipLaunchKernelGGL(locate_kernel, dim3(blocks), dim3(64), 0, stream, p);
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}

}  // namespace gpd
