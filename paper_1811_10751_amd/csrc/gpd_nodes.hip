// Node-level error location: the aggregate of Algorithm 1 (Sec. V) over all element codewords
// of a stack, for the error models of Sec. III where a faulty node's whole output is wrong.
//
// gram_kernel makes one pass over the stack and accumulates
//     G = sum_c (H z_c)(H z_c)^T      and      sum_c ||z_c||^2
// The syndromes H z_c are a dense contraction over the nodes (fp32 MFMA 16x16x4: 16 codewords
// x 16 syndromes per instruction, 4 nodes per step), the Gram matrix a contraction over the
// codewords (fp64 MFMA 16x16x4 fed with the syndrome accumulators as they come out of the
// first product: the sum over codewords does not care in which order they are taken).  The
// Gram matrix has to be exact to fp64 rounding: the search subtracts the energy explained by
// a node set from the total, and the total can exceed the threshold by many orders of
// magnitude.  The search itself runs on the host (gpd_host.cpp).
#include <algorithm>
#include <cmath>
#include <cstring>

#include "gpd_internal.hpp"

namespace gpd {
namespace {

typedef double v4d __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr float kWild = 1099511627776.0f;      // 2^40

struct GramParams {
  const float* in;
  const int64_t* in_off;     // [ns] element offset of each present node's block
  const float* H;            // [r][ns] fp32
  int ns, r;
  int64_t ncw;               // codewords = elements per block
  double* part;              // [gridDim.x][NT * 256 + 64]: Gram tiles, then the energy
  int32_t* wild;             // [ns], zeroed before the launch
};

template <int NK, int VEC>
struct ZTile { float v[NK][VEC]; };

// lane l loads VEC codewords starting at 16 VEC it + VEC (l % 16) from node 4 kk + l / 16
template <int NK, int VEC>
__device__ __forceinline__ ZTile<NK, VEC> load_ztile(const GramParams& p, const int64_t (&off)[NK], int64_t it,
                                                     int64_t n_iter, int lj) {
  ZTile<NK, VEC> z;
  const int64_t c0 = it * (16 * VEC) + VEC * lj;
#pragma unroll
  for (int kk = 0; kk < NK; ++kk) {
    if (it < n_iter && off[kk] >= 0 && c0 < p.ncw) {          // VEC = 4 only when 4 divides ncw
      if constexpr (VEC == 4) {
        const float4 v = *reinterpret_cast<const float4*>(p.in + off[kk] + c0);
        z.v[kk][0] = v.x; z.v[kk][1] = v.y; z.v[kk][2] = v.z; z.v[kk][3] = v.w;
      } else {
        z.v[kk][0] = p.in[off[kk] + c0];
      }
    } else {
#pragma unroll
      for (int c = 0; c < VEC; ++c) z.v[kk][c] = 0.f;
    }
  }
  return z;
}

// NK: steps of 4 nodes (ns <= 4 NK); RT: tiles of 16 syndromes (r <= 16 RT); VEC: codewords
// per lane and load.  A wavefront handles 16 VEC consecutive codewords per iteration; the loads
// of its next iteration are in flight while the current one is multiplied.
// PACK (RT = 1, VEC = 4, r <= 16 / PACK): the 16 columns of the syndrome tile are shared by
// PACK groups of codewords (group g owns columns g (16 / PACK) ..., its syndromes come from the
// codewords of load component g (4 / PACK) + q), so one fp64 product gives PACK diagonal
// blocks of Gram matrix at once; the blocks off the diagonal mix two groups and are dropped.
template <int NK, int RT, int VEC, int PACK>
__global__ __launch_bounds__(256) void gram_kernel(GramParams p) {
  static_assert(PACK == 1 || (RT == 1 && VEC == 4), "packing needs one tile and four components");
  constexpr int NT = RT * (RT + 1) / 2;
  constexpr int NH = PACK > 1 ? PACK : RT;       // B operands per node step
  constexpr int WCOL = 16 / PACK;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lj = lane & 15, lk = lane >> 4;

  // B operand of the syndrome product: B[k = node][j = syndrome] = H[j][node]
  float hreg[NK][NH];
  int64_t off[NK];
#pragma unroll
  for (int kk = 0; kk < NK; ++kk) {
    const int node = 4 * kk + lk;
    off[kk] = node < p.ns ? p.in_off[node] : -1;
#pragma unroll
    for (int t = 0; t < NH; ++t) {
      if constexpr (PACK > 1) {
        const int j = lj % WCOL;
        hreg[kk][t] = (node < p.ns && lj / WCOL == t && j < p.r) ? p.H[(int64_t)j * p.ns + node] : 0.f;
      } else {
        const int j = 16 * t + lj;
        hreg[kk][t] = (node < p.ns && j < p.r) ? p.H[(int64_t)j * p.ns + node] : 0.f;
      }
    }
  }

  // two accumulators per tile (RT <= 2): consecutive fp64 MFMAs do not wait for each other
  constexpr int NACC = RT <= 2 ? 2 : 1;
  v4d G[NT], G2[NACC == 2 ? NT : 1];
#pragma unroll
  for (int i = 0; i < NT; ++i) G[i] = v4d{0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int i = 0; i < (NACC == 2 ? NT : 1); ++i) G2[i] = v4d{0.0, 0.0, 0.0, 0.0};
  double energy = 0.0;
  uint32_t wildmask = 0;

  const int64_t n_iter = (p.ncw + 16 * VEC - 1) / (16 * VEC);
  const int64_t n_waves = (int64_t)gridDim.x * 4;
  int64_t it = (int64_t)blockIdx.x * 4 + wave;
  ZTile<NK, VEC> zn = load_ztile<NK, VEC>(p, off, it, n_iter, lj);
  for (; it < n_iter; it += n_waves) {
    ZTile<NK, VEC> z = zn;
    zn = load_ztile<NK, VEC>(p, off, it + n_waves, n_iter, lj);
    // non-finite and huge values: remember the node, take the value as zero
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
#pragma unroll
      for (int c = 0; c < VEC; ++c) {
        if (!(fabsf(z.v[kk][c]) < kWild)) { wildmask |= 1u << kk; z.v[kk][c] = 0.f; }
        const double x = (double)z.v[kk][c];
        energy = fma(x, x, energy);
      }
    }
    if constexpr (PACK > 1) {
#pragma unroll
      for (int q = 0; q < VEC / PACK; ++q) {
        v4f S = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int g = 0; g < PACK; ++g) {
#pragma unroll
          for (int kk = 0; kk < NK; ++kk)
            S = __builtin_amdgcn_mfma_f32_16x16x4f32(z.v[kk][g * (VEC / PACK) + q], hreg[kk][g], S, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          if (v & 1) G2[0] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)S[v], (double)S[v], G2[0], 0, 0, 0);
          else G[0] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)S[v], (double)S[v], G[0], 0, 0, 0);
        }
      }
    } else {
#pragma unroll
      for (int c = 0; c < VEC; ++c) {
        // S^T tile t: rows = 16 codewords, columns = syndromes 16 t .. 16 t + 15
        v4f S[RT];
#pragma unroll
        for (int t = 0; t < RT; ++t) S[t] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) {
#pragma unroll
          for (int t = 0; t < RT; ++t)
            S[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(z.v[kk][c], hreg[kk][t], S[t], 0, 0, 0);
        }
        // register v of lane l holds syndrome 16 t + l % 16 of codeword 4 (l / 16) + v: as the
        // A (and B) operand of the next product that is a 16 x 4 matrix [syndrome][codeword]
        int ti = 0;
#pragma unroll
        for (int t = 0; t < RT; ++t) {
#pragma unroll
          for (int t2 = t; t2 < RT; ++t2) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              if (NACC == 2 && (v & 1))
                G2[ti] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)S[t][v], (double)S[t2][v], G2[ti], 0, 0, 0);
              else
                G[ti] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)S[t][v], (double)S[t2][v], G[ti], 0, 0, 0);
            }
            ++ti;
          }
        }
      }
    }
  }

  if constexpr (NACC == 2) {
#pragma unroll
    for (int i = 0; i < NT; ++i) G[i] += G2[i];
  }

  // nodes that held a wild value
#pragma unroll
  for (int kk = 0; kk < NK; ++kk) {
    const int node = 4 * kk + lk;
    if (((wildmask >> kk) & 1u) && node < p.ns) atomicOr(&p.wild[node], 1);
  }

  // sum the four wavefronts of the workgroup (fixed order), one partial per workgroup
  __shared__ double red[3][256];
  __shared__ double red_e[4];
#pragma unroll
  for (int off2 = 32; off2 > 0; off2 >>= 1) energy += __shfl_xor(energy, off2);
  if (lane == 0) red_e[wave] = energy;
  double* dst = p.part + (int64_t)blockIdx.x * (NT * 256 + 64);
#pragma unroll
  for (int ti = 0; ti < NT; ++ti) {
    if (wave > 0) {
#pragma unroll
      for (int v = 0; v < 4; ++v) red[wave - 1][v * 64 + lane] = G[ti][v];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int v = 0; v < 4; ++v)
        dst[ti * 256 + v * 64 + lane] =
            ((G[ti][v] + red[0][v * 64 + lane]) + red[1][v * 64 + lane]) + red[2][v * 64 + lane];
    }
    __syncthreads();
  }
  if (wave == 0) dst[NT * 256 + lane] = lane == 0 ? ((red_e[0] + red_e[1]) + red_e[2]) + red_e[3] : 0.0;
}

// dst[g][i] = sum of src[w][i] over the g-th of gridDim.y equal ranges of w (fixed order).
__global__ __launch_bounds__(64) void sum_partials_kernel(const double* __restrict__ src, int n_src, int width,
                                                          double* __restrict__ dst) {
  const int i = blockIdx.x * 64 + threadIdx.x;
  const int per = (n_src + gridDim.y - 1) / gridDim.y;
  const int w0 = blockIdx.y * per, w1 = min(n_src, w0 + per);
  double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
  int w = w0;
  for (; w + 4 <= w1; w += 4) {
    a0 += src[(int64_t)w * width + i];
    a1 += src[(int64_t)(w + 1) * width + i];
    a2 += src[(int64_t)(w + 2) * width + i];
    a3 += src[(int64_t)(w + 3) * width + i];
  }
  for (; w < w1; ++w) a0 += src[(int64_t)w * width + i];
  dst[(int64_t)blockIdx.y * width + i] = (a0 + a1) + (a2 + a3);
}

int tiles_of(int r) { return r <= 16 ? 1 : (r <= 32 ? 2 : 4); }

int gram_grid(int64_t ncw, int RT, int vec) {
  const int64_t n_iter = (ncw + 16 * vec - 1) / (16 * vec);
  const int64_t max_wg = RT == 1 ? 2048 : (RT == 2 ? 512 : 256);
  return (int)std::max<int64_t>(1, std::min<int64_t>(max_wg, (n_iter + 3) / 4));
}

constexpr size_t kGramHeader = 512;      // wild[64] int32
constexpr int kGramGroups = 32;          // first reduction stage

// how many groups of codewords share one syndrome tile
int gram_pack(int r, int vec) { return (vec == 4 && r <= 16) ? (r <= 4 ? 4 : (r <= 8 ? 2 : 1)) : 1; }

template <int NK, int RT>
gpd_status_t launch_gram_v(hipStream_t s, const GramParams& p, int vec, int n_wg) {
  const int pack = RT == 1 ? gram_pack(p.r, vec) : 1;
  if constexpr (RT == 1) {
    if (pack == 4) GPD_LAUNCH((gram_kernel<NK, 1, 4, 4>), dim3(n_wg), dim3(256), 0, s, p);
    else if (pack == 2) GPD_LAUNCH((gram_kernel<NK, 1, 4, 2>), dim3(n_wg), dim3(256), 0, s, p);
  }
  if (pack == 1) {
    if (vec == 4) GPD_LAUNCH((gram_kernel<NK, RT, 4, 1>), dim3(n_wg), dim3(256), 0, s, p);
    else GPD_LAUNCH((gram_kernel<NK, RT, 1, 1>), dim3(n_wg), dim3(256), 0, s, p);
  }
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}

gpd_status_t launch_gram(hipStream_t s, const GramParams& p, int RT, int vec, int n_wg) {
  const int NK = p.ns <= 16 ? 4 : (p.ns <= 32 ? 8 : 16);
  if (NK == 4) return launch_gram_v<4, 1>(s, p, vec, n_wg);             // r < ns <= 16
  if (NK == 8) return RT == 1 ? launch_gram_v<8, 1>(s, p, vec, n_wg) : launch_gram_v<8, 2>(s, p, vec, n_wg);
  if (RT == 1) return launch_gram_v<16, 1>(s, p, vec, n_wg);
  if (RT == 2) return launch_gram_v<16, 2>(s, p, vec, n_wg);
  return launch_gram_v<16, 4>(s, p, vec, n_wg);
}

}  // namespace

size_t gram_workspace_bytes(int64_t ncw, int r) {
  const int RT = tiles_of(r), NT = RT * (RT + 1) / 2;
  const size_t width = (size_t)NT * 256 + 64;
  const int n_wg = gram_grid(ncw, RT, 1);            // the scalar path has the most workgroups
  const size_t b = kGramHeader + (1 + kGramGroups + (size_t)n_wg) * width * 8;
  return (b + 255) / 256 * 256;
}

gpd_status_t run_locate_nodes(hipStream_t stream, TableRing* ring, const std::vector<double>& pts,
                              int K, int64_t ncw, const float* Zt, const uint8_t* present, double rho,
                              double abs_floor, void* workspace, size_t workspace_bytes,
                              gpd_node_report_t* rep, double* gram_out, int64_t stride) {
  if (!rep) return fail(GPD_E_INVALID, "locate nodes: null report");
  if (stride == 0) stride = ncw;
  if (stride < ncw) return fail(GPD_E_SHAPE, "locate nodes: node stride smaller than a block");
  std::memset(rep, 0, sizeof(*rep));
  const int P = (int)pts.size();
  std::vector<int> S;
  for (int p = 0; p < P; ++p)
    if (!present || present[p]) S.push_back(p);
  const int ns = (int)S.size(), r = ns - K;
  rep->n_present = ns;
  if (ns < K) {
    rep->status = GPD_E_TOO_FEW;
    return fail(GPD_E_TOO_FEW, "%d responses present, %d needed", ns, K);
  }
  if (ncw == 0) return GPD_OK;
  if (!Zt) return fail(GPD_E_INVALID, "locate nodes: null stack");
  if (ncw > 0x7fffffffLL) return fail(GPD_E_SHAPE, "block has more than 2^31 elements");
  const size_t need = gram_workspace_bytes(ncw, r);
  if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))
    return fail(GPD_E_WORKSPACE, "locate nodes: workspace of %zu aligned bytes needed", need);

  std::vector<double> H;
  gpd_status_t st = parity_check_host(pts, S, K, &H);
  if (st != GPD_OK) { rep->status = st; return st; }

  std::string key("gram");
  key_add(&key, K); key_add(&key, ncw); key_add(&key, stride);
  for (int p = 0; p < P; ++p) key.push_back((!present || present[p]) ? 1 : 0);
  CombineTable t;
  st = ring->cached(key, [&](HostCombineTable* ht) {
    ht->nin = ns; ht->nout = 0; ht->r = r;
    ht->in_off.resize(ns); ht->node.resize(ns);
    for (int q = 0; q < ns; ++q) { ht->in_off[q] = (int64_t)S[q] * stride; ht->node[q] = S[q]; }
    ht->H = H;
    return GPD_OK;
  }, stream, &t);
  if (st != GPD_OK) { rep->status = st; return st; }

  const int RT = tiles_of(r), NT = RT * (RT + 1) / 2;
  const int vec = (ncw % 4 == 0 && ((uintptr_t)Zt % 16) == 0) ? 4 : 1;
  const int n_wg = gram_grid(ncw, RT, vec);
  char* ws = (char*)workspace;
  const int width = NT * 256 + 64;
  GramParams gp;
  gp.in = Zt; gp.in_off = t.in_off; gp.H = t.H; gp.ns = ns; gp.r = r; gp.ncw = ncw;
  gp.wild = (int32_t*)ws;
  double* d_out = (double*)(ws + kGramHeader);                 // [width]
  double* d_stage = d_out + width;                             // [kGramGroups][width]
  gp.part = d_stage + (size_t)kGramGroups * width;             // [n_wg][width]
  st = launch_zero_words(stream, ws, (int)(kGramHeader / 4));
  if (st != GPD_OK) return st;
  st = launch_gram(stream, gp, RT, vec, n_wg);
  if (st != GPD_OK) return st;
  // two reduction stages, both in a fixed order
  const int groups = std::min(kGramGroups, n_wg);
  GPD_LAUNCH(sum_partials_kernel, dim3(width / 64, groups), dim3(64), 0, stream, gp.part, n_wg, width,
                     d_stage);
  GPD_HIP(hipGetLastError());
  GPD_LAUNCH(sum_partials_kernel, dim3(width / 64, 1), dim3(64), 0, stream, d_stage, groups, width, d_out);
  GPD_HIP(hipGetLastError());

  // one copy brings the wild flags, the Gram tiles and the energy back
  std::vector<char> host(kGramHeader + (size_t)width * 8);
  GPD_HIP(hipMemcpyAsync(host.data(), ws, host.size(), hipMemcpyDeviceToHost, stream));
  GPD_HIP(hipStreamSynchronize(stream));
  const int32_t* h_wild = (const int32_t*)host.data();
  const double* tiles = (const double*)(host.data() + kGramHeader);
  const double energy = tiles[(size_t)NT * 256];
  // tile (t, t2), register v of lane l: row 16 t + 4 v + l / 16, column 16 t2 + l % 16
  std::vector<double> G((size_t)r * r, 0.0);
  const int pack = RT == 1 ? gram_pack(r, vec) : 1;
  if (pack > 1) {
    // diagonal blocks of the one tile, one per group of codewords
    const int w = 16 / pack;
    for (int v = 0; v < 4; ++v)
      for (int l = 0; l < 64; ++l) {
        const int row = 4 * v + l / 16, col = l % 16;
        if (row / w != col / w || row % w >= r || col % w >= r) continue;
        G[(size_t)(row % w) * r + col % w] += tiles[v * 64 + l];
      }
  }
  int ti = 0;
  for (int a = 0; a < RT && pack == 1; ++a)
    for (int b = a; b < RT; ++b, ++ti)
      for (int v = 0; v < 4; ++v)
        for (int l = 0; l < 64; ++l) {
          const int i = 16 * a + 4 * v + l / 16, j = 16 * b + l % 16;
          if (i >= r || j >= r) continue;
          const double x = tiles[(size_t)ti * 256 + v * 64 + l];
          G[(size_t)i * r + j] = x;
          if (a != b) G[(size_t)j * r + i] = x;
        }
  if (gram_out) std::copy(G.begin(), G.end(), gram_out);
  std::vector<int> forced;
  for (int q = 0; q < ns; ++q)
    if (h_wild[q]) { forced.push_back(q); rep->wild[S[q]] = 1; }
  NodeSearchResult res;
  st = locate_nodes_host(H, r, ns, G, energy, ncw, rho, abs_floor, forced, &res);
  if (st != GPD_OK) { rep->status = st; return st; }
  fill_node_report(res, S, rep);
  if (res.status == 2) return fail(GPD_E_DECODE_FAIL, "more erroneous nodes than can be located");
  return GPD_OK;
}

// ---------------------------------------------------------------- verification step

namespace {

// z[t][p] = Zt[p][pos_t] for every node p; c[t][q] = entry of output block q at element pos_t
__global__ void gather_check_kernel(const float* __restrict__ Zt, int P, int64_t ncw, int64_t stride, int n_check,
                                    const float* __restrict__ out, int64_t ld_out, int grid_r, int grid_c,
                                    int64_t bh, int64_t bw, float* __restrict__ z, float* __restrict__ c) {
  const int t = blockIdx.x;
  if (t >= n_check) return;
  const int64_t pos = ((int64_t)t * ncw) / n_check;
  const int64_t r = pos / bw, col = pos - r * bw;
  for (int p = threadIdx.x; p < P; p += blockDim.x) z[(int64_t)t * P + p] = Zt[(int64_t)p * stride + pos];
  const int nq = grid_r * grid_c;
  for (int q = threadIdx.x; q < nq; q += blockDim.x) {
    const int i = q / grid_c, k = q - i * grid_c;
    c[(int64_t)t * nq + q] = out[((int64_t)i * bh + r) * ld_out + (int64_t)k * bw + col];
  }
}

}  // namespace

gpd_status_t run_verify(hipStream_t stream, const DecodeJob& job, const float* Zt, const uint8_t* present,
                        int mode, const uint8_t* bad, const float* out, int64_t ld_out, int n_check,
                        void* workspace, size_t workspace_bytes, gpd_verify_report_t* rep) {
  if (!rep) return fail(GPD_E_INVALID, "verify: null report");
  std::memset(rep, 0, sizeof(*rep));
  if (mode != GPD_DEC_FIRST_K && mode != GPD_DEC_LSQ_ALL) return fail(GPD_E_INVALID, "verify: bad mode");
  if (!job.out_cols.empty()) return fail(GPD_E_UNSUPPORTED, "verify: padded output grids are not supported");
  const int P = (int)job.pts->size(), K = job.K;
  const int64_t ncw = job.bh * job.bw;
  const int nq = job.grid_r * job.grid_c;
  if (n_check <= 0) n_check = P;
  if (n_check > 4096) return fail(GPD_E_INVALID, "verify: at most 4096 values are checked");
  if ((int64_t)n_check > ncw) n_check = (int)ncw;
  rep->locations_agree = 1;
  if (ncw == 0) return GPD_OK;
  if (!Zt || !out) return fail(GPD_E_INVALID, "verify: null buffer");
  if (ld_out < job.grid_c * job.bw) return fail(GPD_E_SHAPE, "verify: output leading dimension too small");
  const size_t need = 512 + sizeof(float) * (size_t)n_check * (P + nq);
  if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))
    return fail(GPD_E_WORKSPACE, "verify: workspace of %zu aligned bytes needed", need);

  std::vector<int> S, S_main;
  for (int p = 0; p < P; ++p)
    if (!present || present[p]) {
      S.push_back(p);
      if (!bad || !bad[p]) S_main.push_back(p);
    }
  if ((int)S_main.size() < K) return fail(GPD_E_TOO_FEW, "%d responses left, %d needed", (int)S_main.size(), K);

  float* d_z = (float*)((char*)workspace + 512);
  float* d_c = d_z + (size_t)n_check * P;
  const int64_t stride = job.in_stride ? job.in_stride : ncw;
  if (stride < ncw) return fail(GPD_E_SHAPE, "verify: node stride smaller than a block");
  GPD_LAUNCH(gather_check_kernel, dim3(n_check), dim3(64), 0, stream, Zt, P, ncw, stride, n_check, out, ld_out,
                     job.grid_r, job.grid_c, job.bh, job.bw, d_z, d_c);
  GPD_HIP(hipGetLastError());
  std::vector<float> hz((size_t)n_check * P), hc((size_t)n_check * nq);
  GPD_HIP(hipMemcpyAsync(hz.data(), d_z, sizeof(float) * hz.size(), hipMemcpyDeviceToHost, stream));
  GPD_HIP(hipMemcpyAsync(hc.data(), d_c, sizeof(float) * hc.size(), hipMemcpyDeviceToHost, stream));
  GPD_HIP(hipStreamSynchronize(stream));

  // ---- second node search, on the sampled codewords only
  const int ns = (int)S.size(), r = ns - K;
  std::vector<double> H;
  gpd_status_t st = parity_check_host(*job.pts, S, K, &H);
  if (st != GPD_OK) return st;
  std::vector<double> Zs((size_t)n_check * ns), G((size_t)r * r, 0.0), y(r);
  std::vector<char> wild(ns, 0);
  double energy = 0.0;
  for (int t = 0; t < n_check; ++t) {
    for (int q = 0; q < ns; ++q) {
      double v = hz[(size_t)t * P + S[q]];
      if (!(std::fabs(v) < 1099511627776.0)) { wild[q] = 1; v = 0.0; }
      Zs[(size_t)t * ns + q] = v;
      energy += v * v;
    }
    for (int i = 0; i < r; ++i) {
      double acc = 0.0;
      for (int q = 0; q < ns; ++q) acc += H[(size_t)i * ns + q] * Zs[(size_t)t * ns + q];
      y[i] = acc;
    }
    for (int i = 0; i < r; ++i)
      for (int j = 0; j < r; ++j) G[(size_t)i * r + j] += y[i] * y[j];
  }
  std::vector<int> forced;
  for (int q = 0; q < ns; ++q)
    if (wild[q]) forced.push_back(q);
  NodeSearchResult res;
  st = locate_nodes_host(H, r, ns, G, energy, n_check, job.rho, job.abs_floor, forced, &res);
  if (st != GPD_OK) return st;
  std::vector<char> chk_bad(P, 0);
  for (int q : res.bad) { chk_bad[S[q]] = 1; rep->bad[S[q]] = 1; }
  bool agree = res.status != 2;
  for (int p = 0; p < P; ++p)
    if ((!present || present[p]) && ((bad && bad[p]) != (chk_bad[p] != 0))) agree = false;
  rep->locations_agree = agree ? 1 : 0;

  // ---- second decode of the sampled codewords: least squares over what the search leaves
  std::vector<int> S_chk;
  for (int q = 0; q < ns; ++q)
    if (!chk_bad[S[q]]) S_chk.push_back(S[q]);
  rep->n_checked = n_check;
  if ((int)S_chk.size() < K) {
    rep->status = GPD_E_VERIFY;
    return fail(GPD_E_VERIFY, "verification: the second node search leaves fewer than K nodes");
  }
  std::vector<double> D_main, D_chk;
  st = decode_matrices(*job.pts, S_main, K, job.useful, mode == GPD_DEC_FIRST_K, &D_main, nullptr);
  if (st != GPD_OK) return st;
  st = decode_matrices(*job.pts, S_chk, K, job.useful, false, &D_chk, nullptr);
  if (st != GPD_OK) return st;
  const int nm = (int)S_main.size(), nc = (int)S_chk.size();
  std::vector<double> a_main(nq), a_chk(nq);
  for (int q = 0; q < nq; ++q) {
    double s1 = 0.0, s2 = 0.0;
    for (int x = 0; x < nm; ++x) s1 += D_main[(size_t)q * nm + x] * D_main[(size_t)q * nm + x];
    for (int x = 0; x < nc; ++x) s2 += D_chk[(size_t)q * nc + x] * D_chk[(size_t)q * nc + x];
    a_main[q] = std::sqrt(s1); a_chk[q] = std::sqrt(s2);
  }
  for (int t = 0; t < n_check; ++t) {
    double zn = 0.0;
    std::vector<double> zc(nc);
    for (int x = 0; x < nc; ++x) {
      double v = hz[(size_t)t * P + S_chk[x]];
      if (!std::isfinite(v)) v = 0.0;
      zc[x] = v; zn += v * v;
    }
    zn = std::sqrt(zn);
    double worst = 0.0;
    for (int q = 0; q < nq; ++q) {
      double want = 0.0;
      for (int x = 0; x < nc; ++x) want += D_chk[(size_t)q * nc + x] * zc[x];
      const double tol = std::ldexp(1.0, -20) * (a_main[q] + a_chk[q]) * zn;
      const double got = hc[(size_t)t * nq + q];
      double ratio;
      if (!std::isfinite(got)) ratio = INFINITY;
      else if (tol > 0) ratio = std::fabs(got - want) / tol;
      else ratio = got == want ? 0.0 : INFINITY;
      worst = std::max(worst, ratio);
    }
    rep->max_ratio = std::max(rep->max_ratio, worst);
    if (worst > 1.0) rep->n_value_mismatch += 1;
  }
  if (rep->n_value_mismatch > 0 || !agree) {
    rep->status = GPD_E_VERIFY;
    return fail(GPD_E_VERIFY, "verification: %d of %d checked values disagree, node lists %s", rep->n_value_mismatch,
                n_check, agree ? "agree" : "differ");
  }
  return GPD_OK;
}

}  // namespace gpd
