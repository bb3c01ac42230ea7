// Coded DNN layer step (Sec. VII for mini-batch 1, Sec. IX for mini-batch > 1): the weight
// stays encoded as W~_p = sum_ij W_ij a_p^i b_p^j on every node; only X and Delta are
// encoded and decoded per iteration, and the update is applied to W~_p directly.
//
// Kernels here are the small-batch ("skinny") streaming products, which are HBM-bound on
// reading / rewriting W~:
//   skinny_forward   S~_p = W~_p X~_p                 one wavefront per row of W~_p
//   skinny_backward_update
//                    C~_p = W~_p^T Delta~_p (pre-update W~_p) and
//                    W~_p <- (1-decay) W~_p + eta Dhat_p Xhat_p^T in ONE pass over W~_p
// Larger batches go through the MFMA GEMMs of gpd_gemm.hip.  Element-wise steps C1 / C2
// are at the end.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <string>

#include "gpd_internal.hpp"

namespace gpd {

namespace {

// W~ is read (and rewritten) exactly once per pass: streaming accesses that do not displace the
// small operands from the caches and leave no dirty lines behind for the end of the kernel
typedef float v4f __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 stream_load4(const float* p) {
  const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
  return make_float4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void stream_store4(float* p, float a, float b, float c, float d) {
  v4f t; t.x = a; t.y = b; t.z = c; t.w = d;
  __builtin_nontemporal_store(t, reinterpret_cast<v4f*>(p));
}

constexpr int kSkinnyMaxBatch = 8;      // widest per-node batch the streaming kernels take
constexpr int kRowChunk = 64;           // rows of W~_p one workgroup of the backward pass owns

// ---------------------------------------------------------------- projection on the matrix cores

// out_q[e] = sum_s coef[q][s] in_s[e] for up to 32 input and 32 output blocks of n contiguous
// elements each, outputs possibly overwriting inputs.  With P inputs and P outputs the vector
// units need 2 P^2 flops per element (the projection of a 24-node stack ran at 1.9 TB/s on them);
// as a product coef (32 x nin) times in (nin x 32 elements) it is v_mfma_f32_32x32x2_f32 work:
// A operand coef[q = lane % 32][s = 2 kk + lane / 32], B operand in_s[e0 + 4 (lane % 32) + c] for
// the four components c of one 16-byte load, four accumulators of 32 outputs x 32 elements.  A
// wavefront owns 128 elements: it loads them from every input block before it stores any output
// (in-place safe), and a lane's 16 accumulator values of component c are outputs
// q = 8 (v / 4) + 4 (lane / 32) + v % 4 of element e0 + 4 (lane % 32) + c.
constexpr int kStackMax = 32;
struct StackParams {
  const float* in; float* out; const float* coef;      // coef: device, [nout][nin]
  int32_t nin, nout;
  int64_t n;                                           // elements per block, a multiple of 128
  int64_t in_off[kStackMax], out_off[kStackMax];
};
typedef float floatx16 __attribute__((ext_vector_type(16)));

// KS: pairs of input blocks the kernel is compiled for (nin <= 2 KS)
template <int KS>
__global__ __launch_bounds__(256) void stack_mfma_kernel(const StackParams p) {
  const int lane = threadIdx.x & 63, j = lane & 31, g = lane >> 5;
  const int64_t e0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 128;
  if (e0 >= p.n) return;
  float a[KS];
  float4 v[KS];
  // (table entries are read with uniform indices and selected by lane half afterwards: an index
  // that differs between lanes would turn the kernel-argument reads into vector loads)
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    const int s = 2 * kk + g;
    const bool on = s < p.nin;
    const int s0 = min(2 * kk, p.nin - 1), s1 = min(2 * kk + 1, p.nin - 1);
    const int64_t o0 = p.in_off[s0], o1 = p.in_off[s1];
    a[kk] = (on && j < p.nout) ? p.coef[(int64_t)min(j, p.nout - 1) * p.nin + (g ? s1 : s0)] : 0.f;
    v[kk] = *reinterpret_cast<const float4*>(p.in + (g ? o1 : o0) + e0 + 4 * j);
    if (!on) v[kk] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  floatx16 acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kk], v[kk].x, acc[0], 0, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kk], v[kk].y, acc[1], 0, 0, 0);
    acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kk], v[kk].z, acc[2], 0, 0, 0);
    acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kk], v[kk].w, acc[3], 0, 0, 0);
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int qa = 8 * (i >> 2) + (i & 3), q = qa + 4 * g;
    const int64_t o0 = p.out_off[qa], o1 = p.out_off[qa + 4];
    if (q < p.nout)
      *reinterpret_cast<float4*>(p.out + (g ? o1 : o0) + e0 + 4 * j) = make_float4(acc[0][i], acc[1][i], acc[2][i], acc[3][i]);
  }
}

// ---------------------------------------------------------------- small operand encodes

// The three operand encodes of a small-batch backward / update step (Delta~, Dhat, Xhat: a few
// KB each) in one launch; blockIdx.y is the job.
//   out[p][r][b] = sum_s coef[p][s] * in[off[s] + r * ld + b], block s reading as zero at
//   r >= lim_r[s] or b >= lim_c[s] (zero padding of ragged edge blocks).
constexpr int kSmallMaxIn = 8;
struct SmallEnc {
  const float* in = nullptr;           // the unencoded matrix (device)
  const float* coef = nullptr;         // device, [P][nin]: evaluation point powers
  float* out = nullptr;                // [P][rows][nb]
  int32_t ld = 0, nin = 0, rows = 0, nb = 0;
  int32_t count = 0;                   // P * rows * nb
  int64_t off[kSmallMaxIn] = {};
  int32_t lim_r[kSmallMaxIn] = {}, lim_c[kSmallMaxIn] = {};
};
struct SmallEncJobs { SmallEnc job[3]; };

__global__ __launch_bounds__(256) void encode_small_kernel(const SmallEncJobs jobs) {
  const SmallEnc& j = jobs.job[blockIdx.y];
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;      // count < 2^31 (host-checked)
  if (i >= (uint32_t)j.count) return;
  const uint32_t pr = i / (uint32_t)j.nb;
  const int b = (int)(i - pr * (uint32_t)j.nb);
  const int p = (int)(pr / (uint32_t)j.rows), r = (int)(pr - (uint32_t)p * (uint32_t)j.rows);
  float z[kSmallMaxIn], cs[kSmallMaxIn];
  // one round of loads: blocks beyond nin re-read the last one with weight 0
#pragma unroll
  for (int s = 0; s < kSmallMaxIn; ++s) {
    const int sc = min(s, j.nin - 1);
    cs[s] = s < j.nin ? j.coef[p * j.nin + sc] : 0.f;
    z[s] = (r < j.lim_r[sc] && b < j.lim_c[sc]) ? j.in[j.off[sc] + (int64_t)r * j.ld + b] : 0.f;
  }
  float a = 0.f;
#pragma unroll
  for (int s = 0; s < kSmallMaxIn; ++s) a = fmaf(cs[s], z[s], a);
  j.out[i] = a;
}

// ---------------------------------------------------------------- skinny forward

// S~[p][r][b] = sum_c W~[p][r][c] * X~[p][c][b];  NB = per-node batch (columns of X~_p).
// A workgroup owns FR consecutive rows of W~_p, i.e. one contiguous piece of memory, and
// walks through it like a copy kernel (thread t reads 16 bytes at column 4t, 4t+1024, ...), so
// that concurrent workgroups spread over all HBM channels.  The X~ values of a thread's
// columns are fetched once and reused for every row.  All FR row loads of a strip are issued
// before the first is used; rows beyond the matrix (last group only) re-read its last row and
// are never stored, so that the loop has no branch.  Row sums: wavefront shuffle, then LDS.
constexpr int fwd_rows(int nb) { return nb == 1 ? 2 : 4; }

template <int NB>
__global__ __launch_bounds__(256) void skinny_forward_kernel(const float* __restrict__ Wt,
                                                             const float* __restrict__ Xt,
                                                             float* __restrict__ St, int rows,
                                                             int cols) {
  constexpr int FR = fwd_rows(NB);
  __shared__ float part[4][FR][NB];
  const int p = blockIdx.y;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int row0 = blockIdx.x * FR;
  const float* __restrict__ x = Xt + (int64_t)p * cols * NB;
  const int nrows = min(FR, rows - row0);
  const float* wr[FR];
#pragma unroll
  for (int r = 0; r < FR; ++r) wr[r] = Wt + ((int64_t)p * rows + row0 + min(r, nrows - 1)) * cols;
  float acc[FR][NB];
#pragma unroll
  for (int r = 0; r < FR; ++r)
#pragma unroll
    for (int b = 0; b < NB; ++b) acc[r][b] = 0.f;
  if ((cols & 3) == 0) {
    for (int c = tid * 4; c < cols; c += 1024) {
      float4 wv[FR];
#pragma unroll
      for (int r = 0; r < FR; ++r) wv[r] = stream_load4(wr[r] + c);
      float xv[4 * NB];                      // X~[c .. c+3][0 .. NB-1], contiguous
      if constexpr ((NB & 3) == 0 || NB == 1) {
#pragma unroll
        for (int q = 0; q < NB; ++q) {
          const float4 t = *reinterpret_cast<const float4*>(x + (int64_t)c * NB + 4 * q);
          xv[4 * q] = t.x; xv[4 * q + 1] = t.y; xv[4 * q + 2] = t.z; xv[4 * q + 3] = t.w;
        }
      } else {
#pragma unroll
        for (int q = 0; q < 4 * NB; ++q) xv[q] = x[(int64_t)c * NB + q];
      }
#pragma unroll
      for (int r = 0; r < FR; ++r) {
        const float we[4] = {wv[r].x, wv[r].y, wv[r].z, wv[r].w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int b = 0; b < NB; ++b) acc[r][b] = fmaf(we[e], xv[e * NB + b], acc[r][b]);
      }
    }
  } else {
    for (int c = tid; c < cols; c += 256) {
      float wv[FR];
#pragma unroll
      for (int r = 0; r < FR; ++r) wv[r] = wr[r][c];
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const float xb = x[(int64_t)c * NB + b];
#pragma unroll
        for (int r = 0; r < FR; ++r) acc[r][b] = fmaf(wv[r], xb, acc[r][b]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < FR; ++r)
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      float v = acc[r][b];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
      if (lane == 0) part[wave][r][b] = v;
    }
  __syncthreads();
  if (tid < FR * NB) {
    const int r = tid / NB, b = tid % NB;
    if (r < nrows)
      St[((int64_t)p * rows + row0 + r) * NB + b] = (part[0][r][b] + part[1][r][b]) + (part[2][r][b] + part[3][r][b]);
  }
}

// ---------------------------------------------------------------- skinny backward + update

// One workgroup owns rows [chunk*kRowChunk, ...) of W~_p and all columns; a thread owns 4
// consecutive columns per 1024-column strip.
//   part[p][chunk][c][b2] = sum_{r in chunk} W~[p][r][c] * Dt[p][r][b2]        (DO_BWD)
//   W~[p][r][c] = keep * W~[p][r][c] + eta * sum_b Dh[p][r][b] * Xh[p][c][b]   (DO_UPD)
template <int NB2, int NBU, bool DO_BWD, bool DO_UPD>
__global__ __launch_bounds__(256) void skinny_backward_update_kernel(
    float* __restrict__ Wt, const float* __restrict__ Dt, const float* __restrict__ Dh,
    const float* __restrict__ Xh, float* __restrict__ part, int rows, int cols, int nchunks,
    float keep, float eta) {
  const int p = blockIdx.z, chunk = blockIdx.y;
  const int c0 = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (c0 >= cols) return;
  const int r0 = chunk * kRowChunk;
  const int r1 = min(rows, r0 + kRowChunk);
  const bool vec = c0 + 3 < cols;
  float xh[4][NBU > 0 ? NBU : 1];
  if constexpr (DO_UPD) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int b = 0; b < NBU; ++b)
        xh[e][b] = (c0 + e < cols) ? Xh[((int64_t)p * cols + c0 + e) * NBU + b] : 0.f;
  }
  float cs[4][NB2 > 0 ? NB2 : 1];
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int b = 0; b < (NB2 > 0 ? NB2 : 1); ++b) cs[e][b] = 0.f;

  // one row: w is the old value; returns through nw the updated one
  auto row_math = [&](int r, const float (&w)[4], float (&nw)[4]) {
    if constexpr (DO_BWD) {
      const float* __restrict__ d = Dt + ((int64_t)p * rows + r) * NB2;
#pragma unroll
      for (int b = 0; b < NB2; ++b) {
        const float dv = d[b];
#pragma unroll
        for (int e = 0; e < 4; ++e) cs[e][b] = fmaf(w[e], dv, cs[e][b]);
      }
    }
    if constexpr (DO_UPD) {
      const float* __restrict__ dh = Dh + ((int64_t)p * rows + r) * NBU;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float u = 0.f;
#pragma unroll
        for (int b = 0; b < NBU; ++b) u = fmaf(dh[b], xh[e][b], u);
        nw[e] = fmaf(keep, w[e], eta * u);
      }
    }
  };
  int r = r0;
  if (vec) {
    // eight rows in flight per thread: all loads first, then the arithmetic and the stores
    constexpr int RU = 8;
    for (; r + RU <= r1; r += RU) {
      float* wp = Wt + ((int64_t)p * rows + r) * cols + c0;
      float4 t[RU];
#pragma unroll
      for (int k = 0; k < RU; ++k) t[k] = stream_load4(wp + (int64_t)k * cols);
#pragma unroll
      for (int k = 0; k < RU; ++k) {
        const float w[4] = {t[k].x, t[k].y, t[k].z, t[k].w};
        float nw[4];
        row_math(r + k, w, nw);
        if constexpr (DO_UPD)
          stream_store4(wp + (int64_t)k * cols, nw[0], nw[1], nw[2], nw[3]);
      }
    }
  }
  for (; r < r1; ++r) {
    float* wp = Wt + ((int64_t)p * rows + r) * cols + c0;
    float w[4] = {0.f, 0.f, 0.f, 0.f}, nw[4];
    if (vec) {
      const float4 t = *reinterpret_cast<const float4*>(wp);
      w[0] = t.x; w[1] = t.y; w[2] = t.z; w[3] = t.w;
    } else {
      for (int e = 0; e < 4; ++e) if (c0 + e < cols) w[e] = wp[e];
    }
    row_math(r, w, nw);
    if constexpr (DO_UPD) {
      if (vec) {
        *reinterpret_cast<float4*>(wp) = make_float4(nw[0], nw[1], nw[2], nw[3]);
      } else {
        for (int e = 0; e < 4; ++e) if (c0 + e < cols) wp[e] = nw[e];
      }
    }
  }
  if constexpr (DO_BWD) {
    float* __restrict__ out = part + (((int64_t)p * nchunks + chunk) * cols + c0) * NB2;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (c0 + e < cols)
#pragma unroll
        for (int b = 0; b < NB2; ++b) out[e * NB2 + b] = cs[e][b];
  }
}

// Largest finite |x| of up to two arrays (blockIdx.y = array), as kAmaxParts partial maxima per
// array: for non-negative floats the order of the bit patterns is the order of the values, so
// the partial results are plain unsigned maxima (order-free, hence reproducible).
constexpr int kAmaxParts = 256;
struct AbsMaxJobs { const float* x[2]; int64_t n[2]; uint32_t* parts; };

__global__ __launch_bounds__(256) void absmax_kernel(const AbsMaxJobs j) {
  __shared__ uint32_t wmax[4];
  const float* __restrict__ x = j.x[blockIdx.y];
  const int64_t n = j.n[blockIdx.y];
  uint32_t m = 0;
  auto take = [&](float v) {
    const uint32_t b = __float_as_uint(v) & 0x7fffffffu;
    if (b < 0x7f800000u) m = max(m, b);
  };
  const int64_t n4 = ((uintptr_t)x % 16 == 0) ? n / 4 : 0;          // 16-byte pieces, then the rest
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)kAmaxParts * 256) {
    const float4 v = reinterpret_cast<const float4*>(x)[i];
    take(v.x); take(v.y); take(v.z); take(v.w);
  }
  for (int64_t i = 4 * n4 + (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)kAmaxParts * 256) take(x[i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off));
  if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0)
    j.parts[blockIdx.y * kAmaxParts + blockIdx.x] = max(max(wmax[0], wmax[1]), max(wmax[2], wmax[3]));
}

// Ct[p][c][b] = sum_chunk part[p][chunk][c][b], in chunk order (deterministic).
__global__ void reduce_chunks_kernel(const float* __restrict__ part, float* __restrict__ Ct,
                                     int64_t per_node, int nchunks, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int64_t p = i / per_node, e = i - p * per_node;
  float s = 0.f;
  for (int k = 0; k < nchunks; ++k) s += part[((int64_t)p * nchunks + k) * per_node + e];
  Ct[i] = s;
}

// ---------------------------------------------------------------- element-wise steps

__global__ void sigmoid_fwd_kernel(const float* __restrict__ s, float* __restrict__ y, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) y[i] = 1.f / (1.f + expf(-s[i]));
}
__global__ void sigmoid_bwd_kernel(const float* __restrict__ c, const float* __restrict__ y,
                                   float* __restrict__ d, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) d[i] = c[i] * y[i] * (1.f - y[i]);
}
// rho_hat[i] = mean over the batch of y[i][:]: one wavefront per row, lanes stride over the
// columns, tree sum in a fixed order
__global__ __launch_bounds__(256) void row_mean_kernel(const float* __restrict__ y, int64_t rows, int64_t cols,
                                                       float* __restrict__ mean) {
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int lane = threadIdx.x & 63;
  float acc = 0.f;
  for (int64_t c = lane; c < cols; c += 64) acc += y[row * cols + c];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
  if (lane == 0) mean[row] = acc / (float)cols;
}
// delta = (c - scale * Q(rho_hat_row)) * y (1 - y),  Q(r) = -rho / r + (1 - rho) / (1 - r)
__global__ void sigmoid_bwd_sparse_kernel(const float* __restrict__ c, const float* __restrict__ y,
                                          const float* __restrict__ rho_hat, float rho, float scale,
                                          float* __restrict__ d, int64_t cols, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float r = rho_hat[i / cols];
  const float q = -rho / r + (1.f - rho) / (1.f - r);
  d[i] = (c[i] - scale * q) * y[i] * (1.f - y[i]);
}
__global__ void l2_delta_kernel(const float* __restrict__ y, const float* __restrict__ yh, float scale,
                                float* __restrict__ d, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) d[i] = scale * (y[i] - yh[i]) * yh[i] * (1.f - yh[i]);
}

// ---------------------------------------------------------------- vector stage of a whole iteration

// Everything the master does between two coded products of a small-batch training iteration
// (Sec. VII: decoding, the element-wise steps C1 / C2 or the last layer's error, and the encoding of
// the next product's operands), in one launch.  The vectors are a few thousand elements long, so
// the work is nothing; what it costs as four or five dependent launches is their latency.
//   phase 1  t[e][p] = sum_k in[p][k][r(e)][b(e)]             responses of node p (forward: one
//            term; backward: the partial column sums of the row chunks, added in chunk order)
//   phase 2  v[e] = f(sum_p D[q(e)][p] t[e][p])                decode, then the element-wise step f;
//            v is written to the decoded vector (an activation or an error Delta)
//   phase 3  out_j[p][r'][b] = sum_s coef_j[p][s] v[(s, r', b)]  up to three encodes of that vector
//            (the next product's X~ / Delta~ and the update operands X^ / D^), each over the same G
//            blocks of bh rows
// A workgroup owns `tile` rows r' of the G blocks; e = (s, r' - r0, b).  The decoded vector's row
// g = s * bh + r' lies in decode block q = g / len, row r = g % len; rows g >= N are zero padding.
// The arithmetic (order of the sums, the expressions of the element-wise steps) is that of
// combine_kernel, reduce_chunks_kernel, encode_small_kernel and the element-wise kernels, so an
// iteration made of these launches leaves bit for bit the weights the per-layer calls leave.
constexpr int kStageJobs = 3;
struct StageJob { const float* coef; float* out; };     // coef [P][G] (device), out [P][bh][nb]
struct StageParams {
  const float* in;
  int64_t node_stride, red_stride;     // elements between nodes / between the terms of phase 1
  int32_t P, nred, len, nb;
  const float* D;                      // [nblk][P] decoding rows (device, fp32)
  int32_t nblk;                        // decode blocks (rows of D)
  int32_t N;                           // rows of the decoded vector that exist
  int32_t epi;                         // 0 none, 1 logistic, 2 times y (1 - y), 3 logistic, then the L2 error
  const float* epi_y;                  // epi 2: y; epi 3: the targets Y; laid out like the decoded vector
  float scale;                         // epi 3: 2 / batch
  float* out;                          // decoded vector after the element-wise step ([N][nb])
  float* out2;                         // epi 3: the error Delta ([N][nb]); `out` then holds the network output
  int32_t bh, G, tile, njobs;
  StageJob job[kStageJobs];
};

__global__ __launch_bounds__(256) void vector_stage_kernel(const StageParams p) {
  // Everything that does not depend on another phase is requested at once, at the start: the
  // responses of phase 1, the decoding rows and the encode coefficients (into LDS), the operand of
  // the element-wise step.  The kernel then has one memory round trip in front of its arithmetic,
  // not one per phase; its running time is latency, not work.
  extern __shared__ float stage_lds[];
  const int E = p.G * p.tile * p.nb;
  float* tsum = stage_lds;                     // [P][E]
  float* vals = tsum + (size_t)p.P * E;        // [E]
  float* Dl = vals + E;                        // [nblk][P]
  float* cl = Dl + (size_t)p.nblk * p.P;       // [njobs][P][G]
  const int r0 = blockIdx.x * p.tile;
  const int tid = threadIdx.x;
  auto row_of = [&](int e, int* rr, int* b) {
    const int s = e / (p.tile * p.nb), rem = e - s * (p.tile * p.nb);
    *rr = rem / p.nb; *b = rem - *rr * p.nb;
    return s * p.bh + r0 + *rr;                // row g of the decoded vector
  };
  // operand of the element-wise step for the element this thread decodes in phase 2 (E <= 256)
  float epi_in = 0.f;
  int g2 = 0, rr2 = 0, b2 = 0;
  bool live2 = false;
  if (tid < E) {
    g2 = row_of(tid, &rr2, &b2);
    live2 = r0 + rr2 < p.bh && g2 < p.N;
    if (live2 && p.epi >= 2) epi_in = p.epi_y[(int64_t)g2 * p.nb + b2];
  }
  for (int idx = tid; idx < p.nblk * p.P; idx += 256) Dl[idx] = p.D[idx];
  for (int j = 0; j < p.njobs; ++j)
    for (int idx = tid; idx < p.P * p.G; idx += 256) cl[j * p.P * p.G + idx] = p.job[j].coef[idx];
  for (int idx = tid; idx < p.P * E; idx += 256) {
    const int node = idx / E, e = idx - node * E;
    int rr, b;
    const int g = row_of(e, &rr, &b);
    float t = 0.f;
    if (r0 + rr < p.bh && g < p.N) {
      const float* src = p.in + (int64_t)node * p.node_stride + (int64_t)(g % p.len) * p.nb + b;
      if (p.nred == 1) {
        t = src[0];
      } else {
        // (chunk order, as reduce_chunks_kernel adds them; four loads in flight at a time)
        int k = 0;
        for (; k + 4 <= p.nred; k += 4) {
          const float a0 = src[(int64_t)k * p.red_stride], a1 = src[(int64_t)(k + 1) * p.red_stride];
          const float a2 = src[(int64_t)(k + 2) * p.red_stride], a3 = src[(int64_t)(k + 3) * p.red_stride];
          t += a0; t += a1; t += a2; t += a3;
        }
        for (; k < p.nred; ++k) t += src[(int64_t)k * p.red_stride];
      }
    }
    tsum[idx] = t;
  }
  __syncthreads();
  if (tid < E) {
    float v = 0.f;
    if (live2) {
      const float* drow = Dl + (g2 / p.len) * p.P;
      float acc = 0.f;
      for (int node = 0; node < p.P; ++node) acc = fmaf(drow[node], tsum[node * E + tid], acc);
      const int64_t o = (int64_t)g2 * p.nb + b2;
      if (p.epi == 1) {
        v = 1.f / (1.f + expf(-acc));
      } else if (p.epi == 2) {
        v = acc * epi_in * (1.f - epi_in);
      } else if (p.epi == 3) {
        const float yh = 1.f / (1.f + expf(-acc));
        p.out[o] = yh;
        v = p.scale * (epi_in - yh) * yh * (1.f - yh);
      } else {
        v = acc;
      }
      (p.epi == 3 ? p.out2 : p.out)[o] = v;
    }
    vals[tid] = v;
  }
  __syncthreads();
  const int per_job = p.P * p.tile * p.nb;
  for (int idx = tid; idx < p.njobs * per_job; idx += 256) {
    const int j = idx / per_job, rem = idx - j * per_job;
    const int node = rem / (p.tile * p.nb), rb = rem - node * (p.tile * p.nb);
    const int rr = rb / p.nb;
    if (r0 + rr >= p.bh) continue;
    const float* crow = cl + (j * p.P + node) * p.G;
    float a = 0.f;
    for (int s = 0; s < p.G; ++s) a = fmaf(crow[s], vals[s * p.tile * p.nb + rb], a);
    p.job[j].out[((int64_t)node * p.bh + r0) * p.nb + rb] = a;
  }
}

size_t align256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace
}  // namespace gpd

using namespace gpd;

// ---------------------------------------------------------------- layer object

struct gpd_layer {
  gpd_layer_desc_t desc;
  Code fwd;                        // plan of W~ X~ (m, n, d1)
  std::vector<int> eD, eCb;        // [m*d2] exponent of Delta block (i,k); [n*d2] useful of C block (j,k)
  int Kb = 0;
  std::vector<int> eUd, eUx;       // update exponents of Delta_i and X_j
  int64_t N_out_pad = 0, N_in_pad = 0, wr = 0, wc = 0, nb1 = 0, nb2 = 0;
  hipStream_t stream = nullptr;
  double rho = 0, abs_floor = 0;
  TableRing ring;
  // workspace layout (byte offsets)
  size_t off_Xt = 0, off_St = 0, off_Dt = 0, off_Ct = 0, off_Dh = 0, off_Xh = 0, off_part = 0,
         off_dec = 0, ws_bytes = 0;
  bool upd_planes = false;         // update operands stored as planes: three bf16 planes, or
  bool upd_fp16 = false;           // (bf16 layers) two fp16 planes of the operand / 2^E
  int exp_Dh = 0, exp_Xh = 0;      // bits the encoded update operands can exceed Delta, X by
  size_t off_scal = 0;             // partial maxima of |Delta|, |X| and the two exponents E
  size_t off_delta = 0;            // this layer's error Delta (N_out x batch) in gpd_mlp_step
  int nchunks = 0;
  int64_t flag_cap = 0, loc_cap = 0;
  size_t dec_bytes = 0;
};

namespace {

std::vector<int32_t> limits(int64_t total, int64_t block, int nblocks) {
  std::vector<int32_t> v(nblocks);
  for (int i = 0; i < nblocks; ++i) {
    int64_t left = total - (int64_t)i * block;
    v[i] = (int32_t)std::max<int64_t>(0, std::min<int64_t>(block, left));
  }
  return v;
}

// limits for a grid_r x grid_c grid of bh x bw blocks covering a rows x cols matrix
void grid_limits(int64_t rows, int64_t cols, int grid_r, int grid_c, int64_t bh, int64_t bw,
                 std::vector<int32_t>* lr, std::vector<int32_t>* lc) {
  lr->clear(); lc->clear();
  if (rows == grid_r * bh && cols == grid_c * bw) return;      // nothing ragged
  std::vector<int32_t> r = limits(rows, bh, grid_r), c = limits(cols, bw, grid_c);
  for (int i = 0; i < grid_r; ++i)
    for (int j = 0; j < grid_c; ++j) { lr->push_back(r[i]); lc->push_back(c[j]); }
}

}  // namespace

extern "C" gpd_status_t gpd_layer_create(const gpd_layer_desc_t* d, gpd_layer_t** out) {
  if (!d || !out) return fail(GPD_E_INVALID, "gpd_layer_create: null argument");
  *out = nullptr;
  if (d->N_out < 1 || d->N_in < 1 || d->batch < 1 || d->d1 < 1 || d->d2 < 1)
    return fail(GPD_E_INVALID, "layer sizes must be >= 1");
  if (d->batch % d->d1 || d->batch % d->d2) return fail(GPD_E_SHAPE, "d1 and d2 must divide the batch");
  if (d->worker_dtype != GPD_F32 && d->worker_dtype != GPD_BF16 && d->worker_dtype != GPD_F32_SPLIT)
    return fail(GPD_E_INVALID, "unknown worker dtype");
  if (d->m < 1 || d->n < 1) return fail(GPD_E_INVALID, "m, n must be >= 1");
  if (d->m * d->d2 > GPD_MAX_BLOCKS || d->n * d->d2 > GPD_MAX_BLOCKS)
    return fail(GPD_E_INVALID, "block grid larger than GPD_MAX_BLOCKS");
  gpd_layer_t* L = new (std::nothrow) gpd_layer_t();
  if (!L) return fail(GPD_E_DEVICE, "out of host memory");
  L->desc = *d;
  L->desc.points = nullptr;
  int subst = d->subst;
  if (subst == GPD_SUB_AUTO) subst = d->m > d->n ? GPD_SUB_V_UM : GPD_SUB_U_VN;
  gpd_status_t st = make_code(d->m, d->n, d->d1, d->P, subst, d->points, &L->fwd);
  if (st != GPD_OK) { delete L; return st; }
  const Code& c = L->fwd;
  const int m = d->m, n = d->n, d2 = d->d2;
  // Sec. IX backpropagation stage: Delta~^T(w,u) = sum Delta^T_{k,i} w^k u^(m-1-i); C^T_{k,j} is
  // the coefficient of w^k u^(m-1) v^j.
  L->eD.resize(m * d2); L->eCb.resize(n * d2);
  int maxD = 0, maxA = 0;
  for (int i = 0; i < m; ++i)
    for (int k = 0; k < d2; ++k) {
      L->eD[i * d2 + k] = c.ew * k + c.eu * (m - 1 - i);
      maxD = std::max(maxD, L->eD[i * d2 + k]);
    }
  for (int j = 0; j < n; ++j)
    for (int k = 0; k < d2; ++k) L->eCb[j * d2 + k] = c.ew * k + c.eu * (m - 1) + c.ev * j;
  for (int e : c.eA) maxA = std::max(maxA, e);
  L->Kb = maxD + maxA + 1;
  if (L->Kb > d->P) {
    delete L;
    return fail(GPD_E_SHAPE, "backward threshold K_b = %d exceeds P = %d", maxD + maxA + 1, d->P);
  }
  L->eUd.resize(m); L->eUx.resize(n);
  for (int i = 0; i < m; ++i) L->eUd[i] = c.eu * i;      // update: sum_i Delta_i u^i
  for (int j = 0; j < n; ++j) L->eUx[j] = c.ev * j;      //         sum_j X_j v^j
  L->N_out_pad = (d->N_out + m - 1) / m * m;
  L->N_in_pad = (d->N_in + n - 1) / n * n;
  L->wr = L->N_out_pad / m; L->wc = L->N_in_pad / n;
  L->nb1 = d->batch / d->d1; L->nb2 = d->batch / d->d2;
  L->stream = (hipStream_t)d->hip_stream;
  L->rho = d->rho_detect > 0 ? d->rho_detect : (d->worker_dtype == GPD_BF16 ? 0.125 : 1.0 / 4096.0);
  L->abs_floor = d->abs_floor;
  L->nchunks = (int)((L->wr + kRowChunk - 1) / kRowChunk);

  const int64_t P = d->P;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
  L->off_Xt = take((size_t)P * L->wc * L->nb1 * 4);
  L->off_St = take((size_t)P * L->wr * L->nb1 * 4);
  L->off_Dt = take((size_t)P * L->wr * L->nb2 * 4);
  L->off_Ct = take((size_t)P * L->wc * L->nb2 * 4);
  // update operands: fp32 stacks, or (batch a multiple of 64) planes written by the encode itself:
  // three bf16 planes hi / mid / lo (GPD_F32_SPLIT layers: six partial products, fp32-exact) or
  // two fp16 planes hi / lo of the operand divided by a power of two (GPD_BF16 layers: three
  // partial products, error below 2^-20 of a product)
  L->upd_planes = d->worker_dtype != GPD_F32 && d->batch % 64 == 0;
  L->upd_fp16 = L->upd_planes && d->worker_dtype == GPD_BF16;
  {
    // |Dhat_p| <= (sum_i |a_p|^eUd[i]) max |Delta|, likewise Xhat: the bound as a power of two
    double bd = 1, bx = 1;
    for (double x : c.pts) {
      double sd = 0, sx = 0;
      for (int e : L->eUd) sd += std::pow(std::fabs(x), e);
      for (int e : L->eUx) sx += std::pow(std::fabs(x), e);
      bd = std::max(bd, sd); bx = std::max(bx, sx);
    }
    L->exp_Dh = (int)std::ceil(std::log2(bd)); L->exp_Xh = (int)std::ceil(std::log2(bx));
    if (L->exp_Dh > 16 || L->exp_Xh > 16) L->upd_fp16 = false;    // (points far outside [-1, 1])
  }
  const size_t ues = L->upd_planes && !L->upd_fp16 ? 6 : 4;
  L->off_Dh = take((size_t)P * L->wr * d->batch * ues);
  L->off_Xh = take((size_t)P * L->wc * d->batch * ues);
  L->off_part = take((size_t)P * L->nchunks * L->wc * L->nb2 * 4);
  L->off_scal = take((size_t)(2 * kAmaxParts + 2) * 4);
  L->off_delta = take((size_t)L->N_out_pad * d->batch * 4);
  const int64_t ncw = std::max(L->wr * L->nb1, L->wc * L->nb2);
  decode_workspace_layout(ncw, &L->flag_cap, &L->loc_cap, &L->dec_bytes);
  // the node search needs room for its partial Gram matrices (forward, backward and weight stacks)
  L->dec_bytes = std::max(L->dec_bytes, gram_workspace_bytes(L->wr * L->nb1, (int)P - c.K));
  L->dec_bytes = std::max(L->dec_bytes, gram_workspace_bytes(L->wc * L->nb2, (int)P - L->Kb));
  L->dec_bytes = std::max(L->dec_bytes, gram_workspace_bytes(L->wr * L->wc, (int)P - m * n));
  L->off_dec = take(L->dec_bytes);
  L->ws_bytes = off;

  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) { delete L; return fail(GPD_E_DEVICE, "no HIP device"); }
  HostCombineTable probe;
  size_t slot = 0;
  auto grow = [&](int nin, int nout, int r) {
    probe.nin = nin; probe.nout = nout; probe.r = r;
    slot = std::max(slot, probe.bytes());
  };
  grow(m * n, (int)P, 0); grow(n * d->d1, (int)P, 0); grow(m * d2, (int)P, 0);
  grow((int)P, m * d->d1, (int)P); grow((int)P, n * d2, (int)P); grow((int)P, m * n, 0);
  grow((int)P, (int)P, 0);                    // projection onto the code
  st = L->ring.init(slot);
  if (st != GPD_OK) { L->ring.destroy(); delete L; return st; }
  *out = L;
  return GPD_OK;
}

extern "C" gpd_status_t gpd_layer_info(const gpd_layer_t* L, int32_t* Kf, int32_t* Kb, int64_t* wt_rows,
                                       int64_t* wt_cols, size_t* workspace_bytes) {
  if (!L) return fail(GPD_E_INVALID, "gpd_layer_info: null layer");
  if (Kf) *Kf = L->fwd.K;
  if (Kb) *Kb = L->Kb;
  if (wt_rows) *wt_rows = L->wr;
  if (wt_cols) *wt_cols = L->wc;
  if (workspace_bytes) *workspace_bytes = L->ws_bytes;
  return GPD_OK;
}

extern "C" gpd_status_t gpd_layer_workspace_view(const gpd_layer_t* L, int32_t which, size_t* byte_offset,
                                                 int64_t* rows, int64_t* cols) {
  if (!L || !byte_offset || !rows || !cols) return fail(GPD_E_INVALID, "gpd_layer_workspace_view: null argument");
  switch (which) {
    case 0: *byte_offset = L->off_Xt; *rows = L->wc; *cols = L->nb1; break;
    case 1: *byte_offset = L->off_St; *rows = L->wr; *cols = L->nb1; break;
    case 2: *byte_offset = L->off_Dt; *rows = L->wr; *cols = L->nb2; break;
    case 3: *byte_offset = L->off_Ct; *rows = L->wc; *cols = L->nb2; break;
    case 4: *byte_offset = L->off_Dh; *rows = L->wr; *cols = L->desc.batch; break;
    case 5: *byte_offset = L->off_Xh; *rows = L->wc; *cols = L->desc.batch; break;
    case 6:
      if (!L->upd_fp16) return fail(GPD_E_INVALID, "gpd_layer_workspace_view: the layer holds no fp16 planes");
      *byte_offset = L->off_scal + (size_t)2 * kAmaxParts * 4; *rows = 1; *cols = 2; break;
    case 7: *byte_offset = L->off_delta; *rows = L->N_out_pad; *cols = L->desc.batch; break;
    default: return fail(GPD_E_INVALID, "gpd_layer_workspace_view: unknown buffer %d", which);
  }
  return GPD_OK;
}

extern "C" void gpd_layer_destroy(gpd_layer_t* L) {
  if (!L) return;
  L->ring.destroy();
  delete L;
}

extern "C" gpd_status_t gpd_layer_encode_weights(const gpd_layer_t* Lc, const float* W, int64_t ldw,
                                                 float* Wt) {
  gpd_layer_t* L = const_cast<gpd_layer_t*>(Lc);
  if (!L || !W || !Wt) return fail(GPD_E_INVALID, "gpd_layer_encode_weights: null argument");
  if (ldw < L->desc.N_in) return fail(GPD_E_SHAPE, "ldw smaller than N_in");
  const Code& c = L->fwd;
  CombineTable t;
  std::string key("encW");
  key_add(&key, ldw);
  gpd_status_t st = L->ring.cached(key, [&](HostCombineTable* ht) {
    *ht = encode_table(c.pts, c.eA, c.m, c.n, L->wr, L->wc, ldw);
    grid_limits(L->desc.N_out, L->desc.N_in, c.m, c.n, L->wr, L->wc, &ht->in_rows, &ht->in_cols);
    return GPD_OK;
  }, L->stream, &t);
  if (st != GPD_OK) return st;
  ScreenArgs none;
  return launch_combine(L->stream, t, W, ldw, Wt, L->wc, false, L->wr, L->wc, none);
}

extern "C" gpd_status_t gpd_layer_decode_weights(const gpd_layer_t* Lc, const float* Wt,
                                                 const uint8_t* present, float* W, int64_t ldw) {
  gpd_layer_t* L = const_cast<gpd_layer_t*>(Lc);
  if (!L || !W || !Wt) return fail(GPD_E_INVALID, "gpd_layer_decode_weights: null argument");
  if (ldw < L->desc.N_in) return fail(GPD_E_SHAPE, "ldw smaller than N_in");
  const Code& c = L->fwd;
  // W~(b) = sum W_ij b^eA(i,j): a polynomial with mn coefficients (footnote on regeneration)
  DecodeJob job;
  job.pts = &c.pts; job.K = c.m * c.n; job.useful = c.eA;
  job.grid_r = c.m; job.grid_c = c.n; job.bh = L->wr; job.bw = L->wc;
  job.rho = L->rho; job.abs_floor = L->abs_floor;
  job.flag_cap = 0; job.loc_cap = 0; job.workspace_bytes = 0;
  grid_limits(L->desc.N_out, L->desc.N_in, c.m, c.n, L->wr, L->wc, &job.out_rows, &job.out_cols);
  return run_decode(L->stream, &L->ring, job, Wt, present, GPD_DEC_LSQ_ALL, 0, W, ldw, nullptr, 0, nullptr);
}

// ---------------------------------------------------------------- node-level faults

extern "C" gpd_status_t gpd_layer_locate_nodes(const gpd_layer_t* Lc, int32_t which, const float* stack,
                                               const uint8_t* present, void* workspace,
                                               size_t workspace_bytes, gpd_node_report_t* report,
                                               double* gram) {
  gpd_layer_t* L = const_cast<gpd_layer_t*>(Lc);
  if (!L || !stack || !report) return fail(GPD_E_INVALID, "gpd_layer_locate_nodes: null argument");
  if (!workspace || workspace_bytes < L->ws_bytes || ((uintptr_t)workspace & 255))
    return fail(GPD_E_WORKSPACE, "layer: workspace of %zu aligned bytes needed", L->ws_bytes);
  const Code& c = L->fwd;
  int K = 0;
  int64_t ncw = 0;
  double rho = L->rho;
  switch (which) {
    case GPD_STACK_WEIGHTS:
      K = c.m * c.n; ncw = L->wr * L->wc;
      rho = L->desc.rho_detect > 0 ? L->desc.rho_detect : 1.0 / 4096.0;    // stored in fp32
      break;
    case GPD_STACK_FORWARD: K = c.K; ncw = L->wr * L->nb1; break;
    case GPD_STACK_BACKWARD: K = L->Kb; ncw = L->wc * L->nb2; break;
    default: return fail(GPD_E_INVALID, "gpd_layer_locate_nodes: unknown stack %d", which);
  }
  return run_locate_nodes(L->stream, &L->ring, c.pts, K, ncw, stack, present, rho, L->abs_floor,
                          (char*)workspace + L->off_dec, L->dec_bytes, report, gram);
}

namespace {

// Table that re-evaluates the polynomial W~(b) (mn coefficients), interpolated through the
// nodes in `from` (all of them by least squares, or the first mn), at the nodes in `to`.
gpd_status_t reevaluate_table(const gpd_layer_t* L, const std::vector<int>& from, const std::vector<int>& to,
                              bool first_k, HostCombineTable* ht) {
  const Code& c = L->fwd;
  const int Kw = c.m * c.n;
  std::vector<int> all_e(Kw);
  for (int e = 0; e < Kw; ++e) all_e[e] = e;
  std::vector<double> D;                       // [Kw][from.size()]: coefficients from node values
  gpd_status_t st = decode_matrices(c.pts, from, Kw, all_e, first_k, &D, nullptr);
  if (st != GPD_OK) return st;
  const int nf = (int)from.size();
  std::vector<int> used;
  for (int q = 0; q < nf; ++q) {
    bool nz = false;
    for (int e = 0; e < Kw && !nz; ++e) nz = D[(size_t)e * nf + q] != 0.0;
    if (nz) used.push_back(q);
  }
  ht->nin = (int)used.size(); ht->nout = (int)to.size(); ht->r = 0;
  ht->in_off.resize(ht->nin); ht->node.resize(ht->nin); ht->out_off.resize(ht->nout);
  ht->coef.assign((size_t)ht->nout * ht->nin, 0.0);
  const int64_t blk = L->wr * L->wc;
  for (int u = 0; u < ht->nin; ++u) { ht->in_off[u] = from[used[u]] * blk; ht->node[u] = from[used[u]]; }
  for (int o = 0; o < ht->nout; ++o) {
    ht->out_off[o] = to[o] * blk;
    for (int u = 0; u < ht->nin; ++u) {
      double acc = 0.0;                        // sum_e b_to^e D[e][q]
      for (int e = 0; e < Kw; ++e) acc += ipow(c.pts[to[o]], e) * D[(size_t)e * nf + used[u]];
      ht->coef[(size_t)o * ht->nin + u] = acc;
    }
  }
  return GPD_OK;
}

}  // namespace

extern "C" gpd_status_t gpd_layer_regenerate(const gpd_layer_t* Lc, float* Wt, const uint8_t* bad,
                                             int32_t mode) {
  gpd_layer_t* L = const_cast<gpd_layer_t*>(Lc);
  if (!L || !Wt || !bad) return fail(GPD_E_INVALID, "gpd_layer_regenerate: null argument");
  if (mode != GPD_DEC_FIRST_K && mode != GPD_DEC_LSQ_ALL)
    return fail(GPD_E_INVALID, "gpd_layer_regenerate: bad mode");
  const int P = L->desc.P, Kw = L->fwd.m * L->fwd.n;
  std::vector<int> good, todo;
  for (int p = 0; p < P; ++p) (bad[p] ? todo : good).push_back(p);
  if ((int)good.size() < Kw) return fail(GPD_E_TOO_FEW, "%d good nodes, %d needed", (int)good.size(), Kw);
  if (todo.empty()) return GPD_OK;
  std::string key("regen");
  key_add(&key, mode);
  key_add_bytes(&key, bad, P);
  CombineTable t;
  gpd_status_t st = L->ring.cached(key, [&](HostCombineTable* ht) {
    return reevaluate_table(L, good, todo, mode == GPD_DEC_FIRST_K, ht);
  }, L->stream, &t);
  if (st != GPD_OK) return st;
  ScreenArgs none;
  return launch_combine(L->stream, t, Wt, L->wc, Wt, L->wc, false, L->wr, L->wc, none);
}

extern "C" gpd_status_t gpd_layer_project(const gpd_layer_t* Lc, float* Wt, const uint8_t* present) {
  gpd_layer_t* L = const_cast<gpd_layer_t*>(Lc);
  if (!L || !Wt) return fail(GPD_E_INVALID, "gpd_layer_project: null argument");
  const int P = L->desc.P, Kw = L->fwd.m * L->fwd.n;
  std::vector<int> from, all;
  for (int p = 0; p < P; ++p) {
    all.push_back(p);
    if (!present || present[p]) from.push_back(p);
  }
  if ((int)from.size() < Kw) return fail(GPD_E_TOO_FEW, "%d nodes present, %d needed", (int)from.size(), Kw);
  std::string key("proj");
  for (int p = 0; p < P; ++p) key.push_back((!present || present[p]) ? 1 : 0);
  CombineTable t;
  gpd_status_t st = L->ring.cached(key, [&](HostCombineTable* ht) {
    return reevaluate_table(L, from, all, false, ht);
  }, L->stream, &t);
  if (st != GPD_OK) return st;
  const int64_t n = L->wr * L->wc;
  if (t.k_offsets && t.nin <= kStackMax && t.nout <= kStackMax && n > 0 && n % 128 == 0 && (uintptr_t)Wt % 16 == 0) {
    // P blocks -> P blocks is matrix-core work
    StackParams sp;
    sp.in = Wt; sp.out = Wt; sp.coef = t.coef; sp.nin = t.nin; sp.nout = t.nout; sp.n = n;
    for (int q = 0; q < kStackMax; ++q) {
      sp.in_off[q] = q < t.nin ? t.k_in_off[q] : 0;
      sp.out_off[q] = q < t.nout ? t.k_out_off[q] : 0;
      if ((sp.in_off[q] | sp.out_off[q]) & 3) return fail(GPD_E_SHAPE, "projection: block offsets not 16-byte aligned");
    }
    const dim3 grid((unsigned)((n / 128 + 3) / 4)), block(256);
    if (t.nin <= 16) GPD_LAUNCH(stack_mfma_kernel<8>, grid, block, 0, L->stream, sp);
    else if (t.nin <= 24) GPD_LAUNCH(stack_mfma_kernel<12>, grid, block, 0, L->stream, sp);
    else GPD_LAUNCH(stack_mfma_kernel<16>, grid, block, 0, L->stream, sp);
    GPD_HIP(hipGetLastError());
    return GPD_OK;
  }
  // in place: a thread reads every input block's value of its element before it writes any output
  ScreenArgs none;
  return launch_combine(L->stream, t, Wt, L->wc, Wt, L->wc, false, L->wr, L->wc, none);
}

// ---------------------------------------------------------------- products

namespace {

template <int NB>
void launch_skinny_fwd(hipStream_t s, const float* Wt, const float* Xt, float* St, int rows, int cols, int P) {
  constexpr int FR = fwd_rows(NB);
  GPD_LAUNCH((skinny_forward_kernel<NB>), dim3((rows + FR - 1) / FR, P), dim3(256), 0, s, Wt, Xt,
                     St, rows, cols);
}

gpd_status_t skinny_forward(hipStream_t s, const float* Wt, const float* Xt, float* St, int64_t rows,
                            int64_t cols, int P, int nb) {
  if (rows == 0 || cols == 0) return GPD_OK;
  switch (nb) {
    case 1: launch_skinny_fwd<1>(s, Wt, Xt, St, (int)rows, (int)cols, P); break;
    case 2: launch_skinny_fwd<2>(s, Wt, Xt, St, (int)rows, (int)cols, P); break;
    case 3: launch_skinny_fwd<3>(s, Wt, Xt, St, (int)rows, (int)cols, P); break;
    case 4: launch_skinny_fwd<4>(s, Wt, Xt, St, (int)rows, (int)cols, P); break;
    case 5: launch_skinny_fwd<5>(s, Wt, Xt, St, (int)rows, (int)cols, P); break;
    case 6: launch_skinny_fwd<6>(s, Wt, Xt, St, (int)rows, (int)cols, P); break;
    case 7: launch_skinny_fwd<7>(s, Wt, Xt, St, (int)rows, (int)cols, P); break;
    case 8: launch_skinny_fwd<8>(s, Wt, Xt, St, (int)rows, (int)cols, P); break;
    default: return fail(GPD_E_UNSUPPORTED, "skinny forward: batch %d", nb);
  }
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}

template <int NB2, int NBU>
gpd_status_t launch_skinny_bu(hipStream_t s, float* Wt, const float* Dt, const float* Dh, const float* Xh,
                              float* part, int rows, int cols, int nchunks, int P, float keep, float eta,
                              bool do_bwd) {
  dim3 grid((cols + 1023) / 1024, nchunks, P), block(256);
  if (do_bwd)
    GPD_LAUNCH((skinny_backward_update_kernel<NB2, NBU, true, true>), grid, block, 0, s, Wt, Dt, Dh, Xh,
                       part, rows, cols, nchunks, keep, eta);
  else
    GPD_LAUNCH((skinny_backward_update_kernel<0, NBU, false, true>), grid, block, 0, s, Wt, Dt, Dh, Xh,
                       part, rows, cols, nchunks, keep, eta);
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}

template <int NB2>
gpd_status_t skinny_bu_nbu(hipStream_t s, float* Wt, const float* Dt, const float* Dh, const float* Xh,
                           float* part, int rows, int cols, int nchunks, int P, float keep, float eta,
                           bool do_bwd, int nbu) {
  switch (nbu) {
    case 1: return launch_skinny_bu<NB2, 1>(s, Wt, Dt, Dh, Xh, part, rows, cols, nchunks, P, keep, eta, do_bwd);
    case 2: return launch_skinny_bu<NB2, 2>(s, Wt, Dt, Dh, Xh, part, rows, cols, nchunks, P, keep, eta, do_bwd);
    case 4: return launch_skinny_bu<NB2, 4>(s, Wt, Dt, Dh, Xh, part, rows, cols, nchunks, P, keep, eta, do_bwd);
    case 8: return launch_skinny_bu<NB2, 8>(s, Wt, Dt, Dh, Xh, part, rows, cols, nchunks, P, keep, eta, do_bwd);
    default: return fail(GPD_E_UNSUPPORTED, "skinny update: batch %d", nbu);
  }
}

// In-kernel form of an encode table over a grid_r x grid_c grid of bh x bw blocks of a
// total_rows x total_cols matrix; false when the table does not fit it.
bool make_small(const CombineTable& t, const float* in, int64_t ld, int64_t total_rows, int64_t total_cols,
                int grid_r, int grid_c, int64_t bh, int64_t bw, float* out, int P, SmallEnc* f) {
  if (!t.k_offsets || t.nin != grid_r * grid_c || t.nin > kSmallMaxIn || t.nout != P || ld > INT32_MAX ||
      bh > INT32_MAX || bw > INT32_MAX)
    return false;
  f->in = in; f->coef = t.coef; f->out = out;
  f->ld = (int32_t)ld; f->nin = t.nin; f->rows = (int32_t)bh; f->nb = (int32_t)bw;
  if ((int64_t)P * bh * bw > INT32_MAX - 256) return false;
  f->count = (int32_t)(P * bh * bw);
  const std::vector<int32_t> lr = limits(total_rows, bh, grid_r), lc = limits(total_cols, bw, grid_c);
  for (int i = 0; i < grid_r; ++i)
    for (int j = 0; j < grid_c; ++j) {
      const int q = i * grid_c + j;
      f->off[q] = t.k_in_off[q]; f->lim_r[q] = lr[i]; f->lim_c[q] = lc[j];
    }
  return true;
}

bool skinny_ok(const gpd_layer_t* L) {
  const int64_t b = L->desc.batch;
  const bool bu = b == 1 || b == 2 || b == 4 || b == 8;
  const int64_t n2 = L->nb2;
  return bu && L->nb1 <= kSkinnyMaxBatch && (n2 == 1 || n2 == 2 || n2 == 4 || n2 == 8);
}

}  // namespace

extern "C" gpd_status_t gpd_coded_layer_step(gpd_layer_t* L, int32_t phase, float* Wt, const float* X,
                                             const float* Dlt, float eta, float decay, float* out,
                                             const uint8_t* present, int32_t correct_errors,
                                             void* workspace, size_t workspace_bytes,
                                             gpd_report_t* report) {
  if (!L || !Wt || !X) return fail(GPD_E_INVALID, "gpd_coded_layer_step: null argument");
  // the element-wise step after the decode (C1: logistic function of S; C2: Hadamard product of
  // C with X (1 - X), X being the logistic output of the layer below) on request in the same pass
  const bool fuse_act = (phase & GPD_STEP_FUSE_SIGMOID) != 0;
  phase &= ~GPD_STEP_FUSE_SIGMOID;
  if (phase != GPD_STEP_FORWARD && phase != GPD_STEP_BACKWARD_UPDATE)
    return fail(GPD_E_INVALID, "unknown phase %d", phase);
  // a decode with element-wise correction patches single outputs after the pass: the step then
  // follows as a launch of its own
  const bool act_in_decode = fuse_act && correct_errors != GPD_CORRECT_ELEMENTS && correct_errors != GPD_CORRECT_ELEMENTS_L1;
  auto act_after = [&](gpd_status_t dst, float* o, int64_t n) -> gpd_status_t {
    if (!fuse_act || act_in_decode || !o || n == 0 || (dst != GPD_OK && dst != GPD_E_DECODE_FAIL)) return dst;
    const std::string why = dst == GPD_OK ? std::string() : std::string(gpd_last_error());
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    if (phase == GPD_STEP_FORWARD) GPD_LAUNCH(sigmoid_fwd_kernel, grid, block, 0, L->stream, o, o, n);
    else GPD_LAUNCH(sigmoid_bwd_kernel, grid, block, 0, L->stream, o, X, o, n);
    GPD_HIP(hipGetLastError());
    if (dst != GPD_OK) return fail(dst, "%s", why.c_str());
    return dst;
  };
  if (!workspace || workspace_bytes < L->ws_bytes || ((uintptr_t)workspace & 255))
    return fail(GPD_E_WORKSPACE, "layer step: workspace of %zu aligned bytes needed", L->ws_bytes);
  const gpd_layer_desc_t& d = L->desc;
  const Code& c = L->fwd;
  const int P = d.P;
  char* ws = (char*)workspace;
  float* Xt = (float*)(ws + L->off_Xt);
  float* St = (float*)(ws + L->off_St);
  float* Dt = (float*)(ws + L->off_Dt);
  float* Ct = (float*)(ws + L->off_Ct);
  float* Dh = (float*)(ws + L->off_Dh);
  float* Xh = (float*)(ws + L->off_Xh);
  float* part = (float*)(ws + L->off_part);
  uint32_t* scal = (uint32_t*)(ws + L->off_scal);
  int32_t* exps = (int32_t*)(scal + 2 * kAmaxParts);
  void* dec_ws = ws + L->off_dec;
  hipStream_t s = L->stream;
  ScreenArgs none;
  gpd_status_t st;
  const bool split = d.worker_dtype == GPD_F32_SPLIT;
  const bool bf16 = d.worker_dtype == GPD_BF16 || split;       // products on the bf16 matrix cores
  const bool skinny = skinny_ok(L) && !bf16;
  const bool xt_bf16 = bf16 && !split;      // X~_p, Delta~_p are stored in bf16

  if (phase == GPD_STEP_FORWARD) {
    if (!out) return fail(GPD_E_INVALID, "forward: out is null");
    // X~_p = sum_jk X_jk b_p^eB(j,k)   (feedforward stage)
    CombineTable t;
    st = L->ring.cached("encX", [&](HostCombineTable* ht) {
      *ht = encode_table(c.pts, c.eB, c.n, c.d, L->wc, L->nb1, d.batch);
      grid_limits(d.N_in, d.batch, c.n, c.d, L->wc, L->nb1, &ht->in_rows, &ht->in_cols);
      return GPD_OK;
    }, s, &t);
    if (st != GPD_OK) return st;
    // (bf16 layers: rounded to bf16 here instead of on the way into the product's LDS tile: the
    // same round-to-nearest-even of the same fp32 value, half the bytes for the product to read)
    st = launch_combine(s, t, X, d.batch, Xt, L->nb1, xt_bf16 ? 1 : 0, L->wc, L->nb1, none);
    if (st != GPD_OK) return st;
    // S~_p = W~_p X~_p   (step O1 on every node)
    if (skinny) {
      st = skinny_forward(s, Wt, Xt, St, L->wr, L->wc, P, (int)L->nb1);
    } else {
      GemmArgs g;
      g.A = Wt; g.B = Xt; g.C = St;
      g.M = L->wr; g.K = L->wc; g.N = L->nb1;
      g.lda = L->wc; g.ldb = L->nb1; g.ldc = L->nb1;
      g.strideA = L->wr * L->wc; g.strideB = L->wc * L->nb1; g.strideC = L->wr * L->nb1;
      g.batch = P; g.mfma_bf16 = bf16; g.split3 = split; g.b_bf16 = xt_bf16;
      st = launch_gemm(s, g);
    }
    if (st != GPD_OK) return st;
    DecodeJob job;
    job.pts = &c.pts; job.K = c.K; job.useful = c.eC;
    job.grid_r = c.m; job.grid_c = c.d; job.bh = L->wr; job.bw = L->nb1;
    job.rho = L->rho; job.abs_floor = L->abs_floor;
    job.flag_cap = L->flag_cap; job.loc_cap = L->loc_cap; job.workspace_bytes = L->dec_bytes;
    grid_limits(d.N_out, d.batch, c.m, c.d, L->wr, L->nb1, &job.out_rows, &job.out_cols);
    if (act_in_decode) job.epi.kind = 1;
    return act_after(run_decode(s, &L->ring, job, St, present, GPD_DEC_LSQ_ALL, correct_errors, out, d.batch,
                                dec_ws, L->dec_bytes, report), out, d.N_out * d.batch);
  }

  // ---- BACKWARD_UPDATE
  if (!Dlt) return fail(GPD_E_INVALID, "backward: Dlt is null");
  const bool do_bwd = out != nullptr;
  CombineTable tD, tDh, tXh;
  if (do_bwd) {
    // Delta~_p = sum_{i,k} Delta_{i,k} b_p^eD(i,k), stored (N_out/m) x (batch/d2)
    st = L->ring.cached("encD", [&](HostCombineTable* ht) {
      *ht = encode_table(c.pts, L->eD, c.m, d.d2, L->wr, L->nb2, d.batch);
      grid_limits(d.N_out, d.batch, c.m, d.d2, L->wr, L->nb2, &ht->in_rows, &ht->in_cols);
      return GPD_OK;
    }, s, &tD);
    if (st != GPD_OK) return st;
  }
  // update operands: Dhat_p = sum_i Delta_i a_p^i,  Xhat_p = sum_j X_j b_p^j
  st = L->ring.cached("encDh", [&](HostCombineTable* hd) {
    *hd = encode_table(c.pts, L->eUd, c.m, 1, L->wr, d.batch, d.batch);
    grid_limits(d.N_out, d.batch, c.m, 1, L->wr, d.batch, &hd->in_rows, &hd->in_cols);
    return GPD_OK;
  }, s, &tDh);
  if (st != GPD_OK) return st;
  st = L->ring.cached("encXh", [&](HostCombineTable* hx) {
    *hx = encode_table(c.pts, L->eUx, c.n, 1, L->wc, d.batch, d.batch);
    grid_limits(d.N_in, d.batch, c.n, 1, L->wc, d.batch, &hx->in_rows, &hx->in_cols);
    return GPD_OK;
  }, s, &tXh);
  if (st != GPD_OK) return st;
  // small batches on the streaming path: the two or three encodes (a few KB each) in one launch
  SmallEncJobs sj;
  int nj = 0;
  bool small = skinny;
  if (small && do_bwd)
    small = make_small(tD, Dlt, d.batch, d.N_out, d.batch, c.m, d.d2, L->wr, L->nb2, Dt, P, &sj.job[nj++]);
  small = small && make_small(tDh, Dlt, d.batch, d.N_out, d.batch, c.m, 1, L->wr, d.batch, Dh, P, &sj.job[nj++]) &&
          make_small(tXh, X, d.batch, d.N_in, d.batch, c.n, 1, L->wc, d.batch, Xh, P, &sj.job[nj++]);
  if (small) {
    int64_t most = 0;
    for (int q = 0; q < nj; ++q) most = std::max<int64_t>(most, sj.job[q].count);
    if (most > 0) {
      GPD_LAUNCH(encode_small_kernel, dim3((unsigned)((most + 255) / 256), nj), dim3(256), 0, s, sj);
      GPD_HIP(hipGetLastError());
    }
  } else {
    if (do_bwd) {
      st = launch_combine(s, tD, Dlt, d.batch, Dt, L->nb2, xt_bf16 ? 1 : 0, L->wr, L->nb2, none);
      if (st != GPD_OK) return st;
    }
    const int kind = L->upd_fp16 ? 3 : (L->upd_planes ? 2 : 0);
    PlaneScale sd, sx;
    if (L->upd_fp16) {
      // the fp16 planes hold the operands divided by a power of two chosen from the largest
      // finite |Delta| and |X| of this call (one small pass over both, results stay on the device)
      AbsMaxJobs aj;
      aj.x[0] = Dlt; aj.n[0] = d.N_out * d.batch; aj.x[1] = X; aj.n[1] = d.N_in * d.batch;
      aj.parts = scal;
      GPD_LAUNCH(absmax_kernel, dim3(kAmaxParts, 2), dim3(256), 0, s, aj);
      GPD_HIP(hipGetLastError());
      sd.amax_parts = scal; sd.amax_n = kAmaxParts; sd.exp_extra = L->exp_Dh; sd.exp_out = exps;
      sx.amax_parts = scal + kAmaxParts; sx.amax_n = kAmaxParts; sx.exp_extra = L->exp_Xh; sx.exp_out = exps + 1;
    }
    st = launch_combine(s, tDh, Dlt, d.batch, Dh, d.batch, kind, L->wr, d.batch, none, P * L->wr * d.batch,
                        Epilogue(), sd);
    if (st != GPD_OK) return st;
    st = launch_combine(s, tXh, X, d.batch, Xh, d.batch, kind, L->wc, d.batch, none, P * L->wc * d.batch,
                        Epilogue(), sx);
    if (st != GPD_OK) return st;
  }
  const float keep = 1.f - decay;
  if (skinny) {
    // one pass over W~: C~_p from the pre-update values, then the coded update in place
    const int nb2 = (int)L->nb2, nbu = (int)d.batch;
    const int rows = (int)L->wr, cols = (int)L->wc;
    switch (do_bwd ? nb2 : 1) {
      case 1: st = skinny_bu_nbu<1>(s, Wt, Dt, Dh, Xh, part, rows, cols, L->nchunks, P, keep, eta, do_bwd, nbu); break;
      case 2: st = skinny_bu_nbu<2>(s, Wt, Dt, Dh, Xh, part, rows, cols, L->nchunks, P, keep, eta, do_bwd, nbu); break;
      case 4: st = skinny_bu_nbu<4>(s, Wt, Dt, Dh, Xh, part, rows, cols, L->nchunks, P, keep, eta, do_bwd, nbu); break;
      case 8: st = skinny_bu_nbu<8>(s, Wt, Dt, Dh, Xh, part, rows, cols, L->nchunks, P, keep, eta, do_bwd, nbu); break;
      default: st = fail(GPD_E_UNSUPPORTED, "skinny backward: batch %d", nb2);
    }
    if (st != GPD_OK) return st;
    if (do_bwd) {
      const int64_t per_node = L->wc * L->nb2, total = per_node * P;
      GPD_LAUNCH(reduce_chunks_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, part, Ct,
                         per_node, L->nchunks, total);
      GPD_HIP(hipGetLastError());
    }
  } else {
    if (do_bwd) {
      // C~_p = W~_p^T Delta~_p   (step O2, pre-update weights)
      GemmArgs g;
      g.A = Wt; g.transA = true; g.B = Dt; g.C = Ct;
      g.M = L->wc; g.K = L->wr; g.N = L->nb2;
      g.lda = L->wc; g.ldb = L->nb2; g.ldc = L->nb2;
      g.strideA = L->wr * L->wc; g.strideB = L->wr * L->nb2; g.strideC = L->wc * L->nb2;
      g.batch = P; g.mfma_bf16 = bf16; g.split3 = split; g.b_bf16 = xt_bf16;
      st = launch_gemm(s, g);
      if (st != GPD_OK) return st;
    }
    // W~_p <- keep * W~_p + eta * Dhat_p Xhat_p^T   (step O3 in coded form, fp32: on the fp32
    // matrix cores for fp32 layers, as six bf16 or three fp16 partial products otherwise)
    GemmArgs g;
    g.A = Dh; g.B = Xh; g.transB = true; g.C = Wt;
    g.M = L->wr; g.K = d.batch; g.N = L->wc;
    g.lda = d.batch; g.ldb = d.batch; g.ldc = L->wc;
    g.strideA = L->wr * d.batch; g.strideB = L->wc * d.batch; g.strideC = L->wr * L->wc;
    g.batch = P; g.alpha = eta; g.beta = keep;
    g.mfma_bf16 = g.split3 = bf16;
    if (L->upd_planes) { g.planeA = P * L->wr * d.batch; g.planeB = P * L->wc * d.batch; }
    if (L->upd_fp16) g.plane_exps = exps;
    st = launch_gemm(s, g);
    if (st != GPD_OK) return st;
  }
  if (!do_bwd) {
    if (report) {
      // (the caller's list and its capacity stay as they were given, as in every decode)
      gpd_located_t* keep_ptr = report->located;
      const int64_t keep_cap = report->located_cap;
      std::memset(report, 0, sizeof(*report));
      report->located = keep_ptr; report->located_cap = keep_cap;
      report->n_present = P;
    }
    return GPD_OK;
  }
  DecodeJob job;
  job.pts = &c.pts; job.K = L->Kb; job.useful = L->eCb;
  job.grid_r = c.n; job.grid_c = d.d2; job.bh = L->wc; job.bw = L->nb2;
  job.rho = L->rho; job.abs_floor = L->abs_floor;
  job.flag_cap = L->flag_cap; job.loc_cap = L->loc_cap; job.workspace_bytes = L->dec_bytes;
  grid_limits(d.N_in, d.batch, c.n, d.d2, L->wc, L->nb2, &job.out_rows, &job.out_cols);
  if (act_in_decode) { job.epi.kind = 2; job.epi.y = X; }
  return act_after(run_decode(s, &L->ring, job, Ct, present, GPD_DEC_LSQ_ALL, correct_errors, out, d.batch,
                              dec_ws, L->dec_bytes, report), out, d.N_in * d.batch);
}

// ---------------------------------------------------------------- a whole iteration, small batches

namespace {

// Rows `useful` of the least-squares decoding matrix over all P nodes, as a device table [nout][P].
gpd_status_t decode_rows(gpd_layer_t* L, int K, const std::vector<int>& useful, const char* name, CombineTable* t) {
  const Code& c = L->fwd;
  std::string key(name);
  key_add(&key, K);
  return L->ring.cached(key, [&](HostCombineTable* ht) {
    const int P = (int)c.pts.size();
    std::vector<int> S(P);
    for (int q = 0; q < P; ++q) S[q] = q;
    std::vector<double> D;
    gpd_status_t st = decode_matrices(c.pts, S, K, useful, false, &D, nullptr);
    if (st != GPD_OK) return st;
    ht->nin = P; ht->nout = (int)useful.size(); ht->r = 0;
    ht->in_off.assign(P, 0); ht->out_off.assign(ht->nout, 0); ht->node.resize(P);
    for (int q = 0; q < P; ++q) ht->node[q] = q;
    ht->coef = D;
    return GPD_OK;
  }, L->stream, t);
}

gpd_status_t launch_stage(hipStream_t s, StageParams sp) {
  // rows per workgroup: few enough for some 256 workgroups (the kernel is latency, the chip is
  // empty otherwise), and a thread of phase 2 per decoded element (at most 256 per workgroup)
  int tile = std::max(1, std::min(sp.bh / 256, 16));
  while (tile > 1 && sp.G * tile * sp.nb > 256) --tile;
  if (sp.G * tile * sp.nb > 256) return fail(GPD_E_UNSUPPORTED, "mlp step: vectors too wide for the fused stage");
  sp.tile = tile;
  const size_t E = (size_t)sp.G * tile * sp.nb;
  const size_t lds = ((size_t)(sp.P + 1) * E + (size_t)sp.nblk * sp.P + (size_t)sp.njobs * sp.P * sp.G) * sizeof(float);
  if (lds > 60 * 1024) return fail(GPD_E_UNSUPPORTED, "mlp step: vectors too wide for the fused stage");
  GPD_LAUNCH(vector_stage_kernel, dim3((unsigned)((sp.bh + tile - 1) / tile)), dim3(256), lds, s, sp);
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}

}  // namespace

extern "C" gpd_status_t gpd_mlp_step(gpd_layer_t* const* layers, int32_t n_layers, float* const* Wt,
                                     const float* X, const float* Y, float eta, float decay,
                                     float* const* acts, void* const* workspaces,
                                     const size_t* workspace_bytes) {
  if (!layers || n_layers < 1 || !Wt || !X || !Y || !acts || !workspaces || !workspace_bytes)
    return fail(GPD_E_INVALID, "gpd_mlp_step: null argument");
  if (n_layers > 64) return fail(GPD_E_INVALID, "gpd_mlp_step: more than 64 layers");
  // ---- what this path covers; anything else is the caller's per-layer loop
  for (int l = 0; l < n_layers; ++l) {
    const gpd_layer_t* L = layers[l];
    if (!L || !Wt[l] || !acts[l] || !workspaces[l]) return fail(GPD_E_INVALID, "gpd_mlp_step: null entry for layer %d", l);
    if (workspace_bytes[l] < L->ws_bytes || ((uintptr_t)workspaces[l] & 255))
      return fail(GPD_E_WORKSPACE, "gpd_mlp_step: layer %d needs a workspace of %zu aligned bytes", l, L->ws_bytes);
    const gpd_layer_desc_t& d = L->desc;
    if (d.worker_dtype != GPD_F32 || !skinny_ok(L) || d.d1 != 1 || d.d2 != 1 || d.batch != layers[0]->desc.batch ||
        L->stream != layers[0]->stream || d.m > kSmallMaxIn || d.n > kSmallMaxIn)
      return fail(GPD_E_UNSUPPORTED, "gpd_mlp_step: layer %d is outside the small-batch fp32 path "
                                     "(batch 1, 2, 4 or 8, d1 = d2 = 1, fp32 workers, one stream)", l);
    if (l > 0 && d.N_in != layers[l - 1]->desc.N_out)
      return fail(GPD_E_SHAPE, "gpd_mlp_step: layer %d takes %lld inputs, layer %d gives %lld", l,
                  (long long)d.N_in, l - 1, (long long)layers[l - 1]->desc.N_out);
    if (L->wr * d.batch > INT32_MAX / 64 || L->wc * d.batch > INT32_MAX / 64)
      return fail(GPD_E_UNSUPPORTED, "gpd_mlp_step: layer %d too large", l);
  }
  hipStream_t s = layers[0]->stream;
  const int nb = (int)layers[0]->desc.batch;
  const float keep = 1.f - decay;
  gpd_status_t st;

  struct Tables { CombineTable X, Xh, D, Dh, decF, decB; };
  std::vector<Tables> tab(n_layers);
  for (int l = 0; l < n_layers; ++l) {
    gpd_layer_t* L = layers[l];
    const gpd_layer_desc_t& d = L->desc;
    const Code& c = L->fwd;
    st = L->ring.cached("encX", [&](HostCombineTable* ht) {
      *ht = encode_table(c.pts, c.eB, c.n, c.d, L->wc, L->nb1, d.batch);
      grid_limits(d.N_in, d.batch, c.n, c.d, L->wc, L->nb1, &ht->in_rows, &ht->in_cols);
      return GPD_OK;
    }, s, &tab[l].X);
    if (st != GPD_OK) return st;
    st = L->ring.cached("encXh", [&](HostCombineTable* hx) {
      *hx = encode_table(c.pts, L->eUx, c.n, 1, L->wc, d.batch, d.batch);
      grid_limits(d.N_in, d.batch, c.n, 1, L->wc, d.batch, &hx->in_rows, &hx->in_cols);
      return GPD_OK;
    }, s, &tab[l].Xh);
    if (st != GPD_OK) return st;
    st = L->ring.cached("encD", [&](HostCombineTable* ht) {
      *ht = encode_table(c.pts, L->eD, c.m, d.d2, L->wr, L->nb2, d.batch);
      grid_limits(d.N_out, d.batch, c.m, d.d2, L->wr, L->nb2, &ht->in_rows, &ht->in_cols);
      return GPD_OK;
    }, s, &tab[l].D);
    if (st != GPD_OK) return st;
    st = L->ring.cached("encDh", [&](HostCombineTable* hd) {
      *hd = encode_table(c.pts, L->eUd, c.m, 1, L->wr, d.batch, d.batch);
      grid_limits(d.N_out, d.batch, c.m, 1, L->wr, d.batch, &hd->in_rows, &hd->in_cols);
      return GPD_OK;
    }, s, &tab[l].Dh);
    if (st != GPD_OK) return st;
    st = decode_rows(L, c.K, c.eC, "rowsF", &tab[l].decF);
    if (st != GPD_OK) return st;
    st = decode_rows(L, L->Kb, L->eCb, "rowsB", &tab[l].decB);
    if (st != GPD_OK) return st;
    if (tab[l].decF.nin != d.P || tab[l].decB.nin != d.P || tab[l].X.nin != c.n || tab[l].Xh.nin != c.n ||
        tab[l].D.nin != c.m || tab[l].Dh.nin != c.m)
      return fail(GPD_E_UNSUPPORTED, "gpd_mlp_step: unexpected table shape for layer %d", l);
    // all tables of the iteration are fetched before the first launch: each must be one that stays
    // where it is (the layer's table arena can be full after thousands of distinct erasure patterns)
    if (!(tab[l].decF.persistent && tab[l].decB.persistent && tab[l].X.persistent && tab[l].Xh.persistent &&
          tab[l].D.persistent && tab[l].Dh.persistent))
      return fail(GPD_E_UNSUPPORTED, "gpd_mlp_step: the table arena of layer %d is full", l);
  }
  auto ws = [&](int l, size_t off) { return (float*)((char*)workspaces[l] + off); };

  // ---- feedforward stage: X~ and X^ of the first layer from the input, then product and vector stage per layer
  {
    gpd_layer_t* L = layers[0];
    const gpd_layer_desc_t& d = L->desc;
    const Code& c = L->fwd;
    SmallEncJobs sj;
    const int P = d.P;
    if (!make_small(tab[0].X, X, d.batch, d.N_in, d.batch, c.n, c.d, L->wc, L->nb1, ws(0, L->off_Xt), P, &sj.job[0]) ||
        !make_small(tab[0].Xh, X, d.batch, d.N_in, d.batch, c.n, 1, L->wc, d.batch, ws(0, L->off_Xh), P, &sj.job[1]))
      return fail(GPD_E_UNSUPPORTED, "gpd_mlp_step: the first layer's encodes do not fit the small-operand kernel");
    const int64_t most = std::max<int64_t>(sj.job[0].count, sj.job[1].count);
    if (most > 0) {
      GPD_LAUNCH(encode_small_kernel, dim3((unsigned)((most + 255) / 256), 2), dim3(256), 0, s, sj);
      GPD_HIP(hipGetLastError());
    }
  }
  for (int l = 0; l < n_layers; ++l) {
    gpd_layer_t* L = layers[l];
    const gpd_layer_desc_t& d = L->desc;
    const int P = d.P;
    st = skinny_forward(s, Wt[l], ws(l, L->off_Xt), ws(l, L->off_St), L->wr, L->wc, P, nb);   // step O1
    if (st != GPD_OK) return st;
    StageParams sp{};
    sp.in = ws(l, L->off_St); sp.node_stride = L->wr * nb; sp.red_stride = 0;
    sp.P = P; sp.nred = 1; sp.len = (int)L->wr; sp.nb = nb;
    sp.D = tab[l].decF.coef; sp.nblk = tab[l].decF.nout; sp.N = (int)d.N_out;
    sp.out = acts[l];
    if (l + 1 < n_layers) {
      // C1, then the next layer's X~ and X^
      gpd_layer_t* Ln = layers[l + 1];
      sp.epi = 1;
      sp.bh = (int)Ln->wc; sp.G = Ln->fwd.n; sp.njobs = 2;
      sp.job[0] = StageJob{tab[l + 1].X.coef, ws(l + 1, Ln->off_Xt)};
      sp.job[1] = StageJob{tab[l + 1].Xh.coef, ws(l + 1, Ln->off_Xh)};
    } else {
      // C1, the error of the L2 loss, then this layer's Delta~ and D^
      sp.epi = 3; sp.epi_y = Y; sp.scale = 2.f / (float)nb; sp.out2 = ws(l, L->off_delta);
      sp.bh = (int)L->wr; sp.G = L->fwd.m; sp.njobs = l > 0 ? 2 : 1;
      sp.job[0] = StageJob{tab[l].Dh.coef, ws(l, L->off_Dh)};
      sp.job[1] = StageJob{tab[l].D.coef, ws(l, L->off_Dt)};
    }
    st = launch_stage(s, sp);
    if (st != GPD_OK) return st;
  }
  // ---- backpropagation and update stages, from the last layer to the first
  for (int l = n_layers - 1; l >= 0; --l) {
    gpd_layer_t* L = layers[l];
    const gpd_layer_desc_t& d = L->desc;
    const int P = d.P;
    const bool do_bwd = l > 0;
    const int rows = (int)L->wr, cols = (int)L->wc;
    float* part = ws(l, L->off_part);
    // steps O2 (from the pre-update weights) and O3 in one pass over W~
    switch (nb) {
      case 1: st = skinny_bu_nbu<1>(s, Wt[l], ws(l, L->off_Dt), ws(l, L->off_Dh), ws(l, L->off_Xh), part, rows, cols, L->nchunks, P, keep, eta, do_bwd, nb); break;
      case 2: st = skinny_bu_nbu<2>(s, Wt[l], ws(l, L->off_Dt), ws(l, L->off_Dh), ws(l, L->off_Xh), part, rows, cols, L->nchunks, P, keep, eta, do_bwd, nb); break;
      case 4: st = skinny_bu_nbu<4>(s, Wt[l], ws(l, L->off_Dt), ws(l, L->off_Dh), ws(l, L->off_Xh), part, rows, cols, L->nchunks, P, keep, eta, do_bwd, nb); break;
      case 8: st = skinny_bu_nbu<8>(s, Wt[l], ws(l, L->off_Dt), ws(l, L->off_Dh), ws(l, L->off_Xh), part, rows, cols, L->nchunks, P, keep, eta, do_bwd, nb); break;
      default: st = fail(GPD_E_UNSUPPORTED, "gpd_mlp_step: batch %d", nb);
    }
    if (st != GPD_OK) return st;
    if (!do_bwd) break;
    // chunk sums, decode, C2 with this layer's input, then the layer below's Delta~ and D^
    gpd_layer_t* Lp = layers[l - 1];
    StageParams sp{};
    sp.in = part; sp.node_stride = (int64_t)L->nchunks * cols * nb; sp.red_stride = (int64_t)cols * nb;
    sp.P = P; sp.nred = L->nchunks; sp.len = cols; sp.nb = nb;
    sp.D = tab[l].decB.coef; sp.nblk = tab[l].decB.nout; sp.N = (int)d.N_in;
    sp.epi = 2; sp.epi_y = l == 0 ? X : acts[l - 1];
    sp.out = ws(l - 1, Lp->off_delta);
    sp.bh = (int)Lp->wr; sp.G = Lp->fwd.m; sp.njobs = l - 1 > 0 ? 2 : 1;
    sp.job[0] = StageJob{tab[l - 1].Dh.coef, ws(l - 1, Lp->off_Dh)};
    sp.job[1] = StageJob{tab[l - 1].D.coef, ws(l - 1, Lp->off_Dt)};
    st = launch_stage(s, sp);
    if (st != GPD_OK) return st;
  }
  return GPD_OK;
}

// ---------------------------------------------------------------- element-wise steps

extern "C" gpd_status_t gpd_sigmoid_fwd(const float* s, float* y, int64_t n, void* stream) {
  if (n < 0 || (n > 0 && (!s || !y))) return fail(GPD_E_INVALID, "gpd_sigmoid_fwd: bad argument");
  if (n == 0) return GPD_OK;
  GPD_LAUNCH(sigmoid_fwd_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, s, y, n);
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}

extern "C" gpd_status_t gpd_sigmoid_bwd(const float* c, const float* y, float* d, int64_t n, void* stream) {
  if (n < 0 || (n > 0 && (!c || !y || !d))) return fail(GPD_E_INVALID, "gpd_sigmoid_bwd: bad argument");
  if (n == 0) return GPD_OK;
  GPD_LAUNCH(sigmoid_bwd_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, c, y, d, n);
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}

extern "C" gpd_status_t gpd_row_mean(const float* y, int64_t rows, int64_t cols, float* mean, void* stream) {
  if (rows < 0 || cols < 1 || (rows > 0 && (!y || !mean))) return fail(GPD_E_INVALID, "gpd_row_mean: bad argument");
  if (rows == 0) return GPD_OK;
  GPD_LAUNCH(row_mean_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, (hipStream_t)stream, y, rows,
                     cols, mean);
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}

extern "C" gpd_status_t gpd_sigmoid_bwd_sparse(const float* c, const float* y, const float* rho_hat, float rho,
                                               float scale, float* d, int64_t rows, int64_t cols, void* stream) {
  const int64_t n = rows * cols;
  if (rows < 0 || cols < 1 || (n > 0 && (!c || !y || !rho_hat || !d)) || !(rho > 0.f && rho < 1.f))
    return fail(GPD_E_INVALID, "gpd_sigmoid_bwd_sparse: bad argument");
  if (n == 0) return GPD_OK;
  GPD_LAUNCH(sigmoid_bwd_sparse_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                     c, y, rho_hat, rho, scale, d, cols, n);
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}

extern "C" gpd_status_t gpd_l2_delta(const float* y, const float* yhat, float scale, float* d, int64_t n,
                                     void* stream) {
  if (n < 0 || (n > 0 && (!y || !yhat || !d))) return fail(GPD_E_INVALID, "gpd_l2_delta: bad argument");
  if (n == 0) return GPD_OK;
  GPD_LAUNCH(l2_delta_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, y, yhat,
                     scale, d, n);
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}
