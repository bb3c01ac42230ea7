// Streaming "linear combination of blocks" kernel: the encode step (Sec. IV, equations for
// W~(u,v) and X~(v,w)), the erasure decode (remark after Thm 2) and, fused into the decode
// pass, the fp32 soft-error screen (Sec. V Algorithm 1 step 1; appendix "Decoding Methods").
//
//   out_q[r][c] = sum_s coef[q][s] * in_s[r][c]        q < nout, s < nin
//
// HBM-bound: every input element is read once, every output element written once.  Each
// thread owns VEC consecutive columns of one row, holds the nin input values in registers
// and produces the nout outputs one after the other; the coefficient table is read with
// wave-uniform addresses (scalar loads), so no LDS is needed.
#include "gpd_internal.hpp"
#include <cstring>
#include <type_traits>

namespace gpd {

namespace {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

// two fp32 -> packed bf16, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const floatx2 f = {lo, hi};
  union { bf16x2 h; uint32_t u; } cv;
  cv.h = __builtin_convertvector(f, bf16x2);
  return cv.u;
}

template <int VEC> struct VecT;
template <> struct VecT<4> { using f = float4; };
template <> struct VecT<2> { using f = float2; };
template <> struct VecT<1> { using f = float; };

// NT: streaming (nontemporal) load, for inputs that are read exactly once
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
template <int VEC, bool NT = false>
__device__ __forceinline__ void load_vec(const float* p, float (&v)[VEC]) {
  if constexpr (NT && VEC == 4) {
    const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  } else if constexpr (NT && VEC == 2) {
    const v2f t = __builtin_nontemporal_load(reinterpret_cast<const v2f*>(p));
    v[0] = t.x; v[1] = t.y;
  } else if constexpr (NT) {
    v[0] = __builtin_nontemporal_load(p);
  } else if constexpr (VEC == 4) {
    float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  } else if constexpr (VEC == 2) {
    float2 t = *reinterpret_cast<const float2*>(p);
    v[0] = t.x; v[1] = t.y;
  } else {
    v[0] = *p;
  }
}

// NT: streaming (nontemporal) store, for large outputs written exactly once
template <int VEC, bool NT = false>
__device__ __forceinline__ void store_vec(float* p, const float (&v)[VEC]) {
  if constexpr (NT && VEC == 4) {
    v4f t; t.x = v[0]; t.y = v[1]; t.z = v[2]; t.w = v[3];
    __builtin_nontemporal_store(t, reinterpret_cast<v4f*>(p));
  } else if constexpr (NT && VEC == 2) {
    v2f t; t.x = v[0]; t.y = v[1];
    __builtin_nontemporal_store(t, reinterpret_cast<v2f*>(p));
  } else if constexpr (NT) {
    __builtin_nontemporal_store(v[0], p);
  } else if constexpr (VEC == 4) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  } else if constexpr (VEC == 2) {
    *reinterpret_cast<float2*>(p) = make_float2(v[0], v[1]);
  } else {
    *p = v[0];
  }
}

template <int VEC>
__device__ __forceinline__ void store_vec_bf16(uint16_t* p, const float (&v)[VEC]) {
  if constexpr (VEC == 4) {
    uint2 t;
    t.x = pack_bf16(v[0], v[1]);
    t.y = pack_bf16(v[2], v[3]);
    *reinterpret_cast<uint2*>(p) = t;
  } else if constexpr (VEC == 2) {
    *reinterpret_cast<uint32_t*>(p) = pack_bf16(v[0], v[1]);
  } else {
    *p = (uint16_t)(pack_bf16(v[0], 0.f) & 0xffffu);
  }
}

// An fp32 value as three bf16 values (hi = bf16(x), mid = bf16(x - hi), lo = bf16(x - hi - mid),
// round-to-nearest-even, both subtractions exact), stored in three planes `plane` elements apart.
template <int VEC>
__device__ __forceinline__ void store_vec_split3(uint16_t* p, int64_t plane, const float (&v)[VEC]) {
  float r[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) r[e] = v[e];
#pragma unroll
  for (int pl = 0; pl < 3; ++pl) {
    store_vec_bf16<VEC>(p + pl * plane, r);
    if (pl < 2) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const uint32_t h = pack_bf16(r[e], 0.f) & 0xffffu;
        r[e] -= __uint_as_float(h << 16);
      }
    }
  }
}

// An fp32 value, scaled by the power of two `inv`, as two fp16 values (hi = fp16(x), lo =
// fp16(x - hi), round-to-nearest-even, the subtraction exact), stored in two planes `plane`
// elements apart: |x - hi - lo| <= 2^-22 |x| while lo is a normal fp16 number.
__device__ __forceinline__ uint32_t f16_bits(float x) {
  union { _Float16 h; uint16_t u; } cv;
  cv.h = (_Float16)x;
  return cv.u;
}
template <int VEC>
__device__ __forceinline__ void store_vec_split2h(uint16_t* p, int64_t plane, const float (&v)[VEC], float inv) {
  uint32_t hi[VEC], lo[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    const float x = v[e] * inv;
    union { _Float16 h; uint16_t u; } cv;
    cv.h = (_Float16)x;
    hi[e] = cv.u;
    lo[e] = f16_bits(x - (float)cv.h);
  }
#pragma unroll
  for (int pl = 0; pl < 2; ++pl) {
    const uint32_t* w = pl == 0 ? hi : lo;
    uint16_t* q = p + pl * plane;
    if constexpr (VEC == 4) {
      uint2 t;
      t.x = w[0] | (w[1] << 16);
      t.y = w[2] | (w[3] << 16);
      *reinterpret_cast<uint2*>(q) = t;
    } else if constexpr (VEC == 2) {
      *reinterpret_cast<uint32_t*>(q) = w[0] | (w[1] << 16);
    } else {
      *q = (uint16_t)w[0];
    }
  }
}

struct CombineParams {
  const float* in;
  int64_t in_ld;
  void* out;
  int64_t out_ld;
  int64_t out_plane;         // elements between the three planes of a split output
  int64_t rows, cols;        // block shape in elements
  int64_t cols_vec;          // cols / VEC
  int nin, nout, r;
  int q_chunk;               // outputs per thread: blockIdx.y selects [y*q_chunk, (y+1)*q_chunk)
  const int64_t* in_off;
  const int64_t* out_off;
  const float* coef;         // [nout][nin]
  const float* H;            // [r][nin]
  const int32_t* in_rows; const int32_t* in_cols;      // block limits (LIMITS only)
  const int32_t* out_rows; const int32_t* out_cols;
  float rho_screen;          // flagged iff !(sigma <= rho_screen*max(|z|,floor) - margin*|z|)
  float abs_floor;
  float rho;                 // for the ratio statistic
  uint32_t* counters;
  unsigned long long* flag_bits;   // the screen's bit map (bit = codeword index row * cols + col)
  int64_t flag_words;
  // Tables as kernel arguments (scalar loads, independent of the vector memory counter: a
  // table entry read from memory between two stores of the output loop would have to wait for
  // the first store to complete).  The block offsets always; coef and H when karg is set (they
  // fit), else those two are read from memory.
  int32_t karg;
  // bit 0: the inputs are read with streaming loads, bit 1: fp32 outputs are written with streaming
  // stores (large launches in which every input element is read once: measured on 16 MiB blocks,
  // decode 4.8 -> 5.3 TB/s, encode 4.8 -> 5.4 TB/s, before any spreading of the blocks)
  int32_t streaming;
  // element-wise step on fp32 outputs: 0 none, 1 logistic function, 2 times y (1 - y) with y
  // read from epi_y at the output's own offset
  int32_t epi;
  const float* epi_y;
  // output kind 3 (two fp16 planes of out / 2^E): E = exponent of the largest finite input
  // magnitude (amax_parts: amax_n partial maxima as float bit patterns) - 14 + exp_extra, so
  // that |out| / 2^E < 2^15; written to exp_out for the kernel that reads the planes
  const uint32_t* amax_parts;
  int32_t amax_n, exp_extra;
  int32_t* exp_out;
  int64_t in_off_k[64];
  int64_t out_off_k[64];
  float coef_k[256 + 64];    // (64 more, zero: a row is always read NIN_MAX entries long)
  float H_k[256 + 64];
};

static_assert(sizeof(CombineParams) <= 4096, "kernel arguments are limited to 4 KB");

// NIN_MAX: compile-time bound on nin (register array); VEC: columns per thread.
// OUT: 0 fp32, 1 bf16, 2 three bf16 planes (hi, mid, lo of the fp32 value), each block stored
// k-blocked: 16 consecutive columns of a row are contiguous, rows next, column groups outermost;
// 3 two fp16 planes (hi, lo) of the value divided by a power of two, k-blocked in the same way
// TAB: the coefficient tables come through LDS (too large for the kernel arguments); else they
// are kernel arguments.  Two kernels, so that neither carries the other's code and registers.
// The low 64 / VEC bits of x moved to every VEC-th bit position (bit j to bit j * VEC).
template <int VEC>
__device__ __forceinline__ unsigned long long spread_bits(unsigned long long x) {
  if constexpr (VEC == 4) {
    x = (x | (x << 24)) & 0x000000ff000000ffull;
    x = (x | (x << 12)) & 0x000f000f000f000full;
    x = (x | (x << 6)) & 0x0303030303030303ull;
    x = (x | (x << 3)) & 0x1111111111111111ull;
  } else if constexpr (VEC == 2) {
    x = (x | (x << 16)) & 0x0000ffff0000ffffull;
    x = (x | (x << 8)) & 0x00ff00ff00ff00ffull;
    x = (x | (x << 4)) & 0x0f0f0f0f0f0f0f0full;
    x = (x | (x << 2)) & 0x3333333333333333ull;
    x = (x | (x << 1)) & 0x5555555555555555ull;
  }
  return x;
}

// EXACT: nin == NIN_MAX and no block limits, so no input has to be masked out (idle threads of
// the last workgroup compute on the first input's first element and store nothing).
template <int NIN_MAX, int VEC, int OUT, bool SCREEN, bool LIMITS, bool TAB, bool EXACT = false>
__global__ __launch_bounds__(64) void combine_kernel(CombineParams p) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = p.rows * p.cols_vec;
  const bool active = idx < total;
  int64_t row, col;
  if constexpr (OUT >= 2) {
    // threads follow the k-blocked output order (16 / VEC threads per row of a 16-column group,
    // rows next): the stores of a wavefront are contiguous in every plane, and the inputs, whose
    // rows are then read in pieces, are P times smaller than the outputs
    constexpr int TPR = 16 / VEC;
    const int64_t rc = active ? idx / TPR : 0;
    const int64_t kb = rc / p.rows;
    row = rc - kb * p.rows;
    col = kb * 16 + (active ? idx % TPR : 0) * VEC;
  } else {
    row = active ? idx / p.cols_vec : 0;
    col = active ? (idx - row * p.cols_vec) * VEC : 0;
  }

  // Tables that do not travel as kernel arguments go through LDS (dynamic, sized by the host; none
  // when karg): the rows this workgroup needs, padded with zeros to NIN_MAX entries so that a row
  // is read whole and without a branch, like the kernel-argument form.  LDS reads do not share a
  // counter with the output stores, so they never wait for them.  The screening decode always
  // takes this form: with its r + nout rows of kernel arguments, read one row per trip of a loop,
  // every trip waited for a scalar load (decode + screen of 16 nodes: 78 us against 61 us).
  // The table entries are requested after the inputs (below): every workgroup of the launch reads
  // the same few hundred words, and with those requests first the inputs waited behind them (the
  // same launch: 74 us against 60 us).
  constexpr bool karg = !TAB;
  extern __shared__ float tab_lds[];
  const int q_first = blockIdx.y * p.q_chunk;
  const int q_count = min(p.nout, q_first + p.q_chunk) - q_first;
  float* coef_s = tab_lds;
  float* H_s = tab_lds + p.q_chunk * NIN_MAX;
  const int n_coef = q_count * NIN_MAX;
  const int n_tab = n_coef + (SCREEN ? p.r * NIN_MAX : 0);
  // (entry e of the coefficient rows followed by the parity-check rows; an entry of the padding is
  // read from the table's first word and replaced by zero, so that the load is unconditional)
  auto tab_entry = [&](int e) -> float {
    const bool c = e < n_coef;
    const int e2 = c ? e : e - n_coef, row2 = e2 / NIN_MAX, s2 = e2 - row2 * NIN_MAX;
    const bool valid = e < n_tab && s2 < p.nin;
    const float* src = c ? p.coef + (int64_t)(q_first + row2) * p.nin + s2 : p.H + (int64_t)row2 * p.nin + s2;
    const float v = *(valid ? src : p.coef);
    return valid ? v : 0.f;
  };
  auto tab_slot = [&](int e) -> float* { return e < n_coef ? coef_s + e : H_s + (e - n_coef); };

  // All inputs are requested back to back: the address of an input that is not to be read
  // (beyond nin, beyond a block limit, an idle thread) is replaced by that of the first input's
  // first element and the value discarded afterwards, so that there is no branch, and no wait
  // for a table entry, between two loads.  The block offsets are kernel arguments.
  // (the screen's running maximum of ||Hz|| / tau, requested together with the inputs; used below
  // to skip most of the atomics)
  uint32_t ratio_seen = 0;
  if constexpr (SCREEN) ratio_seen = __hip_atomic_load(&p.counters[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  float z[NIN_MAX][VEC];
  const int64_t lane_off = row * p.in_ld + col;
  bool take[NIN_MAX];
#pragma unroll
  for (int s = 0; s < NIN_MAX; ++s) {
    take[s] = s < p.nin && active;
    if constexpr (LIMITS) take[s] = take[s] && row < p.in_rows[s < p.nin ? s : 0] && col < p.in_cols[s < p.nin ? s : 0];
  }
  if (p.streaming & 1) {
#pragma unroll
    for (int s = 0; s < NIN_MAX; ++s)
      load_vec<VEC, true>(p.in + (take[s] ? p.in_off_k[s] + lane_off : p.in_off_k[0]), z[s]);
  } else {
#pragma unroll
    for (int s = 0; s < NIN_MAX; ++s)
      load_vec<VEC>(p.in + (take[s] ? p.in_off_k[s] + lane_off : p.in_off_k[0]), z[s]);
  }
  if constexpr (!EXACT) {
#pragma unroll
    for (int s = 0; s < NIN_MAX; ++s)
#pragma unroll
      for (int v = 0; v < VEC; ++v) z[s][v] = take[s] ? z[s][v] : 0.f;
  }
  if constexpr (!karg) {
    for (int e = (int)threadIdx.x; e < n_tab; e += 64) *tab_slot(e) = tab_entry(e);
    __syncthreads();                                 // the tables are in LDS
  }

  float inv = 1.f;
  if constexpr (OUT == 3) {
    // (one wavefront per workgroup) largest partial maximum, its exponent, the scale
    uint32_t m = 0;
    for (int i = threadIdx.x; i < p.amax_n; i += 64) m = max(m, p.amax_parts[i]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off));
    const int E = max((int)(m >> 23) - 127, -100) - 14 + p.exp_extra;
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *p.exp_out = E;
    inv = ldexpf(1.f, -E);
  }

  // non-finite responses are replaced by zero everywhere (and always passed on, below)
  // (The sum of squares tells whether anything is non-finite: one multiply-add per value.  Only a
  // wavefront that holds such a value, or one so large that its square overflows, goes through
  // the value-by-value test; comparing every value of every wavefront took a quarter of the
  // kernel's vector instructions.)
  bool bad[VEC];
  float nz2[VEC];
  if constexpr (SCREEN) {
    bool odd = false;
#pragma unroll
    for (int v = 0; v < VEC; ++v) { bad[v] = false; nz2[v] = 0.f; }
#pragma unroll
    for (int s = 0; s < NIN_MAX; ++s)
#pragma unroll
      for (int v = 0; v < VEC; ++v) nz2[v] = fmaf(z[s][v], z[s][v], nz2[v]);
#pragma unroll
    for (int v = 0; v < VEC; ++v) odd = odd || !(nz2[v] <= 3.4028234664e38f);
    if (__ballot(odd) != 0ull) {                         // (wave-uniform, rare)
#pragma unroll
      for (int v = 0; v < VEC; ++v) nz2[v] = 0.f;
#pragma unroll
      for (int s = 0; s < NIN_MAX; ++s) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          const float x = z[s][v];
          if (!(fabsf(x) <= 3.4028234664e38f)) { bad[v] = true; z[s][v] = 0.f; }
          nz2[v] = fmaf(z[s][v], z[s][v], nz2[v]);
        }
      }
    }
  }
  if (SCREEN && blockIdx.y == 0) {
    // Algorithm 1 step 1 in fp32, with a threshold below tau so that every codeword the
    // fp64 check could flag is passed on.
    float sig2[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) sig2[v] = 0.f;
    auto syndromes = [&](auto from_args) __attribute__((always_inline)) {
      constexpr bool K = decltype(from_args)::value;
      // (two rows per trip: both rows' table entries are requested before either is used, which
      // halves the number of waits for a scalar load)
#pragma unroll 2
      for (int i = 0; i < p.r; ++i) {
        float y[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) y[v] = 0.f;
        if constexpr (K) {
          const float* __restrict__ hrow = p.H_k + i * p.nin;
          float h[NIN_MAX];
#pragma unroll
          for (int s = 0; s < NIN_MAX; ++s) h[s] = hrow[s];
#pragma unroll
          for (int s = 0; s < NIN_MAX; ++s)
#pragma unroll
            for (int v = 0; v < VEC; ++v) y[v] = fmaf(h[s], z[s][v], y[v]);
        } else {
          const float* hrow = H_s + i * NIN_MAX;
          float h[NIN_MAX];
#pragma unroll
          for (int s = 0; s < NIN_MAX; ++s) h[s] = hrow[s];
#pragma unroll
          for (int s = 0; s < NIN_MAX; ++s)
#pragma unroll
            for (int v = 0; v < VEC; ++v) y[v] = fmaf(h[s], z[s][v], y[v]);
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) sig2[v] = fmaf(y[v], y[v], sig2[v]);
      }
    };
    syndromes(std::integral_constant<bool, karg>{});
    // The codewords passed on are marked in a bit map, bit row * cols + col of 64-bit words: a
    // wavefront covers 64 * VEC consecutive codewords, lane l the VEC codewords from l * VEC on, and
    // writes the VEC words of its own (all of them, also when no bit is set: nothing has to be
    // cleared beforehand, nothing is counted and no wavefront waits for another's atomic).
    float ratio = 0.f;
    unsigned long long words[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) words[k] = 0ull;
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      // (square roots and the reciprocal by the hardware's one-ulp instructions: this test only
      // preselects, with a margin of a factor two, and the ratio is a statistic)
      const float nz = __builtin_amdgcn_sqrtf(nz2[v]);
      const float sig = __builtin_amdgcn_sqrtf(sig2[v]);
      const float base = fmaxf(nz, p.abs_floor);
      const float thr = fmaxf(p.rho_screen * base - 1.52587890625e-05f * nz, 0.f);
      const bool flag = active && (bad[v] || !(sig <= thr));
      if (!flag && active) {
        const float tau = p.rho * base;
        if (tau > 0.f) ratio = fmaxf(ratio, sig * __builtin_amdgcn_rcpf(tau));
      }
      const unsigned long long b = __ballot(flag);       // bit l: lane l, component v
#pragma unroll
      for (int k = 0; k < VEC; ++k)
        words[k] |= spread_bits<VEC>((b >> (k * (64 / VEC))) & (~0ull >> (64 - 64 / VEC))) << v;
    }
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
      for (int k = 0; k < VEC; ++k) p.flag_bits[(int64_t)blockIdx.x * VEC + k] = words[k];
    }
    // wave-wide maximum, one atomic per wave
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ratio = fmaxf(ratio, __shfl_xor(ratio, off));
    // (A running maximum.  Atomics to one address, or to one cache line, are served one after the
    // other, some 10 ns each: 16 384 wavefronts must not all send one.  Almost none has a value above
    // the maximum it read when it started; the few that have read it again, now, and only those
    // still above it send the atomic.  Reading it only here held every wavefront for a memory round
    // trip in front of its outputs; reading it only at the start let the first thousands of
    // wavefronts, which all saw zero, send an atomic each.)
    if ((threadIdx.x & 63) == 0 && ratio > 0.f) {
      const uint32_t bits = __float_as_uint(ratio);
      if (bits > ratio_seen &&
          bits > __hip_atomic_load(&p.counters[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        atomicMax(&p.counters[1], bits);
    }
  }

  if (!active) return;
  const int q_begin = blockIdx.y * p.q_chunk;
  const int q_end = min(p.nout, q_begin + p.q_chunk);
  // (two copies of the loop, so that the copy that reads its tables from the kernel arguments
  // contains no vector load at all and its stores are never waited for)
  auto outputs = [&](auto from_args) __attribute__((always_inline)) {
    constexpr bool K = decltype(from_args)::value;
#pragma unroll 2
    for (int q = q_begin; q < q_end; ++q) {
      float acc[VEC];
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
      if constexpr (K) {
        // the whole row in one go (entries beyond nin meet inputs that are zero)
        const float* __restrict__ crow = p.coef_k + q * p.nin;
        float c[NIN_MAX];
#pragma unroll
        for (int s = 0; s < NIN_MAX; ++s) c[s] = crow[s];
#pragma unroll
        for (int s = 0; s < NIN_MAX; ++s)
#pragma unroll
          for (int v = 0; v < VEC; ++v) acc[v] = fmaf(c[s], z[s][v], acc[v]);
      } else {
        const float* crow = coef_s + (q - q_first) * NIN_MAX;
        float c[NIN_MAX];
#pragma unroll
        for (int s = 0; s < NIN_MAX; ++s) c[s] = crow[s];
#pragma unroll
        for (int s = 0; s < NIN_MAX; ++s)
#pragma unroll
          for (int v = 0; v < VEC; ++v) acc[v] = fmaf(c[s], z[s][v], acc[v]);
      }
      if constexpr (LIMITS) {
        if (!(row < p.out_rows[q] && col < p.out_cols[q])) continue;
      }
      const int64_t oq = p.out_off_k[q];
      const int64_t o = oq + row * p.out_ld + col;
      if constexpr (OUT >= 2) {
        // k-blocked: [col / 16][row][col % 16], what the split GEMM reads as one contiguous stage
        const int64_t ob = oq + ((col >> 4) * p.rows + row) * 16 + (col & 15);
        if constexpr (OUT == 2) store_vec_split3<VEC>(reinterpret_cast<uint16_t*>(p.out) + ob, p.out_plane, acc);
        else store_vec_split2h<VEC>(reinterpret_cast<uint16_t*>(p.out) + ob, p.out_plane, acc, inv);
      } else if constexpr (OUT == 1) store_vec_bf16<VEC>(reinterpret_cast<uint16_t*>(p.out) + o, acc);
      else {
        if constexpr (!SCREEN) {
          if (p.epi == 1) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] = 1.f / (1.f + expf(-acc[v]));
          } else if (p.epi == 2) {
            float y[VEC];
            load_vec<VEC>(p.epi_y + o, y);
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] = acc[v] * y[v] * (1.f - y[v]);
          }
        }
        if (SCREEN || (p.streaming & 2)) store_vec<VEC, true>(reinterpret_cast<float*>(p.out) + o, acc);
        else store_vec<VEC, false>(reinterpret_cast<float*>(p.out) + o, acc);
      }
    }
  };
  outputs(std::integral_constant<bool, karg>{});
}

template <int NIN_MAX, int VEC>
gpd_status_t launch_t(hipStream_t stream, const CombineParams& p, int out_kind, bool screen) {
  const int64_t total = p.rows * p.cols_vec;
  if (total == 0) return GPD_OK;
  // one wavefront per workgroup: a finished wavefront is replaced at once instead of waiting for
  // the rest of a larger workgroup (decode launches measured 6-9 % faster than with 256 threads)
  const int64_t blocks = (total + 63) / 64;
  if (blocks > 0x7fffffffLL) return fail(GPD_E_SHAPE, "block too large for one launch");
  if (screen && blocks * VEC > p.flag_words)
    return fail(GPD_E_WORKSPACE, "combine: the screen's bit map needs %lld words, %lld given",
                (long long)(blocks * VEC), (long long)p.flag_words);
  dim3 grid((unsigned)blocks, (unsigned)((p.nout + p.q_chunk - 1) / p.q_chunk)), block(64);
  const bool lim = p.in_rows != nullptr;
  // tables that do not travel as kernel arguments are staged in LDS: q_chunk coefficient rows and,
  // with the screen, r parity-check rows of NIN_MAX entries each
  const size_t lds = p.karg ? 0 : (size_t)(p.q_chunk + (screen ? p.r : 0)) * NIN_MAX * sizeof(float);
  if (lds > 64 * 1024) return fail(GPD_E_UNSUPPORTED, "combine: tables of %zu bytes do not fit the LDS", lds);
  auto go = [&](auto out_c, auto screen_c) {
    constexpr int O = decltype(out_c)::value;
    constexpr bool S = decltype(screen_c)::value;
    if constexpr (S) {
      if (!lim && p.nin == NIN_MAX) {
        if (p.karg) GPD_LAUNCH((combine_kernel<NIN_MAX, VEC, O, S, false, false, true>), grid, block, lds, stream, p);
        else GPD_LAUNCH((combine_kernel<NIN_MAX, VEC, O, S, false, true, true>), grid, block, lds, stream, p);
        return;
      }
    }
    if (p.karg) {
      if (lim) GPD_LAUNCH((combine_kernel<NIN_MAX, VEC, O, S, true, false>), grid, block, lds, stream, p);
      else GPD_LAUNCH((combine_kernel<NIN_MAX, VEC, O, S, false, false>), grid, block, lds, stream, p);
    } else {
      if (lim) GPD_LAUNCH((combine_kernel<NIN_MAX, VEC, O, S, true, true>), grid, block, lds, stream, p);
      else GPD_LAUNCH((combine_kernel<NIN_MAX, VEC, O, S, false, true>), grid, block, lds, stream, p);
    }
  };
  if (screen) {
    if (out_kind != 0) return fail(GPD_E_UNSUPPORTED, "screen with bf16 output");
    go(std::integral_constant<int, 0>{}, std::true_type{});
  } else if (out_kind == 3) {
    go(std::integral_constant<int, 3>{}, std::false_type{});
  } else if (out_kind == 2) {
    go(std::integral_constant<int, 2>{}, std::false_type{});
  } else if (out_kind == 1) {
    go(std::integral_constant<int, 1>{}, std::false_type{});
  } else {
    go(std::integral_constant<int, 0>{}, std::false_type{});
  }
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}

template <int VEC>
gpd_status_t launch_v(hipStream_t stream, const CombineParams& p, int out_kind, bool screen) {
  if (p.nin <= 4) return launch_t<4, VEC>(stream, p, out_kind, screen);
  if (p.nin <= 8) return launch_t<8, VEC>(stream, p, out_kind, screen);
  if constexpr (VEC == 4) {
    if (p.nin <= 12) return launch_t<12, VEC>(stream, p, out_kind, screen);
  }
  if (p.nin <= 16) return launch_t<16, VEC>(stream, p, out_kind, screen);
  if constexpr (VEC <= 2) {
    if (p.nin <= 32) return launch_t<32, VEC>(stream, p, out_kind, screen);
  }
  if constexpr (VEC == 1) {
    if (p.nin <= 64) return launch_t<64, VEC>(stream, p, out_kind, screen);
  }
  return fail(GPD_E_UNSUPPORTED, "combine: nin = %d too large for VEC = %d", p.nin, VEC);
}

}  // namespace

gpd_status_t launch_combine(hipStream_t stream, const CombineTable& t, const float* in,
                            int64_t in_ld, void* out, int64_t out_ld, int out_kind,
                            int64_t rows, int64_t cols, const ScreenArgs& screen, int64_t out_plane,
                            const Epilogue& epi, const PlaneScale& scale, int streaming) {
  if (t.nin < 1 || t.nin > GPD_MAX_BLOCKS || t.nout < 1)
    return fail(GPD_E_INVALID, "combine: nin = %d, nout = %d", t.nin, t.nout);
  if (rows * cols > 0x7fffffffLL) return fail(GPD_E_SHAPE, "block has more than 2^31 elements");
  CombineParams p;
  p.in = in; p.in_ld = in_ld; p.out = out; p.out_ld = out_ld; p.out_plane = out_plane;
  if (out_kind < 0 || out_kind > 3) return fail(GPD_E_INVALID, "combine: unknown output kind");
  if (out_kind >= 2 && (out_plane % 8 || cols % 16 || out_ld != cols || screen.enabled))
    return fail(GPD_E_INVALID, "combine: split planes need full blocks of a multiple of 16 columns");
  if (out_kind == 3 && (!scale.amax_parts || scale.amax_n < 1 || !scale.exp_out || scale.exp_extra < 0 ||
                        scale.exp_extra > 16))
    return fail(GPD_E_INVALID, "combine: fp16 planes need the partial maxima of the input");
  p.amax_parts = scale.amax_parts; p.amax_n = scale.amax_n; p.exp_extra = scale.exp_extra;
  p.exp_out = scale.exp_out;
  if (epi.kind < 0 || epi.kind > 2 || (epi.kind == 2 && !epi.y) ||
      (epi.kind != 0 && (out_kind != 0 || screen.enabled)))
    return fail(GPD_E_INVALID, "combine: element-wise step needs a plain fp32 output");
  p.epi = epi.kind; p.epi_y = epi.kind == 2 ? epi.y : nullptr;
  p.rows = rows; p.cols = cols;
  p.nin = t.nin; p.nout = t.nout; p.r = screen.enabled ? t.r : 0;
  p.in_off = t.in_off; p.out_off = t.out_off; p.coef = t.coef; p.H = t.H;
  p.in_rows = t.in_rows; p.in_cols = t.in_cols; p.out_rows = t.out_rows; p.out_cols = t.out_cols;
  p.rho = screen.rho; p.rho_screen = 0.5f * screen.rho; p.abs_floor = screen.abs_floor;
  p.counters = screen.counters; p.flag_bits = screen.flag_bits; p.flag_words = screen.flag_words;
  if (!t.k_offsets) return fail(GPD_E_UNSUPPORTED, "combine: more than 64 inputs or outputs");
  std::memcpy(p.in_off_k, t.k_in_off, sizeof(p.in_off_k));
  std::memcpy(p.out_off_k, t.k_out_off, sizeof(p.out_off_k));
  p.karg = t.k_coefs ? 1 : 0;
  if (screen.enabled) {
    // (the screening decode reads its tables from LDS: see the kernel)
    if (!t.coef || (t.r > 0 && !t.H)) return fail(GPD_E_INVALID, "combine: the screen needs its tables in device memory");
    p.karg = 0;
  }
  std::memset(p.coef_k, 0, sizeof(p.coef_k));
  std::memset(p.H_k, 0, sizeof(p.H_k));
  if (p.karg) {
    std::memcpy(p.coef_k, t.k_coef, sizeof(t.k_coef));
    std::memcpy(p.H_k, t.k_H, sizeof(t.k_H));
  }

  // widest vector the shapes, leading dimensions, block offsets and base addresses allow
  const size_t out_elem = out_kind ? 2 : 4;
  auto ok = [&](int vec) {
    if (cols % vec || in_ld % vec || out_ld % vec || t.off_align % vec) return false;
    if (t.in_rows && t.limit_align % vec) return false;
    if (((uintptr_t)in) % (4 * vec) || ((uintptr_t)out) % (out_elem * vec)) return false;
    if (p.epi_y && ((uintptr_t)p.epi_y) % (4 * vec)) return false;
    return true;
  };
  int vec = 1;
  if (t.nin <= 16 && ok(4)) vec = 4;
  else if (t.nin <= 32 && ok(2)) vec = 2;
  p.cols_vec = cols / vec;
  // small launches (the vectors of the batch-1 layer step) are latency-bound: give every
  // output block its own threads instead of looping over the outputs inside one thread
  p.q_chunk = (rows * p.cols_vec < 16384) ? 1 : t.nout;
  // in place (outputs overwrite inputs): a thread must hold all its inputs before any output
  // of its element is written, so the outputs cannot be split over several workgroups
  if ((const void*)in == (const void*)out) p.q_chunk = t.nout;
  // streaming accesses, where the caller asks for them, for launches that move tens of megabytes
  // and read every input once
  {
    const bool big = (double)rows * cols * 4.0 * (t.nin + t.nout) >= 32.0 * 1024 * 1024;
    p.streaming = 0;
    if (big && p.q_chunk == t.nout && (const void*)in != (const void*)out)
      p.streaming = (streaming & kStreamLoads) | (out_kind == 0 ? (streaming & kStreamStores) : 0);
  }
  if (vec == 4) return launch_v<4>(stream, p, out_kind, screen.enabled);
  if (vec == 2) return launch_v<2>(stream, p, out_kind, screen.enabled);
  return launch_v<1>(stream, p, out_kind, screen.enabled);
}

}  // namespace gpd
