// Batched dense products on the matrix cores: the P worker products C~_p = A~_p B~_p
// (Sec. IV, proof of Thm 2), the coded forward / backward products and the rank-B coded
// update of the DNN layer step (Sec. IX).
//
// fp32 path: v_mfma_f32_32x32x2_f32.  A workgroup of 4 wavefronts computes a 128 x 128
// tile of C; each wavefront owns a 64 x 64 sub-tile = 2 x 2 MFMA blocks (64 accumulator
// registers).  Operand tiles of 16 k-values are staged through double-buffered LDS.  The
// order of k inside a tile is permuted so that a lane fetches its four consecutive
// k-values of a k-contiguous operand with one 128-bit LDS read.
#include "gpd_internal.hpp"

namespace gpd {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 16;                 // k-values per LDS stage (fp32 kernel)
constexpr int KC_STRIDE = BK + 4;      // row stride (floats) of a k-contiguous tile  [rows][BK]

// The fp32 kernel comes in two workgroup shapes:
//   small: 128 x 128 tile, 2 x 2 wavefronts (3 workgroups per CU): many tiles, for small or
//          ragged problems;
//   large: 256 x 256 tile, 4 x 4 wavefronts (one 1024-thread workgroup per CU): a quarter of
//          the global-to-LDS traffic per flop; used when both M and N are multiples of 256 and
//          there are enough tiles to fill the chip.
// floats of one LDS operand tile of ROWS rows: k-contiguous [ROWS][BK+4] or row-contiguous [BK][ROWS+4]
template <bool KCONTIG, int ROWS>
constexpr int tile_floats() { return KCONTIG ? ROWS * KC_STRIDE : BK * (ROWS + 4); }

struct GemmParams {
  const float* A; const float* B; float* C;
  int M, N, K;
  int64_t lda, ldb, ldc;
  int64_t sA, sB, sC;
  int batch, tiles_m, tiles_n;
  int total_tiles, tiles_per_xcd;
  float alpha, beta;
};

// One ROWS x 16 operand tile in flight: ROWS*4/NT float4 per thread (NT threads).
//   KCONTIG: memory is [rows][k] (ld = stride between rows): item f -> row f/4, k 4*(f%4)
//   else   : memory is [k][rows]:                  item f -> k f/(ROWS/4), row 4*(f%(ROWS/4))
// MODE 0: tile fully inside, 16-byte aligned; 1: guarded, aligned; 2: guarded, scalar.
template <int ROWS, int NT> struct TileRegs { float4 q[ROWS * 4 / NT]; };

template <bool KCONTIG, int MODE, int ROWS, int NT>
__device__ __forceinline__ TileRegs<ROWS, NT> load_tile(const float* __restrict__ base, int64_t ld, int row0,
                                                        int k0, int nrows, int nk, int tid) {
  TileRegs<ROWS, NT> t;
#pragma unroll
  for (int q = 0; q < ROWS * 4 / NT; ++q) {
    const int f = tid + NT * q;
    int row, k;
    if constexpr (KCONTIG) { row = row0 + (f >> 2); k = k0 + 4 * (f & 3); }
    else { k = k0 + f / (ROWS / 4); row = row0 + 4 * (f % (ROWS / 4)); }
    if constexpr (MODE == 0) {
      const float* p = KCONTIG ? base + (int64_t)row * ld + k : base + (int64_t)k * ld + row;
      t.q[q] = *reinterpret_cast<const float4*>(p);
    } else {
      float v[4] = {0.f, 0.f, 0.f, 0.f};
      if constexpr (KCONTIG) {
        if (row < nrows) {
          const float* p = base + (int64_t)row * ld + k;
          if (MODE == 1 && k + 3 < nk) {
            const float4 x = *reinterpret_cast<const float4*>(p);
            v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) if (k + e < nk) v[e] = p[e];
          }
        }
      } else {
        if (k < nk) {
          const float* p = base + (int64_t)k * ld + row;
          if (MODE == 1 && row + 3 < nrows) {
            const float4 x = *reinterpret_cast<const float4*>(p);
            v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) if (row + e < nrows) v[e] = p[e];
          }
        }
      }
      t.q[q] = make_float4(v[0], v[1], v[2], v[3]);
    }
  }
  return t;
}

template <bool KCONTIG, int ROWS, int NT>
__device__ __forceinline__ void store_tile(float* __restrict__ lds, int tid, const TileRegs<ROWS, NT>& t) {
#pragma unroll
  for (int q = 0; q < ROWS * 4 / NT; ++q) {
    const int f = tid + NT * q;
    if constexpr (KCONTIG) {
      *reinterpret_cast<float4*>(lds + (f >> 2) * KC_STRIDE + 4 * (f & 3)) = t.q[q];
    } else {
      *reinterpret_cast<float4*>(lds + (f / (ROWS / 4)) * (ROWS + 4) + 4 * (f % (ROWS / 4))) = t.q[q];
    }
  }
}

// Fragment of one 32-row block for the four MFMA steps of one 8-wide k group `h`:
// step t multiplies k = 8h + t (lanes 0-31) and k = 8h + 4 + t (lanes 32-63).
template <bool KCONTIG, int ROWS>
__device__ __forceinline__ void read_frag(const float* __restrict__ lds, int row, int h, int g,
                                          float (&f)[4]) {
  if constexpr (KCONTIG) {
    const float4 t = *reinterpret_cast<const float4*>(lds + row * KC_STRIDE + 8 * h + 4 * g);
    f[0] = t.x; f[1] = t.y; f[2] = t.z; f[3] = t.w;
  } else {
#pragma unroll
    for (int t = 0; t < 4; ++t) f[t] = lds[(8 * h + 4 * g + t) * (ROWS + 4) + row];
  }
}

// A_KC: op(A) rows are k-contiguous in memory (A not transposed).
// B_KC: op(B) columns are k-contiguous in memory (B transposed, stored N x K).
// TBM x TBN: workgroup tile; the WGM x WGN wavefronts own (TBM/WGM) x (TBN/WGN) sub-tiles.
template <bool A_KC, bool B_KC, int MODE, int TBM, int TBN, int WGM, int WGN>
// (4-wavefront shape: at least 3 wavefronts per SIMD, i.e. 3 workgroups per CU)
__global__ __launch_bounds__(64 * WGM * WGN, (WGM * WGN == 4) ? 3 : 1) void gemm_f32_kernel(GemmParams g) {
  constexpr int NT = 64 * WGM * WGN;
  constexpr int TA = tile_floats<A_KC, TBM>();
  constexpr int TB = tile_floats<B_KC, TBN>();
  constexpr int WM = TBM / WGM, WN = TBN / WGN, MI = WM / 32, NJ = WN / 32;
  __shared__ __attribute__((aligned(16))) float lds_a[2][TA];
  __shared__ __attribute__((aligned(16))) float lds_b[2][TB];

  // XCD-aware tile order: consecutive workgroup ids go to different XCDs (each with its own
  // L2), so give every XCD one contiguous range of tiles.
  const int xcd = blockIdx.x & 7;
  const int slot = blockIdx.x >> 3;
  const int tile = xcd * g.tiles_per_xcd + slot;
  if (tile >= g.total_tiles) return;
  const int per_batch = g.tiles_m * g.tiles_n;
  const int p = tile / per_batch;
  const int rem = tile - p * per_batch;
  const int tm = rem / g.tiles_n;
  const int tn = rem - tm * g.tiles_n;
  const int m0 = tm * TBM, n0 = tn * TBN;

  const float* __restrict__ A = g.A + (int64_t)p * g.sA;
  const float* __restrict__ B = g.B + (int64_t)p * g.sB;
  float* __restrict__ C = g.C + (int64_t)p * g.sC;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lg = lane >> 5;
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;

  floatx16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nchunks = (g.K + BK - 1) / BK;
  TileRegs<TBM, NT> ra = load_tile<A_KC, MODE, TBM, NT>(A, g.lda, m0, 0, g.M, g.K, tid);
  TileRegs<TBN, NT> rb = load_tile<B_KC, MODE, TBN, NT>(B, g.ldb, n0, 0, g.N, g.K, tid);
  store_tile<A_KC, TBM, NT>(lds_a[0], tid, ra);
  store_tile<B_KC, TBN, NT>(lds_b[0], tid, rb);
  // (the loads of a stage are requested at the end of the stage before the one that moves them to
  // LDS, ahead of the barrier: behind the barrier nothing but the fragment reads stands between a
  // wavefront and its first matrix instruction, and all wavefronts of a SIMD arrive there together)
  if (nchunks > 1) {
    ra = load_tile<A_KC, MODE, TBM, NT>(A, g.lda, m0, BK, g.M, g.K, tid);
    rb = load_tile<B_KC, MODE, TBN, NT>(B, g.ldb, n0, BK, g.N, g.K, tid);
  }
  __syncthreads();

  for (int c = 0; c < nchunks; ++c) {
    const int cur = c & 1;
    const float* __restrict__ as = lds_a[cur];
    const float* __restrict__ bs = lds_b[cur];
#pragma unroll
    for (int h = 0; h < BK / 8; ++h) {
      float fa[MI][4], fb[NJ][4];
#pragma unroll
      for (int i = 0; i < MI; ++i) read_frag<A_KC, TBM>(as, wm + 32 * i + li, h, lg, fa[i]);
#pragma unroll
      for (int j = 0; j < NJ; ++j) read_frag<B_KC, TBN>(bs, wn + 32 * j + li, h, lg, fb[j]);
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < NJ; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][t], fb[j][t], acc[i][j], 0, 0, 0);
    }
    if (c + 1 < nchunks) {
      store_tile<A_KC, TBM, NT>(lds_a[cur ^ 1], tid, ra);
      store_tile<B_KC, TBN, NT>(lds_b[cur ^ 1], tid, rb);
      if (c + 2 < nchunks) {
        ra = load_tile<A_KC, MODE, TBM, NT>(A, g.lda, m0, (c + 2) * BK, g.M, g.K, tid);
        rb = load_tile<B_KC, MODE, TBN, NT>(B, g.ldb, n0, (c + 2) * BK, g.N, g.K, tid);
      }
    }
    __syncthreads();
  }

  // epilogue: accumulator register v of lane (li, lg) holds row 8*(v/4) + 4*lg + v%4, column li
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int col = n0 + wn + 32 * j + li;
      // with beta != 0 all 16 old values of the block are requested before any is used
      float old[16];
      if (g.beta != 0.f) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * lg + (v & 3);
          old[v] = (MODE == 0 || (row < g.M && col < g.N)) ? C[(int64_t)row * g.ldc + col] : 0.f;
        }
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) old[v] = 0.f;
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * lg + (v & 3);
        if (MODE == 0 || (row < g.M && col < g.N))
          C[(int64_t)row * g.ldc + col] = fmaf(g.beta, old[v], g.alpha * acc[i][j][v]);
      }
    }
}

// ------------------------------------------------------------------ bf16 path
//
// v_mfma_f32_32x32x16_bf16: same 128 x 128 workgroup tile and 2 x 2 blocks per wavefront,
// 32 k-values per LDS stage.  Both operand tiles live in LDS as bf16, k-contiguous
// ([row][32 k], row stride 80 bytes), so a lane fetches its 8 consecutive k-values with one
// 128-bit read.  Operands may be fp32 in memory (rounded to nearest even on the way to LDS:
// the coded weights stay fp32 in HBM) and may be k-strided in memory (B of a plain product,
// A of the backward product W~^T Delta~): those are transposed while they are written to
// LDS, with a per-lane rotation of the store order that keeps the 32-bit stores of a
// half-wavefront on 32 different banks.

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// k-values per LDS stage: HK = 32 for the plain kernel, 16 for the three-way split (three planes
// per operand, still double-buffered); a row of a tile is HK + 8 bf16 elements apart from the
// next (80 or 48 bytes: the 128-bit reads of 8 consecutive rows fall on 32 different banks)
constexpr int hk_of(int split) { return split == 1 ? 32 : 16; }


enum { SRC_F32_KC = 0, SRC_BF16_KC = 1, SRC_F32_RC = 2, SRC_BF16_RC = 3 };

struct HGemmParams {
  const void* A; const void* B; float* C;
  int M, N, K;
  int64_t lda, ldb, ldc;
  int64_t sA, sB, sC;
  int64_t planeA, planeB;    // elements between the three planes of a pre-split operand
  int tiles_m, tiles_n, total_tiles, tiles_per_xcd;
  float alpha, beta;
  const int32_t* exps;       // device, {E_A, E_B}: plane operands are two fp16 planes scaled by 2^-E (null: three bf16 planes)
};

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

// two fp32 -> packed bf16, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const floatx2 f = {lo, hi};
  union { bf16x2 h; uint32_t u; } cv;
  cv.h = __builtin_convertvector(f, bf16x2);
  return cv.u;
}

// up to 4 consecutive floats; elements at or beyond nvalid read as zero
template <int MODE>
__device__ __forceinline__ float4 load4f(const float* p, int nvalid) {
  if (MODE == 0 || (nvalid >= 4 && (((uintptr_t)p) & 15) == 0)) return *reinterpret_cast<const float4*>(p);
  float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int e = 0; e < 4; ++e) if (e < nvalid) v[e] = p[e];
  return make_float4(v[0], v[1], v[2], v[3]);
}
// up to 8 consecutive bf16
template <int MODE>
__device__ __forceinline__ uint4 load8h(const uint16_t* p, int nvalid) {
  if (MODE == 0 || (nvalid >= 8 && (((uintptr_t)p) & 15) == 0)) return *reinterpret_cast<const uint4*>(p);
  uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int e = 0; e < 8; ++e) if (e < nvalid) w[e >> 1] |= (uint32_t)p[e] << (16 * (e & 1));
  return make_uint4(w[0], w[1], w[2], w[3]);
}
__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// One operand tile of ROWS rows x HK k in flight, still in source form, spread over NT threads.
// Items per thread: F32_KC ROWS*(HK/4)/NT float4; BF16_KC ROWS*(HK/8)/NT uint4; F32_RC
// ROWS*HK/8/NT patches of 2 k x 4 rows; BF16_RC ROWS*HK/16/NT patches of 2 k x 8 rows (threads
// beyond the patch count idle).
template <int SRC, int ROWS, int NT, int HK> struct HStage;
template <int ROWS, int NT, int HK> struct HStage<SRC_F32_KC, ROWS, NT, HK> { float4 v[ROWS * (HK / 4) / NT]; };
template <int ROWS, int NT, int HK> struct HStage<SRC_BF16_KC, ROWS, NT, HK> { uint4 v[(ROWS * (HK / 8) + NT - 1) / NT]; };
template <int ROWS, int NT, int HK> struct HStage<SRC_F32_RC, ROWS, NT, HK> { float4 v[ROWS * HK / 8 / NT][2]; };
template <int ROWS, int NT, int HK> struct HStage<SRC_BF16_RC, ROWS, NT, HK> { uint4 v[(ROWS * HK / 16 + NT - 1) / NT][2]; };

// base: start of the operand for this batch entry; "row" is the m (or n) index, k the
// contraction index.  KC sources are [row][k] with leading dimension ld, RC sources [k][row].
template <int SRC, int MODE, int ROWS, int NT, int HK>
__device__ __forceinline__ void hload(HStage<SRC, ROWS, NT, HK>& st, const void* base, int64_t ld, int row0,
                                      int k0, int nrows, int nk, int tid) {
  if constexpr (SRC == SRC_F32_KC) {
    const float* b = (const float*)base;
#pragma unroll
    for (int q = 0; q < ROWS * (HK / 4) / NT; ++q) {
      const int f = tid + NT * q;
      const int row = row0 + f / (HK / 4), k = k0 + 4 * (f % (HK / 4));
      const int nv = (MODE == 0) ? 4 : (row < nrows ? clampi(nk - k, 0, 4) : 0);
      st.v[q] = (MODE == 0 || nv > 0) ? load4f<MODE>(b + (int64_t)row * ld + k, nv) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  } else if constexpr (SRC == SRC_BF16_KC) {
    const uint16_t* b = (const uint16_t*)base;
#pragma unroll
    for (int q = 0; q < (ROWS * (HK / 8) + NT - 1) / NT; ++q) {
      const int f = tid + NT * q;
      const int row = row0 + f / (HK / 8), k = k0 + 8 * (f % (HK / 8));
      const bool mine = f < ROWS * (HK / 8);
      const int nv = !mine ? 0 : ((MODE == 0) ? 8 : (row < nrows ? clampi(nk - k, 0, 8) : 0));
      st.v[q] = (nv > 0) ? load8h<MODE>(b + (int64_t)row * ld + k, nv) : make_uint4(0u, 0u, 0u, 0u);
    }
  } else if constexpr (SRC == SRC_F32_RC) {
    const float* b = (const float*)base;
#pragma unroll
    for (int q = 0; q < ROWS * HK / 8 / NT; ++q) {
      const int f = tid + NT * q;
      const int kp = (f & 3) + 4 * (f / ROWS), rq = (f >> 2) % (ROWS / 4);
      const int row = row0 + 4 * rq;
#pragma unroll
      for (int par = 0; par < 2; ++par) {
        const int k = k0 + 2 * kp + par;
        const int nv = (MODE == 0) ? 4 : (k < nk ? clampi(nrows - row, 0, 4) : 0);
        st.v[q][par] = (MODE == 0 || nv > 0) ? load4f<MODE>(b + (int64_t)k * ld + row, nv)
                                             : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
  } else {
    const uint16_t* b = (const uint16_t*)base;
#pragma unroll
    for (int q = 0; q < (ROWS * HK / 16 + NT - 1) / NT; ++q) {
      const int f = tid + NT * q;
      const int kp = (f & 3) + 4 * (f / (ROWS / 2)), rq = (f >> 2) % (ROWS / 8);
      const int row = row0 + 8 * rq;
#pragma unroll
      for (int par = 0; par < 2; ++par) {
        const int k = k0 + 2 * kp + par;
        const bool mine = f < ROWS * HK / 16;
        const int nv = !mine ? 0 : ((MODE == 0) ? 8 : (k < nk ? clampi(nrows - row, 0, 8) : 0));
        st.v[q][par] = (nv > 0) ? load8h<MODE>(b + (int64_t)k * ld + row, nv) : make_uint4(0u, 0u, 0u, 0u);
      }
    }
  }
}

// ---- loads of full tiles through buffer instructions
//
// The descriptor covers one batch entry of the operand, starting at the tile's first row (or
// column); every access of a full tile lies inside it.  voff is the byte offset of the lane's
// first item inside the stage at k = 0; the items of a lane, the two k-rows of a patch and the
// stage itself only add wavefront-uniform amounts.
struct BufSrc {
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t voff;
  uint32_t voff_lane;   // the lane's index in the workgroup
};
__device__ __forceinline__ uint4 bload16(const BufSrc& b, uint32_t soff) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(b.rsrc, b.voff, soff, 0);
  return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ float4 bload16f(const BufSrc& b, uint32_t soff) {
  const uint4 v = bload16(b, soff);
  return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}

template <int SRC, int ROWS, int NT, int HK>
__device__ __forceinline__ BufSrc make_bufsrc(const void* base, int64_t ld, int row0, int nrows, int nk, int tid) {
  BufSrc b;
  // bytes from the tile's origin to the end of the batch entry (the host has checked that this
  // is below 2^31 for every operand that takes this path)
  int64_t origin, extent;
  if constexpr (SRC == SRC_F32_KC) {
    origin = (int64_t)row0 * ld * 4; extent = (((int64_t)nrows - 1) * ld + nk) * 4;
    b.voff = (uint32_t)(((tid / (HK / 4)) * ld + 4 * (tid % (HK / 4))) * 4);
    static_assert(NT % (HK / 4) == 0, "items of a lane differ by whole rows");
  } else if constexpr (SRC == SRC_BF16_KC) {
    origin = (int64_t)row0 * ld * 2; extent = (((int64_t)nrows - 1) * ld + nk) * 2;
    b.voff = (uint32_t)(((tid / (HK / 8)) * ld + 8 * (tid % (HK / 8))) * 2);
    static_assert(NT % (HK / 8) == 0, "items of a lane differ by whole rows");
  } else if constexpr (SRC == SRC_F32_RC) {
    origin = (int64_t)row0 * 4; extent = (((int64_t)nk - 1) * ld + nrows) * 4;
    b.voff = (uint32_t)((2 * ((tid & 3) + 4 * (tid / ROWS)) * ld + 4 * ((tid >> 2) % (ROWS / 4))) * 4);
    static_assert(NT % ROWS == 0 || ROWS % NT == 0, "items of a lane differ by whole k-rows");
  } else {
    static_assert(SRC == SRC_BF16_RC, "four source layouts");
    origin = (int64_t)row0 * 2; extent = (((int64_t)nk - 1) * ld + nrows) * 2;
    b.voff = (uint32_t)((2 * ((tid & 3) + 4 * (tid / (ROWS / 2))) * ld + 8 * ((tid >> 2) % (ROWS / 8))) * 2);
  }
  b.voff_lane = (uint32_t)tid;
  const int64_t left = extent - origin;
  b.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>((const char*)base + origin), 0,
                                             (int)(left > 0x7fffffffLL ? 0x7fffffffLL : left), 0x00020000);
  return b;
}

// the stage at k0 of a full tile (same items and order as hload)
template <int SRC, int ROWS, int NT, int HK>
__device__ __forceinline__ void hload_buf(HStage<SRC, ROWS, NT, HK>& st, const BufSrc& b, int64_t ld, int k0) {
  if constexpr (SRC == SRC_F32_KC) {
    const uint32_t step = (uint32_t)((NT / (HK / 4)) * ld * 4);
#pragma unroll
    for (int q = 0; q < ROWS * (HK / 4) / NT; ++q) st.v[q] = bload16f(b, (uint32_t)k0 * 4u + q * step);
  } else if constexpr (SRC == SRC_BF16_KC) {
    constexpr int COUNT = ROWS * (HK / 8);
    const uint32_t step = (uint32_t)((NT / (HK / 8)) * ld * 2);
#pragma unroll
    for (int q = 0; q < (COUNT + NT - 1) / NT; ++q) {
      const bool mine = COUNT % NT == 0 || (int)(b.voff_lane + NT * q) < COUNT;
      st.v[q] = mine ? bload16(b, (uint32_t)k0 * 2u + q * step) : make_uint4(0u, 0u, 0u, 0u);
    }
  } else if constexpr (SRC == SRC_F32_RC) {
    // f = tid + NT q: kp grows by 4 NT / ROWS per item (NT a multiple of ROWS)
    static_assert(NT % ROWS == 0, "an item step is a whole number of k-pairs");
    const uint32_t row_b = (uint32_t)(ld * 4), step = (uint32_t)(8 * (NT / ROWS)) * row_b;
#pragma unroll
    for (int q = 0; q < ROWS * HK / 8 / NT; ++q)
#pragma unroll
      for (int par = 0; par < 2; ++par) st.v[q][par] = bload16f(b, (uint32_t)k0 * row_b + q * step + par * row_b);
  } else {
    static_assert(SRC == SRC_BF16_RC && NT % (ROWS / 2) == 0, "an item step is a whole number of k-pairs");
    constexpr int COUNT = ROWS * HK / 16;                   // patches per stage; lanes beyond idle
    const uint32_t row_b = (uint32_t)(ld * 2), step = (uint32_t)(8 * (NT / (ROWS / 2))) * row_b;
#pragma unroll
    for (int q = 0; q < (COUNT + NT - 1) / NT; ++q) {
      const bool mine = COUNT % NT == 0 || (int)(b.voff_lane + NT * q) < COUNT;
#pragma unroll
      for (int par = 0; par < 2; ++par)
        st.v[q][par] = mine ? bload16(b, (uint32_t)k0 * row_b + q * step + par * row_b) : make_uint4(0u, 0u, 0u, 0u);
    }
  }
}

// An fp32 value as the sum of three bf16 values (8 + 8 + 8 significand bits; what is left is
// below 2^-26 of the value): hi = bf16(x), mid = bf16(x - hi), lo = bf16(x - hi - mid), all
// round-to-nearest-even, both subtractions exact.  Two values at a time, packed.
__device__ __forceinline__ void split3_pack(float x0, float x1, uint32_t (&w)[3]) {
  w[0] = pack_bf16(x0, x1);
  const float r0 = x0 - __uint_as_float(w[0] << 16), r1 = x1 - __uint_as_float(w[0] & 0xffff0000u);
  w[1] = pack_bf16(r0, r1);
  const float s0 = r0 - __uint_as_float(w[1] << 16), s1 = r1 - __uint_as_float(w[1] & 0xffff0000u);
  w[2] = pack_bf16(s0, s1);
}

// Writes the staged tile to LDS as bf16 [row][k] (row stride HK + 8 elements).  With SPLIT = 3
// (fp32 sources only) three such planes, PLANE elements apart, hold hi / mid / lo.
template <int SRC, int ROWS, int NT, int HK>
constexpr int hstage_items() {
  return SRC == SRC_F32_KC ? ROWS * (HK / 4) / NT
       : SRC == SRC_BF16_KC ? (ROWS * (HK / 8) + NT - 1) / NT
       : SRC == SRC_F32_RC ? ROWS * HK / 8 / NT
                           : (ROWS * HK / 16 + NT - 1) / NT;
}

// item q of the staged tile (one global load's worth per thread)
template <int SRC, int ROWS, int NT, int SPLIT, int PLANE, int HK>
__device__ __forceinline__ void hstore_item(const HStage<SRC, ROWS, NT, HK>& st, int q,
                                            uint16_t* __restrict__ lds, int tid) {
  constexpr int HSTRIDE = HK + 8;
  static_assert(SPLIT == 1 || SRC == SRC_F32_KC || SRC == SRC_F32_RC, "only fp32 sources are split");
  const int f = tid + NT * q;
  if constexpr (SRC == SRC_F32_KC) {
    uint16_t* dst = lds + (f / (HK / 4)) * HSTRIDE + 4 * (f % (HK / 4));
    if constexpr (SPLIT == 1) {
      uint2 w;
      w.x = pack_bf16(st.v[q].x, st.v[q].y);
      w.y = pack_bf16(st.v[q].z, st.v[q].w);
      *reinterpret_cast<uint2*>(dst) = w;
    } else {
      uint32_t a[3], b[3];
      split3_pack(st.v[q].x, st.v[q].y, a);
      split3_pack(st.v[q].z, st.v[q].w, b);
#pragma unroll
      for (int pl = 0; pl < 3; ++pl) *reinterpret_cast<uint2*>(dst + pl * PLANE) = make_uint2(a[pl], b[pl]);
    }
  } else if constexpr (SRC == SRC_BF16_KC) {
    if (f < ROWS * (HK / 8))
      *reinterpret_cast<uint4*>(lds + (f / (HK / 8)) * HSTRIDE + 8 * (f % (HK / 8))) = st.v[q];
  } else if constexpr (SRC == SRC_F32_RC) {
    const int kp = (f & 3) + 4 * (f / ROWS), rq = (f >> 2) % (ROWS / 4);
    const float lo[4] = {st.v[q][0].x, st.v[q][0].y, st.v[q][0].z, st.v[q][0].w};
    const float hi[4] = {st.v[q][1].x, st.v[q][1].y, st.v[q][1].z, st.v[q][1].w};
    const int rot = (rq >> 1) & 3;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int ee = (e + rot) & 3;
      float l = lo[0], h = hi[0];
#pragma unroll
      for (int c = 1; c < 4; ++c) { if (ee == c) { l = lo[c]; h = hi[c]; } }
      uint16_t* dst = lds + (4 * rq + ee) * HSTRIDE + 2 * kp;
      if constexpr (SPLIT == 1) {
        *reinterpret_cast<uint32_t*>(dst) = pack_bf16(l, h);
      } else {
        uint32_t w[3];
        split3_pack(l, h, w);
#pragma unroll
        for (int pl = 0; pl < 3; ++pl) *reinterpret_cast<uint32_t*>(dst + pl * PLANE) = w[pl];
      }
    }
  } else {
    if (f < ROWS * HK / 16) {
      const int kp = (f & 3) + 4 * (f / (ROWS / 2)), rq = (f >> 2) % (ROWS / 8);
      const uint32_t lo[4] = {st.v[q][0].x, st.v[q][0].y, st.v[q][0].z, st.v[q][0].w};
      const uint32_t hi[4] = {st.v[q][1].x, st.v[q][1].y, st.v[q][1].z, st.v[q][1].w};
      const int rot = rq & 7;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int ee = (e + rot) & 7;
        uint32_t l = lo[0], h = hi[0];
#pragma unroll
        for (int c = 1; c < 4; ++c) { if ((ee >> 1) == c) { l = lo[c]; h = hi[c]; } }
        const uint32_t sh = 16u * (ee & 1);
        const uint32_t w = ((l >> sh) & 0xffffu) | (((h >> sh) & 0xffffu) << 16);
        *reinterpret_cast<uint32_t*>(lds + (8 * rq + ee) * HSTRIDE + 2 * kp) = w;
      }
    }
  }
}

template <int SRC, int ROWS, int NT, int SPLIT, int PLANE, int HK>
__device__ __forceinline__ void hstore(const HStage<SRC, ROWS, NT, HK>& st, uint16_t* __restrict__ lds, int tid) {
#pragma unroll
  for (int q = 0; q < hstage_items<SRC, ROWS, NT, HK>(); ++q)
    hstore_item<SRC, ROWS, NT, SPLIT, PLANE, HK>(st, q, lds, tid);
}

// TBM x TBN workgroup tile, WGM x WGN wavefronts, each owning (TBM/WGM) x (TBN/WGN).
// SPLIT = 3: both operands are fp32 in memory and are multiplied as sums of three bf16 values;
// the six partial products of weight >= 2^-16 are accumulated (hi*hi, hi*mid, mid*hi, hi*lo,
// mid*mid, lo*hi), which leaves a relative error below 2^-24 per product of two elements, the
// rounding of one fp32 multiplication.  A stage holds 16 k-values of all three planes of both
// operands; the conversion of the next stage (plain ALU work) overlaps with the products of
// the wavefronts that are still multiplying.
template <int ASRC, int BSRC, int MODE, int TBM, int TBN, int WGM, int WGN, int SPLIT>
__global__ __launch_bounds__(64 * WGM * WGN, (WGM * WGN == 4) ? (SPLIT == 1 ? 3 : 2) : 1) void gemm_bf16_kernel(HGemmParams g) {
  constexpr int NT = 64 * WGM * WGN;
  constexpr int WM = TBM / WGM, WN = TBN / WGN, MI = WM / 32, NJ = WN / 32;
  constexpr int HK = hk_of(SPLIT), HSTRIDE = HK + 8;
  constexpr int PA = TBM * HSTRIDE, PB = TBN * HSTRIDE;          // elements per plane
  __shared__ __attribute__((aligned(16))) uint16_t lds_a[2][SPLIT * PA];
  __shared__ __attribute__((aligned(16))) uint16_t lds_b[2][SPLIT * PB];

  const int xcd = blockIdx.x & 7;
  const int slot = blockIdx.x >> 3;
  const int tile = xcd * g.tiles_per_xcd + slot;
  if (tile >= g.total_tiles) return;
  const int per_batch = g.tiles_m * g.tiles_n;
  const int p = tile / per_batch;
  const int rem = tile - p * per_batch;
  const int tm = rem / g.tiles_n;
  const int tn = rem - tm * g.tiles_n;
  const int m0 = tm * TBM, n0 = tn * TBN;

  constexpr int A_ES = (ASRC == SRC_BF16_KC || ASRC == SRC_BF16_RC) ? 2 : 4;
  constexpr int B_ES = (BSRC == SRC_BF16_KC || BSRC == SRC_BF16_RC) ? 2 : 4;
  const int64_t lda = g.lda, ldb = g.ldb;
  const char* A = (const char*)g.A + (int64_t)p * g.sA * A_ES;
  const char* B = (const char*)g.B + (int64_t)p * g.sB * B_ES;
  float* __restrict__ C = g.C + (int64_t)p * g.sC;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lg = lane >> 5;
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;

  floatx16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // Read-modify-write of the output tile (the coded update): with two workgroups of this shape on
  // a CU there are registers to spare, so the old values are requested before the first stage
  // and have arrived long before the epilogue needs them.
  constexpr bool kPrefetchC = SPLIT == 3 && MI * NJ <= 4;
  float oldc[kPrefetchC ? MI * NJ * 16 : 1];
  if constexpr (kPrefetchC) {
    if (g.beta != 0.f) {
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int row = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * lg + (v & 3);
            const int col = n0 + wn + 32 * j + li;
            oldc[(i * NJ + j) * 16 + v] =
                (MODE == 0 || (row < g.M && col < g.N)) ? C[(int64_t)row * g.ldc + col] : 0.f;
          }
    } else {
#pragma unroll
      for (int v = 0; v < MI * NJ * 16; ++v) oldc[v] = 0.f;
    }
  }

  const int nchunks = (g.K + HK - 1) / HK;
  auto kof = [&](int c) { return c * HK; };
  union Frag { uint4 u; bf16x8 v; };
  // Full tiles are loaded through buffer instructions: the descriptor and the per-stage offset
  // live in scalar registers, and one 32-bit lane offset per operand serves every load (64-bit
  // per-load pointers would cost two registers and an add per load and stage).
  [[maybe_unused]] BufSrc bufA, bufB;
  if constexpr (MODE == 0) {
    bufA = make_bufsrc<ASRC, TBM, NT, HK>(A, lda, m0, g.M, g.K, tid);
    bufB = make_bufsrc<BSRC, TBN, NT, HK>(B, ldb, n0, g.N, g.K, tid);
  }
  auto loadA = [&](HStage<ASRC, TBM, NT, HK>& st, int k0) __attribute__((always_inline)) {
    if constexpr (MODE == 0) hload_buf<ASRC, TBM, NT, HK>(st, bufA, lda, k0);
    else hload<ASRC, MODE, TBM, NT, HK>(st, A, lda, m0, k0, g.M, g.K, tid);
  };
  auto loadB = [&](HStage<BSRC, TBN, NT, HK>& st, int k0) __attribute__((always_inline)) {
    if constexpr (MODE == 0) hload_buf<BSRC, TBN, NT, HK>(st, bufB, ldb, k0);
    else hload<BSRC, MODE, TBN, NT, HK>(st, B, ldb, n0, k0, g.N, g.K, tid);
  };

  // the matrix instructions of one stage held in LDS buffer cur; between(g) runs after group g
  // of MI x NJ instructions (SPLIT == 1: HK / 16 groups, one per 16 k; SPLIT == 3: the six
  // partial products hi*lo, mid*mid, hi*mid, lo*hi, mid*hi, hi*hi)
  auto multiply = [&](int cur, auto&& between) __attribute__((always_inline)) {
    const uint16_t* __restrict__ as = lds_a[cur];
    const uint16_t* __restrict__ bs = lds_b[cur];
    if constexpr (SPLIT == 1) {
#pragma unroll
      for (int h = 0; h < HK / 16; ++h) {
        Frag fa[MI], fb[NJ];
#pragma unroll
        for (int i = 0; i < MI; ++i)
          fa[i].u = *reinterpret_cast<const uint4*>(as + (wm + 32 * i + li) * HSTRIDE + 16 * h + 8 * lg);
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          fb[j].u = *reinterpret_cast<const uint4*>(bs + (wn + 32 * j + li) * HSTRIDE + 16 * h + 8 * lg);
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < NJ; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i].v, fb[j].v, acc[i][j], 0, 0, 0);
        between(h);
      }
    } else {
      static_assert(SPLIT == 1 || HK == 16, "one matrix-instruction step per stage");
      Frag fa[MI][3];
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int pl = 0; pl < 3; ++pl)
          fa[i][pl].u = *reinterpret_cast<const uint4*>(as + pl * PA + (wm + 32 * i + li) * HSTRIDE + 8 * lg);
      int group = 0;
#pragma unroll
      for (int pb = 2; pb >= 0; --pb) {
        Frag fb[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          fb[j].u = *reinterpret_cast<const uint4*>(bs + pb * PB + (wn + 32 * j + li) * HSTRIDE + 8 * lg);
#pragma unroll
        for (int pa = 2 - pb; pa >= 0; --pa) {
#pragma unroll
          for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i][pa].v, fb[j].v, acc[i][j], 0, 0, 0);
          between(group);
          ++group;
        }
      }
    }
  };

  // Deep: the 8-wavefront shapes (256 registers per wavefront) and the split kernels keep two
  // stages of global loads in flight; needs full tiles and an even number of stages (the host
  // sends everything else to the bounds-checked kernel).
  constexpr bool kDeep = (SPLIT == 3 || WGM * WGN == 8) && MODE == 0;
  if constexpr (!kDeep) {
    // one register set: the loads of stage c + 1 are issued before stage c is multiplied and
    // written to the other LDS buffer after it
    HStage<ASRC, TBM, NT, HK> sa;
    HStage<BSRC, TBN, NT, HK> sb;
    loadA(sa, kof(0));
    loadB(sb, kof(0));
    hstore<ASRC, TBM, NT, SPLIT, PA, HK>(sa, lds_a[0], tid);
    hstore<BSRC, TBN, NT, SPLIT, PB, HK>(sb, lds_b[0], tid);
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
      const int cur = c & 1;
      if (c + 1 < nchunks) {
        loadA(sa, kof(c + 1));
        loadB(sb, kof(c + 1));
      }
      multiply(cur, [](int) {});
      if (c + 1 < nchunks) {
        hstore<ASRC, TBM, NT, SPLIT, PA, HK>(sa, lds_a[cur ^ 1], tid);
        hstore<BSRC, TBN, NT, SPLIT, PB, HK>(sb, lds_b[cur ^ 1], tid);
      }
      __syncthreads();
    }
  } else {
    // Two statically addressed register sets.  Stage c is multiplied from LDS buffer c & 1;
    // stage c + 1, already in registers, is converted and written to the other buffer in pieces
    // placed between the groups of matrix instructions (the plain ALU work runs while the
    // matrix pipe is busy); the global loads of stage c + 2 go into the set stage c has left.
    // Rotating the sets by copies would make every iteration wait for the loads it has just
    // issued; and the load counter is relative, so the steady state (every iteration loads: the
    // number of younger loads in flight when a set is needed is always the same) is a loop of
    // its own and the last two stages, after which nothing is loaded, are peeled.
    constexpr int R = 2;
    constexpr int IA = hstage_items<ASRC, TBM, NT, HK>(), IB = hstage_items<BSRC, TBN, NT, HK>();
    constexpr int GROUPS = SPLIT == 3 ? 6 : HK / 16;
    constexpr int PER = (IA + IB + GROUPS - 1) / GROUPS;     // conversion items after each group
    HStage<ASRC, TBM, NT, HK> sa[R];
    HStage<BSRC, TBN, NT, HK> sb[R];
    loadA(sa[0], kof(0));
    loadB(sb[0], kof(0));
    loadA(sa[1], kof(1));
    loadB(sb[1], kof(1));
    hstore<ASRC, TBM, NT, SPLIT, PA, HK>(sa[0], lds_a[0], tid);
    hstore<BSRC, TBN, NT, SPLIT, PB, HK>(sb[0], lds_b[0], tid);
    __syncthreads();
    auto stage = [&](HStage<ASRC, TBM, NT, HK>& la, HStage<BSRC, TBN, NT, HK>& lb,
                     const HStage<ASRC, TBM, NT, HK>& ca, const HStage<BSRC, TBN, NT, HK>& cb, int c, bool load,
                     bool conv) __attribute__((always_inline)) {
      const int cur = c & 1;
      if (load) {
        loadA(la, kof(c + R));
        loadB(lb, kof(c + R));
      }
      multiply(cur, [&](int group) __attribute__((always_inline)) {
        if (conv) {
#pragma unroll
          for (int it = group * PER; it < (group + 1) * PER && it < IA + IB; ++it) {
            if (it < IA) hstore_item<ASRC, TBM, NT, SPLIT, PA, HK>(ca, it, lds_a[cur ^ 1], tid);
            else hstore_item<BSRC, TBN, NT, SPLIT, PB, HK>(cb, it - IA, lds_b[cur ^ 1], tid);
          }
        }
      });
      __syncthreads();
    };
    int c0 = 0;
    for (; c0 + 2 * R <= nchunks; c0 += R) {
      stage(sa[0], sb[0], sa[1], sb[1], c0, true, true);
      stage(sa[1], sb[1], sa[0], sb[0], c0 + 1, true, true);
    }
    stage(sa[0], sb[0], sa[1], sb[1], c0, false, true);
    stage(sa[1], sb[1], sa[0], sb[0], c0 + 1, false, false);
  }

  // Read-modify-write of the output tile.  All old values of a group of 32 x 32 blocks are
  // requested before any is used: one memory latency per group.  Where two workgroups of four
  // wavefronts share a CU the group is the whole tile (the registers of the staging sets and
  // fragments are free by now), elsewhere one block.
  constexpr int NB = MI * NJ, GB = (SPLIT == 3 && MI * NJ <= 4) ? 4 : 1;
  static_assert(NB % GB == 0, "whole groups of blocks");
#pragma unroll
  for (int b0 = 0; b0 < NB; b0 += GB) {
    float old[GB][16];
#pragma unroll
    for (int bb = 0; bb < GB; ++bb) {
      const int i = (b0 + bb) / NJ, j = (b0 + bb) % NJ;
      const int col = n0 + wn + 32 * j + li;
      if constexpr (kPrefetchC) {
#pragma unroll
        for (int v = 0; v < 16; ++v) old[bb][v] = oldc[(i * NJ + j) * 16 + v];
      } else if (g.beta != 0.f) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * lg + (v & 3);
          old[bb][v] = (MODE == 0 || (row < g.M && col < g.N)) ? C[(int64_t)row * g.ldc + col] : 0.f;
        }
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) old[bb][v] = 0.f;
      }
    }
#pragma unroll
    for (int bb = 0; bb < GB; ++bb) {
      const int i = (b0 + bb) / NJ, j = (b0 + bb) % NJ;
      const int col = n0 + wn + 32 * j + li;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * lg + (v & 3);
        if (MODE == 0 || (row < g.M && col < g.N))
          C[(int64_t)row * g.ldc + col] = fmaf(g.beta, old[bb][v], g.alpha * acc[i][j][v]);
      }
    }
  }
}


// ------------------------------------------------------------------ rank-B update from split planes
//
// C_p = beta C_p + alpha A_p B_p^T for operands that arrive as three bf16 planes (hi, mid, lo of
// the fp32 value), k-blocked ([k / 16][row][16]): the coded update W~_p += eta Dhat_p Xhat_p^T with
// a contraction over the mini-batch only, so the read-modify-write of the output tile weighs as
// much as the six partial products.  128 x 128 tile, four wavefronts of 64 x 64, 16 k per stage.
// A stage of a tile is 4 KB per plane and operand, contiguous in memory and stored to LDS as it
// is (32-byte rows; the 16-byte halves of a row are swapped in every second group of four rows,
// which keeps the 128-bit fragment reads of 8 consecutive lanes on 32 different banks without
// padding): 24 KB per stage, two stages, three workgroups per CU, so that while one workgroup
// reads and writes its output tile two others keep the matrix pipe busy.
// FMT 0: three bf16 planes per operand (hi, mid, lo), six partial products; FMT 1: two fp16
// planes (hi, lo) of the operand divided by 2^E (E per operand, g.exps), three partial products,
// the result multiplied by 2^(E_A + E_B).
template <int MODE, int R, int FMT>
__global__ __launch_bounds__(256, 3) void gemm_planes_kernel(HGemmParams g) {
  constexpr int TB = 128, MI = 2, NJ = 2;
  constexpr int NPL = FMT == 0 ? 3 : 2;            // planes per operand
  constexpr int NG = NPL * (NPL + 1) / 2;          // partial products
  constexpr int PLANE_B = TB * 32, STAGE_B = 2 * NPL * PLANE_B;
  __shared__ __attribute__((aligned(16))) unsigned char lds[2][STAGE_B];

  const int xcd = blockIdx.x & 7;
  const int slot = blockIdx.x >> 3;
  const int tile = xcd * g.tiles_per_xcd + slot;
  if (tile >= g.total_tiles) return;
  const int per_batch = g.tiles_m * g.tiles_n;
  const int p = tile / per_batch;
  const int rem = tile - p * per_batch;
  // Tiles that run at the same time should share operand panels: a panel of 128 rows is 96 KB
  // per 128 k, the workgroups of an XCD run about 96 tiles at once, and its L2 holds 4 MB.  Row
  // by row (16 or more tiles of one row of tiles, then the next row) every B panel comes back
  // only after a whole row's worth of traffic and has left the L2 by then; in blocks of 8 x 8
  // tiles 16 panels serve 64 tiles.
  constexpr int SM = 8, SN = 8;            // tiles per block, along m and n
  int tm, tn;
  if (g.tiles_m % SM == 0 && g.tiles_n % SN == 0) {
    const int blk = rem / (SM * SN), in = rem % (SM * SN), bn = g.tiles_n / SN;
    tm = (blk / bn) * SM + in / SN;
    tn = (blk % bn) * SN + in % SN;
  } else {
    tm = rem / g.tiles_n;
    tn = rem - tm * g.tiles_n;
  }
  const int m0 = tm * TB, n0 = tn * TB;
  float* __restrict__ C = g.C + (int64_t)p * g.sC;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lg = lane >> 5;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;

  // one batch entry of each operand behind a buffer descriptor that starts at the tile's first
  // row; a lane's 16 bytes of a stage are at 16 * tid, planes and stages add uniform offsets
  const char* Ab = (const char*)g.A + ((int64_t)p * g.sA + (int64_t)m0 * 16) * 2;
  const char* Bb = (const char*)g.B + ((int64_t)p * g.sB + (int64_t)n0 * 16) * 2;
  const int64_t extA = 2 * (NPL - 1) * g.planeA + (int64_t)(g.K >> 4) * g.M * 32 - (int64_t)m0 * 32;
  const int64_t extB = 2 * (NPL - 1) * g.planeB + (int64_t)(g.K >> 4) * g.N * 32 - (int64_t)n0 * 32;
  const __amdgpu_buffer_rsrc_t rA = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(Ab), 0, (int)extA, 0x00020000);
  const __amdgpu_buffer_rsrc_t rB = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(Bb), 0, (int)extB, 0x00020000);
  const uint32_t voff = 16u * (uint32_t)tid;
  const uint32_t kbA = (uint32_t)g.M * 32u, kbB = (uint32_t)g.N * 32u;
  const uint32_t plA = (uint32_t)(g.planeA * 2), plB = (uint32_t)(g.planeB * 2);
  const bool okA = MODE == 0 || m0 + (tid >> 1) < g.M;
  const bool okB = MODE == 0 || n0 + (tid >> 1) < g.N;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  struct Set { u32x4 a[NPL], b[NPL]; };
  auto load = [&](Set& st, int c) __attribute__((always_inline)) {
#pragma unroll
    for (int pl = 0; pl < NPL; ++pl) {
      st.a[pl] = okA ? __builtin_amdgcn_raw_buffer_load_b128(rA, voff, (uint32_t)c * kbA + pl * plA, 0) : u32x4{0u, 0u, 0u, 0u};
      st.b[pl] = okB ? __builtin_amdgcn_raw_buffer_load_b128(rB, voff, (uint32_t)c * kbB + pl * plB, 0) : u32x4{0u, 0u, 0u, 0u};
    }
  };
  // LDS positions: a lane stores its 16 bytes of row tid / 2, and reads rows wm (wn) + 32 i + li
  const uint32_t swz_w = ((tid & 1) ^ ((tid >> 3) & 1)) * 16u, swz_r = ((uint32_t)lg ^ ((li >> 2) & 1)) * 16u;
  const uint32_t wr_off = (uint32_t)(tid >> 1) * 32u + swz_w;
  const uint32_t rdA = (uint32_t)(wm + li) * 32u + swz_r, rdB = NPL * PLANE_B + (uint32_t)(wn + li) * 32u + swz_r;
  auto put = [&](const Set& st, int buf, int item) __attribute__((always_inline)) {
    *reinterpret_cast<u32x4*>(lds[buf] + wr_off + item * PLANE_B) = item < NPL ? st.a[item] : st.b[item - NPL];
  };
  union Frag { u32x4 u; bf16x8 v; f16x8 h; };
  auto frag = [&](int buf, uint32_t off) __attribute__((always_inline)) {
    Frag f;
    f.u = *reinterpret_cast<const u32x4*>(lds[buf] + off);
    return f;
  };

  floatx16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nchunks = g.K >> 4;            // a multiple of R (the host checks K % 64 == 0)
  Set st[R];
#pragma unroll
  for (int u = 0; u < R; ++u) load(st[u], u);
#pragma unroll
  for (int it = 0; it < 2 * NPL; ++it) put(st[0], 0, it);
  __syncthreads();

  // stage c: the global loads of stage c + R go into the register set stage c has left (set
  // u = c % R, addressed statically: the loop is unrolled R times), stage c + 1 moves from its
  // set to the other LDS buffer between the groups of matrix instructions, and the six partial
  // products hi*lo, mid*mid, hi*mid, lo*hi, mid*hi, hi*hi (fp16 planes: hi*lo, lo*hi, hi*hi) of
  // stage c are accumulated
  auto stage = [&](Set& ld_set, const Set& nx_set, int c, bool do_load, bool do_next) __attribute__((always_inline)) {
    const int cur = c & 1;
    if (do_load) load(ld_set, c + R);
    Frag fa[MI][NPL], fb[NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int pl = 0; pl < NPL; ++pl) fa[i][pl] = frag(cur, rdA + pl * PLANE_B + i * 1024);
    int grp = 0;
#pragma unroll
    for (int pb = NPL - 1; pb >= 0; --pb) {
#pragma unroll
      for (int j = 0; j < NJ; ++j) fb[j] = frag(cur, rdB + pb * PLANE_B + j * 1024);
#pragma unroll
      for (int pa = NPL - 1 - pb; pa >= 0; --pa) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < NJ; ++j) {
            if constexpr (FMT == 0)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i][pa].v, fb[j].v, acc[i][j], 0, 0, 0);
            else
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i][pa].h, fb[j].h, acc[i][j], 0, 0, 0);
          }
        // the 2 NPL pieces of the next stage are spread over the NG groups of matrix instructions
        if (do_next) {
#pragma unroll
          for (int it = grp * 2 * NPL / NG; it < (grp + 1) * 2 * NPL / NG; ++it) put(nx_set, cur ^ 1, it);
        }
        ++grp;
      }
    }
    __syncthreads();
  };
  // steady state with loads in every iteration: the number of younger loads in flight when a
  // set is needed is then the same each time, and the wait for it leaves them in flight (the
  // load counter is relative: code shared with the last R stages, after which nothing is
  // loaded, would have to wait for everything)
  int c0 = 0;
  for (; c0 + 2 * R <= nchunks; c0 += R) {
#pragma unroll
    for (int u = 0; u < R; ++u) stage(st[u], st[(u + 1) % R], c0 + u, true, true);
  }
#pragma unroll
  for (int u = 0; u < R; ++u) stage(st[u], st[(u + 1) % R], c0 + u, false, u + 1 < R);

  // read-modify-write of the output tile, two 32 x 32 blocks at a time: the 32 old values of a
  // pair are requested before any is used.  The tile is touched once: its loads and stores are
  // marked non-temporal so that they do not push the operand panels out of the L2.
  constexpr int GB = 2;
  int esum = 0;                              // fp16 planes: the product is scaled by 2^(E_A + E_B)
  if constexpr (FMT == 1) esum = g.exps[0] + g.exps[1];
#pragma unroll
  for (int b0 = 0; b0 < MI * NJ; b0 += GB) {
    float old[GB][16];
#pragma unroll
    for (int bb = 0; bb < GB; ++bb) {
      const int i = (b0 + bb) / NJ, j = (b0 + bb) % NJ;
      const int col = n0 + wn + 32 * j + li;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * lg + (v & 3);
        old[bb][v] = (g.beta != 0.f && (MODE == 0 || (row < g.M && col < g.N))) ? __builtin_nontemporal_load(&C[(int64_t)row * g.ldc + col]) : 0.f;
      }
    }
#pragma unroll
    for (int bb = 0; bb < GB; ++bb) {
      const int i = (b0 + bb) / NJ, j = (b0 + bb) % NJ;
      const int col = n0 + wn + 32 * j + li;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * lg + (v & 3);
        if (MODE == 0 || (row < g.M && col < g.N))
          __builtin_nontemporal_store(fmaf(g.beta, old[bb][v], FMT == 1 ? ldexpf(g.alpha * acc[i][j][v], esum) : g.alpha * acc[i][j][v]),
                                      &C[(int64_t)row * g.ldc + col]);
      }
    }
  }
}


// ------------------------------------------------ rank-B update from fp16 planes, B panel resident
//
// The same update C_p = beta C_p + alpha A_p B_p^T from two fp16 planes per operand as
// gemm_planes_kernel<.., FMT 1>, organised around what that kernel's counters showed: per 128 x 128
// tile its matrix instructions, its traffic through the vector memory path (operands to LDS, the
// output tile) and its LDS traffic (operands written and read) each take about 6100 cycles of
// their unit, and they added up instead of overlapping.  Here a workgroup owns 128 columns of one
// batch entry for the whole height of C: the B panel of those columns (K <= 256: 128 KB, both
// planes) is copied to LDS once and only read from then on, a wavefront owns a strip of 32 rows x 128
// columns and takes its A fragments straight from memory (in the k-blocked plane layout the
// 32 x 16 fragment of a plane is one contiguous KB, already in the lane order the matrix
// instruction wants), so the loop over k has no LDS write and no barrier, every wavefront runs on
// its own, and per 128 x 128 of output the vector memory path carries a third less and the LDS
// half as much.  Products are accumulated in the order hi*lo, lo*hi, hi*hi per 16 k, as there.
template <int NW, int R>
__global__ __launch_bounds__(64 * NW, 1) void planes_sweep_kernel(HGemmParams g) {
  constexpr int NJ = 4;
  extern __shared__ __attribute__((aligned(16))) unsigned char bpan[];   // [K / 16][plane][128 columns x 32 B]
  const int xcd = blockIdx.x & 7;
  const int slot = blockIdx.x >> 3;
  const int sweep = xcd * g.tiles_per_xcd + slot;
  if (sweep >= g.total_tiles) return;
  const int p = sweep / g.tiles_n;
  const int n0 = (sweep - p * g.tiles_n) * 128;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lg = lane >> 5;
  const int nchunks = g.K >> 4;              // a multiple of R (the host checks)
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

  {
    // stage c, plane pl of the panel is one run of 4 KB in memory (128 columns x 16 k); the halves of
    // its 32-byte rows are swapped in every second group of four rows, which keeps the 128-bit
    // fragment reads of 8 consecutive lanes on 32 different banks
    const char* Bb = (const char*)g.B + ((int64_t)p * g.sB + (int64_t)n0 * 16) * 2;
    const int n_items = nchunks * 2 * 256;   // 16-byte pieces
    for (int base = 0; base < n_items; base += 64 * NW * 4) {
      u32x4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int idx = base + u * 64 * NW + tid;
        const int item = idx >> 8, q = idx & 255;
        v[u] = u32x4{0u, 0u, 0u, 0u};
        if (idx < n_items)
          v[u] = *reinterpret_cast<const u32x4*>(Bb + (int64_t)(item >> 1) * g.N * 32 + (int64_t)(item & 1) * g.planeB * 2 + q * 16);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int idx = base + u * 64 * NW + tid;
        const int item = idx >> 8, q = idx & 255;
        if (idx < n_items)
          *reinterpret_cast<u32x4*>(bpan + item * 4096 + (q >> 1) * 32 + (((q & 1) ^ ((q >> 3) & 1)) * 16)) = v[u];
      }
    }
  }
  __syncthreads();

  union Frag { u32x4 u; f16x8 h; };
  const uint32_t rdB = (uint32_t)li * 32u + ((uint32_t)lg ^ ((li >> 2) & 1)) * 16u;
  auto fragB = [&](int c, int pl, int j) __attribute__((always_inline)) {
    Frag f;
    f.u = *reinterpret_cast<const u32x4*>(bpan + (c * 2 + pl) * 4096 + j * 1024 + rdB);
    return f;
  };
  const char* Ab = (const char*)g.A + (int64_t)p * g.sA * 2;
  const int64_t extA = 2 * g.planeA + (int64_t)nchunks * g.M * 32;
  const __amdgpu_buffer_rsrc_t rA = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(Ab), 0, (int)extA, 0x00020000);
  const uint32_t kbA = (uint32_t)g.M * 32u, plA = (uint32_t)(g.planeA * 2);
  float* __restrict__ Cn = g.C + (int64_t)p * g.sC + n0 + li;
  const int esum = g.exps[0] + g.exps[1];

  for (int s = wave; s < (g.M >> 5); s += NW) {
    const int r0 = s * 32;
    const uint32_t voff = (uint32_t)(r0 + li) * 32u + (uint32_t)lg * 16u;
    Frag fa[R][2];
    auto loadA = [&](int u, int c) __attribute__((always_inline)) {
#pragma unroll
      for (int pl = 0; pl < 2; ++pl) fa[u][pl].u = __builtin_amdgcn_raw_buffer_load_b128(rA, voff, (uint32_t)c * kbA + pl * plA, 0);
    };
#pragma unroll
    for (int u = 0; u < R; ++u) loadA(u, u);
    floatx16 acc[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    auto stage = [&](int u, int c, bool more) __attribute__((always_inline)) {
      Frag fb[NJ];
#pragma unroll
      for (int j = 0; j < NJ; ++j) fb[j] = fragB(c, 1, j);
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[u][0].h, fb[j].h, acc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < NJ; ++j) fb[j] = fragB(c, 0, j);
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[u][1].h, fb[j].h, acc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[u][0].h, fb[j].h, acc[j], 0, 0, 0);
      if (more) loadA(u, c + R);
    };
    int c0 = 0;
    for (; c0 + 2 * R <= nchunks; c0 += R) {
#pragma unroll
      for (int u = 0; u < R; ++u) stage(u, c0 + u, true);
    }
#pragma unroll
    for (int u = 0; u < R; ++u) stage(u, c0 + u, false);

    // read-modify-write of the strip, two 32 x 32 blocks at a time, non-temporal (touched once)
    float* Cs = Cn + (int64_t)(r0 + 4 * lg) * g.ldc;
#pragma unroll
    for (int j0 = 0; j0 < NJ; j0 += 2) {
      float old[2][16];
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          old[jj][v] = g.beta != 0.f ? __builtin_nontemporal_load(Cs + (int64_t)(8 * (v >> 2) + (v & 3)) * g.ldc + 32 * (j0 + jj)) : 0.f;
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          __builtin_nontemporal_store(fmaf(g.beta, old[jj][v], ldexpf(g.alpha * acc[j0 + jj][v], esum)),
                                      Cs + (int64_t)(8 * (v >> 2) + (v & 3)) * g.ldc + 32 * (j0 + jj));
    }
  }
}


gpd_status_t launch_planes(hipStream_t stream, HGemmParams p, int64_t batch) {
  p.tiles_m = (p.M + 127) / 128;
  p.tiles_n = (p.N + 127) / 128;
  // fp16 planes, whole strips and a B panel that fits the LDS: the kernel with the resident panel
  // (measured on the 8192 x 8192 and 8192 x 4096 layers at batch 256: 450 us per launch on average
  // against 488 us; 8 wavefronts with four A stages in flight were as fast as 12 or 16 wavefronts
  // or deeper staging)
  if (p.exps && p.M % 32 == 0 && p.M >= 256 && p.N % 128 == 0 && p.K % 64 == 0 && p.K <= 256) {
    const int64_t sweeps = (int64_t)p.tiles_n * batch;
    if (sweeps > 0x0fffffff) return fail(GPD_E_SHAPE, "gemm: too many tiles");
    p.total_tiles = (int)sweeps;
    p.tiles_per_xcd = (int)((sweeps + 7) / 8);
    const size_t lds = (size_t)(p.K >> 4) * 2 * 4096;      // at most 128 KB
    static bool raised = false;
    if (!raised) {
      GPD_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(planes_sweep_kernel<8, 4>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
      raised = true;
    }
    GPD_LAUNCH((planes_sweep_kernel<8, 4>), dim3((unsigned)(p.tiles_per_xcd * 8)), dim3(512), lds, stream, p);
    GPD_HIP(hipGetLastError());
    return GPD_OK;
  }
  const int64_t total = (int64_t)p.tiles_m * p.tiles_n * batch;
  if (total > 0x0fffffff) return fail(GPD_E_SHAPE, "gemm: too many tiles");
  p.total_tiles = (int)total;
  p.tiles_per_xcd = (int)((total + 7) / 8);
  dim3 grid((unsigned)(p.tiles_per_xcd * 8));
  const bool full = p.M % 128 == 0 && p.N % 128 == 0;
  if (p.exps) {
    if (full) GPD_LAUNCH((gemm_planes_kernel<0, 2, 1>), grid, dim3(256), 0, stream, p);
    else GPD_LAUNCH((gemm_planes_kernel<1, 2, 1>), grid, dim3(256), 0, stream, p);
  } else {
    if (full) GPD_LAUNCH((gemm_planes_kernel<0, 2, 0>), grid, dim3(256), 0, stream, p);
    else GPD_LAUNCH((gemm_planes_kernel<1, 2, 0>), grid, dim3(256), 0, stream, p);
  }
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}

// ---------------------------------------------------------------- bf16 products with very few rows

// C = beta C + alpha A B with M <= 8 rows of fp32 A (row-major) and row-major bf16 B: the
// output layer of a classifier.  A 128-row matrix-core tile would be 1/16 full and its k-loop one
// chain of dependent steps on a few workgroups, so this is a streaming kernel instead: a
// workgroup of 16 wavefronts owns 64 output columns of one batch entry, each wavefront 1/16 of
// k; a lane owns four columns (one 8-byte load per k) of every fourth k of its wavefront, so a
// load instruction covers four rows of B.  A goes through LDS in chunks of kShortKC values of k,
// rounded to bf16 (nearest even) like on the matrix cores; products are summed in fp32, the four
// k-phases of a wavefront by shuffles, the 16 wavefronts through LDS in wavefront order.
constexpr int kShortM = 8, kShortKC = 1024, kShortWaves = 16;

__device__ __forceinline__ float bf16_round(float x) { return __uint_as_float(pack_bf16(x, 0.f) << 16); }

__global__ __launch_bounds__(64 * kShortWaves) void short_m_bf16_kernel(const HGemmParams g) {
  __shared__ float4 As[kShortKC][2];                     // [k][rows 0-3 | rows 4-7], zero beyond M
  __shared__ float part[kShortWaves][kShortM][64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ks = lane >> 4, cg = lane & 15;              // k-phase, group of four columns
  const int n = blockIdx.x * 64 + 4 * cg;
  const int nc = min(n, g.N - 4);                        // groups beyond N re-read the last one (N % 4 == 0)
  const float* __restrict__ A = reinterpret_cast<const float*>(g.A) + (int64_t)blockIdx.y * g.sA;
  const uint16_t* __restrict__ B = reinterpret_cast<const uint16_t*>(g.B) + (int64_t)blockIdx.y * g.sB + nc;
  float acc[kShortM][4];
#pragma unroll
  for (int r = 0; r < kShortM; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;
  constexpr int KW = kShortKC / kShortWaves;             // values of k per wavefront and chunk
  constexpr int U = KW / 4;                              // ... per lane
  for (int kc = 0; kc < g.K; kc += kShortKC) {
    __syncthreads();                                     // the previous chunk has been consumed
    {
      const int k = kc + tid;                            // kShortKC == number of threads
      float a[kShortM];
#pragma unroll
      for (int r = 0; r < kShortM; ++r) a[r] = (r < g.M && k < g.K) ? bf16_round(A[(int64_t)r * g.lda + k]) : 0.f;
      As[tid][0] = make_float4(a[0], a[1], a[2], a[3]);
      As[tid][1] = make_float4(a[4], a[5], a[6], a[7]);
    }
    __syncthreads();
    const int kw = wave * KW + ks;                       // this lane's first k inside the chunk
    uint2 b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int k = min(kc + kw + 4 * u, g.K - 1);       // beyond K: A is zero there
      b[u] = *reinterpret_cast<const uint2*>(B + (int64_t)k * g.ldb);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float4 lo = As[kw + 4 * u][0], hi = As[kw + 4 * u][1];
      const float av[kShortM] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      const float bv[4] = {__uint_as_float(b[u].x << 16), __uint_as_float(b[u].x & 0xffff0000u),
                           __uint_as_float(b[u].y << 16), __uint_as_float(b[u].y & 0xffff0000u)};
#pragma unroll
      for (int r = 0; r < kShortM; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] = fmaf(av[r], bv[c], acc[r][c]);
    }
  }
#pragma unroll
  for (int r = 0; r < kShortM; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float v = acc[r][c];
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      if (ks == 0) part[wave][r][4 * cg + c] = v;
    }
  __syncthreads();
  // thread (r, column) adds the 16 partial sums in wavefront order
  if (tid < kShortM * 64) {
    const int r = tid >> 6, col = blockIdx.x * 64 + lane;
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < kShortWaves; ++w) v += part[w][r][lane];
    if (r < g.M && col < g.N) {
      float* c = g.C + (int64_t)blockIdx.y * g.sC + (int64_t)r * g.ldc + col;
      *c = g.beta != 0.f ? fmaf(g.beta, *c, g.alpha * v) : g.alpha * v;
    }
  }
}

// The same layer's backward product: C = beta C + alpha A^T B with a contraction over at most 8
// rows (A stored K x M fp32, B K x N bf16, both row-major).  Nothing to tile: a thread owns four
// consecutive columns of kShortRows consecutive output rows, reads its K 8-byte pieces of B once
// and K x kShortRows values of A (two 16-byte loads per k, the same for all lanes that share the
// rows), rounds A to bf16 like the matrix cores would, and stores 16 bytes per row; the kernel
// is bound by writing C.
constexpr int kShortRows = 8;

__global__ __launch_bounds__(256) void short_k_bf16_kernel(const HGemmParams g) {
  const int n4 = g.N >> 2;                                   // N % 4 == 0, M % 8 == 0 (host-checked)
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)(g.M / kShortRows) * n4) return;
  const int row = (int)(idx / n4) * kShortRows, n = (int)(idx % n4) * 4;
  const float* __restrict__ A = reinterpret_cast<const float*>(g.A) + (int64_t)blockIdx.y * g.sA + row;
  const uint16_t* __restrict__ B = reinterpret_cast<const uint16_t*>(g.B) + (int64_t)blockIdx.y * g.sB + n;
  float4 a[kShortM][2];
  uint2 b[kShortM];
#pragma unroll
  for (int k = 0; k < kShortM; ++k) {
    const int kc = min(k, g.K - 1);                          // beyond K: re-read the last, weight 0
    a[k][0] = *reinterpret_cast<const float4*>(A + (int64_t)kc * g.lda);
    a[k][1] = *reinterpret_cast<const float4*>(A + (int64_t)kc * g.lda + 4);
    b[k] = k < g.K ? *reinterpret_cast<const uint2*>(B + (int64_t)kc * g.ldb) : make_uint2(0u, 0u);
  }
  float acc[kShortRows][4];
#pragma unroll
  for (int r = 0; r < kShortRows; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;
#pragma unroll
  for (int k = 0; k < kShortM; ++k) {
    const float bv[4] = {__uint_as_float(b[k].x << 16), __uint_as_float(b[k].x & 0xffff0000u),
                         __uint_as_float(b[k].y << 16), __uint_as_float(b[k].y & 0xffff0000u)};
    const float av[kShortRows] = {a[k][0].x, a[k][0].y, a[k][0].z, a[k][0].w, a[k][1].x, a[k][1].y, a[k][1].z, a[k][1].w};
#pragma unroll
    for (int r = 0; r < kShortRows; ++r) {
      const float ar = bf16_round(av[r]);
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[r][c] = fmaf(ar, bv[c], acc[r][c]);
    }
  }
#pragma unroll
  for (int r = 0; r < kShortRows; ++r) {
    float4* c = reinterpret_cast<float4*>(g.C + (int64_t)blockIdx.y * g.sC + (int64_t)(row + r) * g.ldc + n);
    float4 o = make_float4(g.alpha * acc[r][0], g.alpha * acc[r][1], g.alpha * acc[r][2], g.alpha * acc[r][3]);
    if (g.beta != 0.f) {
      const float4 old = *c;
      o = make_float4(fmaf(g.beta, old.x, o.x), fmaf(g.beta, old.y, o.y), fmaf(g.beta, old.z, o.z), fmaf(g.beta, old.w, o.w));
    }
    *c = o;
  }
}

template <int ASRC, int BSRC, int SPLIT>
gpd_status_t launch_bf16_t(hipStream_t stream, HGemmParams p, int64_t batch, bool aligned) {
  // same two workgroup shapes as the fp32 kernel; the large one needs full aligned tiles
  // (the split kernel with a short contraction is dominated by the read-modify-write of its
  // output tile: two small workgroups per CU overlap one's epilogue with the other's products)
  // (the pipelined kernels for full tiles take an even number of stages)
  const bool even = p.K % (2 * hk_of(SPLIT)) == 0;
  const bool large = aligned && even && p.M % 256 == 0 && p.N % 256 == 0 && p.K > 0 &&
                     (int64_t)(p.M / 256) * (p.N / 256) * batch >= 256 && (SPLIT == 1 || p.K >= 1024);
  const int tbm = large ? 256 : 128, tbn = large ? 256 : 128;
  p.tiles_m = (p.M + tbm - 1) / tbm;
  p.tiles_n = (p.N + tbn - 1) / tbn;
  const int64_t total = (int64_t)p.tiles_m * p.tiles_n * batch;
  if (total > 0x0fffffff) return fail(GPD_E_SHAPE, "gemm: too many tiles");
  p.total_tiles = (int)total;
  p.tiles_per_xcd = (int)((total + 7) / 8);
  dim3 grid((unsigned)(p.tiles_per_xcd * 8));
  if (large) {
    // the split kernel keeps three planes of A in registers, and a kernel that streams fp32
    // weights needs two stages of global loads in flight: 8 wavefronts of 128 x 64 (256
    // registers each) instead of 16 of 64 x 64 (128 registers)
    if constexpr (SPLIT == 3 || ASRC == SRC_F32_KC || ASRC == SRC_F32_RC)
      GPD_LAUNCH((gemm_bf16_kernel<ASRC, BSRC, 0, 256, 256, 2, 4, SPLIT>), grid, dim3(512), 0, stream, p);
    else
      GPD_LAUNCH((gemm_bf16_kernel<ASRC, BSRC, 0, 256, 256, 4, 4, SPLIT>), grid, dim3(1024), 0, stream, p);
  } else {
    const bool full = aligned && p.M % 128 == 0 && p.N % 128 == 0 && p.K % hk_of(SPLIT) == 0 && p.K > 0 &&
                      (SPLIT == 1 || even);
    if (full) GPD_LAUNCH((gemm_bf16_kernel<ASRC, BSRC, 0, 128, 128, 2, 2, SPLIT>), grid, dim3(256), 0, stream, p);
    else GPD_LAUNCH((gemm_bf16_kernel<ASRC, BSRC, 1, 128, 128, 2, 2, SPLIT>), grid, dim3(256), 0, stream, p);
  }
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}

template <bool A_KC, bool B_KC, int TBM, int TBN, int WGM, int WGN>
gpd_status_t launch_f32_shape(hipStream_t stream, const GemmParams& p, int mode) {
  dim3 grid((unsigned)(p.tiles_per_xcd * 8)), block(64 * WGM * WGN);
  if (mode == 0) GPD_LAUNCH((gemm_f32_kernel<A_KC, B_KC, 0, TBM, TBN, WGM, WGN>), grid, block, 0, stream, p);
  else if (mode == 1) GPD_LAUNCH((gemm_f32_kernel<A_KC, B_KC, 1, TBM, TBN, WGM, WGN>), grid, block, 0, stream, p);
  else GPD_LAUNCH((gemm_f32_kernel<A_KC, B_KC, 2, TBM, TBN, WGM, WGN>), grid, block, 0, stream, p);
  GPD_HIP(hipGetLastError());
  return GPD_OK;
}

template <bool A_KC, bool B_KC>
gpd_status_t launch_f32(hipStream_t stream, GemmParams p, int64_t batch, bool aligned) {
  // short contractions are dominated by per-tile prologue / epilogue, which only overlap with
  // matrix work when several workgroups share a CU: keep the small shape for them
  const bool large = aligned && p.M % 256 == 0 && p.N % 256 == 0 && p.K % BK == 0 && p.K >= 1024 &&
                     (int64_t)(p.M / 256) * (p.N / 256) * batch >= 256;
  const int tbm = large ? 256 : 128, tbn = large ? 256 : 128;
  p.tiles_m = (p.M + tbm - 1) / tbm;
  p.tiles_n = (p.N + tbn - 1) / tbn;
  const int64_t total = (int64_t)p.tiles_m * p.tiles_n * batch;
  if (total > 0x0fffffff) return fail(GPD_E_SHAPE, "gemm: too many tiles");
  p.total_tiles = (int)total;
  p.tiles_per_xcd = (int)((total + 7) / 8);
  if (large) return launch_f32_shape<A_KC, B_KC, 256, 256, 4, 4>(stream, p, 0);
  const bool full = p.M % 128 == 0 && p.N % 128 == 0 && p.K % BK == 0 && p.K > 0;
  const int mode = !aligned ? 2 : (full ? 0 : 1);
  return launch_f32_shape<A_KC, B_KC, 128, 128, 2, 2>(stream, p, mode);
}

}  // namespace

gpd_status_t launch_gemm(hipStream_t stream, const GemmArgs& a) {
  if (a.M < 0 || a.N < 0 || a.K < 0 || a.batch < 0) return fail(GPD_E_INVALID, "gemm: negative size");
  if (a.M == 0 || a.N == 0 || a.batch == 0) return GPD_OK;
  if (a.M > 0x7fffffff || a.N > 0x7fffffff || a.K > 0x7fffffff)
    return fail(GPD_E_SHAPE, "gemm: dimension above 2^31");
  if ((a.a_bf16 || a.b_bf16) && !a.mfma_bf16)
    return fail(GPD_E_INVALID, "gemm: bf16 operands need the bf16 multiply");
  if (a.split3 && (!a.mfma_bf16 || a.a_bf16 || a.b_bf16))
    return fail(GPD_E_INVALID, "gemm: the three-way split needs fp32 operands and the bf16 multiply");
  const bool planes = a.planeA != 0 || a.planeB != 0;
  if (planes) {
    if (!a.split3 || a.planeA <= 0 || a.planeB <= 0)
      return fail(GPD_E_INVALID, "gemm: split planes need the three-way split, for both operands");
    if (a.K % 64 || a.K < 64 || a.planeA % 8 || a.planeB % 8 || a.strideA % 8 || a.strideB % 8 ||
        (uintptr_t)a.A % 16 || (uintptr_t)a.B % 16)
      return fail(GPD_E_SHAPE, "gemm: split planes need K %% 64 == 0 and 16-byte aligned planes");
    if (a.batch > 1 && (a.strideA < a.M * a.K || a.strideB < a.N * a.K))
      return fail(GPD_E_SHAPE, "gemm: batch stride of a plane operand overlaps");
    if (a.planeA < (a.batch - 1) * a.strideA + a.M * a.K || a.planeB < (a.batch - 1) * a.strideB + a.N * a.K)
      return fail(GPD_E_SHAPE, "gemm: planes overlap");
  }
  if (a.mfma_bf16 && !a.split3 && (a.transB || (a.transA && a.a_bf16)))
    return fail(GPD_E_UNSUPPORTED, "gemm: this operand layout has no bf16 kernel");
  // operand shapes must match what the kernel and its grid assume
  const int64_t a_rows = a.transA ? a.K : a.M, a_cols = a.transA ? a.M : a.K;
  const int64_t b_rows = a.transB ? a.N : a.K, b_cols = a.transB ? a.K : a.N;
  if ((!planes && (a.lda < a_cols || a.ldb < b_cols)) || a.ldc < a.N)
    return fail(GPD_E_SHAPE, "gemm: leading dimension smaller than the row length");
  if (!planes && a.batch > 1 && (a.strideA < (a_rows - 1) * a.lda + a_cols && a.strideA != 0))
    return fail(GPD_E_SHAPE, "gemm: batch stride of A overlaps");
  if (!planes && a.batch > 1 && (a.strideB < (b_rows - 1) * a.ldb + b_cols && a.strideB != 0))
    return fail(GPD_E_SHAPE, "gemm: batch stride of B overlaps");
  if (a.batch > 1 && a.strideC < (a.M - 1) * a.ldc + a.N)
    return fail(GPD_E_SHAPE, "gemm: batch stride of C overlaps");

  if (a.mfma_bf16) {
    HGemmParams h;
    h.A = a.A; h.B = a.B; h.C = a.C;
    h.M = (int)a.M; h.N = (int)a.N; h.K = (int)a.K;
    h.lda = a.lda; h.ldb = a.ldb; h.ldc = a.ldc;
    h.sA = a.strideA; h.sB = a.strideB; h.sC = a.strideC;
    h.alpha = a.alpha; h.beta = a.beta;
    h.planeA = a.planeA; h.planeB = a.planeB;
    h.exps = planes ? a.plane_exps : nullptr;
    const int a_es = a.a_bf16 ? 2 : 4, b_es = a.b_bf16 ? 2 : 4;
    // full tiles are read through buffer instructions with 32-bit offsets: one batch entry of
    // each operand has to stay below 2^31 bytes
    const int64_t ext_a = planes ? 4 * a.planeA + a.M * a.K * 2 : ((a_rows - 1) * a.lda + a_cols) * a_es;
    const int64_t ext_b = planes ? 4 * a.planeB + a.N * a.K * 2 : ((b_rows - 1) * a.ldb + b_cols) * b_es;
    const bool fits = ext_a < 0x7fffffffLL && ext_b < 0x7fffffffLL;
    const bool al = fits && ((uintptr_t)a.A % 16 == 0) && ((uintptr_t)a.B % 16 == 0) &&
                    (a.lda * a_es) % 16 == 0 && (a.ldb * b_es) % 16 == 0 &&
                    (a.strideA * a_es) % 16 == 0 && (a.strideB * b_es) % 16 == 0;
    if (planes) {
      if (!fits) return fail(GPD_E_SHAPE, "gemm: plane operands above 2^31 bytes");
      return launch_planes(stream, h, a.batch);
    }
    if (a.split3) {
      if (!a.transA && !a.transB) return launch_bf16_t<SRC_F32_KC, SRC_F32_RC, 3>(stream, h, a.batch, al);
      if (!a.transA && a.transB) return launch_bf16_t<SRC_F32_KC, SRC_F32_KC, 3>(stream, h, a.batch, al);
      if (a.transA && !a.transB) return launch_bf16_t<SRC_F32_RC, SRC_F32_RC, 3>(stream, h, a.batch, al);
      return launch_bf16_t<SRC_F32_RC, SRC_F32_KC, 3>(stream, h, a.batch, al);
    }
    if (!a.transA && !a.a_bf16 && a.b_bf16 && a.M >= 1 && a.M <= kShortM && a.N >= 4 && a.N % 4 == 0 && a.K > 0 &&
        a.ldb % 4 == 0 && a.strideB % 4 == 0 && (uintptr_t)a.B % 8 == 0 && a.batch > 0 && a.batch <= 65535) {
      static_assert(kShortKC == 64 * kShortWaves, "one thread per value of k of a chunk");
      const dim3 grid((unsigned)((a.N + 63) / 64), (unsigned)a.batch);
      GPD_LAUNCH(short_m_bf16_kernel, grid, dim3(64 * kShortWaves), 0, stream, h);
      GPD_HIP(hipGetLastError());
      return GPD_OK;
    }
    if (a.transA && !a.a_bf16 && a.b_bf16 && a.K >= 1 && a.K <= kShortM && a.M > 0 && a.M % kShortRows == 0 &&
        a.N > 0 && a.N % 4 == 0 && a.lda % 4 == 0 && a.strideA % 4 == 0 && (uintptr_t)a.A % 16 == 0 &&
        a.ldb % 4 == 0 && a.strideB % 4 == 0 && (uintptr_t)a.B % 8 == 0 && a.ldc % 4 == 0 && a.strideC % 4 == 0 &&
        (uintptr_t)a.C % 16 == 0 && a.batch > 0 && a.batch <= 65535 &&
        (a.M / kShortRows) * (a.N / 4) < 0x7fffffffLL * 256) {
      const dim3 grid((unsigned)(((a.M / kShortRows) * (a.N / 4) + 255) / 256), (unsigned)a.batch);
      GPD_LAUNCH(short_k_bf16_kernel, grid, dim3(256), 0, stream, h);
      GPD_HIP(hipGetLastError());
      return GPD_OK;
    }
    if (!a.transA && !a.a_bf16 && !a.b_bf16) return launch_bf16_t<SRC_F32_KC, SRC_F32_RC, 1>(stream, h, a.batch, al);
    if (!a.transA && !a.a_bf16 && a.b_bf16) return launch_bf16_t<SRC_F32_KC, SRC_BF16_RC, 1>(stream, h, a.batch, al);
    if (!a.transA && a.a_bf16 && a.b_bf16) return launch_bf16_t<SRC_BF16_KC, SRC_BF16_RC, 1>(stream, h, a.batch, al);
    if (!a.transA && a.a_bf16 && !a.b_bf16) return launch_bf16_t<SRC_BF16_KC, SRC_F32_RC, 1>(stream, h, a.batch, al);
    if (a.transA && !a.b_bf16) return launch_bf16_t<SRC_F32_RC, SRC_F32_RC, 1>(stream, h, a.batch, al);
    return launch_bf16_t<SRC_F32_RC, SRC_BF16_RC, 1>(stream, h, a.batch, al);
  }

  GemmParams p;
  p.A = (const float*)a.A; p.B = (const float*)a.B; p.C = a.C;
  p.M = (int)a.M; p.N = (int)a.N; p.K = (int)a.K;
  p.lda = a.lda; p.ldb = a.ldb; p.ldc = a.ldc;
  p.sA = a.strideA; p.sB = a.strideB; p.sC = a.strideC;
  p.batch = a.batch;
  p.alpha = a.alpha; p.beta = a.beta;

  const bool aligned = ((uintptr_t)a.A % 16 == 0) && ((uintptr_t)a.B % 16 == 0) &&
                       a.lda % 4 == 0 && a.ldb % 4 == 0 && a.strideA % 4 == 0 && a.strideB % 4 == 0;
  const bool a_kc = !a.transA, b_kc = a.transB;
  if (a_kc && b_kc) return launch_f32<true, true>(stream, p, a.batch, aligned);
  if (a_kc && !b_kc) return launch_f32<true, false>(stream, p, a.batch, aligned);
  if (!a_kc && b_kc) return launch_f32<false, true>(stream, p, a.batch, aligned);
  return launch_f32<false, false>(stream, p, a.batch, aligned);
}

}  // namespace gpd
