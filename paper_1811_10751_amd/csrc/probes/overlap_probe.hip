// Stand-alone probe: do matrix instructions and full-rate HBM traffic overlap on this chip?
//
// The coded update of a batch-256 layer reads and rewrites W~ (32 x 4096 x 2048 fp32 = 1 GiB)
// and multiplies 412 GFLOP of fp16 planes into it.  Its kernels take about the sum of what the
// traffic and the products take alone, whatever is done to overlap them inside a compute unit;
// this probe reproduces that without any operand traffic or LDS use, so that it can be told apart
// from a property of those kernels.  All kernels walk the same 32 x 4096 x 2048 array in the
// access pattern of the 32 x 32 matrix-core accumulator (lane = column, 16 rows per lane) with
// 12 wavefronts per workgroup, one workgroup per 128-column panel of one matrix, a wavefront per
// strip of 32 rows:
//   traffic only            old values in, scaled values out
//   products only           192 v_mfma_f32_32x32x16_f16 per strip on register data
//   both, one wavefront     old values requested, then the products, then the values written
//   both, roles split       8 wavefronts of a workgroup only move data, 4 (one per SIMD) only multiply
//   two kernels, two streams  the traffic-only and the products-only kernel launched side by side
// Build:  hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops
//         overlap_probe.hip -o overlap_probe        (paper_1811_10751_amd/build.py does it)
// Run:    ./overlap_probe          prints microseconds per launch (10 launches after 3 warm-ups)
//         ./overlap_probe V S      repeats variant V (0 .. 3, in the order above) for S seconds, for reading
//                                  clocks and power beside it (rocm-smi --showclocks --showpower)
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("hip error %s at line %d\n", hipGetErrorString(e_), __LINE__); std::exit(1); } } while (0)

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int NB = 32, M = 4096, N = 2048;   // matrices, rows, columns
constexpr int NW = 12;                       // wavefronts per workgroup
constexpr int NMF = 192;                     // matrix instructions per strip: 16 k-steps x 3 products x 4 blocks

__device__ __forceinline__ float* strip_of(float* C, int sweep, int s, int lane) {
  const int p = sweep / (N / 128), n0 = (sweep % (N / 128)) * 128;
  return C + (size_t)p * M * N + (size_t)(s * 32 + 4 * (lane >> 5)) * N + n0 + (lane & 31);
}
__device__ __forceinline__ size_t elem(int j, int v) { return (size_t)(8 * (v >> 2) + (v & 3)) * N + 32 * j; }

__device__ __forceinline__ void operands(int lane, h8& a, h8 (&b)[4]) {
  for (int k = 0; k < 8; ++k) {
    a[k] = (_Float16)(0.001f * (lane + k));
    for (int j = 0; j < 4; ++j) b[j][k] = (_Float16)(0.002f * (lane - k) + 0.01f * j);
  }
}

// MOVE: read and rewrite the strip; MULT: NMF matrix instructions per strip (they depend on the strip
// number, so nothing can be hoisted out of the loop)
template <bool MOVE, bool MULT>
__global__ __launch_bounds__(64 * NW, 1) void one_wavefront_kernel(float* C, float alpha) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  h8 a, b[4];
  operands(lane, a, b);
  float keep = 0.f;
  for (int s = wave; s < M / 32; s += NW) {
    float* Cs = strip_of(C, blockIdx.x, s, lane);
    a[0] = (_Float16)(float)(s & 15);
    float old[4][16];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) old[j][v] = MOVE ? __builtin_nontemporal_load(Cs + elem(j, v)) : 0.f;
    f16v acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    if (MULT) {
      for (int it = 0; it < NMF / 4; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b[j], acc[j], 0, 0, 0);
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        if (MOVE) __builtin_nontemporal_store(old[j][v] * alpha + acc[j][v], Cs + elem(j, v));
        else keep += acc[j][v];
      }
  }
  if (!MOVE && keep == 123.456f) C[0] = keep;          // (never true: keeps the products alive)
}

__global__ __launch_bounds__(64 * NW, 1) void split_roles_kernel(float* C, float alpha) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (wave < 8) {
    for (int s = wave; s < M / 32; s += 8) {
      float* Cs = strip_of(C, blockIdx.x, s, lane);
      float old[4][16];
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) old[j][v] = __builtin_nontemporal_load(Cs + elem(j, v));
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) __builtin_nontemporal_store(old[j][v] * alpha + 1.f, Cs + elem(j, v));
    }
  } else {
    h8 a, b[4];
    operands(lane, a, b);
    float keep = 0.f;
    for (int s = wave - 8; s < M / 32; s += 4) {
      a[0] = (_Float16)(float)(s & 15);
      f16v acc[4];
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
      for (int it = 0; it < NMF / 4; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b[j], acc[j], 0, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) keep += acc[j][v];
    }
    if (keep == 123.456f) C[0] = keep;
  }
}

int main(int argc, char** argv) {
  const size_t n = (size_t)NB * M * N;
  static_assert(M % 32 == 0 && N % 128 == 0, "whole strips and panels");
  // the largest element index any kernel touches: last matrix, last strip, lane 63, j = 3, v = 15
  const size_t last = (size_t)(NB - 1) * M * N + (size_t)((M / 32 - 1) * 32 + 4 + 8 * 3 + 3) * N + (N - 128) + 31 + 96;
  if (last >= n) { std::printf("extent check failed\n"); return 2; }
  float* C = nullptr;
  CK(hipMalloc(&C, n * sizeof(float)));
  CK(hipMemset(C, 0, n * sizeof(float)));
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  const dim3 grid(NB * (N / 128)), block(64 * NW);
  auto time = [&](const char* name, auto launch) {
    for (int i = 0; i < 3; ++i) launch();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    for (int i = 0; i < 10; ++i) launch();
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    CK(hipGetLastError());
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    std::printf("%-34s %8.1f us\n", name, ms * 100.0);
    std::fflush(stdout);
  };
  if (argc == 3) {
    const int variant = std::atoi(argv[1]);
    const double seconds = std::atof(argv[2]);
    if (variant < 0 || variant > 3 || !(seconds > 0.0) || seconds > 30.0) { std::printf("usage: overlap_probe [variant 0..3 seconds<=30]\n"); return 2; }
    int launches = 0;
    float total_ms = 0.f;
    while (total_ms < seconds * 1e3) {
      CK(hipEventRecord(e0));
      for (int i = 0; i < 50; ++i) {
        if (variant == 0) hipLaunchKernelGGL((one_wavefront_kernel<true, false>), grid, block, 0, 0, C, 0.5f);
        else if (variant == 1) hipLaunchKernelGGL((one_wavefront_kernel<false, true>), grid, block, 0, 0, C, 0.5f);
        else if (variant == 2) hipLaunchKernelGGL((one_wavefront_kernel<true, true>), grid, block, 0, 0, C, 0.5f);
        else hipLaunchKernelGGL(split_roles_kernel, grid, block, 0, 0, C, 0.5f);
      }
      CK(hipEventRecord(e1));
      CK(hipEventSynchronize(e1));
      float ms = 0.f;
      CK(hipEventElapsedTime(&ms, e0, e1));
      total_ms += ms;
      launches += 50;
    }
    CK(hipGetLastError());
    std::printf("variant %d: %d launches, %.1f us each\n", variant, launches, total_ms * 1e3 / launches);
    CK(hipFree(C));
    return 0;
  }
  time("traffic only (2.15 GB)", [&] { hipLaunchKernelGGL((one_wavefront_kernel<true, false>), grid, block, 0, 0, C, 0.5f); });
  time("products only (412 GFLOP)", [&] { hipLaunchKernelGGL((one_wavefront_kernel<false, true>), grid, block, 0, 0, C, 0.5f); });
  time("both, in one wavefront", [&] { hipLaunchKernelGGL((one_wavefront_kernel<true, true>), grid, block, 0, 0, C, 0.5f); });
  time("both, roles split over wavefronts", [&] { hipLaunchKernelGGL(split_roles_kernel, grid, block, 0, 0, C, 0.5f); });
  {
    // the two kernels side by side on two streams (default priority): each launch of one is paired with
    // a launch of the other; the time is that of both streams, from a common start
    hipStream_t s1, s2;
    CK(hipStreamCreate(&s1));
    CK(hipStreamCreate(&s2));
    hipEvent_t start, d1, d2;
    CK(hipEventCreate(&start)); CK(hipEventCreate(&d1)); CK(hipEventCreate(&d2));
    for (int rep = 0; rep < 2; ++rep) {
      CK(hipDeviceSynchronize());
      CK(hipEventRecord(start, 0));
      CK(hipStreamWaitEvent(s1, start, 0));
      CK(hipStreamWaitEvent(s2, start, 0));
      for (int i = 0; i < 10; ++i) {
        hipLaunchKernelGGL((one_wavefront_kernel<true, false>), grid, block, 0, s1, C, 0.5f);
        hipLaunchKernelGGL((one_wavefront_kernel<false, true>), grid, block, 0, s2, C, 0.5f);
      }
      CK(hipEventRecord(d1, s1));
      CK(hipEventRecord(d2, s2));
      CK(hipEventSynchronize(d1));
      CK(hipEventSynchronize(d2));
      float m1 = 0.f, m2 = 0.f;
      CK(hipEventElapsedTime(&m1, start, d1));
      CK(hipEventElapsedTime(&m2, start, d2));
      if (rep == 1)
        std::printf("%-34s %8.1f us  (traffic stream done after %.1f us per pair, products stream after %.1f)\n",
                    "two kernels on two streams", (m1 > m2 ? m1 : m2) * 100.0, m1 * 100.0, m2 * 100.0);
    }
    CK(hipGetLastError());
    CK(hipStreamDestroy(s1));
    CK(hipStreamDestroy(s2));
  }
  CK(hipDeviceSynchronize());
  CK(hipFree(C));
  std::printf("done\n");
  return 0;
}
