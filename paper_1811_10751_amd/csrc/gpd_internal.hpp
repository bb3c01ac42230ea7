// Internal declarations shared by the translation units of libgpd (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#if defined(__HIPCC__)
#include <hip/hip_ext.h>   // launches with per-dispatch events: device translation units only
#endif

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <functional>
#include <map>
#include <string>
#include <vector>

#include "gpd.h"

namespace gpd {

// ---------------------------------------------------------------- errors
void set_error(const char* fmt, ...);
gpd_status_t fail(gpd_status_t st, const char* fmt, ...);

#define GPD_HIP(expr)                                                                      \
  do {                                                                                     \
    hipError_t e__ = (expr);                                                               \
    if (e__ != hipSuccess)                                                                 \
      return ::gpd::fail(GPD_E_DEVICE, "%s: %s (%s:%d)", #expr, hipGetErrorString(e__),    \
                         __FILE__, __LINE__);                                              \
  } while (0)

// ---------------------------------------------------------------- kernel timing (gpd_api.hip)

// While a timing tag is set (gpd_timing_tag), every kernel the library launches carries a pair
// of events of its own (start / stop of that one dispatch, as a profiler sees it), filed under the
// tag; gpd_timing_collect adds up the durations.  Off: a plain launch, no event, no cost.
bool timing_take(hipEvent_t* start, hipEvent_t* stop);

#define GPD_LAUNCH(kernel, grid, block, lds, stream, ...)                                        \
  do {                                                                                           \
    hipEvent_t ts__, te__;                                                                       \
    if (::gpd::timing_take(&ts__, &te__))                                                        \
      hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, ts__, te__, 0, __VA_ARGS__);       \
    else                                                                                         \
      hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                         \
  } while (0)

// ---------------------------------------------------------------- host mathematics (gpd_host.cpp)

// Exponents of one coded product after substitution (Sec. IV, Thm 2).
struct Code {
  int m = 0, n = 0, d = 0, P = 0;
  int eu = 0, ev = 0, ew = 0;          // u = b^eu, v = b^ev, w = b^ew
  int K = 0;                           // 1 + degree of the product polynomial
  std::vector<int> eA, eB, eC;         // [m*n], [n*d], [m*d]
  std::vector<double> pts;             // [P]
};

gpd_status_t substitution(int m, int n, int subst, int* eu, int* ev, int* ew);
gpd_status_t make_points(int P, const double* user, std::vector<double>* out);
gpd_status_t make_code(int m, int n, int d, int P, int subst, const double* points, Code* out);
double ipow(double b, int e);

// Decoding matrices for the present nodes `S` (indices into pts), in fp64:
//   D [useful.size()][S.size()]: rows `useful` of the (pseudo-)inverse of the Vandermonde
//     matrix of the nodes used (first K of S for first_k; all of S for lsq);
//     columns of nodes not used are zero.
//   H [(S.size()-K)][S.size()]: orthonormal parity check of the (|S|, K) code (optional).
gpd_status_t decode_matrices(const std::vector<double>& pts, const std::vector<int>& S, int K,
                             const std::vector<int>& useful, bool first_k,
                             std::vector<double>* D, std::vector<double>* H);

// Orthonormal parity check H [(S.size()-K)][S.size()] of the (|S|, K) code alone.
gpd_status_t parity_check_host(const std::vector<double>& pts, const std::vector<int>& S, int K,
                               std::vector<double>* H);

// Algorithm 1 (Sec. V) for errors that sit on the same nodes in every codeword of a stack,
// run on the aggregate G = sum_c (H z_c)(H z_c)^T (r x r, in the basis of H):
//   step 1: trace(G) <= tau^2 = rho^2 max(energy, n_codewords abs_floor^2) -> no errors;
//   step 2: the smallest node set A (containing `forced`) with trace((I - Pi_A) G) <= tau^2,
//           Pi_A the projector on span(H_A); the smallest residual wins inside one size;
//   step 3: only sets of at most r - 1 nodes are accepted.
// Sets of one size are tried exhaustively while there are at most kNodeSearchBudget of them.
constexpr double kNodeSearchBudget = 4194304.0;
struct NodeSearchResult {
  int status = 0;                      // 0 clean, 1 located, 2 failure
  std::vector<int> bad;                // positions in S, ascending
  bool exhaustive = true;
  double energy = 0, syndrome_energy = 0, residual = 0, threshold = 0;
};
gpd_status_t locate_nodes_host(const std::vector<double>& H, int r, int ns, const std::vector<double>& G,
                               double energy, int64_t n_codewords, double rho, double abs_floor,
                               const std::vector<int>& forced, NodeSearchResult* out);
void fill_node_report(const NodeSearchResult& res, const std::vector<int>& S, gpd_node_report_t* rep);

// ---------------------------------------------------------------- device tables

// One "combine" operation: out_q = sum_s coef[q][s] * in_s over equally shaped blocks.
// The table lives in device memory as
//   int64 in_off[nin]; int64 out_off[nout]; float coef[nout*nin]; float H[r*nin];
//   double coef64[nout*nin]; double H64[r*nin]; int32 node[nin]; double pts64[nin] (decode tables)
//   int32 in_rows[nin], in_cols[nin], out_rows[nout], out_cols[nout]   (only with limits)
// With limits, rows/columns of a block at or beyond its limit read as zero (inputs) or are
// not written (outputs): this is how zero-padded ragged edge blocks are handled.
struct CombineTable {
  int nin = 0, nout = 0, r = 0;
  int off_align = 1;                   // largest of 1, 2, 4 dividing every block offset
  const int64_t* in_off = nullptr;
  const int64_t* out_off = nullptr;
  const float* coef = nullptr;
  const float* H = nullptr;
  const double* coef64 = nullptr;
  const double* H64 = nullptr;
  const int32_t* node = nullptr;
  const double* pts64 = nullptr;       // evaluation points of the inputs (tables with H only)
  const int32_t* in_rows = nullptr;    // all four null when there are no limits
  const int32_t* in_cols = nullptr;
  const int32_t* out_rows = nullptr;
  const int32_t* out_cols = nullptr;
  int limit_align = 4;                 // largest of 1, 2, 4 dividing every column limit
  // Host copies of the small parts, handed to the kernels as kernel arguments (those are always
  // read through the scalar cache, whatever the kernel stores meanwhile): the block offsets
  // (nin, nout <= 64) and, when they fit (nout * nin <= 256 and r * nin <= 256), coef and H.
  bool k_offsets = false, k_coefs = false;
  // the device pointers stay valid for the life of the ring (a table in its arena); false: a
  // staging slot that a later upload of the same ring overwrites, good for the next launches only
  bool persistent = false;
  int64_t k_in_off[64] = {}, k_out_off[64] = {};
  float k_coef[256] = {}, k_H[256] = {};
};

struct HostCombineTable {
  int nin = 0, nout = 0, r = 0;
  std::vector<int64_t> in_off, out_off;
  std::vector<double> coef, H;         // fp64 masters
  std::vector<int32_t> node;
  std::vector<double> pts;             // evaluation point of every input (empty = not needed)
  std::vector<int32_t> in_rows, in_cols, out_rows, out_cols;   // empty = no limits
  size_t bytes() const;
  // serialise into `dst` (host) and return the device-side view relative to `dev_base`
  CombineTable pack(void* dst, const void* dev_base) const;
};

// Ring of pinned staging buffers + device slots for per-call tables.
struct TableRing {
  static constexpr int kSlots = 8;
  size_t slot_bytes = 0;
  char* host = nullptr;                // pinned, kSlots * slot_bytes
  char* dev = nullptr;                 // device, kSlots * slot_bytes
  hipEvent_t ev[kSlots] = {};
  bool used[kSlots] = {};
  int next = 0;
  gpd_status_t init(size_t bytes_per_slot);
  void destroy();
  // uploads `t` asynchronously on `stream`; the returned view stays valid until kSlots
  // further uploads have been made.
  gpd_status_t upload(const HostCombineTable& t, hipStream_t stream, CombineTable* out);

  // Tables that recur (same code, same leading dimension, same erasure pattern) are built and
  // uploaded once and then stay in a device arena: `key` identifies the table, `build` makes
  // it on a miss.  A miss stages the table in a pinned ring slot and copies it on an upload
  // stream of the ring's own (the caller's stream waits for the copy's event), so a caller
  // that wants to capture its calls in a HIP graph has to make each distinct call once before
  // capturing (a captured copy would re-read a recycled slot).
  // When the arena is full the table goes through the ring instead.
  static constexpr size_t kArenaBytes = 1 << 20;
  static constexpr size_t kHostOnlyEntries = 4096;   // tables kept on the host alone, at most (about 3 KB each)
  char* arena = nullptr;
  size_t arena_used = 0;
  hipStream_t up = nullptr;            // uploads into the arena (default priority, non-blocking)
  // pinned landing place for the counters a decode with a host report reads back (one
  // stream-ordered copy; the caller waits for the stream afterwards)
  static constexpr size_t kReportBytes = 512;
  char* report_host = nullptr;
  std::map<std::string, CombineTable> cache;
  // args_suffice: the caller launches only kernels that take this table from their kernel
  // arguments when it fits there (block offsets and coefficients, no block limits); such a table
  // is then kept on the host alone: no copy, no event, nothing for the stream to wait for, and the
  // device pointers of the view are null.
  gpd_status_t cached(const std::string& key, const std::function<gpd_status_t(HostCombineTable*)>& build,
                      hipStream_t stream, CombineTable* out, bool args_suffice = false);
};

// appends the raw bytes of v to a cache key
template <typename T>
inline void key_add(std::string* k, const T& v) { k->append((const char*)&v, sizeof(T)); }
inline void key_add_bytes(std::string* k, const void* p, size_t n) { k->append((const char*)p, n); }

// ---------------------------------------------------------------- kernels (launchers)

struct ScreenArgs {               // soft-error screen fused into the decode pass
  bool enabled = false;
  float rho = 0.f, abs_floor = 0.f;
  uint32_t* counters = nullptr;   // [1] max ratio bits
  // bit map of the codewords passed on, bit row*cols+col of 64-bit words; the kernel writes every
  // word that covers a codeword (and up to 3 words after the last of them)
  unsigned long long* flag_bits = nullptr;
  int64_t flag_words = 0;         // words the map can hold
};

// Element-wise step applied to an fp32 output of launch_combine before it is stored (the
// post-processing steps C1 / C2 of Sec. VII done by the kernel that produces their input):
//   1: v -> 1 / (1 + exp(-v));  2: v -> v * y * (1 - y), y read at the output's own position
//   from a matrix laid out like the output (same leading dimension).
struct Epilogue {
  int kind = 0;
  const float* y = nullptr;
};

// For output kind 3 of launch_combine: where the partial maxima of |input| are (device, amax_n
// float bit patterns, non-finite values left out), how many bits the outputs can exceed the
// inputs by (2^exp_extra >= the largest absolute row sum of the coefficients), and where the
// kernel leaves the exponent E it has scaled the planes by (device).
struct PlaneScale {
  const uint32_t* amax_parts = nullptr;
  int amax_n = 0, exp_extra = 0;
  int32_t* exp_out = nullptr;
};

// out_q[r][c] = sum_s coef[q][s] in_s[r][c]; blocks are rows x cols; fp32 in.  out_kind: 0 fp32,
// 1 bf16, 2 the fp32 value as three bf16 planes (hi, mid, lo) out_plane elements apart, each
// block k-blocked ([cols / 16][rows][16]; cols a multiple of 16, out_ld = cols, no block limits);
// 3 the value divided by 2^E as two fp16 planes (hi, lo), k-blocked likewise (PlaneScale).
gpd_status_t launch_combine(hipStream_t stream, const CombineTable& t, const float* in,
                            int64_t in_ld, void* out, int64_t out_ld, int out_kind,
                            int64_t rows, int64_t cols, const ScreenArgs& screen, int64_t out_plane = 0, const Epilogue& epi = Epilogue(),
                            const PlaneScale& scale = PlaneScale(), int streaming = 0);
// `streaming` (launches that move tens of megabytes only): bit 0 = the inputs are read with
// streaming loads (inputs that no kernel touched recently, such as the matrices an encode reads),
// bit 1 = fp32 outputs are written with streaming stores (outputs nothing on the device reads next,
// such as a decoded result).
constexpr int kStreamLoads = 1, kStreamStores = 2;

struct GemmArgs {
  const void* A = nullptr;        // op(A) is M x K
  const void* B = nullptr;        // op(B) is K x N
  float* C = nullptr;             // M x N fp32
  int64_t M = 0, N = 0, K = 0;
  int64_t lda = 0, ldb = 0, ldc = 0;
  int64_t strideA = 0, strideB = 0, strideC = 0;
  int batch = 1;
  bool transA = false;            // A stored K x M
  bool transB = false;            // B stored N x K
  bool a_bf16 = false, b_bf16 = false;   // element types in memory (fp32 otherwise)
  bool mfma_bf16 = false;         // multiply in bf16 (fp32 inputs are rounded on the way)
  bool split3 = false;            // with mfma_bf16 and fp32 operands: each operand as the sum of three
                                  // bf16 values, six partial products: fp32-level accuracy
  // with split3: the operand is already stored as three bf16 planes (hi, mid, lo), plane stride
  // in elements (0: fp32 operand), each batch entry k-blocked: [K / 16][rows][16] with rows = M
  // (N for B); needs K % 64 == 0, ignores lda / transA (ldb / transB); the batch stride then
  // counts bf16 elements of one plane
  int64_t planeA = 0, planeB = 0;
  // plane operands in the other format: two fp16 planes (hi, lo) of the operand divided by
  // 2^E, E_A and E_B in device memory (read by the kernel: no host synchronisation), three
  // partial products, error below 2^-20 of a product's magnitude
  const int32_t* plane_exps = nullptr;
  float alpha = 1.f, beta = 0.f;  // C = beta*C + alpha*op(A)op(B)
};
gpd_status_t launch_gemm(hipStream_t stream, const GemmArgs& g);

struct LocateArgs {
  CombineTable t;
  const float* in = nullptr; int64_t in_ld = 0;
  float* out = nullptr; int64_t out_ld = 0;
  int64_t rows = 0, cols = 0;
  double rho = 0, abs_floor = 0;
  uint32_t* counters = nullptr;   // see gpd_decode.hip for the layout
  const unsigned long long* flag_bits = nullptr;   // the screen's bit map (see ScreenArgs)
  gpd_located_t* located = nullptr; int64_t located_cap = 0;
  int32_t* node_err = nullptr;    // [GPD_MAX_P]
  int locator = 0;                // 0: Algorithm 1's search (helped by the algebraic locator); 1: L1 relaxation
};
gpd_status_t launch_locate(hipStream_t stream, const LocateArgs& a);

gpd_status_t launch_zero_words(hipStream_t stream, void* p, int n_words);

// ---------------------------------------------------------------- shared host helpers (gpd_api.hip)

// Table that evaluates sum_blocks b_p^e(block) * block for every node p: grid_r x grid_c
// blocks of bh x bw inside a matrix with leading dimension ld; output stack [P][bh][bw].
// out_stride: elements between the output blocks of consecutive nodes (0 = bh * bw, packed).
HostCombineTable encode_table(const std::vector<double>& pts, const std::vector<int>& exps,
                              int grid_r, int grid_c, int64_t bh, int64_t bw, int64_t ld,
                              int64_t out_stride = 0);

// One decode of a stack of P responses [P][bh][bw] into a grid_r x grid_c grid of blocks.
struct DecodeJob {
  const std::vector<double>* pts = nullptr;
  int K = 0;
  std::vector<int> useful;                     // exponent of output block q (row-major grid)
  int grid_r = 0, grid_c = 0;
  int64_t bh = 0, bw = 0;
  int64_t in_stride = 0;                       // elements between the blocks of consecutive nodes (0 = bh * bw)
  double rho = 0, abs_floor = 0;
  int64_t flag_cap = 0, loc_cap = 0;   // words of the screen's bit map, entries of the located list
  size_t workspace_bytes = 0;
  std::vector<int32_t> out_rows, out_cols;     // limits of the output blocks (empty = none)
  Epilogue epi;                                // applied to the decoded values (decodes without
                                               // element-wise correction only)
};
gpd_status_t run_decode(hipStream_t stream, TableRing* ring, const DecodeJob& job, const float* Zt,
                        const uint8_t* present, int mode, int correct, float* out, int64_t ld_out,
                        void* workspace, size_t workspace_bytes, gpd_report_t* report);
void decode_workspace_layout(int64_t n_codewords, int64_t* flag_cap, int64_t* loc_cap, size_t* bytes);

// ---------------------------------------------------------------- node-level faults (gpd_nodes.hip)

// device bytes run_locate_nodes needs for a stack of n_codewords-element blocks and r syndromes
size_t gram_workspace_bytes(int64_t n_codewords, int r);

// Gram pass over the stack Zt [P][n_codewords] (node blocks `stride` elements apart, 0 = packed)
// + host search; waits for the stream.
gpd_status_t run_locate_nodes(hipStream_t stream, TableRing* ring, const std::vector<double>& pts,
                              int K, int64_t n_codewords, const float* Zt, const uint8_t* present,
                              double rho, double abs_floor, void* workspace, size_t workspace_bytes,
                              gpd_node_report_t* rep, double* gram_out = nullptr, int64_t stride = 0);

// Verification step: gathers n_check element codewords of Zt and the matching entries of the
// decoded grid, decodes them again on the host in fp64 and compares (see gpd_verify_decode).
gpd_status_t run_verify(hipStream_t stream, const DecodeJob& job, const float* Zt, const uint8_t* present,
                        int mode, const uint8_t* bad, const float* out, int64_t ld_out, int n_check,
                        void* workspace, size_t workspace_bytes, gpd_verify_report_t* rep);

// decode for correct == GPD_CORRECT_NODES: run_locate_nodes, then run_decode without the nodes
// found erroneous; fills the gpd_report_t as documented for gpd_decode.
gpd_status_t run_decode_nodes(hipStream_t stream, TableRing* ring, const DecodeJob& job, const float* Zt,
                              const uint8_t* present, int mode, float* out, int64_t ld_out,
                              void* workspace, size_t workspace_bytes, gpd_report_t* report);

}  // namespace gpd
