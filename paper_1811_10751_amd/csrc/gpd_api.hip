// C ABI of the coded matrix multiplication: gpd_plan / gpd_encode / gpd_worker_products /
// gpd_decode.  Host-side bookkeeping only; every step of the path runs in the kernels of
// gpd_combine.hip, gpd_gemm.hip and gpd_locate.hip.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "gpd_internal.hpp"

namespace gpd {

// ---------------------------------------------------------------- table ring

gpd_status_t TableRing::init(size_t bytes_per_slot) {
  slot_bytes = (bytes_per_slot + 255) / 256 * 256;
  GPD_HIP(hipHostMalloc((void**)&host, slot_bytes * kSlots, hipHostMallocDefault));
  GPD_HIP(hipMalloc((void**)&dev, slot_bytes * kSlots));
  for (int i = 0; i < kSlots; ++i) GPD_HIP(hipEventCreateWithFlags(&ev[i], hipEventDisableTiming));
  GPD_HIP(hipMalloc((void**)&arena, kArenaBytes));
  arena_used = 0;
  GPD_HIP(hipStreamCreateWithFlags(&up, hipStreamNonBlocking));
  GPD_HIP(hipHostMalloc((void**)&report_host, kReportBytes, hipHostMallocDefault));
  return GPD_OK;
}

gpd_status_t TableRing::cached(const std::string& key,
                               const std::function<gpd_status_t(HostCombineTable*)>& build,
                               hipStream_t stream, CombineTable* out, bool args_suffice) {
  auto it = cache.find(key);
  if (it != cache.end()) { *out = it->second; return GPD_OK; }
  HostCombineTable ht;
  gpd_status_t st = build(&ht);
  if (st != GPD_OK) return st;
  const size_t need = ht.bytes();
  if (args_suffice && cache.size() < kHostOnlyEntries) {
    std::vector<char> scratch_host(need);
    CombineTable t = ht.pack(scratch_host.data(), nullptr);
    if (t.k_offsets && t.k_coefs && !t.in_rows) {
      t.in_off = t.out_off = nullptr; t.coef = t.H = nullptr; t.coef64 = t.H64 = nullptr;
      t.node = nullptr; t.pts64 = nullptr;
      *out = t;
      cache.emplace(key, t);
      return GPD_OK;
    }
  }
  if (arena_used + need > kArenaBytes || need > slot_bytes) return upload(ht, stream, out);
  // stage in a pinned ring slot and copy to the arena on the upload stream: the region is written
  // once and never again, so the copy may run while earlier work of `stream` (a long product,
  // say) is still executing; `stream` only waits for the copy's event
  const int sl = next;
  next = (next + 1) % kSlots;
  if (used[sl]) GPD_HIP(hipEventSynchronize(ev[sl]));
  char* h = host + (size_t)sl * slot_bytes;
  char* d = arena + arena_used;
  *out = ht.pack(h, d);
  out->persistent = true;
  GPD_HIP(hipMemcpyAsync(d, h, need, hipMemcpyHostToDevice, up));
  GPD_HIP(hipEventRecord(ev[sl], up));
  GPD_HIP(hipStreamWaitEvent(stream, ev[sl], 0));
  used[sl] = true;
  arena_used += need;
  cache.emplace(key, *out);
  return GPD_OK;
}

void TableRing::destroy() {
  for (int i = 0; i < kSlots; ++i)
    if (ev[i]) { (void)hipEventDestroy(ev[i]); ev[i] = nullptr; }
  if (up) { (void)hipStreamSynchronize(up); (void)hipStreamDestroy(up); up = nullptr; }
  if (host) { (void)hipHostFree(host); host = nullptr; }
  if (report_host) { (void)hipHostFree(report_host); report_host = nullptr; }
  if (dev) { (void)hipFree(dev); dev = nullptr; }
  if (arena) { (void)hipFree(arena); arena = nullptr; }
  cache.clear();
}

gpd_status_t TableRing::upload(const HostCombineTable& t, hipStream_t stream, CombineTable* out) {
  const size_t need = t.bytes();
  if (need > slot_bytes) return fail(GPD_E_INVALID, "table of %zu bytes exceeds slot of %zu", need, slot_bytes);
  const int s = next;
  next = (next + 1) % kSlots;
  if (used[s]) GPD_HIP(hipEventSynchronize(ev[s]));     // the copy that last used this slot is done
  char* h = host + (size_t)s * slot_bytes;
  char* d = dev + (size_t)s * slot_bytes;
  *out = t.pack(h, d);
  GPD_HIP(hipMemcpyAsync(d, h, need, hipMemcpyHostToDevice, stream));
  GPD_HIP(hipEventRecord(ev[s], stream));
  used[s] = true;
  return GPD_OK;
}

// ---------------------------------------------------------------- kernel timing

namespace {
struct TimedLaunch { hipEvent_t start, stop; int tag; };
std::mutex timing_mutex;
std::vector<TimedLaunch> timed;              // launches recorded since the last reset
std::vector<TimedLaunch> spare;              // event pairs ready for re-use
int timing_tag = -1;
constexpr size_t kMaxTimed = 16384;
}  // namespace

bool timing_take(hipEvent_t* start, hipEvent_t* stop) {
  if (timing_tag < 0) return false;          // (unlocked read: the tag is set and cleared by the caller's own thread)
  std::lock_guard<std::mutex> lock(timing_mutex);
  if (timing_tag < 0 || timed.size() >= kMaxTimed) return false;
  TimedLaunch t;
  if (!spare.empty()) {
    t = spare.back();
    spare.pop_back();
  } else if (hipEventCreate(&t.start) != hipSuccess || hipEventCreate(&t.stop) != hipSuccess) {
    return false;
  }
  t.tag = timing_tag;
  timed.push_back(t);
  *start = t.start; *stop = t.stop;
  return true;
}

static size_t max_table_bytes(int nin, int nout, int r) {
  HostCombineTable t;
  t.nin = nin; t.nout = nout; t.r = r;
  return t.bytes();
}

}  // namespace gpd

using namespace gpd;

// ---------------------------------------------------------------- plan object

struct gpd_plan {
  gpd_problem_t prob;
  Code code;
  hipStream_t stream = nullptr;
  int64_t ahA = 0, awA = 0;     // block of A: (N1/m) x (N0/n)
  int64_t ahB = 0, awB = 0;     // block of B: (N0/n) x (Nc/d)
  int64_t ahC = 0, awC = 0;     // block of C: (N1/m) x (Nc/d)
  int64_t sA = 0, sB = 0, sC = 0;   // elements between consecutive nodes' blocks of At, Bt, Ct
  double rho = 0, abs_floor = 0;
  // static tables (device): encode A and encode B for the caller's leading dimensions are
  // built per call because in_off depends on lda/ldb; the coefficient part is fixed.
  TableRing ring;
  int64_t flag_cap = 0, loc_cap = 0;
  size_t workspace_bytes = 0;
};

namespace gpd {

constexpr size_t kHeaderBytes = 512;        // counters[64] + node_err[64]
// Pad between the node blocks of a spread stack.  Measured on MI355X with 2048 x 2048 fp32 blocks
// (16 MiB): against packed blocks a pad of 65 KiB + 1 KiB takes the encode's 16 output streams from
// 5.4 to 6.8 TB/s and the decode's 9 to 16 input streams from 5.3 to 5.7 TB/s.
constexpr int64_t kSpreadPadBytes = 66560;

static int64_t screen_words(int64_t n_codewords) { return (n_codewords + 63) / 64 + 8; }

void decode_workspace_layout(int64_t n_codewords, int64_t* flag_cap, int64_t* loc_cap, size_t* bytes) {
  int64_t cap = std::min<int64_t>(n_codewords, 1 << 18);
  if (cap < 1) cap = 1;
  // one bit per codeword for the screen (plus the words a last, partly idle wavefront writes)
  *flag_cap = screen_words(n_codewords);
  *loc_cap = cap * 8;
  size_t b = kHeaderBytes;
  b += ((size_t)(*flag_cap) * 8 + 255) / 256 * 256;
  b += (size_t)(*loc_cap) * sizeof(gpd_located_t);
  *bytes = (b + 255) / 256 * 256;
}

}  // namespace gpd

extern "C" gpd_status_t gpd_plan(const gpd_problem_t* pr, gpd_plan_t** out) {
  if (!pr || !out) return fail(GPD_E_INVALID, "gpd_plan: null argument");
  *out = nullptr;
  if (pr->N1 < 0 || pr->N0 < 0 || pr->Nc < 0) return fail(GPD_E_INVALID, "negative matrix size");
  if (pr->worker_dtype != GPD_F32 && pr->worker_dtype != GPD_BF16 && pr->worker_dtype != GPD_F32_SPLIT)
    return fail(GPD_E_INVALID, "unknown worker dtype %d", pr->worker_dtype);
  if (pr->subst < GPD_SUB_AUTO || pr->subst > GPD_SUB_V_UM)
    return fail(GPD_E_INVALID, "unknown substitution %d", pr->subst);
  if (!(pr->rho_detect >= 0.0) || !(pr->abs_floor >= 0.0) || !std::isfinite(pr->rho_detect) ||
      !std::isfinite(pr->abs_floor))
    return fail(GPD_E_INVALID, "rho_detect and abs_floor must be finite and >= 0");
  gpd_plan_t* pl = new (std::nothrow) gpd_plan_t();
  if (!pl) return fail(GPD_E_DEVICE, "out of host memory");
  pl->prob = *pr;
  pl->prob.points = nullptr;
  gpd_status_t st = make_code(pr->m, pr->n, pr->d, pr->P, pr->subst, pr->points, &pl->code);
  if (st != GPD_OK) { delete pl; return st; }
  if (pr->N1 % pr->m || pr->N0 % pr->n || pr->Nc % pr->d) {
    delete pl;
    return fail(GPD_E_SHAPE, "m, n, d must divide N1, N0, Nc (%lld %lld %lld by %d %d %d)",
                (long long)pr->N1, (long long)pr->N0, (long long)pr->Nc, pr->m, pr->n, pr->d);
  }
  pl->stream = (hipStream_t)pr->hip_stream;
  pl->ahA = pr->N1 / pr->m; pl->awA = pr->N0 / pr->n;
  pl->ahB = pr->N0 / pr->n; pl->awB = pr->Nc / pr->d;
  pl->ahC = pr->N1 / pr->m; pl->awC = pr->Nc / pr->d;
  if (pr->stack_layout != GPD_LAYOUT_PACKED && pr->stack_layout != GPD_LAYOUT_SPREAD) {
    delete pl;
    return fail(GPD_E_INVALID, "unknown stack layout %d", pr->stack_layout);
  }
  // spread stacks: a pad of kSpreadPadBytes between the blocks (whole 256-byte lines, so every
  // block keeps the alignment of the first)
  {
    const int64_t in_elem = pr->worker_dtype == GPD_BF16 ? 2 : 4;
    const int64_t pad = pr->stack_layout == GPD_LAYOUT_SPREAD ? kSpreadPadBytes : 0;
    pl->sA = pl->ahA * pl->awA + pad / in_elem;
    pl->sB = pl->ahB * pl->awB + pad / in_elem;
    pl->sC = pl->ahC * pl->awC + pad / 4;
  }
  pl->rho = pr->rho_detect > 0 ? pr->rho_detect
                               : (pr->worker_dtype == GPD_BF16 ? 0.125 : 1.0 / 4096.0);
  pl->abs_floor = pr->abs_floor;
  decode_workspace_layout(pl->ahC * pl->awC, &pl->flag_cap, &pl->loc_cap, &pl->workspace_bytes);
  pl->workspace_bytes = std::max(pl->workspace_bytes,
                                 gram_workspace_bytes(pl->ahC * pl->awC, pl->code.P - pl->code.K));

  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
    delete pl;
    return fail(GPD_E_DEVICE, "no HIP device");
  }
  const int mn = pr->m * pr->n, nd = pr->n * pr->d, md = pr->m * pr->d;
  size_t slot = max_table_bytes(mn, pr->P, 0);
  slot = std::max(slot, max_table_bytes(nd, pr->P, 0));
  slot = std::max(slot, max_table_bytes(pr->P, md, pr->P));
  st = pl->ring.init(slot);
  if (st != GPD_OK) { pl->ring.destroy(); delete pl; return st; }
  *out = pl;
  return GPD_OK;
}

extern "C" gpd_status_t gpd_plan_info(const gpd_plan_t* pl, int32_t* K, int32_t* t_max,
                                      size_t* workspace_bytes) {
  if (!pl) return fail(GPD_E_INVALID, "gpd_plan_info: null plan");
  if (K) *K = pl->code.K;
  if (t_max) *t_max = std::max(0, pl->code.P - pl->code.K - 1);
  if (workspace_bytes) *workspace_bytes = pl->workspace_bytes;
  return GPD_OK;
}

extern "C" gpd_status_t gpd_timing_tag(int32_t tag) {
  std::lock_guard<std::mutex> lock(timing_mutex);
  timing_tag = tag < 0 ? -1 : tag;
  return GPD_OK;
}

extern "C" gpd_status_t gpd_timing_collect(int32_t tag, double* total_ms, int32_t* launches) {
  std::lock_guard<std::mutex> lock(timing_mutex);
  double sum = 0.0;
  int n = 0;
  for (const TimedLaunch& t : timed) {
    if (t.tag != tag) continue;
    GPD_HIP(hipEventSynchronize(t.stop));
    float ms = 0.f;
    GPD_HIP(hipEventElapsedTime(&ms, t.start, t.stop));
    sum += ms;
    ++n;
  }
  if (total_ms) *total_ms = sum;
  if (launches) *launches = n;
  return GPD_OK;
}

extern "C" gpd_status_t gpd_timing_reset(void) {
  std::lock_guard<std::mutex> lock(timing_mutex);
  for (const TimedLaunch& t : timed) {
    (void)hipEventSynchronize(t.stop);
    spare.push_back(t);
  }
  timed.clear();
  timing_tag = -1;
  return GPD_OK;
}

extern "C" gpd_status_t gpd_plan_strides(const gpd_plan_t* pl, int64_t* strideA, int64_t* strideB,
                                         int64_t* strideC) {
  if (!pl) return fail(GPD_E_INVALID, "gpd_plan_strides: null plan");
  if (strideA) *strideA = pl->sA;
  if (strideB) *strideB = pl->sB;
  if (strideC) *strideC = pl->sC;
  return GPD_OK;
}

extern "C" gpd_status_t gpd_plan_tables(const gpd_plan_t* pl, double* points, int32_t* eA,
                                        int32_t* eB, int32_t* eC) {
  if (!pl) return fail(GPD_E_INVALID, "gpd_plan_tables: null plan");
  const Code& c = pl->code;
  if (points) std::copy(c.pts.begin(), c.pts.end(), points);
  if (eA) std::copy(c.eA.begin(), c.eA.end(), eA);
  if (eB) std::copy(c.eB.begin(), c.eB.end(), eB);
  if (eC) std::copy(c.eC.begin(), c.eC.end(), eC);
  return GPD_OK;
}

extern "C" void gpd_plan_destroy(gpd_plan_t* pl) {
  if (!pl) return;
  pl->ring.destroy();
  delete pl;
}

// ---------------------------------------------------------------- encode

namespace gpd {

// Table that evaluates sum_blocks b_p^e(block) * block for every node p.
//   grid_r x grid_c blocks of bh x bw inside a matrix with leading dimension ld;
//   exps[grid_r*grid_c]; output stack [P][bh][bw].
HostCombineTable encode_table(const std::vector<double>& pts, const std::vector<int>& exps,
                              int grid_r, int grid_c, int64_t bh, int64_t bw, int64_t ld,
                              int64_t out_stride) {
  if (out_stride == 0) out_stride = bh * bw;
  HostCombineTable t;
  const int P = (int)pts.size();
  t.nin = grid_r * grid_c; t.nout = P; t.r = 0;
  t.in_off.resize(t.nin); t.out_off.resize(P); t.coef.resize((size_t)P * t.nin);
  t.node.assign(t.nin, 0);
  for (int i = 0; i < grid_r; ++i)
    for (int j = 0; j < grid_c; ++j) t.in_off[i * grid_c + j] = (int64_t)i * bh * ld + (int64_t)j * bw;
  for (int p = 0; p < P; ++p) {
    t.out_off[p] = (int64_t)p * out_stride;
    for (int s = 0; s < t.nin; ++s) t.coef[(size_t)p * t.nin + s] = ipow(pts[p], exps[s]);
  }
  return t;
}

// Table that decodes the useful coefficients from the present nodes.
//   inputs: stack [P][bh][bw]; outputs: grid_r x grid_c blocks in a matrix with leading
//   dimension ld, block q <-> exponent useful[q].
gpd_status_t decode_table(const std::vector<double>& pts, int K, const uint8_t* present,
                          bool first_k, bool with_H, const std::vector<int>& useful, int grid_r,
                          int grid_c, int64_t bh, int64_t bw, int64_t ld, int64_t in_stride,
                          HostCombineTable* t, int* n_present) {
  const int P = (int)pts.size();
  std::vector<int> S;
  for (int p = 0; p < P; ++p)
    if (!present || present[p]) S.push_back(p);
  if (n_present) *n_present = (int)S.size();
  std::vector<double> D, H;
  gpd_status_t st = decode_matrices(pts, S, K, useful, first_k, &D, with_H ? &H : nullptr);
  if (st != GPD_OK) return st;
  const int ns = (int)S.size();
  // nodes whose column of D is zero everywhere need not be read unless the screen needs them
  std::vector<int> keep;
  for (int s = 0; s < ns; ++s) {
    bool nz = with_H;
    for (size_t u = 0; u < useful.size() && !nz; ++u) nz = D[u * ns + s] != 0.0;
    if (nz) keep.push_back(s);
  }
  t->nin = (int)keep.size(); t->nout = (int)useful.size(); t->r = with_H ? ns - K : 0;
  t->in_off.resize(t->nin); t->node.resize(t->nin);
  t->out_off.resize(t->nout);
  t->coef.resize((size_t)t->nout * t->nin);
  t->H.resize((size_t)t->r * t->nin);
  if (with_H) t->pts.resize(t->nin);
  for (int c = 0; c < t->nin; ++c) {
    t->node[c] = S[keep[c]];
    if (with_H) t->pts[c] = pts[S[keep[c]]];
    t->in_off[c] = (int64_t)S[keep[c]] * in_stride;
    for (int u = 0; u < t->nout; ++u) t->coef[(size_t)u * t->nin + c] = D[(size_t)u * ns + keep[c]];
    for (int i = 0; i < t->r; ++i) t->H[(size_t)i * t->nin + c] = H[(size_t)i * ns + keep[c]];
  }
  for (int i = 0; i < grid_r; ++i)
    for (int j = 0; j < grid_c; ++j) t->out_off[i * grid_c + j] = (int64_t)i * bh * ld + (int64_t)j * bw;
  return GPD_OK;
}

}  // namespace gpd

extern "C" gpd_status_t gpd_encode(const gpd_plan_t* plc, const float* A, int64_t lda,
                                   const float* B, int64_t ldb, void* At, void* Bt) {
  gpd_plan_t* pl = const_cast<gpd_plan_t*>(plc);
  if (!pl) return fail(GPD_E_INVALID, "gpd_encode: null plan");
  // a pair is skipped when both of its pointers are NULL or when it has no elements
  const bool emptyA = pl->prob.N1 == 0 || pl->prob.N0 == 0;
  const bool emptyB = pl->prob.N0 == 0 || pl->prob.Nc == 0;
  if (!emptyA && (A == nullptr) != (At == nullptr))
    return fail(GPD_E_INVALID, "gpd_encode: A and At must be given together");
  if (!emptyB && (B == nullptr) != (Bt == nullptr))
    return fail(GPD_E_INVALID, "gpd_encode: B and Bt must be given together");
  if (emptyA) A = nullptr;
  if (emptyB) B = nullptr;
  const Code& c = pl->code;
  const bool bf16 = pl->prob.worker_dtype == GPD_BF16;
  ScreenArgs none;
  if (A) {
    if (lda < pl->prob.N0) return fail(GPD_E_SHAPE, "lda smaller than N0");
    CombineTable t;
    std::string key("encA");
    key_add(&key, lda);
    gpd_status_t st = pl->ring.cached(key, [&](HostCombineTable* ht) {
      *ht = encode_table(c.pts, c.eA, c.m, c.n, pl->ahA, pl->awA, lda, pl->sA);
      return GPD_OK;
    }, pl->stream, &t, true);
    if (st != GPD_OK) return st;
    // (A and B were last touched a whole product ago: streaming loads; At and Bt are the next
    // kernel's operands: ordinary stores, which measured faster for the step as a whole)
    st = launch_combine(pl->stream, t, A, lda, At, pl->awA, bf16, pl->ahA, pl->awA, none, 0, Epilogue(),
                        PlaneScale(), kStreamLoads);
    if (st != GPD_OK) return st;
  }
  if (B) {
    if (ldb < pl->prob.Nc) return fail(GPD_E_SHAPE, "ldb smaller than Nc");
    CombineTable t;
    std::string key("encB");
    key_add(&key, ldb);
    gpd_status_t st = pl->ring.cached(key, [&](HostCombineTable* ht) {
      *ht = encode_table(c.pts, c.eB, c.n, c.d, pl->ahB, pl->awB, ldb, pl->sB);
      return GPD_OK;
    }, pl->stream, &t, true);
    if (st != GPD_OK) return st;
    st = launch_combine(pl->stream, t, B, ldb, Bt, pl->awB, bf16, pl->ahB, pl->awB, none, 0, Epilogue(),
                        PlaneScale(), kStreamLoads);
    if (st != GPD_OK) return st;
  }
  return GPD_OK;
}

// ---------------------------------------------------------------- worker products

extern "C" gpd_status_t gpd_worker_products(const gpd_plan_t* pl, const void* At, const void* Bt,
                                            float* Ct) {
  if (!pl) return fail(GPD_E_INVALID, "gpd_worker_products: null plan");
  if (pl->ahC == 0 || pl->awC == 0) return GPD_OK;                    // no output elements
  if (!Ct || (pl->awA > 0 && (!At || !Bt)))
    return fail(GPD_E_INVALID, "gpd_worker_products: null argument");
  GemmArgs g;
  g.A = At; g.B = Bt; g.C = Ct;
  g.M = pl->ahA; g.K = pl->awA; g.N = pl->awB;
  g.lda = pl->awA; g.ldb = pl->awB; g.ldc = pl->awC;
  g.strideA = pl->sA; g.strideB = pl->sB; g.strideC = pl->sC;
  g.batch = pl->code.P;
  const bool bf16 = pl->prob.worker_dtype == GPD_BF16;
  g.a_bf16 = g.b_bf16 = bf16;
  g.split3 = pl->prob.worker_dtype == GPD_F32_SPLIT;
  g.mfma_bf16 = bf16 || g.split3;
  return launch_gemm(pl->stream, g);
}

// ---------------------------------------------------------------- decode

namespace gpd {

gpd_status_t run_decode(hipStream_t stream, TableRing* ring, const DecodeJob& job, const float* Zt,
                        const uint8_t* present, int mode, int correct, float* out, int64_t ld_out,
                        void* workspace, size_t workspace_bytes, gpd_report_t* report) {
  const bool empty = job.bh == 0 || job.bw == 0;
  if (!empty && (!Zt || !out)) return fail(GPD_E_INVALID, "decode: null buffer");
  if (mode != GPD_DEC_FIRST_K && mode != GPD_DEC_LSQ_ALL) return fail(GPD_E_INVALID, "decode: bad mode");
  // with block limits (zero-padded ragged edges) the caller of run_decode vouches for ld_out
  if (job.out_cols.empty() && ld_out < job.grid_c * job.bw)
    return fail(GPD_E_SHAPE, "decode: output leading dimension too small");
  if (correct == GPD_CORRECT_NODES)
    return run_decode_nodes(stream, ring, job, Zt, present, mode, out, ld_out, workspace,
                            workspace_bytes, report);
  if (correct != GPD_CORRECT_NONE && correct != GPD_CORRECT_ELEMENTS && correct != GPD_CORRECT_ELEMENTS_L1)
    return fail(GPD_E_INVALID, "decode: unknown correct_errors %d", correct);
  const bool corr = correct != 0;
  if (corr) {
    if (!workspace || workspace_bytes < job.workspace_bytes || ((uintptr_t)workspace & 255))
      return fail(GPD_E_WORKSPACE, "decode: workspace of %zu aligned bytes needed", job.workspace_bytes);
  }
  const int P = (int)job.pts->size();
  int n_present = 0;
  for (int p = 0; p < P; ++p) n_present += (!present || present[p]) ? 1 : 0;
  if (report) {
    gpd_located_t* keep_ptr = report->located;
    const int64_t keep_cap = report->located_cap;
    std::memset(report, 0, sizeof(*report));
    report->located = keep_ptr; report->located_cap = keep_cap;
    report->n_present = n_present;
  }
  if (n_present < job.K) {
    if (report) report->status = GPD_E_TOO_FEW;
    return fail(GPD_E_TOO_FEW, "%d responses present, %d needed", n_present, job.K);
  }
  if (empty) return GPD_OK;
  const bool first_k = !corr && mode == GPD_DEC_FIRST_K;
  std::string key("dec");
  key_add(&key, job.K); key_add(&key, job.grid_r); key_add(&key, job.grid_c);
  const int64_t in_stride = job.in_stride ? job.in_stride : job.bh * job.bw;
  if (in_stride < job.bh * job.bw) return fail(GPD_E_SHAPE, "decode: node stride smaller than a block");
  key_add(&key, job.bh); key_add(&key, job.bw); key_add(&key, ld_out); key_add(&key, in_stride);
  key_add(&key, first_k); key_add(&key, corr);
  key_add_bytes(&key, job.useful.data(), job.useful.size() * sizeof(int));
  key_add_bytes(&key, job.out_rows.data(), job.out_rows.size() * sizeof(int32_t));
  key_add_bytes(&key, job.out_cols.data(), job.out_cols.size() * sizeof(int32_t));
  for (int p = 0; p < P; ++p) key.push_back((!present || present[p]) ? 1 : 0);
  CombineTable t;
  gpd_status_t st = ring->cached(key, [&](HostCombineTable* ht) {
    gpd_status_t s2 = decode_table(*job.pts, job.K, present, first_k, corr, job.useful, job.grid_r,
                                   job.grid_c, job.bh, job.bw, ld_out, in_stride, ht, nullptr);
    if (s2 != GPD_OK) return s2;
    ht->out_rows = job.out_rows; ht->out_cols = job.out_cols;
    return GPD_OK;
  }, stream, &t, !corr);
  if (report) report->status = st;
  if (st != GPD_OK) return st;

  ScreenArgs sc;
  char* ws = (char*)workspace;
  uint32_t* counters = nullptr;
  int32_t* node_err = nullptr;
  unsigned long long* flag_bits = nullptr;
  int64_t flag_words = 0;
  gpd_located_t* located = nullptr;
  if (corr) {
    counters = (uint32_t*)ws;
    node_err = (int32_t*)(ws + 256);
    // (the map and the list of located entries are laid out for the largest block of the plan or
    // layer; a smaller block uses the front of each)
    flag_bits = (unsigned long long*)(ws + kHeaderBytes);
    flag_words = screen_words(job.bh * job.bw);
    if (flag_words > job.flag_cap)
      return fail(GPD_E_WORKSPACE, "decode: the screen's bit map does not fit the workspace");
    located = (gpd_located_t*)(ws + kHeaderBytes + ((size_t)job.flag_cap * 8 + 255) / 256 * 256);
    st = launch_zero_words(stream, ws, (int)(kHeaderBytes / 4));
    if (st != GPD_OK) return st;
    sc.enabled = true; sc.rho = (float)job.rho; sc.abs_floor = (float)job.abs_floor;
    sc.counters = counters; sc.flag_bits = flag_bits; sc.flag_words = flag_words;
  }
  if (corr && job.epi.kind != 0) return fail(GPD_E_INVALID, "decode: element-wise step with element correction");
  // (the responses were written by the product just before: ordinary loads; the decoded result is
  // read by nothing on the device next: streaming stores)
  st = launch_combine(stream, t, Zt, job.bw, out, ld_out, false, job.bh, job.bw, sc, 0, job.epi, PlaneScale(),
                      kStreamStores);
  if (st != GPD_OK) return st;
  if (corr) {
    LocateArgs la;
    la.t = t; la.in = Zt; la.in_ld = job.bw; la.out = out; la.out_ld = ld_out;
    la.rows = job.bh; la.cols = job.bw; la.rho = job.rho; la.abs_floor = job.abs_floor;
    la.counters = counters; la.flag_bits = flag_bits;
    la.located = located; la.located_cap = job.loc_cap; la.node_err = node_err;
    la.locator = correct == GPD_CORRECT_ELEMENTS_L1 ? 1 : 0;
    st = launch_locate(stream, la);
    if (st != GPD_OK) return st;
  }
  if (!report) return GPD_OK;

  // counters and per-node counts (the workspace's first 512 bytes) come back with one
  // stream-ordered copy into pinned memory; the wait for the stream covers it
  static_assert(kHeaderBytes <= TableRing::kReportBytes, "report staging too small");
  if (corr) GPD_HIP(hipMemcpyAsync(ring->report_host, ws, kHeaderBytes, hipMemcpyDeviceToHost, stream));
  GPD_HIP(hipStreamSynchronize(stream));
  if (corr) {
    uint32_t hc[64];
    int32_t hn[64];
    std::memcpy(hc, ring->report_host, sizeof(hc));
    std::memcpy(hn, ring->report_host + 256, sizeof(hn));
    report->n_screened = hc[0];
    report->n_flagged = hc[2];
    report->n_failed = hc[3];
    report->n_located = hc[4];
    float ratio;
    std::memcpy(&ratio, &hc[1], 4);
    report->max_syndrome_ratio = ratio;
    for (int p = 0; p < GPD_MAX_P; ++p) report->node_err_count[p] = hn[p];
    const int64_t have = std::min<int64_t>(hc[4], job.loc_cap);
    if (have > 0) {
      std::vector<gpd_located_t> tmp((size_t)have);
      GPD_HIP(hipMemcpy(tmp.data(), located, sizeof(gpd_located_t) * have, hipMemcpyDeviceToHost));
      // the caller gets the first located_cap entries in (node, row, column) order: only those
      // need to be put in order (a full sort of several 100 000 entries took longer than the kernels)
      if (report->located && report->located_cap > 0) {
        const int64_t n = std::min<int64_t>(have, report->located_cap);
        std::partial_sort(tmp.begin(), tmp.begin() + n, tmp.end(), [](const gpd_located_t& a, const gpd_located_t& b) {
          if (a.node != b.node) return a.node < b.node;
          if (a.row != b.row) return a.row < b.row;
          return a.col < b.col;
        });
        std::memcpy(report->located, tmp.data(), sizeof(gpd_located_t) * n);
      }
    }
    if (hc[3] > 0) {
      report->status = GPD_E_DECODE_FAIL;
      return fail(GPD_E_DECODE_FAIL, "decoding failure on %u codewords", hc[3]);
    }
  }
  report->status = GPD_OK;
  return GPD_OK;
}

gpd_status_t run_decode_nodes(hipStream_t stream, TableRing* ring, const DecodeJob& job, const float* Zt,
                              const uint8_t* present, int mode, float* out, int64_t ld_out,
                              void* workspace, size_t workspace_bytes, gpd_report_t* report) {
  const int P = (int)job.pts->size();
  const int64_t ncw = job.bh * job.bw;
  gpd_located_t* keep_ptr = report ? report->located : nullptr;
  const int64_t keep_cap = report ? report->located_cap : 0;
  gpd_node_report_t nr;
  gpd_status_t st = run_locate_nodes(stream, ring, *job.pts, job.K, ncw, Zt, present, job.rho,
                                     job.abs_floor, workspace, workspace_bytes, &nr, nullptr, job.in_stride);
  if (report) {
    std::memset(report, 0, sizeof(*report));
    report->located = keep_ptr; report->located_cap = keep_cap;
    report->n_present = nr.n_present;
    report->status = st;
  }
  if (st != GPD_OK && st != GPD_E_DECODE_FAIL) return st;
  const bool failed = st == GPD_E_DECODE_FAIL;
  const std::string why = failed ? std::string(gpd_last_error()) : std::string();
  // nodes found erroneous are left out like stragglers; after a failure all present nodes are used
  uint8_t keep[GPD_MAX_P];
  for (int p = 0; p < P; ++p) keep[p] = ((!present || present[p]) && (failed || !nr.bad[p])) ? 1 : 0;
  st = run_decode(stream, ring, job, Zt, keep, mode, GPD_CORRECT_NONE, out, ld_out, nullptr, 0, nullptr);
  if (st != GPD_OK) { if (report) report->status = st; return st; }
  if (report) {
    const bool detected = failed || nr.n_bad > 0;
    report->n_flagged = detected ? ncw : 0;
    report->n_failed = failed ? ncw : 0;
    report->n_located = failed ? 0 : (int64_t)nr.n_bad * ncw;
    for (int p = 0; p < P; ++p)
      report->node_err_count[p] = (!failed && nr.bad[p]) ? (int32_t)std::min<int64_t>(ncw, 0x7fffffff) : 0;
    report->max_syndrome_ratio = nr.threshold > 0 ? (float)std::sqrt(nr.residual / nr.threshold) : 0.f;
    report->status = failed ? GPD_E_DECODE_FAIL : GPD_OK;
    GPD_HIP(hipStreamSynchronize(stream));
  }
  if (failed) return fail(GPD_E_DECODE_FAIL, "%s", why.c_str());
  return GPD_OK;
}

}  // namespace gpd

extern "C" gpd_status_t gpd_locate_nodes(const gpd_plan_t* plc, const float* Ct, const uint8_t* present,
                                         void* workspace, size_t workspace_bytes,
                                         gpd_node_report_t* report, double* gram) {
  gpd_plan_t* pl = const_cast<gpd_plan_t*>(plc);
  if (!pl || !report) return fail(GPD_E_INVALID, "gpd_locate_nodes: null argument");
  return run_locate_nodes(pl->stream, &pl->ring, pl->code.pts, pl->code.K, pl->ahC * pl->awC, Ct, present,
                          pl->rho, pl->abs_floor, workspace, workspace_bytes, report, gram, pl->sC);
}

extern "C" gpd_status_t gpd_verify_decode(const gpd_plan_t* plc, const float* Ct, const uint8_t* present,
                                          int32_t mode, const uint8_t* bad, const float* C, int64_t ldc,
                                          int32_t n_check, void* workspace, size_t workspace_bytes,
                                          gpd_verify_report_t* report) {
  gpd_plan_t* pl = const_cast<gpd_plan_t*>(plc);
  if (!pl || !report) return fail(GPD_E_INVALID, "gpd_verify_decode: null argument");
  DecodeJob job;
  job.pts = &pl->code.pts; job.K = pl->code.K; job.useful = pl->code.eC;
  job.grid_r = pl->code.m; job.grid_c = pl->code.d;
  job.bh = pl->ahC; job.bw = pl->awC; job.in_stride = pl->sC;
  job.rho = pl->rho; job.abs_floor = pl->abs_floor;
  return run_verify(pl->stream, job, Ct, present, mode, bad, C, ldc, n_check, workspace, workspace_bytes, report);
}

// ---------------------------------------------------------------- decode without a workspace argument

namespace {

// Scratch of gpd_decode_static: the same layout run_decode gives a caller's workspace (counters
// and per-node counts, the screen's bit map, the list of located entries), sized for blocks of up
// to kStaticMaxCodewords codewords and a list of kStaticLocCap entries.  Every GPU the library
// runs on holds its own copy until the process ends.
constexpr int64_t kStaticMaxCodewords = (int64_t)GPD_STATIC_MAX_CODEWORDS;
constexpr int64_t kStaticLocCap = (int64_t)GPD_STATIC_LOCATED_CAP;
constexpr int64_t kStaticFlagWords = (kStaticMaxCodewords + 63) / 64 + 8;
constexpr size_t kStaticScratchBytes =
    gpd::kHeaderBytes + ((size_t)kStaticFlagWords * 8 + 255) / 256 * 256 + (size_t)kStaticLocCap * sizeof(gpd_located_t);

static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];

// The array's address on the current device (the name `scratch` is a host-side stand-in, never
// passed to a kernel): asked for once per device, with that device current, and kept.
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices] = {};

gpd_status_t scratch_of_current_device(void** out) {
  int dev = -1;
  GPD_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(GPD_E_DEVICE, "gpd_decode_static: device index %d", dev);
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* ptr = nullptr;
    GPD_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr || ((uintptr_t)ptr & 255)) return fail(GPD_E_DEVICE, "gpd_decode_static: bad scratch address");
    scratch_ptr[dev] = ptr;
  }
  *out = scratch_ptr[dev];
  return GPD_OK;
}

}  // namespace

extern "C" gpd_status_t gpd_decode_static(const gpd_plan_t* plc, const float* Ct, const uint8_t* present,
                                          int32_t mode, int32_t correct_errors, float* C, int64_t ldc,
                                          gpd_report_t* report) {
  gpd_plan_t* pl = const_cast<gpd_plan_t*>(plc);
  if (!pl) return fail(GPD_E_INVALID, "gpd_decode_static: null plan");
  if (correct_errors != GPD_CORRECT_NONE && correct_errors != GPD_CORRECT_ELEMENTS &&
      correct_errors != GPD_CORRECT_ELEMENTS_L1)
    return fail(GPD_E_UNSUPPORTED, "gpd_decode_static: correct_errors must be GPD_CORRECT_NONE, GPD_CORRECT_ELEMENTS "
                                   "or GPD_CORRECT_ELEMENTS_L1 (the node search needs a caller's workspace)");
  const int64_t ncw = pl->ahC * pl->awC;
  if (ncw > kStaticMaxCodewords)
    return fail(GPD_E_WORKSPACE, "gpd_decode_static: blocks of %lld elements exceed the limit of %lld",
                (long long)ncw, (long long)kStaticMaxCodewords);
  void* ws = nullptr;
  if (correct_errors != GPD_CORRECT_NONE) {
    gpd_status_t st = scratch_of_current_device(&ws);
    if (st != GPD_OK) return st;
  }
  DecodeJob job;
  job.pts = &pl->code.pts; job.K = pl->code.K; job.useful = pl->code.eC;
  job.grid_r = pl->code.m; job.grid_c = pl->code.d;
  job.bh = pl->ahC; job.bw = pl->awC; job.in_stride = pl->sC;
  job.rho = pl->rho; job.abs_floor = pl->abs_floor;
  job.flag_cap = kStaticFlagWords; job.loc_cap = kStaticLocCap; job.workspace_bytes = kStaticScratchBytes;
  return run_decode(pl->stream, &pl->ring, job, Ct, present, mode, correct_errors, C, ldc,
                    ws, ws ? kStaticScratchBytes : 0, report);
}

extern "C" gpd_status_t gpd_decode(const gpd_plan_t* plc, const float* Ct, const uint8_t* present,
                                   int32_t mode, int32_t correct_errors, float* C, int64_t ldc,
                                   void* workspace, size_t workspace_bytes, gpd_report_t* report) {
  gpd_plan_t* pl = const_cast<gpd_plan_t*>(plc);
  if (!pl) return fail(GPD_E_INVALID, "gpd_decode: null plan");
  DecodeJob job;
  job.pts = &pl->code.pts; job.K = pl->code.K; job.useful = pl->code.eC;
  job.grid_r = pl->code.m; job.grid_c = pl->code.d;
  job.bh = pl->ahC; job.bw = pl->awC; job.in_stride = pl->sC;
  job.rho = pl->rho; job.abs_floor = pl->abs_floor;
  job.flag_cap = pl->flag_cap; job.loc_cap = pl->loc_cap; job.workspace_bytes = pl->workspace_bytes;
  return run_decode(pl->stream, &pl->ring, job, Ct, present, mode, correct_errors, C, ldc,
                    workspace, workspace_bytes, report);
}
