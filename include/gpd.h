/*
 * gpd.h — C ABI of the MI355X (gfx950) Generalized PolyDot coded-computation library.
 *
 * Implements the hot path of "A Unified Coded Deep Neural Network Training Strategy Based
 * on Generalized PolyDot Codes for Matrix Multiplication" (arXiv 1811.10751): encode, the
 * coded products of all P nodes (simulated on one GPU), decode with erasures and
 * soft-error correction, and the coded DNN layer step that keeps the weights encoded.
 *
 * Notation (paper -> here): W -> A (N1 x N0, split into an m x n block grid), X -> B
 * (N0 x Nc, split n x d), S -> C (N1 x Nc, split m x d); b_p, p = 0..P-1, are the distinct
 * evaluation points; K is the recovery threshold = number of coefficients of the product
 * polynomial.
 *
 * Conventions
 *   - Every matrix is row-major with an explicit leading dimension (in elements).
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary host memory owned by the caller.  The library owns only the opaque
 *     plan / layer objects and their small coefficient tables.
 *   - Coded stacks are [P][rows][cols], contiguous unless the plan asks for GPD_LAYOUT_SPREAD;
 *     fp32 unless stated.
 *   - Calls enqueue work on the stream given at plan creation and return without
 *     waiting, except where a host-side report is requested (then the call waits for the
 *     stream before returning).
 *   - Every call returns a gpd_status_t, never throws, never aborts; gpd_last_error()
 *     gives a thread-local message for the last non-OK status.
 *   - A missing GPU or a failed launch is GPD_E_DEVICE; there is no CPU fallback.
 */
#ifndef GPD_H
#define GPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GPD_MAX_P 64          /* largest number of nodes P */
#define GPD_MAX_BLOCKS 64     /* largest m*n, n*d, m*d (blocks combined by one kernel) */

typedef enum {
  GPD_OK = 0,
  GPD_E_INVALID = 1,      /* null pointer, bad enum, m/n/d/P < 1 or above the limits      */
  GPD_E_SHAPE = 2,        /* m does not divide N1, n not N0, d not Nc; or K > P            */
  GPD_E_POINTS = 3,       /* evaluation points not finite or not distinct                  */
  GPD_E_TOO_FEW = 4,      /* fewer than K responses present                                */
  GPD_E_DECODE_FAIL = 5,  /* errors detected that cannot be corrected ("decoding failure",
                             Sec. V Algorithm 1 last step); the output is still written    */
  GPD_E_WORKSPACE = 6,    /* workspace missing, too small or misaligned                    */
  GPD_E_DEVICE = 7,       /* HIP error or no GPU                                           */
  GPD_E_UNSUPPORTED = 8,  /* valid request this build has no kernel for                    */
  GPD_E_VERIFY = 9        /* gpd_verify_decode: the second decoder disagrees                */
} gpd_status_t;

/* How the worker products are multiplied.
 *   GPD_F32:       fp32 operands, fp32 MFMA.
 *   GPD_BF16:      operands stored and multiplied in bf16 (round-to-nearest-even), fp32 accumulation.
 *   GPD_F32_SPLIT: fp32 operands in memory; on the way to the bf16 matrix cores every value is
 *                  written as the sum of three bf16 values and the six partial products of
 *                  weight >= 2^-16 are accumulated in fp32: the error of a product of two
 *                  elements stays below 2^-24, that of one fp32 rounding, at about twice the
 *                  speed of fp32 MFMA.  Values above the bf16 range (3.39e38) overflow. */
typedef enum { GPD_F32 = 0, GPD_BF16 = 1, GPD_F32_SPLIT = 2 } gpd_dtype_t;

/* Substitution that turns the multivariate product polynomial into one variable
 * (Sec. IV proof of Thm 2; appendix on error tolerance, second case):
 *   U_VN: u = v^n, w = v^(mn)   K = mnd + n - 1
 *   V_UM: v = u^m, w = u^(mn)   K = mnd + mn - m
 * AUTO = U_VN for a matmul plan; for a layer, the one with the smaller max(K_f, K_b). */
typedef enum { GPD_SUB_AUTO = 0, GPD_SUB_U_VN = 1, GPD_SUB_V_UM = 2 } gpd_subst_t;

typedef enum {
  GPD_DEC_FIRST_K = 0,    /* interpolate from the first K present nodes, by node index
                             (remark after Thm 2: the master waits for K nodes)            */
  GPD_DEC_LSQ_ALL = 1     /* least squares over every present node                         */
} gpd_decmode_t;

typedef enum {
  GPD_CORRECT_NONE = 0,     /* erasures only                                                  */
  GPD_CORRECT_ELEMENTS = 1, /* Algorithm 1 on every element codeword (errors anywhere)        */
  GPD_CORRECT_NODES = 2,    /* Algorithm 1 once for the whole stack: an erroneous node's whole
                               output is wrong (error models of Sec. III); see gpd_locate_nodes */
  GPD_CORRECT_ELEMENTS_L1 = 3 /* like GPD_CORRECT_ELEMENTS with the search of step 2 replaced by the
                               L1-norm relaxation the remark after Thm 3 names: e* = argmin ||e||_1
                               subject to H e = H z (a linear program, solved exactly by simplex
                               steps per screened codeword; non-finite entries cost nothing), the
                               nodes ranked by |e*|, and the first prefix of that ranking (with the
                               non-finite entries) that meets Algorithm 1's criterion is the support.
                               Polynomial time for any code length, but it locates fewer errors
                               than the search: a codeword whose ranking has no such prefix of at
                               most min(|S| - K - 1, 24) nodes is a decoding failure. */
} gpd_correct_t;

/* How the P blocks of a coded stack (At, Bt, Ct of a matmul plan) lie in memory.
 *   GPD_LAYOUT_PACKED: contiguous [P][rows][cols]: node p's block starts rows * cols elements
 *                      after node p-1's.
 *   GPD_LAYOUT_SPREAD: node p's block starts `stride` elements after node p-1's, with stride =
 *                      rows * cols plus a pad of a few tens of KB chosen by the library
 *                      (gpd_plan_strides): encode and decode read or write all P blocks at the same
 *                      offset at the same time, and blocks a power of two apart put those P
 *                      streams on the same memory channels.  The caller allocates
 *                      (P - 1) * stride + rows * cols elements (P * stride is fine); the pad
 *                      between two blocks is never read or written. */
typedef enum { GPD_LAYOUT_PACKED = 0, GPD_LAYOUT_SPREAD = 1 } gpd_layout_t;

typedef struct gpd_plan gpd_plan_t;
typedef struct gpd_layer gpd_layer_t;

/* ------------------------------------------------------------------ coded matmul */

typedef struct {
  int64_t N1, N0, Nc;       /* A is N1 x N0, B is N0 x Nc                                   */
  int32_t m, n, d;          /* block grids: A m x n, B n x d                                */
  int32_t P;                /* number of nodes / evaluation points, K <= P <= GPD_MAX_P     */
  const double* points;     /* host, P distinct finite reals; NULL = Chebyshev points of the
                               first kind cos((2p+1)pi/(2P))                               */
  int32_t worker_dtype;     /* gpd_dtype_t: type A~_p and B~_p are stored and multiplied in  */
  int32_t subst;            /* gpd_subst_t                                                  */
  double rho_detect;        /* relative detection threshold rho; 0 = default (2^-12 for
                               fp32 workers, 2^-3 for bf16 workers)                        */
  double abs_floor;         /* tau(z) = rho * max(||z||_2, abs_floor)                       */
  void* hip_stream;         /* hipStream_t all work of this plan is enqueued on (0 = null
                               stream)                                                     */
  int32_t stack_layout;     /* gpd_layout_t of At, Bt and Ct                               */
} gpd_problem_t;

/* Code construction (Sec. IV, Thm 2): exponent tables, K, evaluation points, coefficient
 * tables b_p^e (computed in fp64 on the host, stored as fp32 on the device).  Host work
 * plus one small upload.  *out is owned by the library until gpd_plan_destroy. */
gpd_status_t gpd_plan(const gpd_problem_t* problem, gpd_plan_t** out);

/* K = recovery threshold; t_max = P - K - 1 = errors correctable per codeword under the
 * probabilistic model (Thm 3); workspace_bytes = device bytes gpd_decode needs when
 * correct_errors != 0 (0 otherwise is fine).  Any output pointer may be NULL. */
gpd_status_t gpd_plan_info(const gpd_plan_t* plan, int32_t* K, int32_t* t_max,
                           size_t* workspace_bytes);

/* Elements (of the stack's own type) between the blocks of consecutive nodes in At, Bt and Ct:
 * rows * cols for GPD_LAYOUT_PACKED, more for GPD_LAYOUT_SPREAD.  Any pointer may be NULL. */
gpd_status_t gpd_plan_strides(const gpd_plan_t* plan, int64_t* strideA, int64_t* strideB,
                              int64_t* strideC);

/* Copies the P evaluation points (fp64) and the exponents of the blocks of A (m*n, row-major
 * over (i,j)), of B (n*d over (j,k)) and the useful exponents of C (m*d over (i,k)) to host
 * arrays; any pointer may be NULL. */
gpd_status_t gpd_plan_tables(const gpd_plan_t* plan, double* points, int32_t* eA,
                             int32_t* eB, int32_t* eC);

void gpd_plan_destroy(gpd_plan_t* plan);

/* Encode (Sec. IV, equations for W~(u,v) and X~(v,w)):
 *   At[p] = sum_{i,j} b_p^eA(i,j) A_{i,j}      At: device [P][N1/m][N0/n] (node stride: gpd_plan_strides)
 *   Bt[p] = sum_{j,k} b_p^eB(j,k) B_{j,k}      Bt: device [P][N0/n][Nc/d]
 * A, B: device fp32, leading dimensions lda, ldb.  Either pair (A, At) or (B, Bt) may be
 * NULL to skip it.  At/Bt hold fp32 or bf16 (round-to-nearest-even) per worker_dtype. */
gpd_status_t gpd_encode(const gpd_plan_t* plan, const float* A, int64_t lda,
                        const float* B, int64_t ldb, void* At, void* Bt);

/* Worker products (proof of Thm 2: node p multiplies its two coded blocks):
 *   Ct[p] = At[p] * Bt[p]   for all p; Ct: device fp32 [P][N1/m][Nc/d].
 * fp32 operands use fp32 MFMA; bf16 operands use bf16 MFMA with fp32 accumulation. */
gpd_status_t gpd_worker_products(const gpd_plan_t* plan, const void* At, const void* Bt,
                                 float* Ct);

typedef struct { int32_t node, row, col; float magnitude; } gpd_located_t;

/* Host-side decode report.  Before the call the caller sets located (may be NULL) and
 * located_cap; everything else is written by the library. */
typedef struct {
  int32_t status;                      /* gpd_status_t of the decode                         */
  int32_t n_present;                   /* |S|                                                */
  int64_t n_screened;                  /* codewords the fp32 screen passed to the fp64 check  */
  int64_t n_flagged;                   /* codewords with ||Hz|| > tau or a non-finite entry   */
  int64_t n_located;                   /* located (node, row, col) errors in total            */
  int64_t n_failed;                    /* codewords declared "decoding failure"               */
  int32_t node_err_count[GPD_MAX_P];   /* located errors per node                             */
  float max_syndrome_ratio;            /* max over unflagged codewords of ||Hz|| / tau (fp32) */
  int32_t reserved;
  int64_t located_cap;                 /* in: capacity of located[]                           */
  gpd_located_t* located;              /* out: first min(n_located, cap) entries, sorted by
                                          (node, row, col); magnitude = estimated error value,
                                          NaN for a non-finite response                      */
} gpd_report_t;

/* Decode (remark after Thm 2; Sec. V Algorithm 1; appendix "Decoding Methods"):
 * every element position (row, col) of the P blocks of Ct is a received word z of a
 * (|S|, K) real-number MDS code; block (i,k) of C is the coefficient of b^eC(i,k).
 *   present: host uint8[P], non-zero = node responded; NULL = all.  Fewer than K present
 *            -> GPD_E_TOO_FEW, nothing written.
 *   mode:    which present nodes the interpolation uses (see gpd_decmode_t).
 *   correct_errors == GPD_CORRECT_ELEMENTS: all present nodes are used.  Step 1:
 *            ||Hz||_2 <= tau(z) with H an orthonormal parity check of the present nodes;
 *            steps 2-3: smallest support
 *            (at most |S| - K - 1 nodes, smallest least-squares residual inside one size)
 *            whose columns of H explain Hz up to tau(z); then least squares from the
 *            remaining nodes.  Non-finite responses count as located errors.  A codeword
 *            with no such support is a decoding failure: GPD_E_DECODE_FAIL is returned in
 *            the report and its output is the uncorrected least-squares value.
 *            Requires workspace (device, 256-byte aligned, workspace_bytes from
 *            gpd_plan_info).
 *   correct_errors == GPD_CORRECT_NODES: gpd_locate_nodes first (the call waits for the
 *            stream), then the nodes found erroneous are left out like stragglers and the
 *            rest is decoded with `mode`.  In the report n_located = number of bad nodes
 *            times the codewords, node_err_count[p] = codewords for a bad node p, n_flagged
 *            = all codewords if any error was detected, located[] is not written; on
 *            failure (GPD_E_DECODE_FAIL) the output is decoded from all present nodes.
 *   C:       device fp32 N1 x Nc, leading dimension ldc.
 *   report:  host, or NULL.  With a report the call waits for the stream; without one it
 *            is asynchronous and GPD_E_DECODE_FAIL cannot be returned.
 */
gpd_status_t gpd_decode(const gpd_plan_t* plan, const float* Ct, const uint8_t* present,
                        int32_t mode, int32_t correct_errors, float* C, int64_t ldc,
                        void* workspace, size_t workspace_bytes, gpd_report_t* report);

/* gpd_decode for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and
 * same results as gpd_decode, but the scratch memory of the soft-error path (counters, the
 * screen's bit map, the list of located entries) is a fixed array inside the library, about 1.5 MiB
 * on every GPU the library runs on, held until the process ends.  The call allocates no device
 * memory and frees none.
 *   correct_errors: GPD_CORRECT_NONE, GPD_CORRECT_ELEMENTS or GPD_CORRECT_ELEMENTS_L1
 *            (GPD_CORRECT_NODES -> GPD_E_UNSUPPORTED).
 *   limits:  blocks of at most GPD_STATIC_MAX_CODEWORDS elements ((N1/m) * (Nc/d)), else
 *            GPD_E_WORKSPACE and nothing is touched; at most GPD_STATIC_LOCATED_CAP located entries
 *            are listed (n_located still counts all of them).
 *   Every call on one GPU uses that GPU's one array: it keeps the last call's contents (the call
 *   clears what must start at zero itself, with a kernel), and two calls that overlap on one GPU
 *   (different streams or threads) race.  The device that owns the plan's stream must be current.
 * Everything else as for gpd_decode. */
#define GPD_STATIC_MAX_CODEWORDS (1 << 22)
#define GPD_STATIC_LOCATED_CAP (1 << 16)
gpd_status_t gpd_decode_static(const gpd_plan_t* plan, const float* Ct, const uint8_t* present,
                               int32_t mode, int32_t correct_errors, float* C, int64_t ldc,
                               gpd_report_t* report);

/* ------------------------------------------------------------------ node-level faults */

/* Host-side result of a node search. */
typedef struct {
  int32_t status;               /* GPD_OK (no errors, or erroneous nodes located) or
                                   GPD_E_DECODE_FAIL (errors detected, too many to locate)     */
  int32_t n_present;
  int32_t n_bad;                /* number of nodes found erroneous                             */
  int32_t exhaustive;           /* 1 = every node set of each size tried; 0 = some size had more
                                   than 2^22 sets and only the most likely one was tested      */
  uint8_t bad[GPD_MAX_P];       /* 1 = node found erroneous                                    */
  uint8_t wild[GPD_MAX_P];      /* 1 = node held a non-finite value or one of magnitude >= 2^40 */
  double energy;                /* sum over codewords of ||z||^2 (wild values taken as 0)      */
  double syndrome_energy;       /* sum over codewords of ||Hz||^2                              */
  double residual;              /* syndrome energy not explained by the bad nodes              */
  double threshold;             /* tau^2 = rho^2 max(energy, codewords * abs_floor^2)          */
} gpd_node_report_t;

/* Location of erroneous nodes for a whole response stack (Sec. V Algorithm 1 under the error
 * models of Sec. III, where a faulty node's entire output is wrong, so every element codeword
 * has its errors on the same nodes).  One pass over Ct accumulates G = sum_c (H z_c)(H z_c)^T
 * and sum_c ||z_c||^2 on the GPU (fp64 accumulation); the search runs on the host:
 *   step 1: no errors if trace(G) <= tau^2;
 *   step 2: smallest node set A with trace((I - Pi_A) G) <= tau^2, Pi_A the projector on the
 *           span of A's columns of H; inside one size the smallest residual wins;
 *   step 3: at most |S| - K - 1 nodes, else decoding failure.
 * Nodes holding a non-finite value or one of magnitude >= 2^40 are always in A and such
 * values count as zero.  Ct is not modified.  The call waits for the stream.
 *   workspace: device, 256-byte aligned, workspace_bytes from gpd_plan_info.
 * Returns GPD_E_DECODE_FAIL (also in report->status) on failure. */
gpd_status_t gpd_locate_nodes(const gpd_plan_t* plan, const float* Ct, const uint8_t* present,
                              void* workspace, size_t workspace_bytes, gpd_node_report_t* report,
                              double* gram /* host [(|S|-K)^2], basis of gpd_host_parity_check; or NULL */);

/* Host-side result of gpd_verify_decode. */
typedef struct {
  int32_t status;               /* GPD_OK or GPD_E_VERIFY                                      */
  int32_t n_checked;            /* element codewords looked at                                 */
  int32_t n_value_mismatch;     /* of those, how many have a decoded value that disagrees      */
  int32_t locations_agree;      /* 1 = the second node search names exactly the nodes in `bad` */
  uint8_t bad[GPD_MAX_P];       /* nodes the second search found erroneous                     */
  double max_ratio;             /* max |difference| / tolerance over the values compared       */
} gpd_verify_report_t;

/* Verification step for decoding errors (Sec. VII under error model 2; "crosscheck" item of the
 * complexity appendix): n_check pre-decided values of the decoded result (0 = P of them; element
 * t of the block is floor(t * elements / n_check)) are recomputed by a second decoder that shares
 * nothing with gpd_decode's kernels, and compared; the list of nodes found erroneous is compared
 * too.  The second decoder gathers the n_check element codewords and the matching entries of C,
 * and works on the host in fp64: node search on the sampled codewords, then least squares over
 * the present nodes it leaves.  A value disagrees if it differs by more than
 * 2^-20 (a_main + a_check) ||z||, a_* = norm of the decoding row used by either decoder.
 *   present, mode, bad: what the main decode used (bad: host uint8[P] nodes it left out as
 *                       erroneous, or NULL).
 *   C, ldc: the decoded result under test (device).
 * Returns GPD_E_VERIFY (also in report->status) on any disagreement: the caller restores its
 * last checkpoint.  The call waits for the stream.  workspace as for gpd_decode. */
gpd_status_t gpd_verify_decode(const gpd_plan_t* plan, const float* Ct, const uint8_t* present,
                               int32_t mode, const uint8_t* bad, const float* C, int64_t ldc,
                               int32_t n_check, void* workspace, size_t workspace_bytes,
                               gpd_verify_report_t* report);

/* ------------------------------------------------------------------ coded DNN layer */

typedef struct {
  int64_t N_out, N_in, batch;   /* W is N_out x N_in; X is N_in x batch; Delta N_out x batch  */
  int32_t m, n;                 /* W split m x n (rows / cols zero-padded up to multiples)    */
  int32_t d1, d2;               /* X split n x d1 (forward), Delta^T split d2 x m (backward)  */
  int32_t P;
  const double* points;         /* as in gpd_problem_t                                        */
  int32_t worker_dtype;         /* GPD_BF16: forward/backward products in bf16 MFMA; W~ itself,
                                   encode and decode stay fp32.  The update W~_p += eta Dhat Xhat^T
                                   keeps fp32-level accuracy on every layer: fp32 MFMA for GPD_F32
                                   layers; for GPD_F32_SPLIT the three-way bf16 split (see
                                   gpd_dtype_t); for GPD_BF16 each operand, divided by a power of
                                   two taken from the largest finite |Delta| (|X|) of the call, as
                                   the sum of two fp16 values and three partial products (error
                                   below 2^-20 of a product's magnitude; batch a multiple of 64,
                                   else the three-way bf16 split)                              */
  int32_t subst;
  double rho_detect, abs_floor;
  void* hip_stream;
} gpd_layer_desc_t;

typedef enum {
  GPD_STEP_FORWARD = 0,
  GPD_STEP_BACKWARD_UPDATE = 1,
  /* OR-ed into the phase: the master's element-wise step that follows the decode (Sec. VII,
   * steps C1 / C2, logistic activation) is applied by the decode itself:
   *   FORWARD:          out = f(S), f(s) = 1 / (1 + exp(-s))
   *   BACKWARD_UPDATE:  out = C o X o (1 - X)  (Hadamard products): the error Delta of the layer
   *                     below when X, this layer's input, is that layer's logistic output.
   * Same values as gpd_sigmoid_fwd / gpd_sigmoid_bwd applied to the plain output. */
  GPD_STEP_FUSE_SIGMOID = 0x100
} gpd_phase_t;

/* One coded layer (Sec. VII for batch 1, Sec. IX for batch > 1). */
gpd_status_t gpd_layer_create(const gpd_layer_desc_t* desc, gpd_layer_t** out);

/* K_f, K_b: thresholds of the forward / backward product polynomials (Tables I and III give
 * P - K - 1 as the error tolerances); wt_rows x wt_cols: shape of one coded block W~_p;
 * workspace_bytes: device bytes gpd_coded_layer_step needs. */
gpd_status_t gpd_layer_info(const gpd_layer_t* layer, int32_t* Kf, int32_t* Kb,
                            int64_t* wt_rows, int64_t* wt_cols, size_t* workspace_bytes);

/* Initial encoding of W (Sec. VII pre-processing step): Wt device fp32 [P][wt_rows][wt_cols]. */
gpd_status_t gpd_layer_encode_weights(const gpd_layer_t* layer, const float* W, int64_t ldw,
                                      float* Wt);

/* W back from the coded blocks (degree mn-1 polynomial, footnote on regeneration, Sec. VII):
 * least squares over the present nodes (at least mn of them). */
gpd_status_t gpd_layer_decode_weights(const gpd_layer_t* layer, const float* Wt,
                                      const uint8_t* present, float* W, int64_t ldw);

/* One phase of one training iteration of this layer.
 *   FORWARD (step O1):  encode X, S~_p = W~_p X~_p for all p, decode -> out = S = W X,
 *                       device fp32 N_out x batch (pre-activation).
 *   BACKWARD_UPDATE (steps O2, O3): encode Delta^T, C~^T_p = Delta~^T_p W~_p with the
 *                       pre-update W~_p, decode -> out = C = W^T Delta, device fp32
 *                       N_in x batch (before the Hadamard product; NULL skips O2); then
 *                       W~_p <- (1 - decay) W~_p + eta * (sum_i Delta_i a_p^i)(sum_j X_j b_p^j)^T
 *                       in place (Eq. "coded update"; decay = eta * lambda).
 *   X:   device fp32 N_in x batch (ld = batch), the layer input.
 *   Dlt: device fp32 N_out x batch (ld = batch), ignored in FORWARD.
 *   present / correct_errors / report: as in gpd_decode (gpd_correct_t), applied to the P
 *        node outputs.
 *   workspace: device, 256-byte aligned, workspace_bytes from gpd_layer_info.
 */
gpd_status_t gpd_coded_layer_step(gpd_layer_t* layer, int32_t phase, float* Wt,
                                  const float* X, const float* Dlt, float eta, float decay,
                                  float* out, const uint8_t* present, int32_t correct_errors,
                                  void* workspace, size_t workspace_bytes, gpd_report_t* report);

/* Where the per-node intermediates of the last gpd_coded_layer_step live inside the caller's
 * workspace: fp32 stacks [P][rows][cols] at byte_offset.  which: 0 = X~_p (encoded input),
 * 1 = S~_p (forward node outputs, what the all-gather of Sec. VII would carry), 2 = Delta~_p
 * stored (N_out/m) x (batch/d2), 3 = C~_p stored (N_in/n) x (batch/d2) (backward node
 * outputs), 4 = Dhat_p, 5 = Xhat_p (update operands).  For inspection and fault injection.
 * Layers with worker_dtype == GPD_BF16 hold 0 and 2 (the operands of the bf16 products) as bf16
 * stacks of the same shape.
 * Layers with worker_dtype != GPD_F32 and batch % 64 == 0 hold 4 and 5 in another form, as
 * planes P*rows*cols elements apart, every plane [P][cols/16][rows][16] (16 consecutive batch
 * columns of a row contiguous):
 *   GPD_F32_SPLIT: each fp32 value v as three bf16 values hi = bf16(v), mid = bf16(v - hi),
 *                  lo = bf16(v - hi - mid) (round to nearest even);
 *   GPD_BF16:      each value v as two fp16 values of w = v / 2^E: hi = fp16(w), lo = fp16(w - hi);
 *                  which = 6 gives the two exponents (int32 E of Dhat, E of Xhat; rows = 1,
 *                  cols = 2) of the last BACKWARD_UPDATE call, and fails on any other layer.
 * which = 7: the error Delta of this layer as gpd_mlp_step left it: one fp32 matrix (not a stack),
 * rows = N_out padded up to a multiple of m, cols = batch. */
gpd_status_t gpd_layer_workspace_view(const gpd_layer_t* layer, int32_t which, size_t* byte_offset,
                                      int64_t* rows, int64_t* cols);

typedef enum {
  GPD_STACK_WEIGHTS = 0,    /* W~: [P][wt_rows][wt_cols], code of mn coefficients               */
  GPD_STACK_FORWARD = 1,    /* S~: [P][wt_rows][batch/d1], K_f coefficients                     */
  GPD_STACK_BACKWARD = 2    /* C~: [P][wt_cols][batch/d2], K_b coefficients                     */
} gpd_stack_t;

/* gpd_locate_nodes for one of the layer's coded stacks: the stored weights themselves (every
 * element position of the P blocks W~_p is a word of the (P, mn) code, footnote on regeneration,
 * Sec. VII) or the node outputs of the last forward / backward product (the views 1 and 3 of
 * gpd_layer_workspace_view, or any stack of that shape).  The weights are always screened with
 * the fp32 threshold.  workspace: the layer's. */
gpd_status_t gpd_layer_locate_nodes(const gpd_layer_t* layer, int32_t which, const float* stack,
                                    const uint8_t* present, void* workspace, size_t workspace_bytes,
                                    gpd_node_report_t* report, double* gram);

/* Regeneration (Sec. VII): W~_p of every node with bad[p] != 0 is recomputed in place from
 * nodes known to be correct, W~_p = sum_q L_q(b_p) W~_q, where L interpolates the degree mn-1
 * polynomial W~(b): mode GPD_DEC_FIRST_K uses the first mn good nodes by index (the paper's
 * count), GPD_DEC_LSQ_ALL all good nodes.  bad: host uint8[P].  Fewer than mn good nodes ->
 * GPD_E_TOO_FEW.  Asynchronous. */
gpd_status_t gpd_layer_regenerate(const gpd_layer_t* layer, float* Wt, const uint8_t* bad,
                                  int32_t mode);

/* Projection of the stored stack onto the code: every element codeword of W~ is replaced by
 * the nearest word (least squares over the present nodes) that is an exact evaluation of a
 * polynomial with mn coefficients; all P blocks are rewritten in place.  Removes the part of
 * the rounding drift of many coded updates that the decoder would not see anyway and
 * regenerates absent nodes.  Asynchronous. */
gpd_status_t gpd_layer_project(const gpd_layer_t* layer, float* Wt, const uint8_t* present);

/* One whole training iteration of a multi-layer network of coded layers with logistic activations
 * and the L2 loss (Sec. VII: for every layer, first to last, steps O1 and C1; the last layer's error
 * 2 (y - yhat) f'(s) / batch; then for every layer, last to first, steps O2 and O3 in one pass over
 * the coded weights and step C2), for the small-batch path: batch 1, 2, 4 or 8, d1 = d2 = 1, fp32
 * workers, all P nodes present, no error correction, every layer on the same stream, N_in of a
 * layer = N_out of the layer before.  Anything else returns GPD_E_UNSUPPORTED or GPD_E_SHAPE and
 * nothing is launched: the caller then strings gpd_coded_layer_step calls together.
 * What the master does between two coded products (decoding, the element-wise step, the encoding
 * of the next product's operands) is one launch instead of four or five; the arithmetic is that of
 * the per-layer calls, operation for operation, so both leave the same bits in the coded weights.
 *   layers, Wt, acts, workspaces, workspace_bytes: host arrays of n_layers entries.
 *   Wt[l]:    device, the coded weights of layer l, updated in place.
 *   X, Y:     device fp32, N_in(0) x batch inputs and N_out(last) x batch targets.
 *   acts[l]:  device fp32 N_out(l) x batch, written: the output of layer l (acts[last] is the
 *             network output).
 *   workspaces[l]: device, 256-byte aligned, workspace_bytes[l] >= what gpd_layer_info gives.
 * Asynchronous. */
gpd_status_t gpd_mlp_step(gpd_layer_t* const* layers, int32_t n_layers, float* const* Wt,
                          const float* X, const float* Y, float eta, float decay,
                          float* const* acts, void* const* workspaces, const size_t* workspace_bytes);

void gpd_layer_destroy(gpd_layer_t* layer);

/* Element-wise steps C1 / C2 and the last-layer error (Sec. II background; logistic f):
 *   gpd_sigmoid_fwd:  y = 1 / (1 + exp(-s))
 *   gpd_sigmoid_bwd:  delta_prev = c * y * (1 - y)          (g(f(u)) = f'(u))
 *   gpd_l2_delta:     delta = scale * (y - yhat) * yhat * (1 - yhat), scale = 2 / batch
 * All pointers device fp32, count elements, enqueued on hip_stream. */
gpd_status_t gpd_sigmoid_fwd(const float* s, float* y, int64_t count, void* hip_stream);
gpd_status_t gpd_sigmoid_bwd(const float* c, const float* y, float* delta_prev, int64_t count,
                             void* hip_stream);
gpd_status_t gpd_l2_delta(const float* y, const float* yhat, float scale, float* delta,
                          int64_t count, void* hip_stream);

/* The two extra element-wise steps of the sparse autoencoder (Sec. X; lemma on autoencoder
 * backpropagation), y = hidden activations, device fp32 rows x cols (cols = batch):
 *   gpd_row_mean:           rho_hat[i] = (1 / cols) sum_b y[i][b]
 *   gpd_sigmoid_bwd_sparse: delta[i][b] = (c[i][b] - scale * Q(rho_hat[i])) * y (1 - y),
 *                           Q(r) = -rho / r + (1 - rho) / (1 - r); scale = beta / batch makes
 *                           delta the step direction of the loss with the term beta * sum KL.
 * 0 < rho < 1.  Enqueued on hip_stream. */
gpd_status_t gpd_row_mean(const float* y, int64_t rows, int64_t cols, float* mean, void* hip_stream);
gpd_status_t gpd_sigmoid_bwd_sparse(const float* c, const float* y, const float* rho_hat, float rho,
                                    float scale, float* delta, int64_t rows, int64_t cols,
                                    void* hip_stream);

/* ------------------------------------------------------------------ host-only helpers */

/* The code construction of gpd_plan without a GPU (Sec. IV, Thm 2): K and the exponent tables
 * (eA m*n, eB n*d, eC m*d, row-major) and the P evaluation points.  Output pointers may be NULL. */
gpd_status_t gpd_host_code(int32_t m, int32_t n, int32_t d, int32_t P, int32_t subst,
                           const double* points, int32_t* K, int32_t* eA, int32_t* eB, int32_t* eC,
                           double* points_out);

/* The fp64 decoding matrices gpd_decode uploads, without a GPU (appendix on decoding):
 *   D: host [m*d][n_present], rows eC of the inverse (first_k != 0: of the first K present
 *      nodes, other columns zero) or pseudo-inverse (all present nodes) of the Vandermonde matrix;
 *   H: host [(n_present-K)][n_present], orthonormal parity check of the present nodes, or NULL. */
gpd_status_t gpd_host_decode_matrices(int32_t m, int32_t n, int32_t d, int32_t P, int32_t subst,
                                      const double* points, const uint8_t* present, int32_t first_k,
                                      double* D, double* H, int32_t* n_present);

/* Orthonormal parity check H [(n_present-K)][n_present] of the (n_present, K) code on the
 * present nodes (Sec. V, paragraph before Algorithm 1), as the library computes it. */
gpd_status_t gpd_host_parity_check(int32_t P, int32_t K, const double* points,
                                   const uint8_t* present, double* H, int32_t* n_present);

/* The host half of gpd_locate_nodes without a GPU: gram = sum_c (H z_c)(H z_c)^T, row-major
 * [(n_present-K)^2] in the basis of gpd_host_parity_check; forced: host uint8[P] or NULL. */
gpd_status_t gpd_host_locate_nodes(int32_t P, int32_t K, const double* points,
                                   const uint8_t* present, const double* gram, double energy,
                                   int64_t n_codewords, double rho, double abs_floor,
                                   const uint8_t* forced, gpd_node_report_t* report);

/* ------------------------------------------------------------------ misc */

/* Durations of the library's own kernel launches, one by one, for measurements inside a running
 * pipeline: while a tag >= 0 is set, every kernel any entry point launches carries its own pair of
 * HIP events on its stream (start and stop of that one dispatch: nothing is added between two
 * kernels, unlike an event recorded between them) and is filed under the tag; tag < 0 turns the
 * recording off.  gpd_timing_collect waits for the recorded kernels of one tag and returns the sum
 * of their durations in milliseconds and their number; gpd_timing_reset forgets all recordings (at
 * most 16384 launches are kept between two resets; further ones run untimed).  Process-wide. */
gpd_status_t gpd_timing_tag(int32_t tag);
gpd_status_t gpd_timing_collect(int32_t tag, double* total_ms, int32_t* launches);
gpd_status_t gpd_timing_reset(void);

const char* gpd_last_error(void);     /* thread-local, never NULL */
const char* gpd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GPD_H */
