/* slonn.h -- C ABI of the MI355X (gfx950) SLO-NN hot path.
 *
 * The library evaluates a fully-connected network with per-query dynamic node
 * dropout as defined by "SLO-Aware Neural Networks" (arXiv 2204.08400): for every
 * query and every layer that carries a Node Activator, FreeHash codes (Def. 2,
 * Section 3.4) select one bucket in each of L Node Importance tables (Section 3.2,
 * Alg. 1), the ranked node lists found there are merged into the top-k% active set
 * (Fig. 2 steps 3-4, Section 3.3) and only those nodes' weight rows are evaluated;
 * every other node of the layer outputs exactly +0.
 *
 * Conventions
 *   - All tensor arguments are raw pointers.  "device" = HIP device memory on the
 *     current device, "host" = ordinary host memory.  The library never takes
 *     ownership of caller memory; handles (slonn_model, slonn_tables) are owned by
 *     the library and released with the matching *_destroy call.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  The
 *     forward/select calls only enqueue work on it and never synchronise; build,
 *     import and export synchronise (documented per call).
 *   - Every function returns SLONN_OK (0) or a negative slonn_status; nothing throws
 *     or aborts.  slonn_last_error() returns a thread-local description of the last
 *     failure.  Argument validation happens before any device work is enqueued.
 *   - A keep fraction k in (0, 1] becomes a node budget m = min(n, max(1,
 *     floor(k*n + 0.5))) evaluated in double ("rounding to the nearest whole node",
 *     at least one node).  m == n means the layer is computed in full.  Keep fractions
 *     live in device memory and are not validated: values at or below 0 (and NaN) give
 *     m = 1, values above 1 give m = n.
 *   - Matrices are row-major and dense unless a stride is given.
 */
#ifndef SLONN_H
#define SLONN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SLONN_OK = 0,
  SLONN_EINVAL = -1,       /* bad argument (null pointer, bad size, bad enum, ...)        */
  SLONN_ENOMEM = -2,       /* host or device allocation failed / workspace too small      */
  SLONN_EHIP = -3,         /* a HIP runtime call failed                                   */
  SLONN_EUNSUPPORTED = -4, /* valid request the library cannot serve (stated per call)    */
  SLONN_ECAP = -5          /* a budget exceeds list_cap or an output stride               */
} slonn_status;

enum { SLONN_F32 = 0, SLONN_BF16 = 1 };                 /* weight storage type            */
enum { SLONN_ROWS_ARE_NODES = 0, SLONN_ROWS_ARE_INPUTS = 1 };
enum { SLONN_ACT_NONE = 0, SLONN_ACT_RELU = 1, SLONN_ACT_SOFTMAX = 2 };
enum { SLONN_DENSE = 0, SLONN_ELL = 1 };                /* first-layer input format       */

#define SLONN_MAX_K 16      /* bits per key                                               */
#define SLONN_MAX_L 64      /* tables per layer (one wavefront lane per table)            */
#define SLONN_MAX_GRID 16       /* most keep fractions a policy's k grid may hold */
#define SLONN_MAX_BATCH 1048576 /* queries per call, and training inputs per table build   */
#define SLONN_TABLE_BLOB_MAGIC 0x544E4C53u /* "SLNT" */
#define SLONN_TABLE_BLOB_VERSION 1u

typedef struct slonn_model slonn_model;
typedef struct slonn_tables slonn_tables;
typedef struct slonn_policy slonn_policy;
typedef struct slonn_graph slonn_graph;

/* One fully-connected layer y = act(W x + b).  Activations are always fp32.
 * W: device, BORROWED for the lifetime of the model.  ROWS_ARE_NODES: [d_out][d_in],
 * a node's weights are contiguous (required for every layer but the first);
 * ROWS_ARE_INPUTS: [d_in][d_out], only for a first layer fed with SLONN_ELL input.
 * bias: device [d_out], borrowed.
 * K, L > 0 put a Node Activator on the layer: hash_nodes (HOST, [L*K], copied) lists
 * the K*L distinct nodes of this layer whose weights and biases serve as FreeHash
 * functions; entry b*K+j is bit j (little endian) of table b's key.  K = L = 0: the
 * layer is always computed in full.  list_cap bounds the ids stored per bucket when
 * tables are built (>= the largest budget below d_out that will be requested).   */
typedef struct {
  int32_t d_in, d_out;
  int32_t w_dtype;           /* SLONN_F32 | SLONN_BF16                                    */
  int32_t w_layout;          /* SLONN_ROWS_ARE_NODES | SLONN_ROWS_ARE_INPUTS              */
  int32_t act;               /* SLONN_ACT_*  (SOFTMAX only on the last layer)             */
  int32_t K, L;
  int32_t list_cap;
  const void* W;
  const float* bias;
  const int32_t* hash_nodes;
} slonn_layer_desc;

/* A batch of first-layer inputs, device memory, borrowed for the call.
 * SLONN_DENSE: x [B][d0] fp32.  SLONN_ELL: idx/val [B][ell_stride], nnz [B]; row q has
 * nnz[q] <= ell_stride (column, value) pairs, columns distinct and < d0.            */
typedef struct {
  int32_t format;
  const float* x;
  const int32_t* idx;
  const float* val;
  const int32_t* nnz;
  int32_t ell_stride;
} slonn_input;

/* Caller-allocated device outputs of a forward call; any member may be NULL.
 * dense: [B][d_last]; nodes that were not computed hold +0.0f.
 * idx/val/cnt: compact form of the last layer when it carries a Node Activator:
 *   idx[q][t], val[q][t] for t < cnt[q], in selection (priority) order; rows are
 *   `stride` apart.  Ignored (cnt = d_last, idx ascending) when the last layer is
 *   computed in full.
 * argmax: [B] id of the computed node with the largest output (lowest id on ties). */
typedef struct {
  float* dense;
  int32_t* idx;
  float* val;
  int32_t* cnt;
  int32_t stride;
  int32_t* argmax;
} slonn_output;

/* Optional per-layer taps for parity checks: arrays of n_layers device pointers (HOST
 * arrays; each entry may be NULL).  Layers without a Node Activator only fill
 * layer_out.  codes [B][L] uint32; z [B][K*L] fp32 hash projections; active_idx
 * [B][d_out] int32 (selection order) with active_cnt [B]; layer_out [B][d_out].   */
typedef struct {
  uint32_t** codes;
  float** z;
  int32_t** active_idx;
  int32_t** active_cnt;
  float** layer_out;
} slonn_debug_taps;

/* Library / device self-description: fills a short human-readable string.          */
int slonn_version(char* buf, size_t cap);

/* Measurement aid for callers that cannot reach the matrix cores themselves (bench.py): runs a
 * register-only loop of v_mfma_f32_16x16x32_f16 in the order the tile kernels issue them (two
 * workgroups of eight wavefronts per compute unit, a few milliseconds) and reports the rate in
 * TFLOP/s -- what the fp16 matrix cores of this device deliver at the clock they hold under that
 * load, the yardstick beside the published peak.  scratch: DEVICE memory, 4096 bytes per compute
 * unit (written, nothing to read back); tflops: HOST.  Synchronises `stream`.
 * EINVAL: null argument; ENOMEM: scratch too small.                                           */
int slonn_probe_mfma_rate(void* scratch, size_t scratch_bytes, void* stream, double* tflops);

/* Measurement aid: the rate at which compute units read cache-resident rows with 16-byte loads, the
 * bound of the gather kernels wherever the weights sit in L2 (one 1024-thread workgroup per compute
 * unit reads one 2 MiB window over and over).  gbps_all_units: GB/s summed over all compute units
 * busy together; gbps_one_unit: GB/s of one unit with the rest of the device idle (both HOST).
 * scratch: DEVICE memory, 16-byte aligned, 2 MiB + 4096 bytes per compute unit (any contents; the
 * tail is written).  Synchronises `stream`.  EINVAL: null or misaligned argument; ENOMEM: scratch
 * too small.                                                                                    */
int slonn_probe_l_two_read_rate(void* scratch, size_t scratch_bytes, void* stream, double* gbps_all_units,
                                double* gbps_one_unit);

/* Validate and register a network.  Copies the K*L FreeHash rows of each activated
 * layer into library-owned device memory (synchronises the device once).
 * Errors: EINVAL for null/negative sizes, K > SLONN_MAX_K, L > SLONN_MAX_L, K*L >
 * d_out, duplicate or out-of-range hash nodes, d_in mismatch between consecutive
 * layers, SOFTMAX before the last layer; EUNSUPPORTED for ROWS_ARE_INPUTS anywhere
 * but on layer 0 or together with a Node Activator.                                 */
int slonn_model_create(const slonn_layer_desc* layers, int n_layers, slonn_model** out);
int slonn_model_destroy(slonn_model* m);

/* Execution path of slonn_sparse_forward.  The results are the same on every path.
 * SLONN_PATH_LAYERS: one launch sequence per layer (hash projection as a batch-wide
 *   MFMA contraction, select, gathered-row forward); serves every model and size.
 * SLONN_PATH_FUSED: one workgroup carries one query through the whole network with its
 *   activations in LDS, one launch per batch; for models whose layers are small enough
 *   (every weight matrix at most 8 MiB, dense first-layer input, no Node Activator on
 *   the last layer, row lengths a multiple of 16 bytes).  EUNSUPPORTED otherwise.
 *   A second whole-network kernel serves the wide sparse-input models (ELL input, exactly two
 *   layers: a hidden layer of at most 4096 nodes stored input-major without a Node Activator,
 *   then an activated output layer of any width; compact and/or dense output).
 * SLONN_PATH_AUTO (default): FUSED when the model qualifies (for the first kernel: and no
 *   compact output is requested; for the second: and the batch is at most two queries per
 *   compute unit), else LAYERS.                                                      */
enum { SLONN_PATH_AUTO = 0, SLONN_PATH_LAYERS = 1, SLONN_PATH_FUSED = 2 };
int slonn_model_set_path(slonn_model* m, int path);

/* How many batches the caller keeps in flight on this device at a time (calls on n streams, each
 * with its own workspace and outputs).  The whole-network kernels give a query a workgroup of 1024
 * threads while the queries in flight (n times the batch) leave compute units free, and one of 512
 * or 256 threads once they do not, so that several queries share a unit and one's memory waits are
 * the others' work.  A hint: results do not depend on it.  n >= 1 (default 1).
 * EINVAL: null model, n < 1.                                                                    */
int slonn_model_set_batches_in_flight(slonn_model* m, int n);

/* Large batches compute the FreeHash projections on the int8 matrix cores from fixed-point
 * digits of the operands; a projection counts as certain when |z| exceeds `margin` times a
 * rigorous bound on what the fixed-point form loses, every other one is recomputed in fp64.
 * margin >= 1 (default 2).  Results do not depend on it (a huge margin sends every projection
 * through the fp64 recomputation: a diagnostic).  EINVAL: null model, margin < 1 or NaN.      */
int slonn_model_set_hash_margin(slonn_model* m, double margin);

/* Arithmetic of slonn_dense_forward, the all-nodes baseline (Section 3.4, last paragraph).
 * SLONN_DENSE_FP32_MFMA (default): fp32 operands on the fp32 matrix cores.
 * SLONN_DENSE_F16_PARTS: the arithmetic the sparse path uses for large batches of large layers -
 *   rows scaled by powers of two, activations (and fp32 weights) as sums of two fp16 parts (22
 *   significand bits; bf16 weights are one part, exactly), partial products accumulated in fp32 on
 *   the fp16 matrix cores - so that sparse and dense passes can be compared like for like.
 *   Layers or batches that path does not serve (small layers, rows not a multiple of 32 elements, batches
 *   of only a few tiles) stay on the fp32 cores.  Results agree with the default to fp32 rounding.
 * EINVAL: null model, unknown mode.                                                          */
enum { SLONN_DENSE_FP32_MFMA = 0, SLONN_DENSE_F16_PARTS = 1 };
int slonn_model_set_dense_arithmetic(slonn_model* m, int mode);

/* Variant of Section 3.4 ("the hash is free"): the K*L FreeHash projections of a layer are
 * the pre-activations of K*L of its own nodes, so those nodes can always be computed at no
 * further cost, and the Node Activator then need not select them.  on != 0: for every
 * activated layer and every query whose budget m is below the layer's n nodes, the active
 * list is the K*L hash nodes in the order given at model creation, followed by the first
 * max(m - K*L, 0) other nodes in the usual merge order (a hash node met in a ranked list or
 * in the fallback ranking is passed over); active_cnt = max(m, K*L); the outputs of the hash
 * nodes are act(projection).  m == n is unchanged (all nodes, ascending).  The same tables
 * serve both settings.  on == 0 (default): the active set is exactly the m selected nodes.
 * Applies to slonn_select and slonn_sparse_forward on every path.  EINVAL: null model.    */
int slonn_model_set_hash_nodes_always_active(slonn_model* m, int on);

/* Choice of the FreeHash nodes (Section 3.4): the K*L hash nodes of a layer are drawn with
 * probability proportional to the variance of the nodes' activations over the training set of
 * the tables.  Two steps, both before slonn_model_create (hash_nodes is one of its inputs).
 *
 * slonn_activation_variance: A is a device matrix [N][n] (row stride lda >= n, in floats) of
 * one layer's activations over N inputs, e.g. a layer output of slonn_dense_forward.
 * var_out[j] (device, n doubles) = (1/N) sum_i (A[i][j] - mean_j)^2 with mean_j = (1/N) sum_i
 * A[i][j], both sums in fp64 over i ascending per quarter of the rows, the four quarters added
 * in order.  Asynchronous on `stream`.  EINVAL: null pointer, N < 1, n < 1, lda < n.
 *
 * slonn_sample_hash_nodes: host arrays.  variance[n] (negative or non-finite entries count as
 * 0), u[K*L] uniform draws in [0,1) supplied by the caller.  K*L sequential draws without
 * replacement: with P_i the running sum of the remaining variances v_0..v_i in fp64, i
 * ascending, draw j takes the first i with P_i > u[j] * P_{n-1} (the last node if rounding
 * leaves none; from there the next node with v > 0, cyclically, if that one is exhausted) and
 * then sets v_i = 0.  When no variance is left, the lowest node id not drawn yet.
 * hash_nodes_out[j] serves table j / K, bit j % K.  EINVAL: null pointer, K*L < 1, K*L > n.  */
int slonn_activation_variance(const float* A, int64_t N, int n, int64_t lda, double* var_out, void* stream);
int slonn_sample_hash_nodes(const double* variance, int n, int K, int L, const double* u,
                            int32_t* hash_nodes_out);
/* The same draws on the device, so that variance (as slonn_activation_variance leaves it), draws
 * and ids never visit the host: variance [n], u [K*L] and hash_nodes_out [K*L] are DEVICE arrays;
 * asynchronous on `stream`.  Same ids as slonn_sample_hash_nodes, id for id (the running sums are
 * formed in the same order).  EUNSUPPORTED: n above 2^20.  (slonn_model_create takes hash_nodes
 * from the host: copy the K*L ids back once.)                                               */
int slonn_sample_hash_nodes_device(const double* variance, int n, int K, int L, const double* u,
                                   int32_t* hash_nodes_out, void* stream);

/* Online refresh (Section 3.2: the tables can be trained before or after deployment; Section 6:
 * refreshed as the data drifts).  on != 0, set before slonn_build_tables: the tables keep their
 * NodeScore sums on the device (L * 2^K * n doubles per activated layer, plus the whole-set sums),
 * which slonn_tables_refresh needs.  Default off.  EINVAL: null model.                        */
int slonn_model_set_tables_refreshable(slonn_model* m, int on);

/* Alg. 1 for every activated layer, on the device.  X_build holds N training inputs
 * (device).  Input_l is the full network's output of layer l-1 on X_build; the
 * Activation summed into NodeScore is layer l's own output; each bucket keeps its
 * positive-score nodes sorted from the highest sum to the lowest (ties: lower id),
 * at most list_cap of them; the sums over all N inputs give the fallback ranking.
 * Allocates temporary device memory, synchronises `stream`, returns owned tables.
 * N <= SLONN_MAX_BATCH.  Everything runs on the device (layers up to 8192 nodes sort each
 * bucket in LDS; wider layers rank the head of a bucket through a score threshold, or sort
 * whole buckets when lists longer than 8192 ids are asked for or sums are equal in masses).
 * ENOMEM: the NodeScore sums of refreshable tables do not fit.                       */
int slonn_build_tables(const slonn_model* m, const slonn_input* X_build, int64_t N, void* stream,
                       slonn_tables** out);

/* Alg. 1 continued on N more training inputs X_new (device): they are added to the NodeScore
 * sums of the buckets they fall into and to the whole-set sums, every running sum continued in
 * input order; the buckets they touched and the whole-set ranking are sorted again, the other
 * lists are kept.  Afterwards the tables are, bit for bit, those slonn_build_tables gives on all
 * inputs seen so far in the order they arrived.  Synchronises `stream`; replaces the tables'
 * device arrays, so no select / forward call on these tables may be in flight.
 * EUNSUPPORTED: tables without NodeScore sums (trained without
 * slonn_model_set_tables_refreshable, or imported).  After any other failure discard the tables. */
int slonn_tables_refresh(const slonn_model* m, slonn_tables* t, const slonn_input* X_new, int64_t N,
                         void* stream);

/* Table blob (host memory, little endian, all fields 4 bytes wide):
 *   u32 magic, u32 version, u32 n_sets, u32 0
 *   per set: u32 layer, K, L, n, list_cap, total_ids, 0, 0
 *            i32 hash_nodes[L*K]; u32 dir[L][2^K+1]; i32 ids[total_ids]; i32 global_rank[n]
 * dir[b][key] .. dir[b][key+1] delimit bucket (b,key)'s list inside ids; offsets run on
 * from one table to the next.  export: call with buf == NULL to obtain *bytes, then
 * with a buffer of that size.  import checks the blob against the model (layer ids,
 * K, L, n, hash nodes, offsets monotone, ids in range) and uploads it.             */
int slonn_tables_export(const slonn_tables* t, void* host_buf, size_t* bytes);
int slonn_tables_import(const slonn_model* m, const void* host_buf, size_t bytes, slonn_tables** out);
int slonn_tables_destroy(slonn_tables* t);

/* Bytes of device workspace the select / forward calls need for batches up to B_max. */
int slonn_workspace_bytes(const slonn_model* m, int B_max, size_t* out);

/* Node Activator of one layer (Fig. 2 steps 1, 3, 4) on a batch of that layer's
 * inputs X_l (device [B][d_in] fp32): FreeHash projections z = W_h x + b_h, keys, bucket
 * lookup, rank-major merge of the L lists with first-occurrence de-duplication, the
 * whole-set ranking as fallback, until the budget of each query is met.
 * keep: device, query q uses keep[q*keep_stride] (stride 0 broadcasts one value).
 * codes_out [B][L], z_out [B][K*L] nullable.  active_idx [B][idx_stride] receives the
 * chosen ids in selection order, active_cnt [B] their number (== budget).
 * ECAP when idx_stride < d_out (a budget may reach d_out).                          */
int slonn_select(const slonn_model* m, const slonn_tables* t, int layer, const float* X_l, int B,
                 const float* keep, int keep_stride, uint32_t* codes_out, float* z_out,
                 int32_t* active_idx, int32_t* active_cnt, int idx_stride, void* workspace,
                 size_t ws_bytes, void* stream);

/* Whole network with node dropout: for each layer, select (if activated) then evaluate
 * only the active rows; the sparse output feeds the next layer.  keep: device,
 * query q / layer l uses keep[q*keep_qstride + l*keep_lstride] (0 strides broadcast;
 * the paper uses one k per query for all layers: keep_lstride = 0).
 * Numerics: hash codes and active sets do not depend on the batch size or the path (the
 * projections are summed in fp64, or for batches from 256 as exact integer sums of fixed-
 * point digits with every sign certified; only a projection within about 1e-13 of zero can
 * fall either way).  A selected node's output is act(w . x + b) in fp32-class arithmetic:
 * fp32 FMA chains, or - large batches of large layers - exact partial products of fp16 parts
 * of the operands (rows scaled by powers of two, 22 significand bits per operand, bf16 weights
 * exactly) accumulated in fp32 on the matrix cores; the summation order differs
 * between paths and batch sizes, results agree to fp32 rounding.                     */
int slonn_sparse_forward(const slonn_model* m, const slonn_tables* t, const slonn_input* X, int B,
                         const float* keep, int keep_qstride, int keep_lstride, slonn_output* Y,
                         const slonn_debug_taps* taps, void* workspace, size_t ws_bytes,
                         void* stream);

/* slonn_sparse_forward for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments, results and kernels, but the per-batch workspace is a static device array of
 * SLONN_STATIC_SCRATCH_BYTES inside the library, one per GPU, held until the process ends.  The
 * call allocates nothing (no hipMalloc/hipFree, no host allocation).  ECAP when
 * slonn_workspace_bytes(m, B) exceeds SLONN_STATIC_SCRATCH_BYTES (nothing is enqueued).  All calls
 * on one GPU share that GPU's array, which keeps whatever the last call left there (every kernel
 * clears what it needs to start at zero): calls that overlap on one GPU - from different
 * streams or threads - race; serialise them.                                                  */
#define SLONN_STATIC_SCRATCH_BYTES (64u << 20)
int slonn_sparse_forward_static(const slonn_model* m, const slonn_tables* t, const slonn_input* X, int B,
                                const float* keep, int keep_qstride, int keep_lstride, slonn_output* Y,
                                const slonn_debug_taps* taps, void* stream);

/* ---- Choice of k per query (Section 2: ACLO and LCAO; Section 3.2: Confidence LSH tables,
 * latency profiles; Fig. 2 step 2).  Mechanics only: the confidences c(k, x') of the
 * training inputs (the confidence definition of Section 2.1, the first equation) and the latency profile T(k, beta) are supplied by the caller, and
 * an accuracy target reaches the library as the confidence threshold it was calibrated to.
 *
 * A policy holds an ascending grid k_0 < ... < k_{G-1} of keep fractions (HOST, values in
 * (0, 1], G <= SLONN_MAX_GRID), Confidence LSH tables over L tables of K-bit keys, and a
 * latency profile.  The keys are those of the model's first activated layer (the tables
 * share its hash functions), so K and L must equal that layer's.                          */
int slonn_policy_create(int K, int L, const float* k_grid, int G, slonn_policy** out);
int slonn_policy_destroy(slonn_policy* p);

/* Confidence LSH tables.  codes: device [N][L] keys of the N training inputs (as returned
 * by slonn_select's codes_out for the first activated layer), conf: device [N][G] with
 * conf[x][g] = c(k_g, x).  Every bucket receives the sum (double, in input order) and the
 * count of its inputs' confidences; a later call replaces the tables.  Synchronises the
 * stream.  EINVAL: null argument, N outside 1 .. SLONN_MAX_BATCH, a key >= 2^K.            */
int slonn_policy_train_confidence(slonn_policy* p, const uint32_t* codes, const float* conf, int64_t N,
                                  void* stream);

/* Latency profile T: HOST [n_beta][G], T[beta][g] = latency of a pass at k_g under
 * co-location state beta (any unit; tau and t0 below use the same), entries >= 0.        */
int slonn_policy_set_latency_profile(slonn_policy* p, const float* T, int n_beta);

/* ACLO (Section 2.2): minimise k subject to the accuracy constraint.  For query q with keys
 * codes[q][0..L) (device) the estimated confidence (Eq. 4, arithmetic mean) of grid point g is
 *   c_hat(k_g, x) = (sum over tables of the bucket's sum) / (sum over tables of its count),
 * i.e. the mean over the training inputs that share a bucket with x, an input counted once
 * per shared bucket; with no such input, the mean over the whole training set.  keep_out[q]
 * (device) = the smallest k_g with c_hat >= thr[q*thr_stride] (device; stride 0 broadcasts),
 * else k_{G-1}.  grid_idx_out [B] int32 and c_hat_out [B][G] double are nullable (device).
 * EINVAL: null argument, untrained tables, bad B.                                          */
int slonn_policy_keep_aclo(const slonn_policy* p, const uint32_t* codes, int B, const float* thr,
                           int thr_stride, float* keep_out, int32_t* grid_idx_out, double* c_hat_out,
                           void* stream);

/* LCAO (Section 2.3): maximise k subject to t0 + T(k, beta) <= tau.  All arrays device, with
 * element strides (0 broadcasts): keep_out[q] = the largest k_g with
 * t0[q] + T[beta[q]][g] <= tau[q] (evaluated in double); if no grid point fits, or beta[q]
 * is outside 0 .. n_beta-1, the SLO cannot be met: keep_out[q] = k_0 and violated_out[q] = 1
 * (else 0).  grid_idx_out, violated_out nullable.  EINVAL: null argument, no profile set.   */
int slonn_policy_keep_lcao(const slonn_policy* p, int B, const float* tau, int tau_stride, const float* t0,
                           int t0_stride, const int32_t* beta, int beta_stride, float* keep_out,
                           int32_t* grid_idx_out, int32_t* violated_out, void* stream);

/* slonn_sparse_forward with k chosen inside the pass under ACLO (Fig. 2: the Confidence LSH
 * tables are queried once per request, the chosen k serves every layer): the keys of the
 * first activated layer are computed once and used both for the choice of k and for that
 * layer's Node Importance lookup.  thr as in slonn_policy_keep_aclo; keep_out [B] (device)
 * receives the chosen keep fractions.  Everything else as slonn_sparse_forward.  EINVAL also
 * when the policy's K, L differ from the first activated layer's or it is untrained.        */
int slonn_sparse_forward_aclo(const slonn_model* m, const slonn_tables* t, const slonn_policy* p,
                              const slonn_input* X, int B, const float* thr, int thr_stride, float* keep_out,
                              slonn_output* Y, const slonn_debug_taps* taps, void* workspace, size_t ws_bytes,
                              void* stream);

/* A recorded forward pass, for batches so small that launching dominates (the paper serves one
 * query at a time, Section 4): create runs slonn_sparse_forward once with the given arguments
 * (same meaning, no debug taps) and then records the same call into a HIP graph; launch replays
 * it on `stream` as one submission.  Every pointer is baked in: between launches the caller
 * rewrites the input (X), keep and reads the output buffers in place; model, tables, workspace and
 * buffers must outlive the graph, and launches of one graph must not overlap.  create runs its
 * pass on a stream of its own and waits for it: work still in flight on other streams must not
 * use the same workspace or output buffers meanwhile (graphs that share a workspace are created
 * and launched one after another on one stream).  The recording holds kernel launches only (no
 * memory-set nodes).  EINVAL also while per-kernel timing is on.                             */
int slonn_forward_graph_create(const slonn_model* m, const slonn_tables* t, const slonn_input* X, int B,
                               const float* keep, int keep_qstride, int keep_lstride, slonn_output* Y,
                               void* workspace, size_t ws_bytes, slonn_graph** out);
int slonn_forward_graph_launch(slonn_graph* g, void* stream);
int slonn_forward_graph_destroy(slonn_graph* g);

/* The full network (all nodes), the baseline every speed-up is measured against:
 * per layer an MFMA GEMM + bias + activation.  Y device [B][d_last]; argmax nullable.
 * layer_out: optional HOST array of n_layers device pointers ([B][d_out] each).     */
int slonn_dense_forward(const slonn_model* m, const slonn_input* X, int B, float* Y, int32_t* argmax,
                        float** layer_out, void* workspace, size_t ws_bytes, void* stream);

/* Per-kernel timing for measurement runs.  Between begin and end every kernel the
 * select / forward calls launch is bracketed by two HIP events recorded on the launch
 * stream (at most max_launches of them; later launches go untimed).  end synchronises
 * the device, adds up the elapsed time and launch count per kernel kind into the two
 * caller arrays of SLONN_PROF_KINDS entries (HOST), and switches timing off again.
 * Not thread-safe; costs two event records per launch while on.                     */
enum { SLONN_PROF_HASH = 0, SLONN_PROF_SELECT = 1, SLONN_PROF_GATHER = 2, SLONN_PROF_DENSE = 3,
       SLONN_PROF_ELL = 4, SLONN_PROF_FINALIZE = 5, SLONN_PROF_FUSED = 6,
       SLONN_PROF_TILES = 7,   /* selected pairs evaluated as masked tiles on the matrix cores */
       SLONN_PROF_KINDS = 8 };
int slonn_profile_begin(int max_launches);
int slonn_profile_end(double* ms_per_kind, int64_t* launches_per_kind);

const char* slonn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SLONN_H */
