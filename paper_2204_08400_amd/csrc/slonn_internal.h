// Internal declarations shared by the host side of libslonn and its kernel launchers.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "slonn.h"

namespace slonn {

void set_error(const char* fmt, ...);

#define SLONN_FAIL(code, ...)        \
  do {                               \
    ::slonn::set_error(__VA_ARGS__); \
    return (code);                   \
  } while (0)

#define SLONN_HIP(call)                                                                    \
  do {                                                                                     \
    hipError_t e_ = (call);                                                                \
    if (e_ != hipSuccess) {                                                                \
      ::slonn::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__,  \
                         __LINE__);                                                        \
      return SLONN_EHIP;                                                                   \
    }                                                                                      \
  } while (0)

struct Layer {
  int d_in = 0, d_out = 0;
  int w_dtype = SLONN_F32, w_layout = SLONN_ROWS_ARE_NODES, act = SLONN_ACT_NONE;
  int K = 0, L = 0, list_cap = 0;
  const void* W = nullptr;       // borrowed device
  const float* bias = nullptr;   // borrowed device
  std::vector<int32_t> hash_nodes;
  // library-owned device copies of the FreeHash rows (always fp32) and their biases
  float* Wh = nullptr;           // [H][d_in]
  float* bh = nullptr;           // [H]
  float* WhT = nullptr;          // small layers: the same rows input-major [d_in][(H + 3) & ~3] (zero-padded columns)
  int16_t* hslot = nullptr;      // [d_out] device: index of the node among the hash rows, or -1
  int32_t* hnodes = nullptr;     // [H] device copy of hash_nodes
  uint16_t* Wt = nullptr;        // large layers: the weights as scaled fp16 parts for the tile kernel [d_out][wt_parts d_in]
  int32_t* wt_exp = nullptr;     // [d_out] the rows' exponents
  int wt_parts = 0;              // 2 (fp32 weights) or 1 (bf16 weights)
  int8_t* Whd = nullptr;         // the FreeHash rows as interleaved 7-bit digits [H][hash_int_digits() * d_in] (int8 cores)
  int32_t* ewh = nullptr;        // [H] their fixed-point exponents
  int H() const { return K * L; }
  bool activated() const { return K > 0 && L > 0; }
};

struct TableSet {                 // Node Importance tables of one layer
  int layer = -1, K = 0, L = 0, n = 0, list_cap = 0;
  std::vector<uint32_t> dir;      // host copy [L][2^K+1]
  std::vector<int32_t> ids;       // host staging of the lists (import only; emptied after the upload)
  std::vector<int32_t> global_rank;
  size_t n_ids = 0;               // list entries held in d_ids
  uint32_t* d_dir = nullptr;      // device copies
  void* d_ids = nullptr;          // the lists: uint16_t entries when narrow, else int32_t
  bool narrow = false;            // layers of up to 65 536 nodes store 2-byte node ids
  int32_t* d_global_rank = nullptr;
  // NodeScore state kept for online refresh (tables trained with slonn_model_set_tables_refreshable)
  double* d_score = nullptr;         // [L][2^K][n] NodeScore sums
  double* d_global_score = nullptr;  // [n] sums over all training inputs
  uint32_t* d_npos = nullptr;        // [L][2^K] nodes with a positive sum per bucket
  unsigned long long nonempty = 0;   // buckets that hold a list
  long long n_trained = 0;           // training inputs seen so far
};

}  // namespace slonn

struct slonn_model {
  std::vector<slonn::Layer> layers;
  int path = SLONN_PATH_AUTO;
  bool path_grouped = true;       // allow the grouped (cross-query) evaluation on the per-layer path
  bool hash_first = false;        // hash nodes always computed, never selected (Section 3.4 variant)
  double hash_margin = 2.0;       // integer hash projections: |z| must exceed this many error bounds
  bool tables_refreshable = false; // slonn_build_tables keeps the NodeScore sums for slonn_tables_refresh
  int batches_in_flight = 1;      // batches the caller keeps in flight on the device (sizes the whole-network workgroups)
  int dense_arith = 0;            // slonn_dense_forward: 0 fp32 matrix cores, 1 fp16 parts on the fp16 matrix cores
  int max_lds_bytes = 65536;      // per-workgroup LDS the device grants on request
  int n_cu = 256;
};

struct slonn_tables {
  const slonn_model* model = nullptr;
  std::vector<slonn::TableSet> sets;            // one per activated layer
  const slonn::TableSet* for_layer(int l) const {
    for (const auto& s : sets)
      if (s.layer == l) return &s;
    return nullptr;
  }
};

namespace slonn {

// Optional per-kernel timing (slonn_profile_begin/end): a scope brackets one launch with
// two events on the launch stream.  Does nothing unless profiling is switched on.
struct ProfScope {
  ProfScope(int kind, hipStream_t s);
  ~ProfScope();
  int slot;
  hipStream_t stream;
};

// Confidence tables as the whole-network kernel sees them (sum == nullptr: keep fractions
// come from the caller).
struct PolicyArgs {
  const double* sum = nullptr;     // [L][2^K][G]
  const uint32_t* cnt = nullptr;   // [L][2^K]
  const double* total = nullptr;   // [G]
  const float* grid = nullptr;     // [G]
  const float* thr = nullptr;      // [B] (stride thr_stride)
  float* keep_out = nullptr;       // [B]
  long long N = 0;
  int G = 0, thr_stride = 0, layer = -1;
};

// Arguments of the whole-network kernel (passed by value as kernel arguments).
constexpr int FUSED_MAX_LAYERS = 8;
struct FusedLayer {
  const void* W;
  const float* bias;
  const float* WhT;                // FreeHash rows input-major [d_in][(H + 3) & ~3]
  const float* bh;
  const int16_t* hslot;
  const int32_t* hnodes;
  const uint32_t* dir;
  const void* ids;                 // uint16_t entries when ids_narrow, else int32_t
  const int32_t* global_rank;
  uint32_t* tap_codes;
  float* tap_z;
  int32_t* tap_idx;
  int32_t* tap_cnt;
  float* tap_out;
  int d_in, d_out, act, w_dtype, K, L, ids_narrow;
};
struct FusedArgs {
  FusedLayer layer[FUSED_MAX_LAYERS];
  const float* X;
  const float* keep;
  float* Y;
  int32_t* argmax;
  int ldx, keep_qstride, keep_lstride, n_layers;
  int hash_first;                  // hash nodes always computed, never selected
  PolicyArgs pol;                  // choice of k inside the kernel (ACLO)
  int max_dim, max_H, max_na;      // LDS carve-up: activations, projections, active list
};
size_t fused_lds_bytes(const FusedArgs& a);
int launch_fused_forward(const FusedArgs& a, int B, int in_flight, int n_cu, int max_lds, hipStream_t s);

// Arguments of the whole-network kernel for wide sparse-input models (ELL input, one small
// hidden layer stored input-major, activated output layer).
struct FusedWideArgs {
  // hidden layer
  const void* W0; const float* b0;
  const int32_t* idx; const float* val; const int32_t* nnz;
  int w0_dtype, act0, d0, n1, n1p, ccp, ell_stride, ellp;
  // output layer and its Node Activator
  const void* W1; const float* b1; const float* WhT; const float* bh;   // WhT: hash rows input-major [n1][Hp]
  const uint32_t* dir; const void* ids; const int32_t* global_rank;
  const int32_t* hnodes; const int16_t* hslot;
  int w1_dtype, act1, n2, K, L, Hp, hash_first, ids_narrow;
  const float* keep; int keep_qstride;
  // outputs (list, vals, cnt always; dense, argmax and the taps nullable)
  int32_t* list; int list_stride;
  float* vals; int vals_stride;
  int32_t* cnt;
  float* dense; int32_t* argmax;
  uint32_t* tap_codes; float* tap_z; float* tap_out0;
};
size_t fused_wide_lds_bytes(const FusedWideArgs& a);
int launch_fused_wide(const FusedWideArgs& a, int B, int in_flight, int n_cu, int max_lds, hipStream_t s);

// Active lists regrouped by weight-row block, so that the workgroups running at the same
// time read the same few megabytes of the weight matrix (L2-sized blocks of rows).
struct RowBlocking {
  int rows_per_block = 0, nblk = 0, stride = 0;
  int32_t* part_idx = nullptr;   // [B][stride]  node ids, grouped by row block
  int32_t* part_pos = nullptr;   // [B][stride]  position of each id in the selection order
  int32_t* blk_off = nullptr;    // [B][nblk+1]  start of each row block's group
  // A selected node that is also a hash node already has its pre-activation among the
  // projections (Section 3.4): the regrouping step writes its output from there and leaves
  // it out of the groups, so its row is not fetched a second time.  hslot == nullptr: off.
  const int16_t* hslot = nullptr; // [n] index among the hash rows or -1
  float* y = nullptr;             // [B][ldy] dense outputs (nullable)
  float* yc = nullptr;            // [B][ldc] outputs in selection order (nullable)
  int ldy = 0, ldc = 0, relu = 0;
  // > 0: the masked tiles follow and serve every tile of 128 queries whose list lengths add up
  // to at least this much per query (launch_masked_tiles with the same threshold); the queries
  // of such a tile are not regrouped.  B: the batch (the last tile may be short).
  long long served_min_per_query = 0;
  int B = 0;
  // mask != nullptr: the select kernel itself writes what the tile kernel reads -- for a query of
  // a served tile one bit per node of its list (mask[q][(n + 31) / 32]), and per tile the decision
  // (flags[q / 16 .. + 7] for the tile's first query q) -- so that no pass over the lists follows.
  uint32_t* mask = nullptr;
  int32_t* flags = nullptr;
};
constexpr int MAX_ROW_BLOCKS = 1024;

// Section 3.4 variant: the K*L hash nodes are always computed and the Node Activator never
// selects them.  The active list then starts with the hash nodes in sampled order and
// continues with the first max(m - K*L, 0) other nodes of the merge.  hnodes == nullptr: off.
struct HashFirst {
  const int32_t* hnodes = nullptr;   // [K*L] device
  const int16_t* hslot = nullptr;    // [n] device: index among the hash rows or -1
};

// A hash projection whose reduction is still split in S partial sums (medium batches): the
// select kernel adds them.  part: [S][B][H] fp64 device; Z: [B][H] receives the projections.
struct HashSplit {
  const double* part = nullptr;
  int S = 0;
  int B = 0;
  const float* bh = nullptr;
  float* Z = nullptr;
};

// Tile kernels and the eight XCDs.  Workgroups are dealt to the XCDs in turn by their linear id,
// and each XCD has an L2 of its own: the workgroups of one XCD should share operand tiles.  For an
// nx x ny grid of tiles (x: tiles of the first operand, y: of the second) the XCDs are laid out
// sx x (8 / sx) over the grid and every XCD takes a compact block of nx / sx by ny / (8 / sx) tiles.
// xcd_split picks sx (0: leave the grid as it is) from the bytes of one tile of either operand.
inline int xcd_split(int nx, int ny, double x_tile_bytes, double y_tile_bytes) {
  int best = 0;
  double best_cost = 0.0;
  for (int sx = 1; sx <= 8; sx *= 2) {
    const int sy = 8 / sx;
    if (nx % sx != 0 || ny % sy != 0) continue;
    const double cost = (double)(nx / sx) * x_tile_bytes + (double)(ny / sy) * y_tile_bytes;
    if (best == 0 || cost < best_cost) { best = sx; best_cost = cost; }
  }
  return best;
}
#if defined(__HIPCC__)
__device__ __forceinline__ void xcd_tile(int bx, int by, int nx, int ny, int sx, int& tx, int& ty) {
  if (sx == 0) { tx = bx; ty = by; return; }
  const int sy = 8 / sx;
  const int w = bx + nx * by, xcd = w & 7, slot = w >> 3;
  const int rx = nx / sx, ry = ny / sy;
  tx = (xcd % sx) * rx + slot % rx;
  ty = (xcd / sx) * ry + slot / rx;
}
#endif

// ---- kernel launchers (each validates nothing: callers have checked shapes) ----

// Z[q][h] = Wh[h] . X[q] + bh[h], fp64 accumulation, rounded once to fp32.
// split_scratch (nullable): hash_split_workspace_bytes() of device memory; with it a medium
// batch splits the reduction dimension over workgroups (hash_split_factor > 1 tells when).
// pending (nullable): when the reduction was split, receives the partial sums for launch_select
// to add, and Z is not written here; without it a small kernel adds them right away.
int launch_hash_project(const float* X, int ldx, const float* Wh, const float* bh, float* Z, int B,
                        int H, int d, void* split_scratch, HashSplit* pending, hipStream_t s);
size_t hash_split_workspace_bytes();
int hash_split_factor(int B, int H, int d);

// The same projections for a large batch on the int8 matrix cores: fixed-point digits, exact
// integer dot products, every sign certified against a rigorous error bound, the uncertain
// projections recomputed in fp64.  Wd, ew: the hash rows through launch_slice_digits (model set-up),
// hash_int_digits() bytes per element.
// d a multiple of 64 and two tile buffers within the LDS the device grants (hash_int_supported).  scratch: hash_int_workspace_bytes(B, H, d) bytes.
bool hash_int_supported(int d, int max_lds);
int hash_int_digits();
size_t hash_int_workspace_bytes(int B, int H, int d);
int launch_slice_digits(const float* X, int64_t ldx, int64_t rows, int d, int8_t* out, int32_t* expo,
                        int32_t* nonzeros, hipStream_t s);   // nonzeros: nullable, per row the count of non-zero elements
int launch_hash_project_int(const float* X, int ldx, const float* Wh, const int8_t* Wd, const int32_t* ew,
                            const float* bh, float* Z, int B, int H, int d, double margin, void* scratch,
                            hipStream_t s);
// after launch_hash_project_int: the exponents of the rows of X it left in its scratch (largest magnitude of
// row q below 2^e[q], INT_MIN for a row with a non-finite element)
const int32_t* hash_int_row_exponents(const void* scratch, int B, int d);

// keys + bucket lookup + merge for one layer.  yzero (nullable): [B][ldy] rows to clear.
// ids: the lists, uint16_t entries when ids_narrow, else int32_t
int launch_select(const float* Z, int K, int L, int n, const uint32_t* dir, const void* ids, bool ids_narrow,
                  const int32_t* global_rank, const float* keep, int keep_stride, int B,
                  uint32_t* codes, int32_t* active, int32_t* cnt, int idx_stride, float* yzero,
                  int ldy, int max_lds, const RowBlocking* rb, const HashFirst* hash_first,
                  const HashSplit* split, const int32_t* order, hipStream_t s);
// order (nullable): [B] permutation of the queries; workgroup i serves query order[i].
// launch_order_by_budget fills it with the queries in descending order of their budgets, for
// batches that do not fit the device at once (select_wants_order).
bool select_wants_order(int n, int B, int max_lds, int n_cu);
int launch_order_by_budget(const float* keep, int keep_stride, int B, int32_t* order, hipStream_t s);
// true when launch_select will fill rb for a layer of n nodes (the workgroup kernel is used)
bool select_fills_row_blocks(int n, int max_lds);

// batches up to this size fetch every selected row with a workgroup of its own
constexpr int GATHER_ROW_MAX_BATCH = 6;

// Same result as launch_gather_forward from row-block-grouped lists: workgroup (q, block)
// evaluates the rows of query q that fall into that block of the weight matrix.
// skip_group (nullable): [ceil(B/16)] flags; queries of a flagged group are left to the
// grouped evaluation below.
int launch_gather_blocked(const void* W, int w_dtype, const float* bias, const float* X, int ldx,
                          const RowBlocking& rb, float* Y, int ldy, float* yc, int ldc, int B, int d,
                          int n, int act, const int32_t* skip_group, hipStream_t s);

// Selected hash nodes in the grouped evaluation: nodes with hslot[node] >= 0 are left out of the
// unions (their outputs come from the hash projections, Section 3.4).  With Z set the union
// step also writes those outputs, Y[q][node] = act(Z[q][hslot[node]]); with Z null somebody else
// already has (the row-block regrouping step).  hslot null: no reuse.
struct GroupedReuse {
  const int16_t* hslot = nullptr;
  const float* Z = nullptr;      // [B][H] projections
  int H = 0, relu = 0;
};

// Groups of 16 queries: the union of their active rows evaluated as dense tiles on the matrix
// cores, selected (query, node) pairs written to Y.  A group whose union is too large
// relative to its lists is flagged 0 in *gflag_out (device array, [ceil(B/16)]) and left
// untouched (with bf16 weights on the bf16 cores every group is taken).  served (nullable,
// device, one per 16 queries): groups with a non-zero entry were evaluated another way and are
// skipped altogether.  scratch:
// grouped_workspace_bytes(B, n, d) bytes of device memory.
// d_bf16: widest input of an activated layer with bf16 weights (0: none); its activations are
// split into three bf16 parts for the bf16 matrix cores.
size_t grouped_workspace_bytes(int B, int n, int d_bf16);
bool grouped_supported(int n, int max_lds);
bool grouped_uses_bf16_cores(const void* W, int w_dtype, int d);
int launch_gather_grouped(const void* W, int w_dtype, const float* bias, const float* X, int ldx,
                          const int32_t* active, const int32_t* cnt, int idx_stride, float* Y, int ldy,
                          int B, int d, int n, int act, const GroupedReuse* reuse, const int32_t* served,
                          void* scratch, int max_lds, int32_t** gflag_out, hipStream_t s);

// Large batches of a large layer: the selected (query, node) pairs evaluated as masked dense
// tiles on the fp16 matrix cores (rows scaled by powers of two, activations and fp32 weights as
// two fp16 parts, bf16 weights as one).  Wp, wexp: the weights through launch_split_weights
// (tile_weights_bytes(w_dtype, n, d) bytes, n exponents), w_parts 2 for fp32 weights, 1 for bf16.
// Per 128 queries the select kernel has decided whether the tiles serve them (RowBlocking::mask,
// ::flags, placed in scratch by masked_tiles_buffers): *flags_out (device, one per 16 queries) is
// 1 where they do.  X: 16-byte aligned fp32 rows; xexp (nullable, device): their exponents
// (largest magnitude of row q below 2^xexp[q], INT_MIN for a row with a non-finite element)
// where a kernel before this one has found them.  scratch: masked_tiles_workspace_bytes(B, n, d)
// bytes.
bool masked_tiles_supported(int d, int n, int max_lds);
size_t masked_tiles_workspace_bytes(int B, int n, int d);
// where in that scratch the pair masks [B][(n + 31) / 32] and the per-16-queries flags live
void masked_tiles_buffers(void* scratch, int B, int n, uint32_t** mask, int32_t** flags);
size_t tile_weights_bytes(int w_dtype, int n, int d);
int launch_split_weights(const void* W, int w_dtype, int n, int d, uint16_t* out, int32_t* wexp, hipStream_t s);
// measurement aid: workgroups that read one L2-resident 2 MiB window with 16-byte loads (returns the bytes read)
double launch_l2_read_probe(void* buf, int workgroups, int passes, hipStream_t s);
// measurement aid: a register-only loop of the tile kernel's MFMAs (returns the flops of the launch)
double launch_mfma_rate_probe(float* out, int workgroups, int iters, hipStream_t s);
int launch_dense_tiles(const uint16_t* Wp, int w_parts, const int32_t* wexp, const float* bias, const float* X, int ldx,
                       float* Y, int ldy, int B, int d, int n, int act, void* scratch, hipStream_t s);
int launch_masked_tiles(const uint16_t* Wp, int w_parts, const int32_t* wexp, const float* bias, const float* X, int ldx,
                        const int32_t* xexp, float* Y, int ldy, int B, int d, int n, int act, void* scratch,
                        int32_t** flags_out, hipStream_t s);

// y[q][j] = act(W[j] . X[q] + b[j]) for the listed rows (active == nullptr: all n rows).
// yc (nullable) receives the values in list order.
int launch_gather_forward(const void* W, int w_dtype, const float* bias, const float* X, int ldx,
                          const int32_t* active, const int32_t* cnt, int idx_stride, int max_rows,
                          float* Y, int ldy, float* yc, int ldc, int B, int d, int n, int act,
                          hipStream_t s);

// First layer on ELL input: y[q][j] = act(sum_t val[q][t] * W(j, idx[q][t]) + b[j]).
int launch_ell_layer(const void* W, int w_dtype, int w_layout, const float* bias, const int32_t* idx,
                     const float* val, const int32_t* nnz, int ell_stride, float* Y, int ldy, int B,
                     int d, int n, int act, hipStream_t s);

// Softmax over the computed nodes (in place on Y and yc) and/or argmax, one wave per query.
int launch_finalize(float* Y, int ldy, int n, const int32_t* active, const int32_t* cnt,
                    int idx_stride, float* yc, int ldc, int do_softmax, int32_t* argmax, int B,
                    hipStream_t s);

// Dense layer Y = act(X W^T + b) as an MFMA GEMM (fp32 matrix cores).  split_scratch (nullable):
// dense_split_workspace_bytes(B, n, d) bytes; with it a problem of only a few tiles (a skinny
// output layer) splits its reduction over more workgroups.
int launch_dense_layer(const void* W, int w_dtype, const float* bias, const float* X, int ldx,
                       float* Y, int ldy, int B, int d, int n, int act, void* split_scratch, hipStream_t s,
                       bool batch_invariant = false);
size_t dense_split_workspace_bytes(int B, int n, int d);

// true when a problem of fewer than 256 tiles of 64x64 can take the small-shape MFMA kernel
// (operands straight from L2); otherwise such shapes are better served by the row gather.
bool dense_small_supported(const void* W, int w_dtype, const float* X, int ldx, int d);

// k per query from the confidence tables (ACLO): keys from codes [B][L] or, when codes is
// null, from the projections Z [B][K*L].
int launch_policy_aclo(const slonn_policy* p, const uint32_t* codes, const float* Z, int B, const float* thr,
                       int thr_stride, float* keep_out, int32_t* g_out, double* chat_out, hipStream_t s);
void policy_fused_args(const slonn_policy* p, PolicyArgs* a);
bool policy_matches(const slonn_policy* p, int K, int L);
bool policy_trained(const slonn_policy* p);

// Wh[h][0..d) = row hnodes[h] of W widened to fp32, bh[h] = bias[hnodes[h]] (model set-up).
int launch_gather_hash_rows(const void* W, int w_dtype, const float* bias, const int32_t* hnodes, int H, int d,
                            float* Wh, float* bh, hipStream_t s);
// WhT[j][h] = Wh[h][j] for h < H, 0 for H <= h < Hp (model set-up; the whole-network kernel walks
// the non-zero inputs of a query and reads one contiguous row of WhT per input).
int launch_transpose_hash_rows(const float* Wh, int H, int d, int Hp, float* WhT, hipStream_t s);

int launch_fill_iota(int32_t* idx, int stride, int32_t* cnt, int n, int B, hipStream_t s);

// Alg. 1 on the device for one layer; fills ts (host + device copies).
int build_layer_tables(const slonn_model* m, int layer, const float* X_l, int64_t N, const float* act,
                       TableSet* ts, bool refresh, hipStream_t s);
// Ranking by a full sort, for what the LDS sorts of the table build do not cover: for every
// segment seg < segs (score + seg * n, n sums each) with len[seg] > 0 (and, when only is given,
// only[seg] != only[seg + 1]) the len[seg] best node ids by (sum descending, id ascending) go to
// out + off[seg].  Allocates temporary device memory.
int rank_by_sort(const double* score, int n, int segs, const uint32_t* off, const uint32_t* len,
                 const uint32_t* only, int32_t* out, hipStream_t s);
// device copies from the host vectors; the lists come from d_ids_src (device, ts->n_ids
// entries) when given, else from ts->ids
int upload_table_set(TableSet* ts, const int32_t* d_ids_src = nullptr);
// the lists of a table set as 4-byte ids in host memory (ts->n_ids of them)
int download_ids(const TableSet* ts, int32_t* host_out);
void free_table_set(TableSet* ts);

}  // namespace slonn
