// SLO-NN reference oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
//
// A plain, slow, scalar CPU implementation of the per-query dynamic node-dropout
// path of SLO-Aware Neural Networks, written from the paper so that each function
// can be checked against the text by eye.  It shares no code with the HIP library
// and must only be used by the tests, the smoke check and the CPU-baseline leg of
// the benchmark.
//
// Arithmetic: weights, biases and inputs are fp32 values (bf16 weights widen
// exactly to fp32).  Every dot product is accumulated in double, in index order,
// the bias is added in double, and the sum is rounded once to fp32; that fp32
// value is what the next step sees.  No blocking, no SIMD intrinsics, no BLAS.
//
// Readings taken where the paper is silent (each is restated at its function):
//   * sign(0): a hash bit is 1 iff the pre-activation is > 0 (Def. 2).
//   * bit/table order: the j-th hash node serves table j/K, bit j%K, little endian.
//   * a bucket's list holds only nodes whose activation sum is > 0, sorted from the
//     highest sum to the lowest (Section 3.2), equal sums by ascending node id.
//   * the L per-table lists are merged rank-major, table-minor, first occurrence
//     wins; when they run out the ranking over the whole training set continues
//     (it is Alg. 1 with K = 0, i.e. one bucket).
//   * a keep fraction becomes a node count by rounding to the nearest whole node,
//     at least one node.
//   * softmax / argmax run over the computed nodes only.
//   * (variant) hash nodes always computed and never selected: so_select_hash_first.
//   * confidence estimate with L tables: pooled mean over the L buckets (so_conf_estimate).
//
// Parity with the authors' own implementation is unpinned (no code or printed
// vectors exist); the pins in tests/ check this file against the definitions.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <unordered_map>
#include <vector>

namespace {

enum { W_F32 = 0, W_BF16 = 1 };
enum { ACT_NONE = 0, ACT_RELU = 1, ACT_SOFTMAX = 2 };

inline float weight_at(const void* W, int w_dtype, int64_t i) {
  if (w_dtype == W_F32) return static_cast<const float*>(W)[i];
  uint32_t bits = static_cast<uint32_t>(static_cast<const uint16_t*>(W)[i]) << 16;
  float f;
  std::memcpy(&f, &bits, 4);
  return f;
}

// w_j . x + b_j, accumulated in double in index order, rounded once to fp32.
inline float pre_activation(const void* W, int w_dtype, const float* bias, int d, int64_t j,
                            const float* x) {
  double s = 0.0;
  for (int i = 0; i < d; ++i)
    s += static_cast<double>(weight_at(W, w_dtype, j * d + i)) * static_cast<double>(x[i]);
  s += static_cast<double>(bias[j]);
  return static_cast<float>(s);
}

inline float relu(float z) { return z > 0.0f ? z : 0.0f; }

// Softmax over the listed nodes only; out[] holds logits on entry at those nodes.
void softmax_over(const int32_t* ids, int cnt, float* out) {
  if (cnt <= 0) return;
  double mx = out[ids[0]];
  for (int t = 1; t < cnt; ++t) mx = std::max(mx, static_cast<double>(out[ids[t]]));
  double sum = 0.0;
  std::vector<double> e(cnt);
  for (int t = 0; t < cnt; ++t) {
    e[t] = std::exp(static_cast<double>(out[ids[t]]) - mx);
    sum += e[t];
  }
  for (int t = 0; t < cnt; ++t) out[ids[t]] = static_cast<float>(e[t] / sum);
}

template <class F>
void parallel_for(int64_t N, int threads, F fn) {
  if (threads <= 1 || N <= 1) {
    for (int64_t q = 0; q < N; ++q) fn(q);
    return;
  }
  int T = static_cast<int>(std::min<int64_t>(threads, N));
  std::vector<std::thread> pool;
  for (int t = 0; t < T; ++t)
    pool.emplace_back([=] {
      for (int64_t q = t; q < N; q += T) fn(q);
    });
  for (auto& th : pool) th.join();
}

// Node Importance tables of one layer (Section 3.2, Alg. 1): Rank and, for the
// pins, the NodeScore sums they were sorted from.
struct Tables {
  int n = 0, K = 0, L = 0, list_cap = 0;
  int64_t N = 0;
  bool keep_scores = false;
  // per table: bucket key -> data
  std::vector<std::unordered_map<uint32_t, std::vector<double>>> score;   // NodeScore[b][key]
  std::vector<std::unordered_map<uint32_t, std::vector<int32_t>>> rank;   // Rank[b][key]
  std::vector<std::unordered_map<uint32_t, int64_t>> count;               // inputs per bucket
  std::vector<double> global_score;                                        // sum over all inputs
  std::vector<int32_t> global_rank;                                        // all n ids
};

// ids of positive-score nodes, highest score first, equal scores by ascending id.
std::vector<int32_t> rank_positive(const std::vector<double>& s, int cap) {
  std::vector<int32_t> ids;
  for (int j = 0; j < static_cast<int>(s.size()); ++j)
    if (s[j] > 0.0) ids.push_back(j);
  std::sort(ids.begin(), ids.end(), [&](int32_t a, int32_t b) {
    if (s[a] != s[b]) return s[a] > s[b];
    return a < b;
  });
  if (cap >= 0 && static_cast<int>(ids.size()) > cap) ids.resize(cap);
  return ids;
}

}  // namespace

extern "C" {

// Keep fraction -> node budget: nearest whole node, at least one, at most n.
int32_t so_budget(float keep, int32_t n) {
  double m = std::floor(static_cast<double>(keep) * static_cast<double>(n) + 0.5);
  if (!(m >= 1.0)) m = 1.0;   // values at or below zero, and a fraction that is not a number
  if (m > n) m = n;           // values above one
  return static_cast<int32_t>(m);
}

// Full layer: every node computed.  pre (nullable) receives w_j.x+b_j, out receives
// act(pre).  ReLU(z) = max(z, 0); softmax is taken over all n nodes.
int so_dense_layer(const void* W, int w_dtype, const float* bias, int d, int n, int act,
                   const float* X, int64_t N, float* pre, float* out, int threads) {
  std::vector<int32_t> all(n);
  for (int j = 0; j < n; ++j) all[j] = j;
  parallel_for(N, threads, [&](int64_t q) {
    const float* x = X + q * d;
    float* o = out + q * n;
    for (int j = 0; j < n; ++j) {
      float z = pre_activation(W, w_dtype, bias, d, j, x);
      if (pre) pre[q * n + j] = z;
      o[j] = (act == ACT_RELU) ? relu(z) : z;
    }
    if (act == ACT_SOFTMAX) softmax_over(all.data(), n, o);
  });
  return 0;
}

// FreeHash projections (Def. 2): z_h = w_i.x + b_i for the H = K*L sampled nodes i.
int so_hash_project(const void* W, int w_dtype, const float* bias, int d, const int32_t* hash_nodes,
                    int H, const float* X, int64_t N, float* Z, int threads) {
  parallel_for(N, threads, [&](int64_t q) {
    for (int h = 0; h < H; ++h)
      Z[q * H + h] = pre_activation(W, w_dtype, bias, d, hash_nodes[h], X + q * d);
  });
  return 0;
}

// Keys (Alg. 1, key := (h_1(x),...,h_K(x)) per table): bit j of table b's key is 1 iff
// z[b*K+j] > 0.  tie[q] (nullable) is set when any |z| < tie_eps, i.e. when the key
// depends on rounding order and must be left out of bit-exact comparisons.
int so_keys(const float* Z, int64_t N, int K, int L, uint32_t* keys, uint8_t* tie, float tie_eps) {
  for (int64_t q = 0; q < N; ++q) {
    uint8_t t = 0;
    for (int b = 0; b < L; ++b) {
      uint32_t key = 0;
      for (int j = 0; j < K; ++j) {
        float z = Z[q * (int64_t)K * L + b * K + j];
        if (z > 0.0f) key |= (1u << j);
        if (std::fabs(z) < tie_eps) t = 1;
      }
      keys[q * L + b] = key;
    }
    if (tie) tie[q] = t;
  }
  return 0;
}

// Alg. 1 at one layer.  For every training input (in order) and every table b:
// NodeScore[b][key_b] += Activation, where Activation is the layer's own output on
// that input.  Then Rank[b][key] := nodes sorted by NodeScore, highest first.  The
// same sums taken over all inputs give the fallback ranking.
void* so_tables_build(int n, int K, int L, int list_cap, const uint32_t* keys, const float* act,
                      int64_t N, int keep_scores, int threads) {
  Tables* t = new Tables;
  t->n = n; t->K = K; t->L = L; t->list_cap = list_cap; t->N = N;
  t->keep_scores = keep_scores != 0;
  t->score.resize(L); t->rank.resize(L); t->count.resize(L);
  // Tables are independent; within a table inputs are visited in order so every
  // NodeScore entry is summed in training-set order.
  parallel_for(L, threads, [&](int64_t b) {
    auto& sc = t->score[b];
    auto& ct = t->count[b];
    for (int64_t x = 0; x < N; ++x) {
      uint32_t key = keys[x * L + b];
      auto it = sc.find(key);
      if (it == sc.end()) it = sc.emplace(key, std::vector<double>(n, 0.0)).first;
      std::vector<double>& v = it->second;
      const float* a = act + x * n;
      for (int j = 0; j < n; ++j) v[j] += static_cast<double>(a[j]);
      ct[key] += 1;
    }
    for (auto& kv : sc) t->rank[b][kv.first] = rank_positive(kv.second, list_cap);
    if (!t->keep_scores) sc.clear();
  });
  t->global_score.assign(n, 0.0);
  for (int64_t x = 0; x < N; ++x)
    for (int j = 0; j < n; ++j) t->global_score[j] += static_cast<double>(act[x * n + j]);
  // Whole-set ranking: all n ids (zero-score nodes included, after the rest).
  t->global_rank.resize(n);
  for (int j = 0; j < n; ++j) t->global_rank[j] = j;
  const std::vector<double>& g = t->global_score;
  std::sort(t->global_rank.begin(), t->global_rank.end(), [&](int32_t a, int32_t b) {
    if (g[a] != g[b]) return g[a] > g[b];
    return a < b;
  });
  return t;
}

void so_tables_free(void* h) { delete static_cast<Tables*>(h); }

// Online refresh of a Node Activator (Section 3.2: the tables may be trained before or after
// deployment; Section 6 names refreshing them as data drifts): Alg. 1 goes on where it stopped.
// The N new inputs (their keys and the layer's activations for them, in order) are added to the
// NodeScore of the buckets they fall into and to the whole-set sums, continuing every running
// sum in input order; the buckets they touched and the whole-set ranking are sorted again.
// Needs tables that kept their NodeScore (keep_scores).  Returns 0, or -1 without that state.
int so_tables_refresh(void* h, const uint32_t* keys, const float* act, int64_t N) {
  Tables* t = static_cast<Tables*>(h);
  if (!t->keep_scores) return -1;
  const int n = t->n, L = t->L;
  for (int b = 0; b < L; ++b) {
    auto& sc = t->score[b];
    std::vector<uint32_t> touched;
    for (int64_t x = 0; x < N; ++x) {
      const uint32_t key = keys[x * L + b];
      auto it = sc.find(key);
      if (it == sc.end()) it = sc.emplace(key, std::vector<double>(n, 0.0)).first;
      std::vector<double>& v = it->second;
      const float* a = act + x * n;
      for (int j = 0; j < n; ++j) v[j] += static_cast<double>(a[j]);
      t->count[b][key] += 1;
      touched.push_back(key);
    }
    for (uint32_t key : touched) t->rank[b][key] = rank_positive(sc[key], t->list_cap);
  }
  for (int64_t x = 0; x < N; ++x)
    for (int j = 0; j < n; ++j) t->global_score[j] += static_cast<double>(act[x * n + j]);
  for (int j = 0; j < n; ++j) t->global_rank[j] = j;
  const std::vector<double>& g = t->global_score;
  std::sort(t->global_rank.begin(), t->global_rank.end(), [&](int32_t a, int32_t b) {
    if (g[a] != g[b]) return g[a] > g[b];
    return a < b;
  });
  t->N += N;
  return 0;
}

// Tables from explicit lists (used to load a table set built elsewhere): dir has
// L*(2^K+1) offsets into ids, table-major.
void* so_tables_from_lists(int n, int K, int L, int list_cap, const uint32_t* dir, const int32_t* ids,
                           const int32_t* global_rank) {
  Tables* t = new Tables;
  t->n = n; t->K = K; t->L = L; t->list_cap = list_cap;
  t->score.resize(L); t->rank.resize(L); t->count.resize(L);
  const int64_t nb = int64_t(1) << K;
  for (int b = 0; b < L; ++b)
    for (int64_t key = 0; key < nb; ++key) {
      uint32_t lo = dir[b * (nb + 1) + key], hi = dir[b * (nb + 1) + key + 1];
      if (hi > lo) t->rank[b][static_cast<uint32_t>(key)].assign(ids + lo, ids + hi);
    }
  t->global_rank.assign(global_rank, global_rank + n);
  t->global_score.assign(n, 0.0);
  return t;
}

// Length of Rank[b][key] (0 when the bucket was never hit); copies up to cap ids.
int32_t so_tables_bucket(const void* h, int b, uint32_t key, int32_t* ids_out, int32_t cap) {
  const Tables* t = static_cast<const Tables*>(h);
  auto it = t->rank[b].find(key);
  if (it == t->rank[b].end()) return 0;
  int32_t len = static_cast<int32_t>(it->second.size());
  for (int32_t i = 0; i < len && i < cap; ++i) ids_out[i] = it->second[i];
  return len;
}

// Flat copy of Rank: dir[b*(2^K+1)+key] = offset of Rank[b][key] in ids, offsets
// running on across tables.  ids may be null to size the copy; returns the id count.
int64_t so_tables_csr(const void* h, uint32_t* dir, int32_t* ids) {
  const Tables* t = static_cast<const Tables*>(h);
  const int64_t nb = int64_t(1) << t->K;
  int64_t off = 0;
  for (int b = 0; b < t->L; ++b) {
    for (int64_t key = 0; key < nb; ++key) {
      if (dir) dir[b * (nb + 1) + key] = static_cast<uint32_t>(off);
      auto it = t->rank[b].find(static_cast<uint32_t>(key));
      if (it == t->rank[b].end()) continue;
      if (ids) std::copy(it->second.begin(), it->second.end(), ids + off);
      off += static_cast<int64_t>(it->second.size());
    }
    if (dir) dir[b * (nb + 1) + nb] = static_cast<uint32_t>(off);
  }
  return off;
}

int64_t so_tables_bucket_count(const void* h, int b, uint32_t key) {
  const Tables* t = static_cast<const Tables*>(h);
  auto it = t->count[b].find(key);
  return it == t->count[b].end() ? 0 : it->second;
}

// NodeScore[b][key] (needs keep_scores); returns 0 when the bucket is empty.
int so_tables_bucket_scores(const void* h, int b, uint32_t key, double* out) {
  const Tables* t = static_cast<const Tables*>(h);
  auto it = t->score[b].find(key);
  if (it == t->score[b].end()) return 0;
  std::copy(it->second.begin(), it->second.end(), out);
  return 1;
}

int so_tables_global(const void* h, int32_t* rank_out, double* score_out) {
  const Tables* t = static_cast<const Tables*>(h);
  if (rank_out) std::copy(t->global_rank.begin(), t->global_rank.end(), rank_out);
  if (score_out) std::copy(t->global_score.begin(), t->global_score.end(), score_out);
  return 0;
}

// Selection for one layer (Fig. 2 steps 3-4; Section 3.3): look up one bucket per
// table, then walk rank r = 0,1,2,... and within a rank the tables b = 0..L-1,
// appending every node not chosen before, until m nodes are chosen.  If the lists
// run out first, continue down the whole-set ranking.  m == n selects every node in
// ascending id order without touching the tables.  active rows are emitted in the
// order the nodes were chosen.
int so_select(const void* h, const uint32_t* keys, const float* keep, int64_t keep_stride, int64_t N,
              int32_t* active, int32_t* cnt, int64_t stride) {
  const Tables* t = static_cast<const Tables*>(h);
  const int n = t->n, L = t->L;
  std::vector<uint8_t> chosen(n);
  std::vector<const std::vector<int32_t>*> lists(L);
  for (int64_t q = 0; q < N; ++q) {
    const int32_t m = so_budget(keep[q * keep_stride], n);
    if (m > stride) return -1;
    int32_t* out = active + q * stride;
    int32_t c = 0;
    if (m == n) {
      for (int j = 0; j < n; ++j) out[j] = j;
      cnt[q] = n;
      continue;
    }
    std::fill(chosen.begin(), chosen.end(), 0);
    size_t longest = 0;
    for (int b = 0; b < L; ++b) {
      auto it = t->rank[b].find(keys[q * L + b]);
      lists[b] = (it == t->rank[b].end()) ? nullptr : &it->second;
      if (lists[b]) longest = std::max(longest, lists[b]->size());
    }
    for (size_t r = 0; r < longest && c < m; ++r)
      for (int b = 0; b < L && c < m; ++b) {
        if (!lists[b] || r >= lists[b]->size()) continue;
        int32_t node = (*lists[b])[r];
        if (chosen[node]) continue;
        chosen[node] = 1;
        out[c++] = node;
      }
    for (int i = 0; i < n && c < m; ++i) {
      int32_t node = t->global_rank[i];
      if (chosen[node]) continue;
      chosen[node] = 1;
      out[c++] = node;
    }
    cnt[q] = c;
  }
  return 0;
}

// Selection when the hash nodes are always computed (Section 3.4: their pre-activations are
// forward-pass values that exist as soon as the keys do, so they cost nothing more; the text
// the authors left commented out there adds that the Node Activator therefore never selects
// them).  Reading taken: the active set is the H = K*L hash nodes, in sampled order, followed
// by the first max(m - H, 0) OTHER nodes in the merge order of so_select (a hash node met in
// a list or in the whole-set ranking is passed over); so |active| = max(m, H).  m == n still
// means every node in ascending id order.
int so_select_hash_first(const void* h, const uint32_t* keys, const float* keep, int64_t keep_stride,
                         int64_t N, const int32_t* hash_nodes, int32_t* active, int32_t* cnt,
                         int64_t stride) {
  const Tables* t = static_cast<const Tables*>(h);
  const int n = t->n, L = t->L, H = t->K * t->L;
  std::vector<uint8_t> chosen(n);
  for (int64_t q = 0; q < N; ++q) {
    const int32_t m = so_budget(keep[q * keep_stride], n);
    const int32_t total = std::max<int32_t>(m, H);
    if (total > stride) return -1;
    int32_t* out = active + q * stride;
    if (m == n) {
      for (int j = 0; j < n; ++j) out[j] = j;
      cnt[q] = n;
      continue;
    }
    std::fill(chosen.begin(), chosen.end(), 0);
    int32_t c = 0;
    for (int i = 0; i < H; ++i) {
      chosen[hash_nodes[i]] = 1;
      out[c++] = hash_nodes[i];
    }
    // rank r = 0, 1, ...; within a rank tables 0 .. L-1
    bool any = true;
    for (size_t r = 0; any && c < total; ++r) {
      any = false;
      for (int b = 0; b < L && c < total; ++b) {
        auto it = t->rank[b].find(keys[q * L + b]);
        if (it == t->rank[b].end() || r >= it->second.size()) continue;
        any = true;
        const int32_t node = it->second[r];
        if (chosen[node]) continue;
        chosen[node] = 1;
        out[c++] = node;
      }
    }
    for (int i = 0; i < n && c < total; ++i) {
      const int32_t node = t->global_rank[i];
      if (chosen[node]) continue;
      chosen[node] = 1;
      out[c++] = node;
    }
    cnt[q] = c;
  }
  return 0;
}

// Sparse layer: y_j = act(w_j.x + b_j) for the active nodes, exactly +0 for the rest.
// pre (nullable) receives the active nodes' pre-activations (0 elsewhere).  A softmax
// layer normalises over the active nodes only.
int so_sparse_layer(const void* W, int w_dtype, const float* bias, int d, int n, int act,
                    const float* X, int64_t N, const int32_t* active, const int32_t* cnt,
                    int64_t stride, float* pre, float* out, int threads) {
  parallel_for(N, threads, [&](int64_t q) {
    const float* x = X + q * d;
    float* o = out + q * n;
    for (int j = 0; j < n; ++j) o[j] = 0.0f;
    if (pre) for (int j = 0; j < n; ++j) pre[q * n + j] = 0.0f;
    const int32_t* ids = active + q * stride;
    for (int32_t t = 0; t < cnt[q]; ++t) {
      int32_t j = ids[t];
      float z = pre_activation(W, w_dtype, bias, d, j, x);
      if (pre) pre[q * n + j] = z;
      o[j] = (act == ACT_RELU) ? relu(z) : z;
    }
    if (act == ACT_SOFTMAX) softmax_over(ids, cnt[q], o);
  });
  return 0;
}

// First layer of a sparse-input model: x has nnz[q] non-zeros (col idx, value); the
// dot product visits them in stored order.  Weight (node j, input i) sits at j*d+i,
// or at i*n+j when rows_are_inputs is set (the transposed storage wide sparse-input
// layers use).
int so_dense_layer_ell(const void* W, int w_dtype, int rows_are_inputs, const float* bias, int d,
                       int n, int act,
                       const int32_t* idx, const float* val, const int32_t* nnz, int64_t ell_stride,
                       int64_t N, float* out, int threads) {
  std::vector<int32_t> all(n);
  for (int j = 0; j < n; ++j) all[j] = j;
  parallel_for(N, threads, [&](int64_t q) {
    float* o = out + q * n;
    for (int j = 0; j < n; ++j) {
      double s = 0.0;
      for (int32_t t = 0; t < nnz[q]; ++t)
      {
        int64_t i = idx[q * ell_stride + t];
        int64_t at = rows_are_inputs ? i * n + j : (int64_t)j * d + i;
        s += static_cast<double>(weight_at(W, w_dtype, at)) *
             static_cast<double>(val[q * ell_stride + t]);
      }
      s += static_cast<double>(bias[j]);
      float z = static_cast<float>(s);
      o[j] = (act == ACT_RELU) ? relu(z) : z;
    }
    if (act == ACT_SOFTMAX) softmax_over(all.data(), n, o);
  });
  return 0;
}

// ---------------------------------------------------------------------------
// Choice of k per query (Section 2: ACLO and LCAO; Section 3.2: Confidence LSH tables and
// latency profiles).  Mechanics only: the confidences c(k, x') of the training inputs and
// the latency profile T(k, beta) are inputs.
// ---------------------------------------------------------------------------

// Confidence LSH tables: per table and bucket, the sum over the training inputs hashed
// there of c(k_g, x') for every k_g of the grid, and how many inputs that is.
struct ConfTables {
  int K = 0, L = 0, G = 0;
  int64_t N = 0;
  std::vector<std::unordered_map<uint32_t, std::vector<double>>> sum;   // [b][key] -> G sums
  std::vector<std::unordered_map<uint32_t, int64_t>> count;             // [b][key]
  std::vector<double> total;                                             // G sums over all inputs
};

// Training: every input x' (in order) adds c(k_g, x') to its bucket in each table.
void* so_conf_build(int K, int L, int G, const uint32_t* keys, const float* conf, int64_t N) {
  ConfTables* t = new ConfTables;
  t->K = K; t->L = L; t->G = G; t->N = N;
  t->sum.resize(L); t->count.resize(L);
  t->total.assign(G, 0.0);
  for (int64_t x = 0; x < N; ++x) {
    for (int b = 0; b < L; ++b) {
      const uint32_t key = keys[x * L + b];
      auto it = t->sum[b].find(key);
      if (it == t->sum[b].end()) it = t->sum[b].emplace(key, std::vector<double>(G, 0.0)).first;
      for (int g = 0; g < G; ++g) it->second[g] += static_cast<double>(conf[x * G + g]);
      t->count[b][key] += 1;
    }
    for (int g = 0; g < G; ++g) t->total[g] += static_cast<double>(conf[x * G + g]);
  }
  return t;
}

void so_conf_free(void* h) { delete static_cast<ConfTables*>(h); }

// Eq. 4 with the arithmetic mean as aggregation: c_hat(k_g, x) = mean of c(k_g, x') over the
// training inputs x' that share a bucket with x.  Reading taken for L tables: LSH(x) is the
// union of x's L buckets with multiplicity (an input that shares several buckets with x
// counts once per bucket), i.e. (sum over tables of the bucket sums) / (sum over tables of
// the bucket counts), tables visited in order.  With no bucket-mate at all the mean over the
// whole training set stands in.  mates (nullable) receives the denominator.
int so_conf_estimate(const void* h, const uint32_t* keys, int64_t Q, double* chat, int64_t* mates) {
  const ConfTables* t = static_cast<const ConfTables*>(h);
  const int L = t->L, G = t->G;
  std::vector<double> s(G);
  for (int64_t q = 0; q < Q; ++q) {
    std::fill(s.begin(), s.end(), 0.0);
    int64_t c = 0;
    for (int b = 0; b < L; ++b) {
      auto it = t->sum[b].find(keys[q * L + b]);
      if (it == t->sum[b].end()) continue;
      for (int g = 0; g < G; ++g) s[g] += it->second[g];
      c += t->count[b].at(keys[q * L + b]);
    }
    for (int g = 0; g < G; ++g)
      chat[q * G + g] = c > 0 ? s[g] / static_cast<double>(c) : t->total[g] / static_cast<double>(t->N);
    if (mates) mates[q] = c;
  }
  return 0;
}

// ACLO (Section 2.2): minimise k subject to the accuracy constraint.  The constraint reaches
// this code as a confidence threshold thr[q] (the calibration that ties a threshold to an
// accuracy on held-out data is outside): the answer is the smallest k of the ascending grid
// whose estimated confidence is at least the threshold; if none qualifies, the largest k.
int so_choose_aclo(const void* h, const uint32_t* keys, int64_t Q, const float* k_grid, const float* thr,
                   int64_t thr_stride, float* keep_out, int32_t* g_out) {
  const ConfTables* t = static_cast<const ConfTables*>(h);
  const int G = t->G;
  std::vector<double> chat(G);
  for (int64_t q = 0; q < Q; ++q) {
    so_conf_estimate(h, keys + q * t->L, 1, chat.data(), nullptr);
    int pick = G - 1;
    for (int g = 0; g < G; ++g)
      if (chat[g] >= static_cast<double>(thr[q * thr_stride])) { pick = g; break; }
    keep_out[q] = k_grid[pick];
    if (g_out) g_out[q] = pick;
  }
  return 0;
}

// LCAO (Section 2.3): maximise k subject to t0 + T(k, beta) <= tau.  T is the latency
// profile [n_beta][G] (row beta[q] = the machine's current co-location state).  If no k of
// the grid fits, the SLO cannot be met: the smallest k is returned and violated[q] is set.
int so_choose_lcao(const float* k_grid, int G, const float* T, int n_beta, const float* tau,
                   const float* t0, const int32_t* beta, int64_t Q, float* keep_out, int32_t* g_out,
                   uint8_t* violated) {
  for (int64_t q = 0; q < Q; ++q) {
    if (beta[q] < 0 || beta[q] >= n_beta) return -1;
    const float* row = T + static_cast<int64_t>(beta[q]) * G;
    int pick = -1;
    for (int g = 0; g < G; ++g)
      if (static_cast<double>(t0[q]) + static_cast<double>(row[g]) <= static_cast<double>(tau[q])) pick = g;
    if (violated) violated[q] = pick < 0 ? 1 : 0;
    if (pick < 0) pick = 0;
    keep_out[q] = k_grid[pick];
    if (g_out) g_out[q] = pick;
  }
  return 0;
}

// Prediction: the computed node with the largest output, lowest id on equal values.
// ids == nullptr means every node was computed.
int so_argmax(const float* out, int n, int64_t N, const int32_t* active, const int32_t* cnt,
              int64_t stride, int32_t* pred) {
  for (int64_t q = 0; q < N; ++q) {
    int32_t best = -1;
    float bv = 0.0f;
    int32_t c = active ? cnt[q] : n;
    for (int32_t t = 0; t < c; ++t) {
      int32_t j = active ? active[q * stride + t] : t;
      float v = out[q * n + j];
      if (best < 0 || v > bv || (v == bv && j < best)) { best = j; bv = v; }
    }
    pred[q] = best;
  }
  return 0;
}

}  // extern "C"
