// Node Activator training on the device (Alg. 1, Section 3.2).  For one layer:
//   keys       every training input is hashed into one bucket of each of the L tables;
//   NodeScore  per bucket, the layer's output activations of its inputs are summed
//              (double, in training-set order, so repeated builds are bit-identical);
//   Rank       per bucket, nodes with a positive sum sorted from the highest sum to the
//              lowest (equal sums: lower id first), truncated to list_cap;
//   fallback   the same ranking over the sums of all inputs (all n nodes).
// This is set-up work and is not timed; it favours determinism and small code.
#include <algorithm>

#include "bucket_lists.h"
#include "slonn_internal.h"

namespace slonn {
namespace {

constexpr int SORT_MAX = 8192;   // largest layer the LDS sort handles

__global__ void keys_kernel(const float* __restrict__ Z, int K, int L, int64_t N,
                            uint32_t* __restrict__ keys) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // (input, table)
  if (e >= N * L) return;
  const float* z = Z + e * K;      // Z is [N][L*K]: entry e = x*L + b starts at (x*L + b)*K
  uint32_t key = 0;
  for (int j = 0; j < K; ++j) key |= (z[j] > 0.0f ? 1u : 0u) << j;
  keys[e] = key;
}

// NodeScore[key][j] = sum of act[x][j] over the bucket's members, in order.  accumulate != 0
// (online refresh): the sums continue from the kept NodeScore, and buckets without new members
// are left as they are (npos[key] must have been cleared for the others).
__global__ void node_score_kernel(const float* __restrict__ act, int n, const uint32_t* __restrict__ start,
                                  const uint32_t* __restrict__ members, double* __restrict__ score,
                                  uint32_t* __restrict__ npos, int accumulate) {
  const int key = blockIdx.y;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  uint32_t i = start[key];
  const uint32_t end = start[key + 1];
  if (accumulate && i == end) return;
  double s = accumulate ? score[(size_t)key * n + j] : 0.0;
  for (; i + 8 <= end; i += 8) {        // eight loads in flight, added in input order
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = act[(size_t)members[i + u] * n + j];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += (double)v[u];
  }
  for (; i < end; ++i) s += (double)act[(size_t)members[i] * n + j];
  score[(size_t)key * n + j] = s;
  if (s > 0.0) atomicAdd(&npos[key], 1u);
}

__global__ void total_score_kernel(const float* __restrict__ act, int n, int64_t N,
                                   double* __restrict__ score, int accumulate) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  double s = accumulate ? score[j] : 0.0;
  int64_t x = 0;
  for (; x + 8 <= N; x += 8) {          // eight loads in flight, added in input order
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = act[(x + u) * n + j];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += (double)v[u];
  }
  for (; x < N; ++x) s += (double)act[x * n + j];
  score[j] = s;
}

// List lengths and places of one table: len[k] = min(npos[k], cap), off[k] = running offset
// into the id array (continuing from *base, which is advanced by the table's total), and the
// table's directory row dir[0..nb].  One workgroup.
__global__ __launch_bounds__(256) void layout_kernel(const uint32_t* __restrict__ npos, int nb, uint32_t cap,
                                                    uint32_t* __restrict__ base, uint32_t* __restrict__ off,
                                                    uint32_t* __restrict__ len, uint32_t* __restrict__ dir) {
  __shared__ uint32_t wsum[4];
  __shared__ uint32_t carry_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) carry_s = base[0];
  __syncthreads();
  for (int k0 = 0; k0 < nb; k0 += 256) {
    const int k = k0 + tid;
    const uint32_t v = k < nb ? min(npos[k], cap) : 0u;
    uint32_t incl = v;
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    uint32_t before = carry_s;
    for (int w = 0; w < wave; ++w) before += wsum[w];
    if (k < nb) { len[k] = v; off[k] = before + incl - v; dir[k] = before + incl - v; }
    __syncthreads();
    if (tid == 0) carry_s += wsum[0] + wsum[1] + wsum[2] + wsum[3];
    __syncthreads();
  }
  if (tid == 0) { dir[nb] = carry_s; base[0] = carry_s; }
}

// number of non-empty buckets over all tables
__global__ void count_nonempty_kernel(const uint32_t* __restrict__ hist, int64_t cells, unsigned long long* out) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool ne = e < cells && hist[e] != 0u;
  const unsigned long long votes = __ballot(ne);
  if ((threadIdx.x & 63) == 0 && votes) atomicAdd(out, (unsigned long long)__popcll(votes));
}

__device__ __forceinline__ bool ranks_before(int a, int b, const double* sc) {
  // -1 marks an absent entry and sorts last
  if (a < 0) return false;
  if (b < 0) return true;
  const double sa = sc[a], sb = sc[b];
  return sa > sb || (sa == sb && a < b);
}

__device__ __forceinline__ bool pair_before(double sa, int a, double sb, int b) {
  if (a < 0) return false;
  if (b < 0) return true;
  return sa > sb || (sa == sb && a < b);
}

// Bitonic sort of one bucket's (score, node id) pairs in LDS (12 bytes per node: P doubles,
// then P ids).  positive_only: nodes with a sum <= 0 are left out.  Writes the first
// out_len[bucket] ids at out + out_off[bucket].
// members (nullable): start offsets of the buckets' new member lists; a bucket without new members
// (members[bucket] == members[bucket + 1]) is skipped (online refresh copies its old list instead).
__global__ __launch_bounds__(256) void rank_kernel(const double* __restrict__ score, int n, int P,
                                                  int positive_only, const uint32_t* __restrict__ out_off,
                                                  const uint32_t* __restrict__ out_len,
                                                  int32_t* __restrict__ out, const uint32_t* __restrict__ members) {
  extern __shared__ __align__(16) unsigned char rank_smem[];
  double* key = reinterpret_cast<double*>(rank_smem);
  int32_t* ids = reinterpret_cast<int32_t*>(key + P);
  const int bucket = blockIdx.x;
  const uint32_t len = out_len[bucket];
  if (len == 0) return;
  if (members && members[bucket] == members[bucket + 1]) return;
  const double* sc = score + (size_t)bucket * n;
  for (int i = threadIdx.x; i < P; i += 256) {
    int v = -1;
    double sv = 0.0;
    if (i < n) {
      sv = sc[i];
      if (!positive_only || sv > 0.0) v = i;
    }
    ids[i] = v;
    key[i] = sv;
  }
  __syncthreads();
  for (int k = 2; k <= P; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = threadIdx.x; t < (P >> 1); t += 256) {
        // t-th pair of this stage: i has bit j clear
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int p = i | j;
        const int a = ids[i], b = ids[p];
        const double sa = key[i], sb = key[p];
        const bool up = (i & k) == 0;          // ascending block: best first
        const bool swap = up ? pair_before(sb, b, sa, a) : pair_before(sa, a, sb, b);
        if (swap) { ids[i] = b; ids[p] = a; key[i] = sb; key[p] = sa; }
      }
      __syncthreads();
    }
  }
  int32_t* dst = out + out_off[bucket];
  for (uint32_t i = threadIdx.x; i < len; i += 256) dst[i] = ids[i];
}

// Layers wider than the LDS sort: only the best out_len[bucket] <= SORT_MAX nodes of a
// bucket are wanted, so a score threshold is estimated from a sorted strided sample, checked
// (and moved if needed) by counting passes over the bucket's scores, the nodes at or above it
// are compacted into LDS in id order, sorted there with the exact (score, id) comparison and
// the head of the result is written out.  fail[0] is set if no threshold isolates between
// out_len and SORT_MAX candidates (masses of exactly equal scores).
constexpr int SAMPLE = 4096;

__device__ __forceinline__ int block_count_ge(const double* sc, int n, double thr, int* red) {
  int c = 0;
  for (int i = threadIdx.x; i < n; i += 256) c += (sc[i] >= thr && sc[i] > 0.0) ? 1 : 0;
  for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = c;
  __syncthreads();
  const int total = red[0] + red[1] + red[2] + red[3];
  __syncthreads();
  return total;
}

__global__ __launch_bounds__(256) void rank_wide_kernel(const double* __restrict__ score, int n,
                                                       const uint32_t* __restrict__ out_off,
                                                       const uint32_t* __restrict__ out_len,
                                                       int32_t* __restrict__ out, int* __restrict__ fail,
                                                       const uint32_t* __restrict__ members) {
  __shared__ double samp[SAMPLE];          // 32 KB, reused as the candidate id buffer
  __shared__ int red[8];
  int32_t* ids = reinterpret_cast<int32_t*>(samp);
  const int bucket = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int len = (int)out_len[bucket];
  if (len == 0) return;
  if (members && members[bucket] == members[bucket + 1]) return;
  const double* sc = score + (size_t)bucket * n;

  // threshold: start from the sample value whose rank predicts about four times len candidates
  for (int i = tid; i < SAMPLE; i += 256) samp[i] = sc[(size_t)i * n / SAMPLE];
  __syncthreads();
  for (int k = 2; k <= SAMPLE; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < (SAMPLE >> 1); t += 256) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1)), p = i | j;
        const double a = samp[i], b = samp[p];
        const bool up = (i & k) == 0;                       // descending order overall
        if (up ? (b > a) : (a > b)) { samp[i] = b; samp[p] = a; }
      }
      __syncthreads();
    }
  int r = (int)((4.0 * len * SAMPLE) / n) + 16;
  if (r > SAMPLE - 1) r = SAMPLE - 1;
  double thr = samp[r];
  int lo = 0, hi = SAMPLE - 1;                              // bracket of sample ranks still possible
  int total = 0;
  for (int it = 0; it < 14; ++it) {
    total = block_count_ge(sc, n, thr, red);
    if (total >= len && total <= SORT_MAX) break;
    if (total < len) lo = r + 1; else hi = r - 1;
    if (lo > hi) break;
    r = (total < len) ? min(hi, 2 * r + 32) : max(lo, r / 2);
    if (r < lo) r = lo;
    if (r > hi) r = hi;
    thr = samp[r];
  }
  if (total < len) {                                        // the whole sample is above: take every positive
    thr = 0.0;
    total = block_count_ge(sc, n, thr, red);
  }
  if (total < len || total > SORT_MAX) {
    if (tid == 0) atomicExch(fail, 1);
    return;
  }
  __syncthreads();                                          // the sample is no longer needed

  // compact candidates in id order: ballot + prefix within a wave, wave totals through LDS
  int P = 1;
  while (P < total) P <<= 1;
  if (P < 2) P = 2;
  for (int i = tid; i < P; i += 256) ids[i] = -1;
  __syncthreads();
  int base = 0;
  for (int i0 = 0; i0 < n; i0 += 256) {
    const int i = i0 + tid;
    const bool take = i < n && sc[i] >= thr && sc[i] > 0.0;
    const unsigned long long votes = __ballot(take);
    if (lane == 0) red[wave] = __popcll(votes);
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wave; ++w) before += red[w];
    const int all = red[0] + red[1] + red[2] + red[3];
    if (take) ids[base + before + __popcll(votes & ((lane == 0) ? 0ull : (~0ull >> (64 - lane))))] = i;
    base += all;
    __syncthreads();
  }
  // exact ordering of the candidates
  for (int k = 2; k <= P; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < (P >> 1); t += 256) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1)), p = i | j;
        const int a = ids[i], b = ids[p];
        const bool up = (i & k) == 0;
        const bool swap = up ? ranks_before(b, a, sc) : ranks_before(a, b, sc);
        if (swap) { ids[i] = b; ids[p] = a; }
      }
      __syncthreads();
    }
  int32_t* dst = out + out_off[bucket];
  for (int i = tid; i < len; i += 256) dst[i] = ids[i];
}

// buckets that received new members start again from no positive node (online refresh)
__global__ void clear_touched_npos_kernel(const uint32_t* __restrict__ start, int nb, uint32_t* __restrict__ npos) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k < nb && start[k] != start[k + 1]) npos[k] = 0u;
}

// 4-byte ids <-> the 2-byte ids that layers of up to 65 536 nodes store
__global__ void narrow_ids_kernel(const int32_t* __restrict__ src, uint16_t* __restrict__ dst, size_t count) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) dst[i] = (uint16_t)src[i];
}
__global__ void widen_ids_kernel(const uint16_t* __restrict__ src, int32_t* __restrict__ dst, size_t count) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) dst[i] = (int32_t)src[i];
}

// Online refresh: a bucket without new members keeps its list; it moves to its new place in the
// id array (old_dir: the table's old directory row; its length has not changed).
template <typename IdT>
__global__ __launch_bounds__(256) void copy_untouched_lists_kernel(const uint32_t* __restrict__ start,
                                                                  const uint32_t* __restrict__ old_dir,
                                                                  const IdT* __restrict__ old_ids,
                                                                  const uint32_t* __restrict__ off,
                                                                  const uint32_t* __restrict__ len,
                                                                  int32_t* __restrict__ out) {
  const int bucket = blockIdx.x;
  if (start[bucket] != start[bucket + 1]) return;
  const uint32_t l = len[bucket], from = old_dir[bucket], to = off[bucket];
  for (uint32_t i = threadIdx.x; i < l; i += 256) out[to + i] = (int32_t)old_ids[from + i];
}

template <class T>
struct DevBuf {
  T* p = nullptr;
  ~DevBuf() { if (p) (void)hipFree(p); }
  hipError_t alloc(size_t count) { return hipMalloc(&p, std::max<size_t>(count, 1) * sizeof(T)); }
  T* release() { T* q = p; p = nullptr; return q; }
};

}  // namespace

void free_table_set(TableSet* ts) {
  if (ts->d_dir) (void)hipFree(ts->d_dir);
  if (ts->d_ids) (void)hipFree(ts->d_ids);
  if (ts->d_global_rank) (void)hipFree(ts->d_global_rank);
  if (ts->d_score) (void)hipFree(ts->d_score);
  if (ts->d_global_score) (void)hipFree(ts->d_global_score);
  if (ts->d_npos) (void)hipFree(ts->d_npos);
  ts->d_dir = nullptr; ts->d_ids = nullptr; ts->d_global_rank = nullptr;
  ts->d_score = nullptr; ts->d_global_score = nullptr; ts->d_npos = nullptr;
}

int upload_table_set(TableSet* ts, const int32_t* d_ids_src) {
  if (!d_ids_src) ts->n_ids = ts->ids.size();
  // layers of up to 65 536 nodes keep their lists as 2-byte ids: half the table memory and half
  // the bytes a query's merge reads
  ts->narrow = ts->n <= 65536;
  SLONN_HIP(hipMalloc(&ts->d_dir, std::max<size_t>(ts->dir.size(), 1) * 4));
  SLONN_HIP(hipMalloc(&ts->d_ids, std::max<size_t>(ts->n_ids, 1) * (ts->narrow ? 2 : 4)));
  SLONN_HIP(hipMalloc(&ts->d_global_rank, std::max<size_t>(ts->global_rank.size(), 1) * 4));
  SLONN_HIP(hipMemcpy(ts->d_dir, ts->dir.data(), ts->dir.size() * 4, hipMemcpyHostToDevice));
  if (ts->n_ids && !ts->narrow) {
    SLONN_HIP(hipMemcpy(ts->d_ids, d_ids_src ? d_ids_src : ts->ids.data(), ts->n_ids * 4,
                        d_ids_src ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice));
  } else if (ts->n_ids && d_ids_src) {
    hipLaunchKernelGGL(narrow_ids_kernel, dim3((unsigned)((ts->n_ids + 255) / 256)), dim3(256), 0, nullptr, d_ids_src,
                       static_cast<uint16_t*>(ts->d_ids), ts->n_ids);
    SLONN_HIP(hipGetLastError());
    SLONN_HIP(hipStreamSynchronize(nullptr));
  } else if (ts->n_ids) {
    std::vector<uint16_t> small(ts->n_ids);
    for (size_t i = 0; i < ts->n_ids; ++i) small[i] = (uint16_t)ts->ids[i];
    SLONN_HIP(hipMemcpy(ts->d_ids, small.data(), ts->n_ids * 2, hipMemcpyHostToDevice));
  }
  std::vector<int32_t>().swap(ts->ids);        // the lists live on the device from here on
  SLONN_HIP(hipMemcpy(ts->d_global_rank, ts->global_rank.data(), ts->global_rank.size() * 4,
                      hipMemcpyHostToDevice));
  return SLONN_OK;
}

int download_ids(const TableSet* ts, int32_t* host_out) {
  if (!ts->n_ids) return SLONN_OK;
  if (!ts->narrow) {
    SLONN_HIP(hipMemcpy(host_out, ts->d_ids, ts->n_ids * 4, hipMemcpyDeviceToHost));
    return SLONN_OK;
  }
  // widened on the device through a staging buffer, 64 Mi ids at a time
  const size_t step = std::min<size_t>(ts->n_ids, (size_t)64 << 20);
  DevBuf<int32_t> stage;
  SLONN_HIP(stage.alloc(step));
  const uint16_t* src = static_cast<const uint16_t*>(ts->d_ids);
  for (size_t at = 0; at < ts->n_ids; at += step) {
    const size_t c = std::min(step, ts->n_ids - at);
    hipLaunchKernelGGL(widen_ids_kernel, dim3((unsigned)((c + 255) / 256)), dim3(256), 0, nullptr, src + at, stage.p, c);
    SLONN_HIP(hipGetLastError());
    SLONN_HIP(hipMemcpy(host_out + at, stage.p, c * 4, hipMemcpyDeviceToHost));
  }
  return SLONN_OK;
}

// Alg. 1 for one layer on N training inputs X_l (act: the layer's own output for them).
// refresh == false: from nothing.  refresh == true: ts holds the NodeScore sums of the inputs seen
// so far (tables trained with slonn_model_set_tables_refreshable); the new inputs are added to
// the buckets they hit and to the whole-set sums, every running sum continued in input order, the
// touched buckets and the whole-set ranking are sorted again, the other lists are copied.
int build_layer_tables(const slonn_model* m, int layer, const float* X_l, int64_t N, const float* act,
                       TableSet* ts, bool refresh, hipStream_t s) {
  const Layer& Ly = m->layers[layer];
  const int n = Ly.d_out, K = Ly.K, L = Ly.L, H = Ly.H();
  const bool wide = n > SORT_MAX;
  if (N <= 0 || N > 0x7FFFFFFF) SLONN_FAIL(SLONN_EINVAL, "build: bad training-set size");
  const int nb = 1 << K;
  int P = 1;
  while (P < n) P <<= 1;
  if (P < 2) P = 2;
  const int cap = std::min(Ly.list_cap, n);
  // wide layers rank the head of each bucket through a threshold when the lists are short enough
  // for an LDS sort of the candidates, otherwise (and when masses of equal sums defeat the
  // threshold) through a radix sort of the whole bucket
  bool use_sort = wide && cap > SORT_MAX;
  const size_t rank_lds = (size_t)P * 12;           // (score, id) pairs of the LDS sort
  if (!wide && rank_lds > 65536)
    SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(rank_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)rank_lds));
  const bool keep = refresh || m->tables_refreshable;
  if (refresh && (!ts->d_score || !ts->d_npos || !ts->d_global_score))
    SLONN_FAIL(SLONN_EUNSUPPORTED, "refresh: the tables of layer %d hold no NodeScore sums", layer);

  if (!refresh) {
    ts->layer = layer; ts->K = K; ts->L = L; ts->n = n; ts->list_cap = Ly.list_cap;
    ts->dir.assign((size_t)L * (nb + 1), 0);
    ts->ids.clear();
    ts->global_rank.assign(n, 0);
    ts->nonempty = 0;
  }

  DevBuf<float> Z;
  DevBuf<uint32_t> keys, hist, start, cursor, members, npos_tmp, off, len, dir, base;
  DevBuf<unsigned long long> nonempty;
  DevBuf<double> score_tmp, gscore_tmp;
  DevBuf<int32_t> out, gr;
  DevBuf<int> fail;
  SLONN_HIP(fail.alloc(1));
  SLONN_HIP(hipMemsetAsync(fail.p, 0, sizeof(int), s));
  SLONN_HIP(Z.alloc((size_t)N * H));
  SLONN_HIP(keys.alloc((size_t)N * L));
  SLONN_HIP(hist.alloc((size_t)L * nb));
  SLONN_HIP(start.alloc((size_t)L * (nb + 1)));
  SLONN_HIP(cursor.alloc((size_t)L * nb));
  SLONN_HIP(members.alloc((size_t)L * N));
  SLONN_HIP(off.alloc(nb));
  SLONN_HIP(len.alloc(nb));
  SLONN_HIP(dir.alloc((size_t)L * (nb + 1)));
  SLONN_HIP(base.alloc(1));
  SLONN_HIP(nonempty.alloc(1));
  SLONN_HIP(gr.alloc(n));
  double* score = nullptr;       // [L][nb][n] when kept, else [nb][n] reused by every table
  uint32_t* npos = nullptr;      // [L][nb]
  double* gscore = nullptr;      // [n]
  if (keep) {
    if (!refresh) {
      hipError_t e = hipMalloc(&ts->d_score, (size_t)L * nb * n * sizeof(double));
      if (e == hipSuccess) e = hipMalloc(&ts->d_npos, (size_t)L * nb * 4);
      if (e == hipSuccess) e = hipMalloc(&ts->d_global_score, (size_t)n * sizeof(double));
      if (e != hipSuccess) {
        (void)hipGetLastError();
        SLONN_FAIL(SLONN_ENOMEM, "build: layer %d: the NodeScore sums kept for online refresh need %zu bytes", layer,
                   (size_t)L * nb * n * sizeof(double));
      }
    }
    score = ts->d_score; npos = ts->d_npos; gscore = ts->d_global_score;
  } else {
    SLONN_HIP(score_tmp.alloc((size_t)nb * n));
    SLONN_HIP(npos_tmp.alloc((size_t)L * nb));
    SLONN_HIP(gscore_tmp.alloc(n));
    score = score_tmp.p; npos = npos_tmp.p; gscore = gscore_tmp.p;
  }

  int rc = launch_hash_project(X_l, Ly.d_in, Ly.Wh, Ly.bh, Z.p, (int)N, H, Ly.d_in, nullptr, nullptr, s);
  if (rc) return rc;
  const int64_t tot_keys = N * L;
  hipLaunchKernelGGL(keys_kernel, dim3((unsigned)((tot_keys + 255) / 256)), dim3(256), 0, s, Z.p, K, L, N, keys.p);
  SLONN_HIP(hipGetLastError());

  // bucket member lists of all L tables at once
  SLONN_HIP(hipMemsetAsync(hist.p, 0, (size_t)L * nb * 4, s));
  SLONN_HIP(hipMemsetAsync(nonempty.p, 0, 8, s));
  hipLaunchKernelGGL(bucket_hist_kernel, dim3((unsigned)((tot_keys + 255) / 256)), dim3(256), 0, s, keys.p, N, L, nb,
                     hist.p);
  SLONN_HIP(hipGetLastError());
  hipLaunchKernelGGL(bucket_scan_kernel, dim3(L), dim3(256), 0, s, hist.p, nb, start.p, cursor.p);
  SLONN_HIP(hipGetLastError());
  hipLaunchKernelGGL(bucket_members_kernel, dim3(L), dim3(64), 0, s, keys.p, N, L, K, nb, cursor.p, members.p);
  SLONN_HIP(hipGetLastError());
  const int64_t cells = (int64_t)L * nb;
  hipLaunchKernelGGL(count_nonempty_kernel, dim3((unsigned)((cells + 255) / 256)), dim3(256), 0, s, hist.p, cells,
                     nonempty.p);
  SLONN_HIP(hipGetLastError());
  // every bucket with a list keeps at most cap ids: size the id array once, for all tables (after a
  // refresh: the buckets that had a list before plus the buckets the new inputs hit)
  unsigned long long h_nonempty = 0;
  SLONN_HIP(hipMemcpyAsync(&h_nonempty, nonempty.p, 8, hipMemcpyDeviceToHost, s));
  SLONN_HIP(hipStreamSynchronize(s));
  const unsigned long long id_bound =
      std::min<unsigned long long>(h_nonempty + (refresh ? ts->nonempty : 0), (unsigned long long)cells) *
      (unsigned long long)cap;
  if (id_bound > 0xFFFFFFFFull)
    SLONN_FAIL(SLONN_EUNSUPPORTED, "build: layer %d: up to %llu list entries do not fit 32-bit offsets", layer,
               id_bound);
  SLONN_HIP(out.alloc((size_t)id_bound));

  // per table: NodeScore sums, list lengths and places, ranking -- no host round trip
  auto run_tables = [&](bool sums, bool by_sort) -> int {
    SLONN_HIP(hipMemsetAsync(base.p, 0, 4, s));
    if (sums && !refresh) SLONN_HIP(hipMemsetAsync(npos, 0, (size_t)L * nb * 4, s));
    for (int b = 0; b < L; ++b) {
      const uint32_t* st = start.p + (size_t)b * (nb + 1);
      double* sc = keep ? score + (size_t)b * nb * n : score;
      uint32_t* np_b = npos + (size_t)b * nb;
      if (sums) {
        if (refresh) {
          hipLaunchKernelGGL(clear_touched_npos_kernel, dim3((nb + 255) / 256), dim3(256), 0, s, st, nb, np_b);
          SLONN_HIP(hipGetLastError());
        }
        hipLaunchKernelGGL(node_score_kernel, dim3((n + 255) / 256, nb), dim3(256), 0, s, act, n, st,
                           members.p + (size_t)b * N, sc, np_b, refresh ? 1 : 0);
        SLONN_HIP(hipGetLastError());
      }
      hipLaunchKernelGGL(layout_kernel, dim3(1), dim3(256), 0, s, np_b, nb, (uint32_t)cap, base.p, off.p, len.p,
                         dir.p + (size_t)b * (nb + 1));
      SLONN_HIP(hipGetLastError());
      const uint32_t* only = refresh ? st : nullptr;      // a refresh ranks the buckets with new members
      if (by_sort) {
        const int rc2 = rank_by_sort(sc, n, nb, off.p, len.p, only, out.p, s);
        if (rc2) return rc2;
      } else if (wide) {
        hipLaunchKernelGGL(rank_wide_kernel, dim3(nb), dim3(256), 0, s, sc, n, off.p, len.p, out.p, fail.p, only);
      } else {
        hipLaunchKernelGGL(rank_kernel, dim3(nb), dim3(256), rank_lds, s, sc, n, P, 1, off.p, len.p, out.p, only);
      }
      SLONN_HIP(hipGetLastError());
      if (refresh) {
        if (ts->narrow)
          hipLaunchKernelGGL(copy_untouched_lists_kernel<uint16_t>, dim3(nb), dim3(256), 0, s, st,
                             ts->d_dir + (size_t)b * (nb + 1), static_cast<const uint16_t*>(ts->d_ids), off.p, len.p,
                             out.p);
        else
          hipLaunchKernelGGL(copy_untouched_lists_kernel<int32_t>, dim3(nb), dim3(256), 0, s, st,
                             ts->d_dir + (size_t)b * (nb + 1), static_cast<const int32_t*>(ts->d_ids), off.p, len.p,
                             out.p);
        SLONN_HIP(hipGetLastError());
      }
    }
    return SLONN_OK;
  };
  rc = run_tables(true, use_sort);
  if (rc) return rc;
  if (wide && !use_sort) {
    int h_fail = 0;
    SLONN_HIP(hipMemcpyAsync(&h_fail, fail.p, sizeof(int), hipMemcpyDeviceToHost, s));
    SLONN_HIP(hipStreamSynchronize(s));
    if (h_fail) {
      // some bucket holds so many exactly equal sums that no threshold isolates the head of its
      // list: rank every bucket by a full sort instead (equal sums fall in ascending id order).
      // Kept sums are final already; sums in the per-table buffer are formed again.
      use_sort = true;
      rc = run_tables(!keep, true);
      if (rc) return rc;
    }
  }
  uint32_t h_total = 0;
  std::vector<uint32_t> h_dir((size_t)L * (nb + 1));
  SLONN_HIP(hipMemcpyAsync(&h_total, base.p, 4, hipMemcpyDeviceToHost, s));
  SLONN_HIP(hipMemcpyAsync(h_dir.data(), dir.p, (size_t)L * (nb + 1) * 4, hipMemcpyDeviceToHost, s));

  // whole-set ranking: every node, zero sums included
  hipLaunchKernelGGL(total_score_kernel, dim3((n + 255) / 256), dim3(256), 0, s, act, n, N, gscore, refresh ? 1 : 0);
  SLONN_HIP(hipGetLastError());
  const uint32_t zero = 0, all = (uint32_t)n;
  SLONN_HIP(hipMemcpyAsync(off.p, &zero, 4, hipMemcpyHostToDevice, s));
  SLONN_HIP(hipMemcpyAsync(len.p, &all, 4, hipMemcpyHostToDevice, s));
  if (wide) {
    rc = rank_by_sort(gscore, n, 1, off.p, len.p, nullptr, gr.p, s);
    if (rc) return rc;
  } else {
    hipLaunchKernelGGL(rank_kernel, dim3(1), dim3(256), rank_lds, s, gscore, n, P, 0, off.p, len.p, gr.p, nullptr);
    SLONN_HIP(hipGetLastError());
  }
  std::vector<int32_t> h_gr(n);
  SLONN_HIP(hipMemcpyAsync(h_gr.data(), gr.p, (size_t)n * 4, hipMemcpyDeviceToHost, s));
  SLONN_HIP(hipStreamSynchronize(s));

  // publish: directory, lists (they stay on the device; export copies them out), ranking
  ts->dir.swap(h_dir);
  ts->global_rank.swap(h_gr);
  ts->n_ids = h_total;
  ts->nonempty = 0;
  for (int b = 0; b < L; ++b)
    for (int k = 0; k < nb; ++k)
      if (ts->dir[(size_t)b * (nb + 1) + k + 1] > ts->dir[(size_t)b * (nb + 1) + k]) ++ts->nonempty;
  ts->n_trained += N;
  if (ts->d_dir) (void)hipFree(ts->d_dir);
  if (ts->d_ids) (void)hipFree(ts->d_ids);
  if (ts->d_global_rank) (void)hipFree(ts->d_global_rank);
  ts->d_dir = nullptr; ts->d_ids = nullptr; ts->d_global_rank = nullptr;
  return upload_table_set(ts, out.p);
}

}  // namespace slonn

using namespace slonn;

namespace slonn {
namespace {

int check_training_input(const slonn_model* m, const slonn_input* X, int64_t N) {
  if (!m || !X) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (N <= 0 || N > SLONN_MAX_BATCH) SLONN_FAIL(SLONN_EINVAL, "N must be in 1 .. %d", SLONN_MAX_BATCH);
  if (X->format == SLONN_DENSE) {
    if (!X->x) SLONN_FAIL(SLONN_EINVAL, "dense input pointer is null");
    if (m->layers[0].w_layout != SLONN_ROWS_ARE_NODES)
      SLONN_FAIL(SLONN_EUNSUPPORTED, "dense input needs a node-major first layer");
  } else if (X->format == SLONN_ELL) {
    if (!X->idx || !X->val || !X->nnz || X->ell_stride <= 0)
      SLONN_FAIL(SLONN_EINVAL, "ELL input needs idx, val, nnz and a positive ell_stride");
    if (m->layers[0].activated())
      SLONN_FAIL(SLONN_EUNSUPPORTED, "a Node Activator on a sparse-input first layer is not supported");
  } else {
    SLONN_FAIL(SLONN_EINVAL, "unknown input format %d", X->format);
  }
  return SLONN_OK;
}

// The full network on the training inputs, layer by layer (Input_l is the full network's output
// of layer l-1); every activated layer trains (refresh == false) or refreshes its tables.
int train_tables(const slonn_model* m, slonn_tables* t, const slonn_input* X, int64_t N, bool refresh,
                 hipStream_t s) {
  const int nl = (int)m->layers.size();
  int last_needed = -1;
  for (int l = 0; l < nl; ++l)
    if (m->layers[l].activated()) last_needed = l;
  float* prev = nullptr;
  const float* cur = X->x;
  int rc = SLONN_OK;
  for (int l = 0; l <= last_needed && rc == SLONN_OK; ++l) {
    const Layer& L = m->layers[l];
    float* act = nullptr;
    hipError_t e = hipMalloc(&act, (size_t)N * L.d_out * 4);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      set_error("build: cannot allocate %zu bytes for layer %d activations", (size_t)N * L.d_out * 4, l);
      rc = SLONN_ENOMEM;
      break;
    }
    if (l == 0 && X->format == SLONN_ELL)
      rc = launch_ell_layer(L.W, L.w_dtype, L.w_layout, L.bias, X->idx, X->val, X->nnz, X->ell_stride, act,
                            L.d_out, (int)N, L.d_in, L.d_out, L.act, s);
    else
      // (refreshable tables: one kernel shape for every training-set size, so that an input's
      // activations - and with them every NodeScore sum - are the same whether it arrives in the
      // first training set or in a later refresh)
      rc = launch_dense_layer(L.W, L.w_dtype, L.bias, cur, L.d_in, act, L.d_out, (int)N, L.d_in, L.d_out,
                              L.act, nullptr, s, refresh || m->tables_refreshable);
    if (rc == SLONN_OK && L.act == SLONN_ACT_SOFTMAX)
      rc = launch_finalize(act, L.d_out, L.d_out, nullptr, nullptr, 0, nullptr, 0, 1, nullptr, (int)N, s);
    if (rc == SLONN_OK && L.activated()) {
      if (refresh) {
        TableSet* ts = nullptr;
        for (TableSet& c : t->sets)
          if (c.layer == l) ts = &c;
        rc = build_layer_tables(m, l, cur, N, act, ts, true, s);
      } else {
        TableSet ts;
        rc = build_layer_tables(m, l, cur, N, act, &ts, false, s);
        if (rc == SLONN_OK) t->sets.push_back(std::move(ts));
        else free_table_set(&ts);
      }
    }
    if (hipStreamSynchronize(s) != hipSuccess && rc == SLONN_OK) {
      set_error("build: stream synchronisation failed at layer %d", l);
      rc = SLONN_EHIP;
    }
    if (prev) (void)hipFree(prev);
    prev = act;
    cur = act;
  }
  if (prev) (void)hipFree(prev);
  return rc;
}

}  // namespace
}  // namespace slonn

extern "C" int slonn_build_tables(const slonn_model* m, const slonn_input* X_build, int64_t N, void* stream,
                                  slonn_tables** out) {
  if (!out) SLONN_FAIL(SLONN_EINVAL, "out is null");
  *out = nullptr;
  int rc = check_training_input(m, X_build, N);
  if (rc) return rc;
  slonn_tables* t = new (std::nothrow) slonn_tables;
  if (!t) SLONN_FAIL(SLONN_ENOMEM, "out of host memory");
  t->model = m;
  rc = train_tables(m, t, X_build, N, false, static_cast<hipStream_t>(stream));
  if (rc != SLONN_OK) {
    slonn_tables_destroy(t);
    return rc;
  }
  *out = t;
  return SLONN_OK;
}

extern "C" int slonn_tables_refresh(const slonn_model* m, slonn_tables* t, const slonn_input* X_new, int64_t N,
                                    void* stream) {
  if (!t) SLONN_FAIL(SLONN_EINVAL, "tables are null");
  int rc = check_training_input(m, X_new, N);
  if (rc) return rc;
  if (t->model != m) SLONN_FAIL(SLONN_EINVAL, "tables belong to another model");
  for (size_t l = 0; l < m->layers.size(); ++l)
    if (m->layers[l].activated()) {
      const TableSet* ts = t->for_layer((int)l);
      if (!ts || !ts->d_score || !ts->d_npos || !ts->d_global_score)
        SLONN_FAIL(SLONN_EUNSUPPORTED, "refresh: the tables of layer %zu hold no NodeScore sums (train them after "
                   "slonn_model_set_tables_refreshable; imported tables carry none)", l);
      if (ts->n_trained + N > SLONN_MAX_BATCH * 64ll)
        SLONN_FAIL(SLONN_EUNSUPPORTED, "refresh: more than %lld training inputs in all", SLONN_MAX_BATCH * 64ll);
    }
  // A failure part-way leaves the earlier layers refreshed and the later ones not: the caller
  // should then discard the tables.
  return train_tables(m, t, X_new, N, true, static_cast<hipStream_t>(stream));
}
