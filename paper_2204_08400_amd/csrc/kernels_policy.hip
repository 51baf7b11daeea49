// Choice of k per query (Section 2: the ACLO and LCAO optimisation targets; Section 3.2:
// Confidence LSH tables and latency profiles; Fig. 2 step 2).  Mechanics only: the
// confidences c(k, x') of the training inputs and the latency profile T(k, beta) are inputs.
//
// Confidence LSH tables share the hash functions of the first activated layer's Node
// Importance tables (same K, L and hash nodes), so a query's keys are computed once.  Per
// table and bucket the tables hold the sum over the training inputs hashed there of
// c(k_g, x') for every k_g of the grid, and the number of those inputs.  The estimate of
// Eq. 4 pools the L buckets of a query: (sum of bucket sums) / (sum of bucket counts).
//
// Sums are taken in double in training-set order (a bucket's members are listed in input
// order first), and a query adds its L buckets in table order, so that every decision
// c_hat >= threshold is reproducible bit for bit.
#include <algorithm>
#include <new>

#include "bucket_lists.h"
#include "slonn_internal.h"

struct slonn_policy {
  int K = 0, L = 0, G = 0;
  int64_t N = 0;                  // training inputs behind the confidence tables (0: none yet)
  float* d_grid = nullptr;        // [G] ascending keep fractions
  double* d_sum = nullptr;        // [L][2^K][G]
  uint32_t* d_cnt = nullptr;      // [L][2^K]
  double* d_total = nullptr;      // [G] sums over the whole training set
  float* d_T = nullptr;           // [n_beta][G] latency profile
  int n_beta = 0;
};

namespace slonn {
namespace {

template <class T>
struct DevBuf {
  T* p = nullptr;
  ~DevBuf() { if (p) (void)hipFree(p); }
  hipError_t alloc(size_t count) { return hipMalloc(&p, std::max<size_t>(count, 1) * sizeof(T)); }
};

// flags keys outside 0 .. nb-1 (they would index outside the tables)
__global__ void policy_check_keys_kernel(const uint32_t* __restrict__ keys, int64_t count, int nb,
                                         int* __restrict__ bad) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < count && keys[e] >= (uint32_t)nb) bad[0] = 1;
}

// sum[b][key][g] = sum over the bucket's members, in input order, of conf[x][g]
__global__ void policy_sum_kernel(const float* __restrict__ conf, int G, int64_t N, int nb,
                                  const uint32_t* __restrict__ start, const uint32_t* __restrict__ members,
                                  double* __restrict__ sum, uint32_t* __restrict__ cnt, int L) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;      // ((b, key), g)
  if (e >= (int64_t)L * nb * G) return;
  const int g = (int)(e % G);
  const int64_t bk = e / G;
  const int b = (int)(bk / nb), key = (int)(bk % nb);
  const uint32_t lo = start[(size_t)b * (nb + 1) + key], hi = start[(size_t)b * (nb + 1) + key + 1];
  const uint32_t* mem = members + (size_t)b * N;
  double s = 0.0;
  for (uint32_t i = lo; i < hi; ++i) s += (double)conf[(size_t)mem[i] * G + g];
  sum[e] = s;
  if (g == 0) cnt[bk] = hi - lo;
}

__global__ void policy_total_kernel(const float* __restrict__ conf, int G, int64_t N, double* __restrict__ total) {
  const int g = threadIdx.x;
  if (g >= G) return;
  double s = 0.0;
  for (int64_t x = 0; x < N; ++x) s += (double)conf[x * G + g];
  total[g] = s;
}

// One 16-lane group per query, lane g = grid point g.  Keys come from codes, or from the
// projections Z (bit j of table b = [Z[q][b*K + j] > 0]).
__global__ __launch_bounds__(256) void policy_aclo_kernel(
    const uint32_t* __restrict__ codes, const float* __restrict__ Z, int K, int L, int nb, int G, int B,
    const double* __restrict__ sum, const uint32_t* __restrict__ cnt, const double* __restrict__ total,
    int64_t N, const float* __restrict__ grid, const float* __restrict__ thr, int thr_stride,
    float* __restrict__ keep_out, int32_t* __restrict__ g_out, double* __restrict__ chat_out) {
  __shared__ uint32_t skey[16][64];
  const int grp = threadIdx.x >> 4, g = threadIdx.x & 15;
  const int q = blockIdx.x * 16 + grp;
  const bool liveq = q < B;
  if (liveq)
    for (int b = g; b < L; b += 16) {
      uint32_t key;
      if (codes) {
        key = codes[(size_t)q * L + b];
      } else {
        key = 0;
        const float* z = Z + ((size_t)q * L + b) * K;
        for (int j = 0; j < K; ++j) key |= (z[j] > 0.0f ? 1u : 0u) << j;
      }
      skey[grp][b] = key < (uint32_t)nb ? key : 0u;
    }
  __syncthreads();
  double s = 0.0;
  unsigned long long c = 0;
  if (liveq && g < G)
    for (int b0 = 0; b0 < L; b0 += 8) {       // eight loads in flight, added in table order
      double v[8];
      uint32_t cb[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int b = min(b0 + u, L - 1);
        const size_t bk = (size_t)b * nb + skey[grp][b];
        v[u] = sum[bk * G + g];               // an empty bucket holds +0 and the count 0
        cb[u] = cnt[bk];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (b0 + u < L) { s += v[u]; c += cb[u]; }
    }
  double chat = 0.0;
  bool ok = false;
  if (liveq && g < G) {
    chat = c > 0 ? s / (double)c : total[g] / (double)N;
    ok = chat >= (double)thr[(size_t)q * thr_stride];
    if (chat_out) chat_out[(size_t)q * G + g] = chat;
  }
  const unsigned long long votes = __ballot(ok);
  const uint32_t mine = (uint32_t)((votes >> (16 * ((threadIdx.x & 63) >> 4))) & 0xFFFFull);
  if (liveq && g == 0) {
    const int pick = mine ? (__ffs((int)mine) - 1) : G - 1;
    keep_out[q] = grid[pick];
    if (g_out) g_out[q] = pick;
  }
}

__global__ void policy_lcao_kernel(const float* __restrict__ grid, int G, const float* __restrict__ T,
                                   int n_beta, const float* __restrict__ tau, int tau_stride,
                                   const float* __restrict__ t0, int t0_stride,
                                   const int32_t* __restrict__ beta, int beta_stride, int B,
                                   float* __restrict__ keep_out, int32_t* __restrict__ g_out,
                                   int32_t* __restrict__ violated) {
  const int q = blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= B) return;
  const int bq = beta[(size_t)q * beta_stride];
  const bool known = bq >= 0 && bq < n_beta;        // an unknown state has no profile: nothing fits
  const float* row = T + (size_t)(known ? bq : 0) * G;
  const double budget = (double)tau[(size_t)q * tau_stride], fixed = (double)t0[(size_t)q * t0_stride];
  int pick = -1;
  for (int g = 0; g < G; ++g)
    if (known && fixed + (double)row[g] <= budget) pick = g;
  if (violated) violated[q] = pick < 0 ? 1 : 0;
  if (pick < 0) pick = 0;
  keep_out[q] = grid[pick];
  if (g_out) g_out[q] = pick;
}

}  // namespace

int launch_policy_aclo(const slonn_policy* p, const uint32_t* codes, const float* Z, int B, const float* thr,
                       int thr_stride, float* keep_out, int32_t* g_out, double* chat_out, hipStream_t s) {
  ProfScope prof_(SLONN_PROF_SELECT, s);
  hipLaunchKernelGGL(policy_aclo_kernel, dim3((B + 15) / 16), dim3(256), 0, s, codes, Z, p->K, p->L, 1 << p->K,
                     p->G, B, p->d_sum, p->d_cnt, p->d_total, p->N, p->d_grid, thr, thr_stride, keep_out, g_out,
                     chat_out);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

void policy_fused_args(const slonn_policy* p, PolicyArgs* a) {
  a->sum = p->d_sum; a->cnt = p->d_cnt; a->total = p->d_total; a->grid = p->d_grid;
  a->G = p->G; a->N = p->N;
}

bool policy_matches(const slonn_policy* p, int K, int L) { return p->K == K && p->L == L; }
bool policy_trained(const slonn_policy* p) { return p->N > 0; }

}  // namespace slonn

using namespace slonn;

extern "C" {

int slonn_policy_create(int K, int L, const float* k_grid, int G, slonn_policy** out) {
  if (!out) SLONN_FAIL(SLONN_EINVAL, "out is null");
  *out = nullptr;
  if (K < 1 || K > SLONN_MAX_K || L < 1 || L > SLONN_MAX_L)
    SLONN_FAIL(SLONN_EINVAL, "K must be in 1 .. %d and L in 1 .. %d", SLONN_MAX_K, SLONN_MAX_L);
  if (!k_grid || G < 1 || G > SLONN_MAX_GRID) SLONN_FAIL(SLONN_EINVAL, "the k grid needs 1 .. %d entries", SLONN_MAX_GRID);
  for (int g = 0; g < G; ++g) {
    if (!(k_grid[g] > 0.0f) || k_grid[g] > 1.0f) SLONN_FAIL(SLONN_EINVAL, "k grid entry %d is outside (0, 1]", g);
    if (g && !(k_grid[g] > k_grid[g - 1])) SLONN_FAIL(SLONN_EINVAL, "the k grid must be strictly ascending");
  }
  const size_t cells = (size_t)L << K;          // at most 64 * 65536 buckets: 512 MiB of sums at G = 16
  slonn_policy* p = new (std::nothrow) slonn_policy;
  if (!p) SLONN_FAIL(SLONN_ENOMEM, "out of host memory");
  p->K = K; p->L = L; p->G = G;
  hipError_t e;
  if ((e = hipMalloc(&p->d_grid, (size_t)G * 4)) != hipSuccess ||
      (e = hipMemcpy(p->d_grid, k_grid, (size_t)G * 4, hipMemcpyHostToDevice)) != hipSuccess ||
      (e = hipMalloc(&p->d_sum, cells * G * sizeof(double))) != hipSuccess ||
      (e = hipMalloc(&p->d_cnt, cells * 4)) != hipSuccess ||
      (e = hipMalloc(&p->d_total, (size_t)G * sizeof(double))) != hipSuccess) {
    set_error("allocating the policy tables failed: %s", hipGetErrorString(e));
    slonn_policy_destroy(p);
    return SLONN_EHIP;
  }
  *out = p;
  return SLONN_OK;
}

int slonn_policy_destroy(slonn_policy* p) {
  if (!p) return SLONN_OK;
  if (p->d_grid) (void)hipFree(p->d_grid);
  if (p->d_sum) (void)hipFree(p->d_sum);
  if (p->d_cnt) (void)hipFree(p->d_cnt);
  if (p->d_total) (void)hipFree(p->d_total);
  if (p->d_T) (void)hipFree(p->d_T);
  delete p;
  return SLONN_OK;
}

int slonn_policy_train_confidence(slonn_policy* p, const uint32_t* codes, const float* conf, int64_t N,
                                  void* stream) {
  if (!p || !codes || !conf) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (N <= 0 || N > SLONN_MAX_BATCH) SLONN_FAIL(SLONN_EINVAL, "N must be in 1 .. %d", SLONN_MAX_BATCH);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int K = p->K, L = p->L, G = p->G, nb = 1 << K;
  DevBuf<uint32_t> hist, start, cursor, members;
  DevBuf<int> bad;
  SLONN_HIP(hist.alloc((size_t)L * nb));
  SLONN_HIP(start.alloc((size_t)L * (nb + 1)));
  SLONN_HIP(cursor.alloc((size_t)L * nb));
  SLONN_HIP(members.alloc((size_t)L * N));
  SLONN_HIP(bad.alloc(1));
  SLONN_HIP(hipMemsetAsync(bad.p, 0, sizeof(int), s));
  SLONN_HIP(hipMemsetAsync(hist.p, 0, (size_t)L * nb * 4, s));
  const int64_t tot = N * L;
  hipLaunchKernelGGL(policy_check_keys_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, s, codes, tot, nb,
                     bad.p);
  SLONN_HIP(hipGetLastError());
  int h_bad = 0;
  SLONN_HIP(hipMemcpyAsync(&h_bad, bad.p, sizeof(int), hipMemcpyDeviceToHost, s));
  SLONN_HIP(hipStreamSynchronize(s));
  if (h_bad) SLONN_FAIL(SLONN_EINVAL, "a training key is outside 0 .. 2^K - 1");
  hipLaunchKernelGGL(bucket_hist_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, s, codes, N, L, nb,
                     hist.p);
  SLONN_HIP(hipGetLastError());
  hipLaunchKernelGGL(bucket_scan_kernel, dim3(L), dim3(256), 0, s, hist.p, nb, start.p, cursor.p);
  SLONN_HIP(hipGetLastError());
  hipLaunchKernelGGL(bucket_members_kernel, dim3(L), dim3(64), 0, s, codes, N, L, K, nb, cursor.p, members.p);
  SLONN_HIP(hipGetLastError());
  const int64_t cells = (int64_t)L * nb * G;
  hipLaunchKernelGGL(policy_sum_kernel, dim3((unsigned)((cells + 255) / 256)), dim3(256), 0, s, conf, G, N, nb,
                     start.p, members.p, p->d_sum, p->d_cnt, L);
  SLONN_HIP(hipGetLastError());
  hipLaunchKernelGGL(policy_total_kernel, dim3(1), dim3(64), 0, s, conf, G, N, p->d_total);
  SLONN_HIP(hipGetLastError());
  SLONN_HIP(hipStreamSynchronize(s));        // the scratch buffers are freed on return
  p->N = N;
  return SLONN_OK;
}

int slonn_policy_set_latency_profile(slonn_policy* p, const float* T, int n_beta) {
  if (!p || !T) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (n_beta < 1 || n_beta > 65536) SLONN_FAIL(SLONN_EINVAL, "n_beta must be in 1 .. 65536");
  for (size_t i = 0; i < (size_t)n_beta * p->G; ++i)
    if (!(T[i] >= 0.0f)) SLONN_FAIL(SLONN_EINVAL, "latency profile entry %zu is negative or not a number", i);
  if (p->d_T) { (void)hipFree(p->d_T); p->d_T = nullptr; p->n_beta = 0; }
  SLONN_HIP(hipMalloc(&p->d_T, (size_t)n_beta * p->G * 4));
  SLONN_HIP(hipMemcpy(p->d_T, T, (size_t)n_beta * p->G * 4, hipMemcpyHostToDevice));
  p->n_beta = n_beta;
  return SLONN_OK;
}

int slonn_policy_keep_aclo(const slonn_policy* p, const uint32_t* codes, int B, const float* thr,
                           int thr_stride, float* keep_out, int32_t* grid_idx_out, double* c_hat_out,
                           void* stream) {
  if (!p || !codes || !thr || !keep_out) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (B <= 0 || B > SLONN_MAX_BATCH) SLONN_FAIL(SLONN_EINVAL, "B must be in 1 .. %d", SLONN_MAX_BATCH);
  if (thr_stride < 0) SLONN_FAIL(SLONN_EINVAL, "negative stride");
  if (p->N <= 0) SLONN_FAIL(SLONN_EINVAL, "the confidence tables have not been trained");
  return launch_policy_aclo(p, codes, nullptr, B, thr, thr_stride, keep_out, grid_idx_out, c_hat_out,
                            static_cast<hipStream_t>(stream));
}

int slonn_policy_keep_lcao(const slonn_policy* p, int B, const float* tau, int tau_stride, const float* t0,
                           int t0_stride, const int32_t* beta, int beta_stride, float* keep_out,
                           int32_t* grid_idx_out, int32_t* violated_out, void* stream) {
  if (!p || !tau || !t0 || !beta || !keep_out) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (B <= 0 || B > SLONN_MAX_BATCH) SLONN_FAIL(SLONN_EINVAL, "B must be in 1 .. %d", SLONN_MAX_BATCH);
  if (tau_stride < 0 || t0_stride < 0 || beta_stride < 0) SLONN_FAIL(SLONN_EINVAL, "negative stride");
  if (!p->d_T) SLONN_FAIL(SLONN_EINVAL, "no latency profile has been set");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(policy_lcao_kernel, dim3((B + 255) / 256), dim3(256), 0, s, p->d_grid, p->G, p->d_T, p->n_beta,
                     tau, tau_stride, t0, t0_stride, beta, beta_stride, B, keep_out, grid_idx_out, violated_out);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

}  // extern "C"
