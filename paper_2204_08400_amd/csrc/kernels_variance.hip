// Choice of the FreeHash nodes (Section 3.4): hash nodes are drawn with probability
// proportional to the variance of the nodes' activations over the tables' training set.
//   activation_variance_kernel   per-node variance of a [N][n] activation matrix, two passes
//                                in fp64 (mean, then squared deviations) with a fixed
//                                summation order: a wavefront owns 64 consecutive nodes and a
//                                quarter of the rows, the four quarters are added in order.
//   slonn_sample_hash_nodes      the K*L sequential draws without replacement, on the host
//                                (K*L passes over n running sums: set-up work);
//   sample_hash_nodes_kernel     the same draws on the device, by one wavefront.
#include <cmath>
#include <vector>

#include "slonn_internal.h"

namespace slonn {
namespace {

// sum over rows [r0, r1) of f(A[r][col]) with eight loads in flight, rows ascending
template <typename F>
__device__ __forceinline__ double column_sum(const float* __restrict__ A, int64_t lda, int64_t r0, int64_t r1,
                                             int col, F f) {
  double acc = 0.0;
  int64_t r = r0;
  for (; r + 8 <= r1; r += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = A[(r + u) * lda + col];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += f((double)v[u]);
  }
  for (; r < r1; ++r) acc += f((double)A[r * lda + col]);
  return acc;
}

__global__ __launch_bounds__(256) void activation_variance_kernel(const float* __restrict__ A, int64_t N, int n,
                                                                 int64_t lda, double* __restrict__ var) {
  __shared__ double part[4][64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = blockIdx.x * 64 + lane;
  const bool live = col < n;
  const int64_t quarter = (N + 3) / 4;
  const int64_t r0 = min(N, wave * quarter), r1 = min(N, r0 + quarter);
  part[wave][lane] = live ? column_sum(A, lda, r0, r1, col, [](double x) { return x; }) : 0.0;
  __syncthreads();
  const double mean = (((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane]) / (double)N;
  __syncthreads();
  part[wave][lane] = live ? column_sum(A, lda, r0, r1, col, [mean](double x) { return (x - mean) * (x - mean); }) : 0.0;
  __syncthreads();
  if (wave == 0 && live)
    var[col] = (((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane]) / (double)N;
}

// The K*L draws on the device, by ONE wavefront: the draws are sequential by definition (each
// removes a node), and so is every running sum (the id a draw lands on is decided by comparing
// fp64 running sums formed in ascending node order, so the order of the additions is part of the
// result).  The wavefront walks the variances 64 at a time: one coalesced load, then the 64
// additions in order, the same in every lane, lane j keeping the sum after element j; a ballot
// finds the first running sum above the target.  Drawn nodes are struck out in an LDS bitmap; the
// variances themselves are only read.
__device__ __forceinline__ double lane_value(double v, int j) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), j);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), j);
  return __hiloint2double(hi, lo);
}

__global__ __launch_bounds__(64) void sample_hash_nodes_kernel(const double* __restrict__ var, int n, int H,
                                                              const double* __restrict__ u,
                                                              int32_t* __restrict__ out) {
  extern __shared__ uint32_t taken[];        // one bit per node: drawn
  const int lane = threadIdx.x;
  const int words = (n + 31) >> 5;
  for (int w = lane; w < words; w += 64) taken[w] = 0u;
  __syncthreads();
  // remaining variance of node i: negative and non-finite entries count as 0, drawn nodes too
  auto value = [&](int i) -> double {
    if (i >= n) return 0.0;
    const double x = var[i];
    const bool ok = x > 0.0 && x <= 1.79769313486231570e308;
    return (ok && !((taken[i >> 5] >> (i & 31)) & 1u)) ? x : 0.0;
  };
  // run += the chunk's 64 values in order; returns the running sum after this lane's element
  auto scan_chunk = [&](double v, double& run) -> double {
    double mine = 0.0;
#pragma unroll
    for (int j = 0; j < 64; ++j) {
      run += lane_value(v, j);
      if (lane == j) mine = run;
    }
    return mine;
  };
  int lowest_free = 0;
  for (int j = 0; j < H; ++j) {
    double run = 0.0;
    double nxt = value(lane);
    for (int c = 0; c < n; c += 64) {          // the total of what is left
      const double v = nxt;
      nxt = value(c + 64 + lane);
      (void)scan_chunk(v, run);
    }
    const double total = run;
    int pick = n - 1;                          // (the last node if rounding leaves no running sum above the target)
    if (total > 0.0) {
      const double target = u[j] * total;
      run = 0.0;
      nxt = value(lane);
      for (int c = 0; c < n; c += 64) {
        const double v = nxt;
        nxt = value(c + 64 + lane);
        const double mine = scan_chunk(v, run);
        const unsigned long long hit = __ballot(c + lane < n && mine > target);
        if (hit) {
          pick = c + __ffsll((long long)hit) - 1;
          break;
        }
      }
      while (!(value(pick) > 0.0)) pick = (pick + 1) % n;      // total > 0: some node still has variance
    } else {                                   // no variance left: the lowest id not drawn yet
      int w = lowest_free >> 5;
      pick = -1;
      while (pick < 0) {
        uint32_t fr = ~taken[w];
        if (w == words - 1 && (n & 31)) fr &= (1u << (n & 31)) - 1u;
        if (fr) pick = w * 32 + __ffs((int)fr) - 1;
        else ++w;
      }
      lowest_free = pick;
    }
    if (lane == 0) {
      out[j] = pick;
      taken[pick >> 5] |= 1u << (pick & 31);
    }
    __syncthreads();
  }
}

}  // namespace
}  // namespace slonn

using namespace slonn;

extern "C" {

int slonn_activation_variance(const float* A, int64_t N, int n, int64_t lda, double* var_out, void* stream) {
  if (!A || !var_out) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (N < 1 || n < 1 || lda < n) SLONN_FAIL(SLONN_EINVAL, "need N >= 1, n >= 1 and lda >= n");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(activation_variance_kernel, dim3((n + 63) / 64), dim3(256), 0, s, A, N, n, lda, var_out);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

int slonn_sample_hash_nodes_device(const double* variance, int n, int K, int L, const double* u,
                                   int32_t* hash_nodes_out, void* stream) {
  if (!variance || !u || !hash_nodes_out) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (n < 1 || K < 1 || L < 1) SLONN_FAIL(SLONN_EINVAL, "need n, K, L >= 1");
  const long long H = (long long)K * L;
  if (H > n) SLONN_FAIL(SLONN_EINVAL, "K*L = %lld exceeds the layer's %d nodes", H, n);
  if (n > (1 << 20)) SLONN_FAIL(SLONN_EUNSUPPORTED, "the device sampler serves layers of up to %d nodes", 1 << 20);
  const size_t lds = (size_t)((n + 31) / 32) * 4;
  if (lds > 65536)
    SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(sample_hash_nodes_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  hipLaunchKernelGGL(sample_hash_nodes_kernel, dim3(1), dim3(64), lds, static_cast<hipStream_t>(stream), variance, n,
                     (int)H, u, hash_nodes_out);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

int slonn_sample_hash_nodes(const double* variance, int n, int K, int L, const double* u,
                            int32_t* hash_nodes_out) {
  if (!variance || !u || !hash_nodes_out) SLONN_FAIL(SLONN_EINVAL, "null argument");
  if (n < 1 || K < 1 || L < 1) SLONN_FAIL(SLONN_EINVAL, "need n, K, L >= 1");
  const long long H = (long long)K * L;
  if (H > n) SLONN_FAIL(SLONN_EINVAL, "K*L = %lld exceeds the layer's %d nodes", H, n);
  std::vector<double> v(n);
  for (int i = 0; i < n; ++i) v[i] = (std::isfinite(variance[i]) && variance[i] > 0.0) ? variance[i] : 0.0;
  std::vector<char> drawn(n, 0);
  int lowest_free = 0;                 // every id below it has been drawn
  for (long long j = 0; j < H; ++j) {
    double total = 0.0;
    for (int i = 0; i < n; ++i) total += v[i];
    int pick = -1;
    if (total > 0.0) {
      const double target = u[j] * total;
      double run = 0.0;
      pick = n - 1;
      for (int i = 0; i < n; ++i) {
        run += v[i];
        if (run > target) { pick = i; break; }
      }
      while (!(v[pick] > 0.0)) pick = (pick + 1) % n;     // total > 0: some node still has variance
    } else {
      while (drawn[lowest_free]) ++lowest_free;            // H <= n: one is left
      pick = lowest_free;
    }
    hash_nodes_out[j] = pick;
    drawn[pick] = 1;
    v[pick] = 0.0;
  }
  return SLONN_OK;
}

}  // extern "C"
