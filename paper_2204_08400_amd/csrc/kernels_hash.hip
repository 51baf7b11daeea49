// FreeHash projections (Def. 2, Section 3.4): z[q][h] = w_h . x_q + b_h for the K*L
// sampled nodes of a layer, shared by every query of the batch -> a dense contraction
// [B x d] . [d x H].  The sign of z is a hash bit, so the sum is carried in fp64: the
// fp32 x fp32 products are exact in fp64 and the result's sign then only depends on
// summation order when |z| is at the 1e-15 level, instead of the 1e-7 level of an
// fp32 accumulator.
#include "slonn_internal.h"

namespace slonn {
namespace {

constexpr int TQ = 32;   // queries per tile
constexpr int TH = 64;   // hash nodes per tile
constexpr int TK = 32;   // reduction chunk

// 256 threads; thread (tq, th) owns queries {tq, tq+16} x hash nodes {th, th+16, th+32, th+48}.
__global__ __launch_bounds__(256) void hash_project_kernel(const float* __restrict__ X, int ldx,
                                                          const float* __restrict__ Wh,
                                                          const float* __restrict__ bh,
                                                          float* __restrict__ Z, int B, int H, int d) {
  __shared__ float xs[TQ][TK + 1];
  __shared__ float ws[TH][TK + 1];
  const int tid = threadIdx.x;
  const int q0 = blockIdx.y * TQ, h0 = blockIdx.x * TH;
  const int tq = tid >> 4, th = tid & 15;
  double acc[2][4] = {};
  for (int k0 = 0; k0 < d; k0 += TK) {
    // stage tiles; consecutive threads read consecutive k (coalesced along a row)
    for (int e = tid; e < TQ * TK; e += 256) {
      int r = e / TK, k = e % TK;
      int q = q0 + r, kk = k0 + k;
      xs[r][k] = (q < B && kk < d) ? X[(size_t)q * ldx + kk] : 0.0f;
    }
    for (int e = tid; e < TH * TK; e += 256) {
      int r = e / TK, k = e % TK;
      int h = h0 + r, kk = k0 + k;
      ws[r][k] = (h < H && kk < d) ? Wh[(size_t)h * d + kk] : 0.0f;
    }
    __syncthreads();
#pragma unroll 8
    for (int k = 0; k < TK; ++k) {
      double x0 = xs[tq][k], x1 = xs[tq + 16][k];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        double w = ws[th + 16 * i][k];
        acc[0][i] = fma(x0, w, acc[0][i]);
        acc[1][i] = fma(x1, w, acc[1][i]);
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    int q = q0 + tq + 16 * r;
    if (q >= B) continue;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int h = h0 + th + 16 * i;
      if (h < H) Z[(size_t)q * H + h] = (float)(acc[r][i] + (double)bh[h]);
    }
  }
}

}  // namespace

int launch_hash_project(const float* X, int ldx, const float* Wh, const float* bh, float* Z, int B,
                        int H, int d, hipStream_t s) {
  ProfScope prof_(SLONN_PROF_HASH, s);
  dim3 grid((H + TH - 1) / TH, (B + TQ - 1) / TQ);
  hipLaunchKernelGGL(hash_project_kernel, grid, dim3(256), 0, s, X, ldx, Wh, bh, Z, B, H, d);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

}  // namespace slonn
