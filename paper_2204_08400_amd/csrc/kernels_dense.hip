// Full layer Y = act(X W^T + b): the baseline every SLO-NN speed-up is measured against
// (Section 3.4: with all nodes computed an SLO-NN does the same work as the full
// network; Section 4 compares against full forward passes).  This is a real dense
// contraction, so it runs on the matrix cores: fp32 MFMA 32x32x2, fp32 accumulate,
// no reduced-precision rounding of the inputs (bf16 weights widen exactly to fp32).
//
// 256 threads = 4 wavefronts in a 2x2 arrangement; a block owns a BM x BN tile of Y,
// each wave a (BM/2) x (BN/2) sub-tile made of 32x32 MFMA blocks.  K is walked in
// chunks of 32 staged through LDS; the next chunk's global loads are issued before
// the current chunk's MFMAs so their latency hides behind the matrix work.
#include <algorithm>

#include "slonn_internal.h"

namespace slonn {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int KC = 32;          // K chunk staged in LDS
constexpr int LDT = KC + 4;     // padded LDS row (keeps 16-byte alignment, staggers banks)

template <int WDT>
__device__ __forceinline__ float4 load4(const void* base, size_t elem_off, bool vec, int valid) {
  // four consecutive K elements starting at elem_off; `valid` of them exist
  float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
  if (valid <= 0) return r;
  if (WDT == SLONN_F32) {
    const float* p = static_cast<const float*>(base) + elem_off;
    if (vec && valid == 4) return *reinterpret_cast<const float4*>(p);
    r.x = p[0];
    if (valid > 1) r.y = p[1];
    if (valid > 2) r.z = p[2];
    if (valid > 3) r.w = p[3];
  } else {
    const uint16_t* p = static_cast<const uint16_t*>(base) + elem_off;
    if (vec && valid == 4) {
      const uint2 u = *reinterpret_cast<const uint2*>(p);
      r.x = __uint_as_float(u.x << 16);
      r.y = __uint_as_float(u.x & 0xFFFF0000u);
      r.z = __uint_as_float(u.y << 16);
      r.w = __uint_as_float(u.y & 0xFFFF0000u);
      return r;
    }
    r.x = __uint_as_float((uint32_t)p[0] << 16);
    if (valid > 1) r.y = __uint_as_float((uint32_t)p[1] << 16);
    if (valid > 2) r.z = __uint_as_float((uint32_t)p[2] << 16);
    if (valid > 3) r.w = __uint_as_float((uint32_t)p[3] << 16);
  }
  return r;
}

template <int WDT, int BM, int BN>
__global__ __launch_bounds__(256) void dense_layer_kernel(const void* __restrict__ W,
                                                         const float* __restrict__ bias,
                                                         const float* __restrict__ X, int ldx,
                                                         float* __restrict__ Y, int ldy, int M, int N,
                                                         int Kd, int act, int vecx, int vecw) {
  constexpr int WM = BM / 2, WN = BN / 2;          // wave tile
  constexpr int MB = WM / 32, NB = WN / 32;        // 32x32 MFMA blocks per wave
  constexpr int PA = BM / 32, PB = BN / 32;        // loader passes (32 rows per pass)
  __shared__ __align__(16) float As[BM * LDT];
  __shared__ __align__(16) float Bs[BN * LDT];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int lrow = tid >> 3, lk = (tid & 7) * 4;   // loader: row within pass, K offset in chunk
  const int half = lane >> 5, l32 = lane & 31;

  f32x16 acc[MB][NB];
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

  float4 ra[PA], rb[PB];
  auto fetch = [&](int k0) {
    const int kk = k0 + lk;
    const int valid = Kd - kk < 4 ? Kd - kk : 4;
#pragma unroll
    for (int p = 0; p < PA; ++p) {
      const int row = m0 + lrow + 32 * p;
      ra[p] = (row < M) ? load4<SLONN_F32>(X, (size_t)row * ldx + kk, vecx, valid)
                        : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int p = 0; p < PB; ++p) {
      const int row = n0 + lrow + 32 * p;
      rb[p] = (row < N) ? load4<WDT>(W, (size_t)row * Kd + kk, vecw, valid)
                        : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int p = 0; p < PA; ++p)
      *reinterpret_cast<float4*>(&As[(lrow + 32 * p) * LDT + lk]) = ra[p];
#pragma unroll
    for (int p = 0; p < PB; ++p)
      *reinterpret_cast<float4*>(&Bs[(lrow + 32 * p) * LDT + lk]) = rb[p];
  };

  fetch(0);
  for (int k0 = 0; k0 < Kd; k0 += KC) {
    stash();
    __syncthreads();
    if (k0 + KC < Kd) fetch(k0 + KC);
#pragma unroll
    for (int ks = 0; ks < KC; ks += 8) {
      // lane (row l32, half) takes K elements ks+4*half .. +3 of its row for A and for B
      float4 fa[MB], fb[NB];
#pragma unroll
      for (int a = 0; a < MB; ++a)
        fa[a] = *reinterpret_cast<const float4*>(&As[(wm * WM + a * 32 + l32) * LDT + ks + 4 * half]);
#pragma unroll
      for (int b = 0; b < NB; ++b)
        fb[b] = *reinterpret_cast<const float4*>(&Bs[(wn * WN + b * 32 + l32) * LDT + ks + 4 * half]);
#pragma unroll
      for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a].x, fb[b].x, acc[a][b], 0, 0, 0);
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a].y, fb[b].y, acc[a][b], 0, 0, 0);
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a].z, fb[b].z, acc[a][b], 0, 0, 0);
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a].w, fb[b].w, acc[a][b], 0, 0, 0);
        }
    }
    __syncthreads();
  }

  // 32x32 block layout: register r of lane (l32, half) is row 8*(r/4) + 4*half + r%4, column l32
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    const int col = n0 + wn * WN + b * 32 + l32;
    if (col >= N) continue;
    const float bv = bias[col];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * WM + a * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
        if (row >= M) continue;
        float z = acc[a][b][r] + bv;
        if (act == SLONN_ACT_RELU) z = z > 0.0f ? z : 0.0f;
        Y[(size_t)row * ldy + col] = z;
      }
  }
}

// Small problems (a batch of a few hundred queries against a layer of about a thousand
// nodes) do not fill the chip with 64x64 tiles and their K loop is pure latency.  Here a
// workgroup owns a 32x32 tile, its KS (4 or 16) wavefronts split the reduction dimension, operands
// go straight from L2 to registers as 16-byte loads (lane (r, half) takes elements
// 8s+4*half .. +3 of row r for both operands, MFMA c of the step consumes element c), U
// steps are loaded ahead, and the partial tiles are added in LDS in a fixed order.  Skinny
// problems (a 100-node output layer) have only a handful of tiles: sixteen wavefronts per tile
// then shorten the latency-bound reduction loop fourfold.
template <int WDT, int U, int KS, bool SPLIT = false>
__global__ __launch_bounds__(64 * KS) void dense_direct_kernel(const void* __restrict__ W,
                                                          const float* __restrict__ bias,
                                                          const float* __restrict__ X, int ldx,
                                                          float* __restrict__ Y, int ldy, int M, int N,
                                                          int Kd, int act, float* __restrict__ split_out,
                                                          int nslices) {
  __shared__ float part[KS - 1][64][16];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 31, half = lane >> 5;
  const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
  const float* xr = X + (size_t)min(m0 + r, M - 1) * ldx;          // surplus rows recompute a valid row
  const size_t wrow = (size_t)min(n0 + r, N - 1) * Kd;
  // blockIdx.z: slice of the reduction dimension (split_out then receives the slice's sums);
  // nslices = gridDim.z, handed over as an argument (cheaper to reach than the dispatch packet)
  const int steps = (Kd + 7) / 8;
  int z_begin = 0, z_end = steps;
  if (SPLIT) {
    const int per_z = (steps + nslices - 1) / nslices;
    z_begin = min(steps, (int)blockIdx.z * per_z);
    z_end = min(steps, z_begin + per_z);
  }
  const int per = (z_end - z_begin + KS - 1) / KS;
  const int s_begin = min(z_end, z_begin + wave * per), s_end = min(z_end, s_begin + per);
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s0 = s_begin; s0 < s_end; s0 += U) {
    float4 a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int k = 8 * (s0 + u) + 4 * half;
      const bool ok = (s0 + u < s_end) && k < Kd;     // Kd is a multiple of 4
      const int kk = ok ? k : 0;
      const float4 xa = *reinterpret_cast<const float4*>(xr + kk);
      float4 wb;
      if (WDT == SLONN_F32) {
        wb = *reinterpret_cast<const float4*>(static_cast<const float*>(W) + wrow + kk);
      } else {
        const uint2 q = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(W) + wrow + kk);
        wb.x = __uint_as_float(q.x << 16);
        wb.y = __uint_as_float(q.x & 0xFFFF0000u);
        wb.z = __uint_as_float(q.y << 16);
        wb.w = __uint_as_float(q.y & 0xFFFF0000u);
      }
      a[u] = ok ? xa : zero4;
      b[u] = ok ? wb : zero4;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u].x, b[u].x, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u].y, b[u].y, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u].z, b[u].z, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u].w, b[u].w, acc, 0, 0, 0);
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int v = 0; v < 16; ++v) part[wave - 1][lane][v] = acc[v];
  }
  __syncthreads();
  if (wave == 0) {
    const int col = n0 + r;
    const float bv = col < N ? bias[col] : 0.0f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = m0 + 8 * (v >> 2) + 4 * half + (v & 3);
      float z = acc[v];
#pragma unroll
      for (int w = 0; w < KS - 1; ++w) z += part[w][lane][v];       // fixed order
      if (SPLIT) {
        if (row < M && col < N) split_out[((size_t)blockIdx.z * M + row) * N + col] = z;
        continue;
      }
      z += bv;
      if (act == SLONN_ACT_RELU) z = z > 0.0f ? z : 0.0f;
      if (row < M && col < N) Y[(size_t)row * ldy + col] = z;
    }
  }
}

// Y = act(sum of the S slices in slice order + bias): the second half of a split reduction.
__global__ __launch_bounds__(256) void dense_split_sum_kernel(const float* __restrict__ part, int S,
                                                             const float* __restrict__ bias, float* __restrict__ Y,
                                                             int ldy, int M, int N, int act) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x, total = (size_t)M * N;
  if (i >= total) return;
  const int row = (int)(i / N), col = (int)(i % N);
  float z = part[i];
  for (int k = 1; k < S; ++k) z += part[(size_t)k * total + i];
  z += bias[col];
  if (act == SLONN_ACT_RELU) z = z > 0.0f ? z : 0.0f;
  Y[(size_t)row * ldy + col] = z;
}

}  // namespace

bool dense_small_supported(const void* W, int w_dtype, const float* X, int ldx, int d) {
  const int wmul = (w_dtype == SLONN_F32) ? 4 : 8;
  return ldx % 4 == 0 && reinterpret_cast<uintptr_t>(X) % 16 == 0 && d % 4 == 0 && d % wmul == 0 &&
         reinterpret_cast<uintptr_t>(W) % (w_dtype == SLONN_F32 ? 16 : 8) == 0;
}

// Slices of the reduction dimension for a problem whose 32x32 tiles leave at least half of the
// compute units idle: up to two workgroups per unit, each slice at least 1024 elements long
// (shorter ones do not repay the second kernel).
static int dense_split_factor(int B, int n, int d) {
  const long tiles32 = (long)((B + 31) / 32) * ((n + 31) / 32);
  int S = 1;
  while (S < 8 && tiles32 <= 128 && tiles32 * S * 2 <= 512 && d / (S * 2) >= 1024) S *= 2;
  return S;
}

// Scratch for the slices: an upper bound that never shrinks as the batch grows (a caller may size
// its workspace for the largest batch and run smaller ones): at most 8 slices of at most 128
// tiles of 32 x 32 sums.
size_t dense_split_workspace_bytes(int B, int n, int d) {
  if (d < 2048) return 0;
  const size_t sums = std::min<size_t>((size_t)B * n, (size_t)128 * 32 * 32);
  return 8 * sums * sizeof(float);
}

int launch_dense_layer(const void* W, int w_dtype, const float* bias, const float* X, int ldx,
                       float* Y, int ldy, int B, int d, int n, int act, void* split_scratch, hipStream_t s,
                       bool batch_invariant) {
  ProfScope prof_(SLONN_PROF_DENSE, s);
  if (B <= 0) return SLONN_OK;
  const int a = (act == SLONN_ACT_RELU) ? SLONN_ACT_RELU : SLONN_ACT_NONE;
  const int vecx = (ldx % 4 == 0) && (reinterpret_cast<uintptr_t>(X) % 16 == 0);
  const int vecw = (d % 4 == 0) && (reinterpret_cast<uintptr_t>(W) % 16 == 0);
  const long big_tiles = (long)((B + 127) / 128) * ((n + 127) / 128);
  // batch_invariant: one kernel shape whatever the batch, so that a query's outputs do not depend on
  // how many queries travel with it (every shape sums a row's products in its own order)
  const bool big = big_tiles >= 512 && !batch_invariant;
  const long tiles64 = (long)((B + 63) / 64) * ((n + 63) / 64);
  if (!batch_invariant && tiles64 < 256 && dense_small_supported(W, w_dtype, X, ldx, d)) {
    const bool few = (long)((n + 31) / 32) * ((B + 31) / 32) < 512 && d >= 1024;
    // a handful of tiles (a skinny output layer): the reduction is split over workgroups as well,
    // a second kernel adds the slices in order
    const int S = (few && split_scratch) ? dense_split_factor(B, n, d) : 1;
    float* split_out = S > 1 ? static_cast<float*>(split_scratch) : nullptr;
    dim3 grid((n + 31) / 32, (B + 31) / 32, S);
#define SLONN_LAUNCH_DIRECT(WDT, KS, SPLIT)                                                             \
  hipLaunchKernelGGL((dense_direct_kernel<WDT, 4, KS, SPLIT>), grid, dim3(64 * KS), 0, s, W, bias, X, ldx, Y, \
                     ldy, B, n, d, a, split_out, S)
    if (w_dtype == SLONN_F32) {
      if (S > 1) SLONN_LAUNCH_DIRECT(SLONN_F32, 16, true);
      else if (few) SLONN_LAUNCH_DIRECT(SLONN_F32, 16, false);
      else SLONN_LAUNCH_DIRECT(SLONN_F32, 4, false);
    } else {
      if (S > 1) SLONN_LAUNCH_DIRECT(SLONN_BF16, 16, true);
      else if (few) SLONN_LAUNCH_DIRECT(SLONN_BF16, 16, false);
      else SLONN_LAUNCH_DIRECT(SLONN_BF16, 4, false);
    }
#undef SLONN_LAUNCH_DIRECT
    SLONN_HIP(hipGetLastError());
    if (S > 1) {
      hipLaunchKernelGGL(dense_split_sum_kernel, dim3((unsigned)(((size_t)B * n + 255) / 256)), dim3(256), 0, s,
                         split_out, S, bias, Y, ldy, B, n, a);
      SLONN_HIP(hipGetLastError());
    }
    return SLONN_OK;
  }
#define SLONN_LAUNCH_DENSE(WDT, BM, BN)                                                            \
  hipLaunchKernelGGL((dense_layer_kernel<WDT, BM, BN>), dim3((n + BN - 1) / BN, (B + BM - 1) / BM), \
                     dim3(256), 0, s, W, bias, X, ldx, Y, ldy, B, n, d, a, vecx, vecw)
  if (w_dtype == SLONN_F32) {
    if (big) SLONN_LAUNCH_DENSE(SLONN_F32, 128, 128); else SLONN_LAUNCH_DENSE(SLONN_F32, 64, 64);
  } else {
    if (big) SLONN_LAUNCH_DENSE(SLONN_BF16, 128, 128); else SLONN_LAUNCH_DENSE(SLONN_BF16, 64, 64);
  }
#undef SLONN_LAUNCH_DENSE
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

}  // namespace slonn
