// FreeHash projections (Def. 2, Section 3.4): z[q][h] = w_h . x_q + b_h for the K*L
// sampled nodes of a layer, shared by every query of the batch -> a dense contraction
// [B x d] . [d x H].  The sign of z is a hash bit, so the sum is carried in fp64: the
// fp32 x fp32 products are exact in fp64 and the result's sign then only depends on
// summation order when |z| is at the 1e-15 level, instead of the 1e-7 level of an
// fp32 accumulator.
//
// hash_project_mfma_kernel: fp64 matrix cores (v_mfma_f64_16x16x4_f64).  A workgroup owns a
// 32x32 (large batches) or 16x16 (small batches) tile of Z; its 4 or 16 wavefronts split
// the reduction dimension and their partial tiles are added in LDS in a fixed order.
// A medium batch (a few dozen queries) has only a few dozen 16x16 tiles, and a tile's operand
// rows would reach one compute unit at that unit's own L2 bandwidth; there the reduction
// dimension is also split over several workgroups (grid.z).  Each writes its partial sums in
// fp64 and hash_split_sum_kernel adds them in split order.
// Operands are read straight from global memory/L2 as 16-byte loads: lane (r = lane%16,
// g = lane/16) fetches elements 16s+4g .. 16s+4g+3 of its row, and MFMA number c of that
// step consumes element c from every lane -- the same K subset for the X and the Wh
// operand, which is all the instruction needs.
// hash_project_kernel: LDS-tiled fp64 FMAs on the vector ALUs, for rows that are not
// 16-byte aligned multiples of four elements.
#include <algorithm>

#include "slonn_internal.h"

namespace slonn {
namespace {

typedef double f64x4 __attribute__((ext_vector_type(4)));

// Lane layout of v_mfma_f64_16x16x4_f64 (checked on gfx950): A[i][k] sits in lane i + 16k,
// B[k][j] in lane j + 16k, D[i][j] in register i / 4 ... precisely: register v of lane l
// holds D[4v + l/16][l%16].
// TM x TN 16x16 MFMA tiles per wavefront; U reduction steps (16 elements each) are
// loaded ahead of the MFMAs that consume them; KS wavefronts split the reduction
// dimension (small batches need the extra wavefronts to cover the load latency).
template <int TM, int TN, int U, int KS, bool SPLIT = false>
__global__ __launch_bounds__(64 * KS) void hash_project_mfma_kernel(const float* __restrict__ X, int ldx,
                                                               const float* __restrict__ Wh,
                                                               const float* __restrict__ bh,
                                                               float* __restrict__ Z, int B, int H, int d,
                                                               double* __restrict__ gpart = nullptr,
                                                               int nslices = 1) {
  __shared__ double part[KS - 1][64][TM * TN * 4];     // partial tiles of waves 1..KS-1
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int q0 = blockIdx.y * (16 * TM), h0 = blockIdx.x * (16 * TN);
  // rows this lane feeds (clamped: surplus rows recompute a valid row and are not stored)
  const float* xr[TM];
  const float* wr[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) xr[i] = X + (size_t)min(q0 + 16 * i + r, B - 1) * ldx;
#pragma unroll
  for (int j = 0; j < TN; ++j) wr[j] = Wh + (size_t)min(h0 + 16 * j + r, H - 1) * d;
  // this wave's share of the reduction dimension, in steps of 16 elements (with SPLIT the
  // workgroup itself owns one of nslices = gridDim.z consecutive ranges of steps; the count
  // comes as an argument, which is quicker to reach than the dispatch packet)
  const int steps = (d + 15) / 16;
  int wg_begin = 0, wg_end = steps;
  if (SPLIT) {
    const int per_wg = (steps + nslices - 1) / nslices;
    wg_begin = min(steps, (int)blockIdx.z * per_wg);
    wg_end = min(steps, wg_begin + per_wg);
  }
  const int per = (wg_end - wg_begin + KS - 1) / KS;
  const int s_begin = min(wg_end, wg_begin + wave * per), s_end = min(wg_end, s_begin + per);

  f64x4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = (f64x4){0.0, 0.0, 0.0, 0.0};

  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
  float4 a[U][TM], b[U][TN];
  auto fetch = [&](int s0) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int k = 16 * (s0 + u) + 4 * g;
      // d is a multiple of 4: a 16-byte load is entirely inside the row or entirely outside
      // (out-of-range steps load element 0 and are zeroed afterwards: the load itself stays an
      // unconditional 16-byte load)
      const bool ok = (s0 + u < s_end) && k < d;
      const int kk = ok ? k : 0;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const float4 v = *reinterpret_cast<const float4*>(xr[i] + kk);
        a[u][i] = ok ? v : zero4;
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const float4 v = *reinterpret_cast<const float4*>(wr[j] + kk);
        b[u][j] = ok ? v : zero4;
      }
    }
  };
  fetch(s_begin);
  for (int s0 = s_begin; s0 < s_end; s0 += U) {
    // widen the current operands, then start the next loads so they fly during the MFMAs
    double da[U][TM][4], db[U][TN][4];
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        da[u][i][0] = a[u][i].x; da[u][i][1] = a[u][i].y; da[u][i][2] = a[u][i].z; da[u][i][3] = a[u][i].w;
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        db[u][j][0] = b[u][j].x; db[u][j][1] = b[u][j].y; db[u][j][2] = b[u][j].z; db[u][j][3] = b[u][j].w;
      }
    }
    if (s0 + U < s_end) fetch(s0 + U);
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(da[u][i][c], db[u][j][c], acc[i][j], 0, 0, 0);
  }

  if (wave > 0) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) part[wave - 1][lane][(i * TN + j) * 4 + v] = acc[i][j][v];
  }
  __syncthreads();
  if (wave != 0) return;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int w = 0; w < KS - 1; ++w) acc[i][j][v] += part[w][lane][(i * TN + j) * 4 + v];
  if (SPLIT) {
    // partial sums [split][query][hash row] in fp64; hash_split_sum_kernel adds them
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int h = h0 + 16 * j + r;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int q = q0 + 16 * i + 4 * v + g;
          if (q < B && h < H) gpart[((size_t)blockIdx.z * B + q) * H + h] = acc[i][j][v];
        }
      }
    return;
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int h = h0 + 16 * j + r;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int q = q0 + 16 * i + 4 * v + g;
        if (q < B && h < H) Z[(size_t)q * H + h] = (float)(acc[i][j][v] + (double)bh[h]);
      }
    }
}

// A handful of queries cannot fill a 16-row MFMA tile: one wavefront per (query, hash row),
// fp64 FMAs on the vector ALUs, x staged in LDS, four 16-byte loads in flight per lane.
__global__ __launch_bounds__(256) void hash_project_rowwise_kernel(const float* __restrict__ X, int ldx,
                                                                  const float* __restrict__ Wh,
                                                                  const float* __restrict__ bh,
                                                                  float* __restrict__ Z, int H, int d) {
  extern __shared__ __align__(16) float xs_hash[];
  const int q = blockIdx.y, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float4* x4 = reinterpret_cast<const float4*>(X + (size_t)q * ldx);
  for (int i = tid; i < (d >> 2); i += 256) reinterpret_cast<float4*>(xs_hash)[i] = x4[i];
  __syncthreads();
  const int h = blockIdx.x * 4 + wave;
  if (h >= H) return;
  const float4* w = reinterpret_cast<const float4*>(Wh + (size_t)h * d);
  const int nv = d >> 2;
  double acc = 0.0;
#pragma unroll 4
  for (int i = lane; i < nv; i += 64) {
    const float4 a = w[i];
    const float4 x = reinterpret_cast<const float4*>(xs_hash)[i];
    acc = fma((double)a.x, (double)x.x, acc);
    acc = fma((double)a.y, (double)x.y, acc);
    acc = fma((double)a.z, (double)x.z, acc);
    acc = fma((double)a.w, (double)x.w, acc);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
  if (lane == 0) Z[(size_t)q * H + h] = (float)(acc + (double)bh[h]);
}

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

// Splitting the reduction over workgroups: at most SPLIT_MAX_WGS workgroups, each with its
// partial 16x16 tile in fp64.
constexpr int SPLIT_MAX_WGS = 512;

__global__ __launch_bounds__(256) void hash_split_sum_kernel(const double* __restrict__ gpart, int S,
                                                            const float* __restrict__ bh,
                                                            float* __restrict__ Z, int B, int H) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= B * H) return;
  double sum = 0.0;
  for (int z = 0; z < S; ++z) sum += gpart[(size_t)z * B * H + i];
  Z[i] = (float)(sum + (double)bh[i % H]);
}

}  // namespace

size_t hash_split_workspace_bytes() { return (size_t)SPLIT_MAX_WGS * 256 * sizeof(double); }

int hash_split_factor(int B, int H, int d) {
  if (B <= 4 || d % 4 != 0) return 1;
  const long tiles32 = (long)((H + 31) / 32) * ((B + 31) / 32);
  if (tiles32 >= 128) return 1;
  const int tiles16 = ((H + 15) / 16) * ((B + 15) / 16);
  const int steps = (d + 15) / 16;
  // at least 8 steps (128 elements of the rows) per workgroup
  const int S = std::min(std::min(8, SPLIT_MAX_WGS / tiles16), steps / 8);
  return S >= 2 ? S : 1;
}

namespace {
int launch_hash_project_chunk(const float* X, int ldx, const float* Wh, const float* bh, float* Z, int B,
                              int H, int d, void* split_scratch, HashSplit* pending, hipStream_t s);
}

int launch_hash_project(const float* X, int ldx, const float* Wh, const float* bh, float* Z, int B,
                        int H, int d, void* split_scratch, HashSplit* pending, hipStream_t s) {
  ProfScope prof_(SLONN_PROF_HASH, s);
  // the batch runs along the grid's y dimension (limit 65535) in tiles of at least 16 queries, one
  // query per y step for the smallest batches: chunks of 2^19 queries stay within it
  constexpr int CHUNK = 1 << 19;
  for (int q0 = 0; q0 < B; q0 += CHUNK) {
    const int nb = std::min(CHUNK, B - q0);
    const int rc = launch_hash_project_chunk(X + (size_t)q0 * ldx, ldx, Wh, bh, Z + (size_t)q0 * H, nb, H, d,
                                             split_scratch, B <= CHUNK ? pending : nullptr, s);
    if (rc) return rc;
  }
  return SLONN_OK;
}

namespace {
int launch_hash_project_chunk(const float* X, int ldx, const float* Wh, const float* bh, float* Z, int B,
                              int H, int d, void* split_scratch, HashSplit* pending, hipStream_t s) {
  const bool vec = (d % 4 == 0) && (ldx % 4 == 0) && (reinterpret_cast<uintptr_t>(X) % 16 == 0) &&
                   (reinterpret_cast<uintptr_t>(Wh) % 16 == 0);
  const int S = (vec && split_scratch) ? hash_split_factor(B, H, d) : 1;
  if (S > 1) {
    double* gpart = static_cast<double*>(split_scratch);
    dim3 g((H + 15) / 16, (B + 15) / 16, S);
    hipLaunchKernelGGL((hash_project_mfma_kernel<1, 1, 4, 4, true>), g, dim3(256), 0, s, X, ldx, Wh, bh, Z, B, H,
                       d, gpart, S);
    SLONN_HIP(hipGetLastError());
    if (pending) {
      pending->part = gpart; pending->S = S; pending->B = B; pending->bh = bh; pending->Z = Z;
      return SLONN_OK;
    }
    hipLaunchKernelGGL(hash_split_sum_kernel, dim3((B * H + 255) / 256), dim3(256), 0, s, gpart, S, bh, Z, B, H);
    SLONN_HIP(hipGetLastError());
    return SLONN_OK;
  }
  if (vec && B <= 4 && (size_t)d * 4 + 64 <= 65536) {
    hipLaunchKernelGGL(hash_project_rowwise_kernel, dim3((H + 3) / 4, B), dim3(256), (size_t)d * 4 + 64, s, X,
                       ldx, Wh, bh, Z, H, d);
    SLONN_HIP(hipGetLastError());
    return SLONN_OK;
  }
  if (vec) {
    // small problems: one 16x16 tile per wavefront so that there are enough workgroups
    const long tiles32 = (long)((H + 31) / 32) * ((B + 31) / 32);
    if (tiles32 >= 128) {
      // Tile shape per workgroup (TM x TN tiles of 16x16): the one whose workgroup count fills
      // the compute units most evenly.  A workgroup count just above a multiple of the unit
      // count leaves most of the chip idle for the last round (C3: 320 workgroups of 2x2 tiles
      // on 256 units, against exactly 256 of 1x5).  Shapes with fewer operand loads per MFMA
      // win ties.
      static const int shapes[4][2] = {{2, 2}, {2, 3}, {1, 5}, {1, 4}};
      static int n_cu = 0;                  // compute units of the device (looked up once)
      if (n_cu == 0) {
        int dev = 0, v = 0;
        n_cu = 256;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
          n_cu = v;
      }
      int best = 0;
      double best_cost = 0.0;
      for (int c = 0; c < 4; ++c) {
        const int tm = shapes[c][0], tn = shapes[c][1];
        const long wgs = (long)((B + 16 * tm - 1) / (16 * tm)) * ((H + 16 * tn - 1) / (16 * tn));
        const long rounds = (wgs + n_cu - 1) / n_cu;
        const double cost = (double)rounds * tm * tn * (1.0 + 0.25 * (tm + tn) / (tm * tn));
        if (c == 0 || cost < best_cost * 0.97) { best = c; best_cost = cost; }
      }
      const int tm = shapes[best][0], tn = shapes[best][1];
      dim3 g((H + 16 * tn - 1) / (16 * tn), (B + 16 * tm - 1) / (16 * tm));
      if (best == 0)
        hipLaunchKernelGGL((hash_project_mfma_kernel<2, 2, 2, 4>), g, dim3(256), 0, s, X, ldx, Wh, bh, Z, B, H, d);
      else if (best == 1)
        hipLaunchKernelGGL((hash_project_mfma_kernel<2, 3, 2, 4>), g, dim3(256), 0, s, X, ldx, Wh, bh, Z, B, H, d);
      else if (best == 2)
        hipLaunchKernelGGL((hash_project_mfma_kernel<1, 5, 2, 4>), g, dim3(256), 0, s, X, ldx, Wh, bh, Z, B, H, d);
      else
        hipLaunchKernelGGL((hash_project_mfma_kernel<1, 4, 2, 4>), g, dim3(256), 0, s, X, ldx, Wh, bh, Z, B, H, d);
    } else {
      dim3 g((H + 15) / 16, (B + 15) / 16);
      hipLaunchKernelGGL((hash_project_mfma_kernel<1, 1, 4, 16>), g, dim3(1024), 0, s, X, ldx, Wh, bh, Z, B, H, d);
    }
    SLONN_HIP(hipGetLastError());
    return SLONN_OK;
  }
  dim3 grid((H + TH - 1) / TH, (B + TQ - 1) / TQ);
  hipLaunchKernelGGL(hash_project_kernel, grid, dim3(256), 0, s, X, ldx, Wh, bh, Z, B, H, d);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}
}  // namespace

// FreeHash rows are borrowed from the layer itself (Def. 2): copy them once into one contiguous
// fp32 matrix so that the projection reads a dense operand.
namespace {
__global__ void gather_hash_rows_kernel(const void* __restrict__ W, int w_dtype, const float* __restrict__ bias,
                                        const int32_t* __restrict__ hnodes, int d, float* __restrict__ Wh,
                                        float* __restrict__ bh) {
  const int h = blockIdx.x;
  const size_t row = (size_t)hnodes[h] * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    float v;
    if (w_dtype == SLONN_F32) v = static_cast<const float*>(W)[row + i];
    else v = __uint_as_float((uint32_t) static_cast<const uint16_t*>(W)[row + i] << 16);
    Wh[(size_t)h * d + i] = v;
  }
  if (threadIdx.x == 0) bh[h] = bias[hnodes[h]];
}
}  // namespace

int launch_gather_hash_rows(const void* W, int w_dtype, const float* bias, const int32_t* hnodes, int H, int d,
                            float* Wh, float* bh, hipStream_t s) {
  hipLaunchKernelGGL(gather_hash_rows_kernel, dim3(H), dim3(256), 0, s, W, w_dtype, bias, hnodes, d, Wh, bh);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

}  // namespace slonn
