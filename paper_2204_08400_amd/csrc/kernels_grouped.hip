// Batched evaluation of the active rows with row reuse across queries (the paper's
// Section 6 names batch inference through micro-batches of similar inputs as future work).
// Queries of one batch select heavily overlapping node sets: inputs that fall into similar
// buckets get similar ranked lists.  Instead of gathering every (query, node) row separately,
// 16 consecutive queries form a group; the union of their active rows is evaluated once as
// dense 16-query tiles on the fp32 matrix cores, and only the (query, node) pairs that were
// actually selected are written.  Every selected pair gets w_j . x_q + b_j exactly as in the
// per-query gather (fp32 products and sums); pairs that were not selected are computed and
// discarded, which is cheaper than fetching each row once per query that wants it.
//
//   union_kernel           one workgroup per group: a 16-bit query mask per node in LDS
//                          (integer OR, order-independent), compacted in node order with
//                          ballot + prefix sums into (row id, mask) lists.
//   gather_grouped_kernel  workgroup = 128 union rows x 16 queries; each wavefront owns 32
//                          rows as two 16x16 MFMA tiles (v_mfma_f32_16x16x4_f32), operands as
//                          16-byte loads straight from L2 (lane (r, g) takes elements
//                          16s+4g .. +3 of weight row r and of query r; MFMA c of the step
//                          consumes element c), U steps of loads kept in flight.
#include <algorithm>

#include "slonn_internal.h"

namespace slonn {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int GQ = 16;            // queries per group
constexpr int ROWS_PER_WG = 128;  // union rows per workgroup pass (4 wavefronts x 32)

constexpr int UNT = 1024;          // threads of the union kernel (few workgroups: one per 16 queries)
constexpr int UNW = UNT / 64;

__global__ __launch_bounds__(UNT) void union_kernel(const int32_t* __restrict__ active,
                                                   const int32_t* __restrict__ cnt, int idx_stride, int B,
                                                   int n, int32_t* __restrict__ urows,
                                                   uint32_t* __restrict__ umask, int32_t* __restrict__ ucnt,
                                                   int32_t* __restrict__ gflag, int ustride,
                                                   const int16_t* __restrict__ skip_hslot,
                                                   const float* __restrict__ Z, int H, int relu,
                                                   float* __restrict__ Y, int ldy, int thr10,
                                                   const int32_t* __restrict__ served) {
  extern __shared__ __align__(16) uint32_t mask2[];      // two 16-bit masks per word
  __shared__ int red[UNW];
  __shared__ int listed;                                 // list entries that take part
  const int g = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (served && served[g]) {             // these 16 queries were evaluated as masked tiles
    if (tid == 0) { ucnt[g] = 0; gflag[g] = 0; }
    return;
  }
  const int q0 = g * GQ, nq = min(GQ, B - q0);
  const int words = (n + 1) >> 1;
  for (int i = tid; i < words; i += UNT) mask2[i] = 0u;
  if (tid == 0) listed = 0;
  __syncthreads();
  int mine = 0;
  for (int qi = wave; qi < nq; qi += UNW) {               // one wavefront per query's list
    const int c = cnt[q0 + qi];
    const int32_t* list = active + (size_t)(q0 + qi) * idx_stride;
#pragma unroll 4
    for (int t = lane; t < c; t += 64) {
      const int node = list[t];
      if (skip_hslot) {
        const int hs = skip_hslot[node];
        if (hs >= 0) {                  // a selected hash node: its output is its projection
          if (Z) {
            float v = Z[(size_t)(q0 + qi) * H + hs];
            if (relu && !(v > 0.0f)) v = 0.0f;
            Y[(size_t)(q0 + qi) * ldy + node] = v;
          }
          continue;
        }
      }
      atomicOr(&mask2[node >> 1], (1u << qi) << (16 * (node & 1)));
      ++mine;
    }
  }
  if (mine) atomicAdd(&listed, mine);
  __syncthreads();
  const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  int base = 0;
  for (int i0 = 0; i0 < n; i0 += UNT) {
    const int i = i0 + tid;
    const uint32_t mk = i < n ? (mask2[i >> 1] >> (16 * (i & 1))) & 0xFFFFu : 0u;
    const unsigned long long votes = __ballot(mk != 0u);
    if (lane == 0) red[wave] = __popcll(votes);
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wave; ++w) before += red[w];
    int all = 0;
    for (int w = 0; w < UNW; ++w) all += red[w];
    if (mk != 0u) {
      const int pos = base + before + __popcll(votes & below);
      urows[(size_t)g * ustride + pos] = i;
      umask[(size_t)g * ustride + pos] = mk;
    }
    base += all;
    __syncthreads();
  }
  if (tid == 0) {
    ucnt[g] = base;
    // Evaluating the union for all 16 queries pays while it is at most about three times one
    // query's own list (measured break-even against the row-block gather on 4096-wide fp32
    // layers: union/list = 2.2 -> 0.74x the time, 3.9 -> 1.3x); otherwise the group stays on
    // the per-query gather.
    gflag[g] = ((long long)base * nq * 10 <= (long long)thr10 * listed) ? 1 : 0;
  }
}

template <int WDT>
__device__ __forceinline__ float4 load_w4(const void* W, size_t elem) {
  if (WDT == SLONN_F32) return *reinterpret_cast<const float4*>(static_cast<const float*>(W) + elem);
  const uint2 q = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(W) + elem);
  float4 r;
  r.x = __uint_as_float(q.x << 16);
  r.y = __uint_as_float(q.x & 0xFFFF0000u);
  r.z = __uint_as_float(q.y << 16);
  r.w = __uint_as_float(q.y & 0xFFFF0000u);
  return r;
}

// Lane layout of v_mfma_f32_16x16x4_f32 (checked on gfx950): A[i][k] in lane i + 16k, B[k][j]
// in lane j + 16k, register v of lane l holds D[4*(l/16) + v][l%16].
template <int WDT, int U>
__global__ __launch_bounds__(256) void gather_grouped_kernel(
    const void* __restrict__ W, const float* __restrict__ bias, const float* __restrict__ X, int ldx,
    const int32_t* __restrict__ urows, const uint32_t* __restrict__ umask,
    const int32_t* __restrict__ ucnt, const int32_t* __restrict__ gflag, int ustride, float* __restrict__ Y,
    int ldy, int B, int d, int act, int ychunks) {      // ychunks = gridDim.y
  const int g = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  if (!gflag[g]) return;                 // this group is served by the per-query gather
  const int r = lane & 15, kg = lane >> 4;
  const int uc = ucnt[g];
  const int q0 = g * GQ, nq = min(GQ, B - q0);
  const int32_t* rows = urows + (size_t)g * ustride;
  const uint32_t* masks = umask + (size_t)g * ustride;
  const float* xq = X + (size_t)(q0 + min(r, nq - 1)) * ldx;       // surplus lanes redo a valid query
  const int steps = (d + 15) / 16;
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);

  for (int r0 = blockIdx.y * ROWS_PER_WG + wave * 32; r0 < uc; r0 += ychunks * ROWS_PER_WG) {
    const size_t wa = (size_t)rows[min(r0 + r, uc - 1)] * d;        // surplus lanes redo a valid row
    const size_t wb = (size_t)rows[min(r0 + 16 + r, uc - 1)] * d;
    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    // Software pipeline of depth U: buffer u holds step s+u; as soon as it has been copied out
    // for the MFMAs its slot is refilled with step s+u+U, so U steps of loads (3 x 16 bytes
    // each) stay in flight behind the matrix work.
    float4 a[U], b[U], x[U];
    auto fetch = [&](int u, int step) {
      const int k = 16 * step + 4 * kg;
      const bool ok = step < steps && k < d;           // d is a multiple of 4
      const int kk = ok ? k : 0;                        // out-of-range steps load element 0 ...
      const float4 va = load_w4<WDT>(W, wa + kk), vb = load_w4<WDT>(W, wb + kk);
      const float4 vx = *reinterpret_cast<const float4*>(xq + kk);
      a[u] = ok ? va : zero4;                           // ... and contribute nothing
      b[u] = ok ? vb : zero4;
      x[u] = ok ? vx : zero4;
    };
#pragma unroll
    for (int u = 0; u < U; ++u) fetch(u, u);
    for (int s0 = 0; s0 < steps; s0 += U) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float4 ca = a[u], cb = b[u], cx = x[u];
        fetch(u, s0 + u + U);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(ca.x, cx.x, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(cb.x, cx.x, acc1, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(ca.y, cx.y, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(cb.y, cx.y, acc1, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(ca.z, cx.z, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(cb.z, cx.z, acc1, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(ca.w, cx.w, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(cb.w, cx.w, acc1, 0, 0, 0);
      }
    }
    // register v of this lane: union row r0 + 16*f + 4*kg + v, query q0 + r
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int ui = r0 + 16 * f + 4 * kg + v;
        if (ui < uc && r < nq) {
          const uint32_t mk = masks[ui];
          if ((mk >> r) & 1u) {
            const int row = rows[ui];
            float z = (f == 0 ? acc0[v] : acc1[v]) + bias[row];
            if (act == SLONN_ACT_RELU) z = z > 0.0f ? z : 0.0f;
            Y[(size_t)(q0 + r) * ldy + row] = z;
          }
        }
      }
  }
}

// ---- bf16 weights: the same evaluation on the bf16 matrix cores at fp32 accuracy ----
// An fp32 activation is the exact sum of three bf16 numbers (8 + 8 + 8 significand bits):
// x = hi + mid + lo.  With bf16 weights every product w * hi, w * mid, w * lo is exact in fp32,
// so three bf16 MFMAs accumulate the same products an fp32 FMA chain would, at sixteen times the
// fp32 MFMA rate.  The kernel is then bound by fetching each union row once per 16 queries
// instead of by arithmetic.  split_x_kernel writes the three parts of a batch of activations;
// gather_grouped_bf16_kernel uses v_mfma_f32_16x16x32_bf16 (lane l feeds row/query l % 16 with
// the eight elements 32 s + 8 (l / 16) .. + 7; register v of lane l holds
// D[4 (l / 16) + v][l % 16], rows from the first operand; checked on gfx950).
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__global__ void split_x_kernel(const float* __restrict__ X, int ldx, int B, int d,
                               uint16_t* __restrict__ xs3, const int32_t* __restrict__ served) {
  const int q = blockIdx.x;                             // one workgroup per query
  if (served && served[q >> 4]) return;                 // evaluated as masked tiles: not needed here
  const size_t plane = (size_t)B * d;
  for (int i = threadIdx.x; i < d; i += 256) {
    const float x = X[(size_t)q * ldx + i];
    const uint32_t hb = __float_as_uint(x) & 0xFFFF0000u;
    const float r1 = x - __uint_as_float(hb);           // exact: hi keeps the leading bits of x
    const uint32_t mb = __float_as_uint(r1) & 0xFFFF0000u;
    const float r2 = r1 - __uint_as_float(mb);          // exact, at most 8 significant bits left
    const size_t at = (size_t)q * d + i;
    xs3[at] = (uint16_t)(hb >> 16);
    xs3[plane + at] = (uint16_t)(mb >> 16);
    xs3[2 * plane + at] = (uint16_t)(__float_as_uint(r2) >> 16);
  }
}

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& v) {
  bf16x8 r;
  __builtin_memcpy(&r, &v, 16);
  return r;
}

// T: 16-row tiles per wavefront (a workgroup pass covers 4 * 16 * T union rows)
template <int T>
__global__ __launch_bounds__(256) void gather_grouped_bf16_kernel(
    const uint16_t* __restrict__ W, const float* __restrict__ bias, const uint16_t* __restrict__ xs3,
    const int32_t* __restrict__ urows, const uint32_t* __restrict__ umask,
    const int32_t* __restrict__ ucnt, const int32_t* __restrict__ gflag, int ustride, float* __restrict__ Y,
    int ldy, int B, int d, int act, int ychunks) {      // ychunks = gridDim.y
  const int g = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  if (!gflag[g]) return;                 // this group is served by the per-query gather
  const int r = lane & 15, kg = lane >> 4;
  const int uc = ucnt[g];
  const int q0 = g * GQ, nq = min(GQ, B - q0);
  const int32_t* rows = urows + (size_t)g * ustride;
  const uint32_t* masks = umask + (size_t)g * ustride;
  const size_t plane = (size_t)B * d;
  const uint16_t* xh = xs3 + (size_t)(q0 + min(r, nq - 1)) * d;    // surplus lanes redo a valid query
  const uint16_t* xm = xh + plane;
  const uint16_t* xl = xm + plane;
  const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
  constexpr int ROWS_WG = 4 * 16 * T;

  for (int r0 = blockIdx.y * ROWS_WG + wave * 16 * T; r0 < uc; r0 += ychunks * ROWS_WG) {
    const uint16_t* wr[T];
#pragma unroll
    for (int t = 0; t < T; ++t) wr[t] = W + (size_t)rows[min(r0 + 16 * t + r, uc - 1)] * d;   // surplus lanes redo a valid row
    f32x4 acc[T];
#pragma unroll
    for (int t = 0; t < T; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // two steps of loads in flight: while the MFMAs of step s run, step s + 1 is on its way.
    // Steps that lie wholly inside the rows need no checks; a ragged last step (d not a
    // multiple of 32) zeroes the lanes beyond the end.
    uint4 a[2][T], bh[2], bm[2], bl[2];
    auto fetch = [&](int u, int step) {
      const int k = 32 * step + 8 * kg;
#pragma unroll
      for (int t = 0; t < T; ++t) a[u][t] = *reinterpret_cast<const uint4*>(wr[t] + k);
      bh[u] = *reinterpret_cast<const uint4*>(xh + k);
      bm[u] = *reinterpret_cast<const uint4*>(xm + k);
      bl[u] = *reinterpret_cast<const uint4*>(xl + k);
    };
    auto compute = [&](int u) {
      const bf16x8 vh = as_bf16x8(bh[u]), vm = as_bf16x8(bm[u]), vl = as_bf16x8(bl[u]);
#pragma unroll
      for (int t = 0; t < T; ++t) {
        const bf16x8 va = as_bf16x8(a[u][t]);
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, vl, acc[t], 0, 0, 0);
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, vm, acc[t], 0, 0, 0);
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, vh, acc[t], 0, 0, 0);
      }
    };
    const int nfull = d / 32;
    if (nfull > 0) fetch(0, 0);
    for (int s0 = 0; s0 < nfull; s0 += 2) {
      if (s0 + 1 < nfull) fetch(1, s0 + 1);
      compute(0);
      if (s0 + 1 < nfull) {
        if (s0 + 2 < nfull) fetch(0, s0 + 2);
        compute(1);
      }
    }
    if (d % 32) {
      const int k = 32 * nfull + 8 * kg;
      const bool ok = k < d;                           // d is a multiple of 8
      const int kk = ok ? k : 0;                        // lanes beyond the end load element 0 ...
#pragma unroll
      for (int t = 0; t < T; ++t) {
        const uint4 v = *reinterpret_cast<const uint4*>(wr[t] + kk);
        a[0][t] = ok ? v : zero;                        // ... and contribute nothing
      }
      const uint4 vh = *reinterpret_cast<const uint4*>(xh + kk);
      const uint4 vm = *reinterpret_cast<const uint4*>(xm + kk);
      const uint4 vl = *reinterpret_cast<const uint4*>(xl + kk);
      bh[0] = ok ? vh : zero;
      bm[0] = ok ? vm : zero;
      bl[0] = ok ? vl : zero;
      compute(0);
    }
    // register v of this lane: union row r0 + 16*t + 4*kg + v, query q0 + r
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int ui = r0 + 16 * t + 4 * kg + v;
        if (ui < uc && r < nq) {
          const uint32_t mk = masks[ui];
          if ((mk >> r) & 1u) {
            const int row = rows[ui];
            float z = acc[t][v] + bias[row];
            if (act == SLONN_ACT_RELU) z = z > 0.0f ? z : 0.0f;
            Y[(size_t)(q0 + r) * ldy + row] = z;
          }
        }
      }
  }
}

}  // namespace

size_t grouped_workspace_bytes(int B, int n, int d_bf16) {
  const size_t ng = (size_t)(B + GQ - 1) / GQ;
  const size_t lists = (ng * n * 8 + ng * 8 + 511) / 256 * 256;
  return lists + (size_t)3 * B * d_bf16 * 2 + 256;        // + the three bf16 parts of the activations
}

bool grouped_supported(int n, int max_lds) { return (size_t)((n + 1) / 2) * 4 + 64 <= (size_t)max_lds; }

bool grouped_uses_bf16_cores(const void* W, int w_dtype, int d) {
  return w_dtype == SLONN_BF16 && d % 8 == 0 && reinterpret_cast<uintptr_t>(W) % 16 == 0;
}

int launch_gather_grouped(const void* W, int w_dtype, const float* bias, const float* X, int ldx,
                          const int32_t* active, const int32_t* cnt, int idx_stride, float* Y, int ldy,
                          int B, int d, int n, int act, const GroupedReuse* reuse, const int32_t* served,
                          void* scratch, int max_lds, int32_t** gflag_out, hipStream_t s) {
  const GroupedReuse ru = reuse ? *reuse : GroupedReuse{};
  const int ng = (B + GQ - 1) / GQ;
  int32_t* urows = static_cast<int32_t*>(scratch);
  uint32_t* umask = reinterpret_cast<uint32_t*>(urows + (size_t)ng * n);
  int32_t* ucnt = reinterpret_cast<int32_t*>(umask + (size_t)ng * n);
  int32_t* gflag = ucnt + ng;
  *gflag_out = gflag;
  const size_t lists = ((size_t)ng * n * 8 + (size_t)ng * 8 + 511) / 256 * 256;
  uint16_t* xs3 = reinterpret_cast<uint16_t*>(static_cast<char*>(scratch) + lists);
  const bool bf16_cores = grouped_uses_bf16_cores(W, w_dtype, d);
  // A group goes to the matrix cores while its union is at most thr10 / 10 times its mean list.
  // fp32 MFMA path (bound by arithmetic): measured break-even 3 on 4096-wide fp32 layers
  // (union/list 2.2 -> 0.74x the time of the row-block gather, 3.9 -> 1.3x).  bf16 path (bound
  // by fetching each union row once per group instead of once per query): ahead of the
  // row-block gather for every group measured (8192-wide bf16 layers, unions up to 6x the mean
  // list: 9.2 -> 6.3 ms of gather per 2048 queries), so every group takes it (a union is never
  // larger than the sum of its lists, i.e. 16x the mean list).
  // (bf16 rows that cannot take the bf16 path -- length not a multiple of 8 -- cost the gather
  // half the bytes of fp32 rows at the same fp32 MFMA work: break-even 1.5)
  const int thr10 = bf16_cores ? 160 : (w_dtype == SLONN_F32 ? 30 : 15);
  const size_t lds = (size_t)((n + 1) / 2) * 4;
  {
    ProfScope prof_(SLONN_PROF_SELECT, s);
    if (lds > (size_t)max_lds) SLONN_FAIL(SLONN_EUNSUPPORTED, "grouped gather: layer too wide for LDS");
    if (lds > 65536)
      SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(union_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(union_kernel, dim3(ng), dim3(UNT), lds, s, active, cnt, idx_stride, B, n, urows, umask,
                       ucnt, gflag, n, ru.hslot, ru.Z, ru.H, ru.relu, Y, ldy, thr10, served);
    SLONN_HIP(hipGetLastError());
    if (bf16_cores) {
      hipLaunchKernelGGL(split_x_kernel, dim3(B), dim3(256), 0, s, X, ldx, B, d, xs3, served);
      SLONN_HIP(hipGetLastError());
    }
  }
  ProfScope prof_(SLONN_PROF_GATHER, s);
  const int a = (act == SLONN_ACT_RELU) ? SLONN_ACT_RELU : SLONN_ACT_NONE;
  if (bf16_cores) {
    // eight 16-row tiles per wavefront: the three activation operands are fetched once per 128
    // rows (measured on C5: 10.0 / 7.4 / 6.3 ms of gather per step with 2 / 4 / 8 tiles)
    constexpr int T = 8;
    int chunks = (n + 64 * T - 1) / (64 * T);
    chunks = std::min(chunks, std::max(4, 4096 / ng));
    hipLaunchKernelGGL((gather_grouped_bf16_kernel<T>), dim3(ng, chunks), dim3(256), 0, s,
                       static_cast<const uint16_t*>(W), bias, xs3, urows, umask, ucnt, gflag, n, Y, ldy, B, d, a, chunks);
    SLONN_HIP(hipGetLastError());
    return SLONN_OK;
  }
  int chunks = (n + ROWS_PER_WG - 1) / ROWS_PER_WG;
  chunks = std::min(chunks, std::max(4, 4096 / ng));
  dim3 grid(ng, chunks);
  if (w_dtype == SLONN_F32)
    hipLaunchKernelGGL((gather_grouped_kernel<SLONN_F32, 4>), grid, dim3(256), 0, s, W, bias, X, ldx, urows,
                       umask, ucnt, gflag, n, Y, ldy, B, d, a, chunks);
  else
    hipLaunchKernelGGL((gather_grouped_kernel<SLONN_BF16, 4>), grid, dim3(256), 0, s, W, bias, X, ldx, urows,
                       umask, ucnt, gflag, n, Y, ldy, B, d, a, chunks);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

}  // namespace slonn
