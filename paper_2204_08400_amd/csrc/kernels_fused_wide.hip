// Whole-network kernel for the wide sparse-input models of Table 1 (Wiki10, AmazonCat-13K,
// Delicious-200K: ~10^5 sparse input features -> one small hidden layer -> 10^4..10^5 labels,
// Node Activator on the output layer only, Section 4 "Model Pruning").  One workgroup
// of 1024 or 512 threads carries one query through both layers in one launch:
//
//   hidden  y1 = act(sum_t val[t] * W0[idx[t]][:] + b0): the first layer is stored input-major,
//           so every non-zero contributes one contiguous row; 16-byte column chunks across
//           lanes, the non-zeros split over lane groups, partial sums added in LDS in a fixed
//           order.  y1 stays in LDS.
//   hash    FreeHash projections of the output layer's K*L sampled nodes on y1 (Def. 2), fp64,
//           over the non-zero hidden activations only, the hash rows read input-major.
//   select  keys -> buckets -> first m distinct nodes (Fig. 2 steps 3-4) with one bit per node
//           in LDS (select_block.h, wide variant); the list is built in LDS while it fits there,
//           else straight in global memory (the caller's compact id array), so its length is
//           not limited by LDS.
//   gather  logits of the listed nodes only, 16 lanes per row, four rows in flight.
//   tail    argmax and softmax over the computed nodes (Section 2.1), compact (id, value)
//           output; the dense row is written only when the caller asks for it.
//
// The separate launches of the per-layer path cost more than their work at these sizes
// (a query moves well under a megabyte); here the query's state never leaves the CU.
#include "select_block.h"
#include "slonn_internal.h"

namespace slonn {
namespace {

constexpr int NT_MAX = 1024;       // threads per workgroup: 1024 or 512
constexpr int VALS_LDS = 4096;     // lists up to this length keep their logits in LDS

__device__ __forceinline__ int budget_of(float keep, int n) {
  double m = floor((double)keep * (double)n + 0.5);
  if (!(m >= 1.0)) m = 1.0;        // also a keep fraction that is not a number
  if (m > (double)n) m = (double)n;
  return (int)m;
}

__device__ __forceinline__ float reduce16(float v) {
  v += __shfl_xor(v, 8, 16);
  v += __shfl_xor(v, 4, 16);
  v += __shfl_xor(v, 2, 16);
  v += __shfl_xor(v, 1, 16);
  return v;
}
__device__ __forceinline__ double reduce16(double v) {
  v += __shfl_xor(v, 8, 16);
  v += __shfl_xor(v, 4, 16);
  v += __shfl_xor(v, 2, 16);
  v += __shfl_xor(v, 1, 16);
  return v;
}

// four consecutive weights starting at element e (a multiple of 4; bf16 widens exactly)
__device__ __forceinline__ float4 load_w4(const void* W, int w_dtype, size_t e) {
  if (w_dtype == SLONN_F32) return *reinterpret_cast<const float4*>(static_cast<const float*>(W) + e);
  const uint2 u = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(W) + e);
  float4 r;
  r.x = __uint_as_float(u.x << 16);
  r.y = __uint_as_float(u.x & 0xFFFF0000u);
  r.z = __uint_as_float(u.y << 16);
  r.w = __uint_as_float(u.y & 0xFFFF0000u);
  return r;
}

__device__ __forceinline__ float dot4(const float4& w, const float* xs, float acc) {
  const float4 x = *reinterpret_cast<const float4*>(xs);
  acc = fmaf(w.x, x.x, acc);
  acc = fmaf(w.y, x.y, acc);
  acc = fmaf(w.z, x.z, acc);
  acc = fmaf(w.w, x.w, acc);
  return acc;
}

template <int LPR>
__device__ __forceinline__ float reduce_group(float v) {
  if (LPR == 16) v += __shfl_xor(v, 8, 16);
  v += __shfl_xor(v, 4, LPR);
  v += __shfl_xor(v, 2, LPR);
  v += __shfl_xor(v, 1, LPR);
  return v;
}

// R rows per LPR-lane group in flight: vals[t] = w_{list[t]} . x + b for t = t0 + k * (NT / LPR).
// Short rows (a few hundred bytes) take 8 lanes so that a pass covers twice as many rows.
template <int R, int LPR, int NT>
__device__ __forceinline__ void gather_pass(const void* __restrict__ W, int w_dtype,
                                            const float* __restrict__ bias, int d, const float* xs,
                                            const int32_t* list, int t0, int count, float* vals) {
  constexpr int NG = NT / LPR;
  const int l = threadIdx.x & (LPR - 1);
  const int nv = d >> 2;
  int t[R], j[R];
  float acc[R];
  uint32_t row4[R];                 // row start in units of four elements (n * d / 4 < 2^32 is checked on the host)
#pragma unroll
  for (int k = 0; k < R; ++k) {
    t[k] = t0 + k * NG;
    const int tt = t[k] < count ? t[k] : t0;
    j[k] = list ? list[tt] : tt;
    acc[k] = 0.f;
    row4[k] = (uint32_t)j[k] * (uint32_t)nv;
  }
#pragma unroll 2
  for (int i = l; i < nv; i += LPR) {
    float4 v[R];
#pragma unroll
    for (int k = 0; k < R; ++k) v[k] = load_w4(W, w_dtype, 4 * ((size_t)row4[k] + i));
#pragma unroll
    for (int k = 0; k < R; ++k) acc[k] = dot4(v[k], xs + 4 * i, acc[k]);
  }
#pragma unroll
  for (int k = 0; k < R; ++k) acc[k] = reduce_group<LPR>(acc[k]);
#pragma unroll
  for (int k = 0; k < R; ++k)
    if (l == k && t[k] < count) vals[t[k]] = acc[k] + bias[j[k]];
}

template <int LPR, int NT>
__device__ __forceinline__ void gather_list(const void* __restrict__ W, int w_dtype,
                                            const float* __restrict__ bias, int d, const float* xs,
                                            const int32_t* list, int total, float* vals) {
  constexpr int NG = NT / LPR;
  constexpr int RMAX = (LPR == 16) ? 6 : 4;
  const int g = threadIdx.x / LPR;
  for (int base = 0; base < total; base += RMAX * NG) {
    const int left = total - base;
    const int t0 = base + g;
    if (t0 >= total) continue;
    if (LPR == 16 && left > 4 * NG) gather_pass<6, LPR, NT>(W, w_dtype, bias, d, xs, list, t0, total, vals);
    else if (left > 3 * NG) gather_pass<4, LPR, NT>(W, w_dtype, bias, d, xs, list, t0, total, vals);
    else if (left > 2 * NG) gather_pass<3, LPR, NT>(W, w_dtype, bias, d, xs, list, t0, total, vals);
    else if (left > NG) gather_pass<2, LPR, NT>(W, w_dtype, bias, d, xs, list, t0, total, vals);
    else gather_pass<1, LPR, NT>(W, w_dtype, bias, d, xs, list, t0, total, vals);
  }
}

template <int NT>
__global__ __launch_bounds__(NT) void fused_wide_kernel(FusedWideArgs a) {
  constexpr int NW = NT / 64, GROUPS = NT / 16;
  extern __shared__ __align__(16) unsigned char smem[];
  // carve-up (every region a multiple of 16 bytes)
  float* part = reinterpret_cast<float*>(smem);                       // [NT][4] partial hidden sums
  float* xs = part + NT * 4;                                          // [n1p] hidden activations
  float* zs = xs + a.n1p;                                             // [Hp] projections
  int32_t* s_idx = reinterpret_cast<int32_t*>(zs + a.Hp);             // [ellp]
  float* s_val = reinterpret_cast<float*>(s_idx + a.ellp);            // [ellp]
  float* red_f = s_val + a.ellp;                                      // [NW] block reductions
  int32_t* red_i = reinterpret_cast<int32_t*>(red_f + NW);            // [NW]
  float* lvals = reinterpret_cast<float*>(red_i + NW);                // [VALS_LDS] logits of a short list
  uint32_t* wide = reinterpret_cast<uint32_t*>(lvals + VALS_LDS);
  const int words = (a.n2 + 31) >> 5;
  const int wordsp = (words + 3) & ~3;
  constexpr int TABLE = SelectWideTable<NT>::entries;
  SelectSharedWide<NT> sh;
  sh.taken = wide;
  sh.tkey = reinterpret_cast<int32_t*>(wide + wordsp);
  sh.tval = wide + wordsp + TABLE;
  sh.s_off = sh.tval + TABLE;
  sh.s_len = sh.s_off + 64;
  sh.wave_cnt = reinterpret_cast<int*>(sh.s_len + 64);
  sh.s_misc = reinterpret_cast<uint32_t*>(sh.wave_cnt + SELECT_MU * NW);

  const int q = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n1 = a.n1, n2 = a.n2;

  // ---- sparse input row into LDS ----
  // (count clamped to the row's slots; an entry whose column lies outside [0, d0) contributes nothing)
  const int c = min(max(a.nnz[q], 0), a.ell_stride);
  for (int t = tid; t < c; t += NT) {
    const int i = a.idx[(size_t)q * a.ell_stride + t];
    const bool ok = (unsigned)i < (unsigned)a.d0;
    s_idx[t] = ok ? i : 0;
    s_val[t] = ok ? a.val[(size_t)q * a.ell_stride + t] : 0.0f;
  }
  __syncthreads();

  // ---- hidden layer: column chunk cc (four nodes) x non-zero group grp ----
  {
    const int cc = tid & (a.ccp - 1), grp = tid / a.ccp, ngrp = NT / a.ccp;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (4 * cc < n1) {
      for (int t0 = grp; t0 < c; t0 += 8 * ngrp) {
        float4 w[8];
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int t = t0 + u * ngrp;
          const int tt = t < c ? t : t0;
          w[u] = load_w4(a.W0, a.w0_dtype, (size_t)s_idx[tt] * n1 + 4 * cc);
          v[u] = t < c ? s_val[tt] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          acc.x = fmaf(w[u].x, v[u], acc.x);
          acc.y = fmaf(w[u].y, v[u], acc.y);
          acc.z = fmaf(w[u].z, v[u], acc.z);
          acc.w = fmaf(w[u].w, v[u], acc.w);
        }
      }
    }
    reinterpret_cast<float4*>(part)[tid] = acc;        // part[grp][cc][0..3]
    __syncthreads();
    const int ngroups = NT / a.ccp;
    for (int j = tid; j < n1; j += NT) {
      float s = 0.0f;
      for (int g = 0; g < ngroups; ++g) s += part[((size_t)g * a.ccp + (j >> 2)) * 4 + (j & 3)];
      s += a.b0[j];
      if (a.act0 == SLONN_ACT_RELU) s = s > 0.0f ? s : 0.0f;
      xs[j] = s;
      if (a.tap_out0) a.tap_out0[(size_t)q * n1 + j] = s;
    }
    __syncthreads();
  }

  // ---- hash: z_h = w_h . y1 + b_h in fp64 over the non-zero hidden activations only (a ReLU layer
  //      leaves about half), the hash rows read input-major: thread (r, c) adds inputs r, r + R, ...
  //      into hash columns 4c .. 4c + 3; partial sums meet in LDS and are added in a fixed order ----
  const int H = a.K * a.L;
  {
    const int Hp = a.Hp;
    int32_t* nz = reinterpret_cast<int32_t*>(lvals);         // [n1 <= VALS_LDS] free until the logits
    double* hpart = reinterpret_cast<double*>(sh.tkey);       // the select tables' room: set up afterwards
    const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    int nnz = 0, it = 0;
    for (int base = 0; base < n1; base += NT, ++it) {
      const int i = base + tid;
      const bool is_nz = i < n1 && xs[i] != 0.0f;
      const unsigned long long votes = __ballot(is_nz);
      int* cnt = sh.wave_cnt + (it & 1) * NW;                 // two sets of counts: one barrier per round
      if (lane == 0) cnt[wave] = __popcll(votes);
      __syncthreads();
      int before = 0, total = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const int c2 = cnt[w];
        before += (w < wave) ? c2 : 0;
        total += c2;
      }
      if (is_nz) nz[nnz + before + __popcll(votes & below)] = i;
      nnz += total;
    }
    __syncthreads();
    const int CG = Hp >> 2, R = NT / CG;
    const int r = tid / CG, cg = tid - r * CG;
    if (r < R) {
      double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
      const float* wt = a.WhT + 4 * cg;
      constexpr int U = 8;
      for (int i0 = r; i0 < nnz; i0 += R * U) {
        float4 w[U];
        float x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int i = i0 + u * R;
          const int j = nz[i < nnz ? i : i0];
          w[u] = *reinterpret_cast<const float4*>(wt + (size_t)j * Hp);
          x[u] = i < nnz ? xs[j] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const double xd = x[u];
          a0 = fma((double)w[u].x, xd, a0);
          a1 = fma((double)w[u].y, xd, a1);
          a2 = fma((double)w[u].z, xd, a2);
          a3 = fma((double)w[u].w, xd, a3);
        }
      }
      double* p = hpart + (size_t)r * Hp + 4 * cg;
      p[0] = a0; p[1] = a1; p[2] = a2; p[3] = a3;
    }
    __syncthreads();
    for (int h = tid; h < H; h += NT) {
      double acc = 0.0;
      for (int k = 0; k < R; ++k) acc += hpart[(size_t)k * Hp + h];
      const float z = (float)(acc + (double)a.bh[h]);
      zs[h] = z;
      if (a.tap_z) a.tap_z[(size_t)q * H + h] = z;
    }
    __syncthreads();
  }
  // the select state, and the dense output row if one is wanted
  for (int i = tid; i < words; i += NT) sh.taken[i] = 0u;
  for (int i = tid; i < TABLE; i += NT) { sh.tkey[i] = -1; sh.tval[i] = 0xFFFFFFFFu; }
  float* y = a.dense ? a.dense + (size_t)q * n2 : nullptr;
  if (y)
    for (int i = tid; i < n2; i += NT) y[i] = 0.0f;
  __syncthreads();

  // ---- select ----
  const int m = budget_of(a.keep[(size_t)q * a.keep_qstride], n2);
  const int Hf = (a.hash_first && m < n2) ? H : 0;       // hash nodes at the head of the list
  const int total = (m == n2 || m > Hf) ? m : Hf;
  // the list is built in LDS while it fits (the room of the hidden layer's partial sums) and goes
  // to the caller's array in one coalesced pass at the end
  int32_t* glist = a.list + (size_t)q * a.list_stride;
  const bool list_lds = m != n2 && total <= NT * 4;
  int32_t* list = list_lds ? reinterpret_cast<int32_t*>(part) : glist;
  if (tid == 0) a.cnt[q] = total;
  if (m == n2) {
    if (a.tap_codes && tid < a.L) {
      uint32_t key = 0;
      for (int j = 0; j < a.K; ++j) key |= (zs[tid * a.K + j] > 0.0f ? 1u : 0u) << j;
      a.tap_codes[(size_t)q * a.L + tid] = key;
    }
    for (int i = tid; i < n2; i += NT) glist[i] = i;
  } else {
    for (int h = tid; h < Hf; h += NT) list[h] = a.hnodes[h];
    if (a.ids_narrow)
      select_block_wide<NT, SELECT_MU, uint16_t>(zs, a.K, a.L, n2, total - Hf, a.dir, static_cast<const uint16_t*>(a.ids),
                                                 a.global_rank, sh,
                                                 a.tap_codes ? a.tap_codes + (size_t)q * a.L : nullptr, list + Hf,
                                                 Hf ? a.hslot : nullptr);
    else
      select_block_wide<NT, SELECT_MU, int32_t>(zs, a.K, a.L, n2, total - Hf, a.dir, static_cast<const int32_t*>(a.ids),
                                                a.global_rank, sh,
                                                a.tap_codes ? a.tap_codes + (size_t)q * a.L : nullptr, list + Hf,
                                                Hf ? a.hslot : nullptr);
  }
  __syncthreads();          // the list is complete and visible to the workgroup

  // ---- logits of the listed nodes (kept in LDS while they fit, else in the caller's array) ----
  float* gv = a.vals + (size_t)q * a.vals_stride;
  float* vals = total <= VALS_LDS ? lvals : gv;
  {
    const int32_t* lp = (m == n2) ? nullptr : list;
    if (n1 <= 256) gather_list<8, NT>(a.W1, a.w1_dtype, a.b1, n1, xs, lp, total, vals);
    else gather_list<16, NT>(a.W1, a.w1_dtype, a.b1, n1, xs, lp, total, vals);
  }
  __syncthreads();

  // ---- argmax (lowest id among equal maxima), activation, outputs ----
  float best = -INFINITY;
  int besti = 0x7FFFFFFF;
  for (int t = tid; t < total; t += NT) {
    const float v = vals[t];
    const int j = (m == n2) ? t : list[t];
    if (v > best || (v == best && j < besti)) { best = v; besti = j; }
  }
  for (int o = 32; o > 0; o >>= 1) {
    const float ob = __shfl_xor(best, o);
    const int oi = __shfl_xor(besti, o);
    if (ob > best || (ob == best && oi < besti)) { best = ob; besti = oi; }
  }
  if (lane == 0) { red_f[wave] = best; red_i[wave] = besti; }
  __syncthreads();
  best = red_f[0];
  besti = red_i[0];
  for (int w = 1; w < NW; ++w) {
    const float ob = red_f[w];
    const int oi = red_i[w];
    if (ob > best || (ob == best && oi < besti)) { best = ob; besti = oi; }
  }
  __syncthreads();
  if (a.argmax && tid == 0) a.argmax[q] = besti;

  float inv = 1.0f;
  if (a.act1 == SLONN_ACT_SOFTMAX) {
    float sum = 0.0f;
    for (int t = tid; t < total; t += NT) sum += expf(vals[t] - best);
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if (lane == 0) red_f[wave] = sum;
    __syncthreads();
    sum = 0.0f;
    for (int w = 0; w < NW; ++w) sum += red_f[w];
    inv = 1.0f / sum;
  }
  for (int t = tid; t < total; t += NT) {
    float v = vals[t];
    if (a.act1 == SLONN_ACT_SOFTMAX) v = expf(v - best) * inv;
    else if (a.act1 == SLONN_ACT_RELU) v = v > 0.0f ? v : 0.0f;
    gv[t] = v;
    const int j = (m == n2) ? t : list[t];
    if (list_lds) glist[t] = j;
    if (y) y[j] = v;
  }
}

}  // namespace

namespace {
template <int NT>
size_t wide_lds_bytes(const FusedWideArgs& a) {
  const size_t words = ((size_t)((a.n2 + 31) >> 5) + 3) & ~(size_t)3;
  return (size_t)NT * 16 + ((size_t)a.n1p + a.Hp + 2 * (size_t)a.ellp + 2 * (NT / 64) + VALS_LDS) * 4 +
         (words + SelectSharedWide<NT>::words_besides_bitmap) * 4;
}
}  // namespace

size_t fused_wide_lds_bytes(const FusedWideArgs& a) { return wide_lds_bytes<NT_MAX>(a); }

namespace {
template <int NT>
int launch_wide_nt(const FusedWideArgs& a, int B, size_t lds, hipStream_t s) {
  if (lds > 65536)
    SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(fused_wide_kernel<NT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  hipLaunchKernelGGL(fused_wide_kernel<NT>, dim3(B), dim3(NT), lds, s, a);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}
}  // namespace

int launch_fused_wide(const FusedWideArgs& a, int B, int in_flight, int n_cu, int max_lds, hipStream_t s) {
  ProfScope prof_(SLONN_PROF_FUSED, s);
  // 1024 threads per query while every query in flight can have a compute unit to itself, else 512
  // (C4, batch 128: one / two / four batches in flight 4.7 / 9.0 / 9.6 M queries/s with 1024
  // threads, 4.1 / 7.5 / 13.1 M with 512)
  const bool wide = (long long)B * in_flight <= n_cu;
  const size_t lds = wide ? wide_lds_bytes<1024>(a) : wide_lds_bytes<512>(a);
  if (lds > (size_t)max_lds)
    SLONN_FAIL(SLONN_EUNSUPPORTED, "wide fused path needs %zu bytes of LDS, device grants %d", lds, max_lds);
  return wide ? launch_wide_nt<1024>(a, B, lds, s) : launch_wide_nt<512>(a, B, lds, s);
}

}  // namespace slonn
