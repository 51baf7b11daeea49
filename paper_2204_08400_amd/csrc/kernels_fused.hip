// Whole-network SLO-aware forward pass for small and medium layers: one workgroup of 256, 512 or
// 1024 threads walks one query through every layer (the "k% forward propagation" loop of
// Section 2.1: for each layer, ask the Node Activator for the active node ids, then
// compute only those nodes).  The query's activations, hash projections, keys, the
// de-duplication map and the active list live in LDS from the first layer to the last;
// HBM/L2 only supplies weight rows, table entries and the query, and receives the
// final output.  One launch per batch replaces seven, which is what matters when a
// whole batch is only tens of microseconds of memory traffic.
//
// Per activated layer:
//   hash    FreeHash projections (Def. 2) of the K*L sampled nodes, fp64 accumulation
//           (the sign is a hash bit).  The hash rows are read input-major and only for the
//           query's non-zero inputs: the bytes fall with the sparsity of the layer before;
//   select  keys -> one bucket per table -> merge in rank-major, table-minor order.
//           Every thread takes a few slots per round (4096 a round); a node's first occurrence is
//           found with an LDS integer min over slot numbers (order-independent, hence
//           deterministic), survivors are compacted in slot order with a ballot and a
//           two-level prefix sum, no atomic counters;
//   reuse   an active node that is also one of the layer's hash nodes already has its
//           pre-activation: the hash projection IS w_j . x + b_j (Section 3.4, the hash is
//           "free").  Its output is taken from there and the node leaves the gather list;
//   gather  y_j = act(w_j . x + b_j) for the remaining active rows, four rows per 16-lane
//           group in flight, written straight into the next layer's input in LDS (dropped
//           nodes were zeroed there beforehand).
#include <type_traits>

#include "select_block.h"
#include "slonn_internal.h"

namespace slonn {
namespace {

// Threads per workgroup: 1024 when the queries in flight leave most compute units free (one query
// per unit), else 512 or 256, so that two to four queries share a unit and fill each other's memory
// waits: every phase of a query is a dependent round trip to L2 or a stream bound by one unit's
// path to L2.
constexpr int NT_MAX = 1024;
constexpr size_t HASH_PART_BYTES = (size_t)NT_MAX * 4 * 8;   // partial hash projections: four doubles per thread
template <int NT> struct SelectMu { static constexpr int value = SELECT_MU * (NT_MAX / NT); };   // 4096 slots per round

__device__ __forceinline__ int budget_of(float keep, int n) {
  double m = floor((double)keep * (double)n + 0.5);
  if (!(m >= 1.0)) m = 1.0;        // also a keep fraction that is not a number
  if (m > (double)n) m = (double)n;
  return (int)m;
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

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

// 16 bytes of a weight row against x (LDS), fp32
template <int WDT>
__device__ __forceinline__ float dot16(const uint4& w, const float* xs, float acc);
template <>
__device__ __forceinline__ float dot16<SLONN_F32>(const uint4& w, const float* xs, float acc) {
  const float4 x = *reinterpret_cast<const float4*>(xs);
  acc = fmaf(__uint_as_float(w.x), x.x, acc);
  acc = fmaf(__uint_as_float(w.y), x.y, acc);
  acc = fmaf(__uint_as_float(w.z), x.z, acc);
  acc = fmaf(__uint_as_float(w.w), x.w, acc);
  return acc;
}
template <>
__device__ __forceinline__ float dot16<SLONN_BF16>(const uint4& w, const float* xs, float acc) {
  const float4 x0 = *reinterpret_cast<const float4*>(xs);
  const float4 x1 = *reinterpret_cast<const float4*>(xs + 4);
  acc = fmaf(bf16_lo(w.x), x0.x, acc);
  acc = fmaf(bf16_hi(w.x), x0.y, acc);
  acc = fmaf(bf16_lo(w.y), x0.z, acc);
  acc = fmaf(bf16_hi(w.y), x0.w, acc);
  acc = fmaf(bf16_lo(w.z), x1.x, acc);
  acc = fmaf(bf16_hi(w.z), x1.y, acc);
  acc = fmaf(bf16_lo(w.w), x1.z, acc);
  acc = fmaf(bf16_hi(w.w), x1.w, acc);
  return acc;
}

__device__ __forceinline__ float reduce64(float v) {
  v += __shfl_xor(v, 32);
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 8);
  v += __shfl_xor(v, 4);
  v += __shfl_xor(v, 2);
  v += __shfl_xor(v, 1);
  return v;
}

// Few rows (a small output layer): one whole wavefront per row, four 16-byte steps in
// flight, so that ten rows keep ten wavefronts busy instead of ten 16-lane groups.
template <int WDT, int NT>
__device__ __forceinline__ void gather_few_rows(const void* __restrict__ W, const float* __restrict__ bias,
                                                int d, const float* xs, const int32_t* list, int count,
                                                int act, float* dst) {
  constexpr int ELEMS = (WDT == SLONN_F32) ? 4 : 8;
  constexpr int ESZ = (WDT == SLONN_F32) ? 4 : 2;
  constexpr int NW = NT / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nv = d / ELEMS;
  for (int t = wave; t < count; t += NW) {
    const int j = list ? list[t] : t;
    const uint4* w = reinterpret_cast<const uint4*>(static_cast<const char*>(W) + (size_t)j * d * ESZ);
    const float b = bias[j];
    float acc = 0.0f;
    for (int i0 = 0; i0 < nv; i0 += 256) {
      uint4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + u * 64 + lane;
        v[u] = (i < nv) ? w[i] : make_uint4(0u, 0u, 0u, 0u);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + u * 64 + lane;
        if (i < nv) acc = dot16<WDT>(v[u], xs + i * ELEMS, acc);
      }
    }
    acc = reduce64(acc);
    if (lane == 0) {
      float z = acc + b;
      if (act == SLONN_ACT_RELU) z = z > 0.0f ? z : 0.0f;
      dst[j] = z;
    }
  }
}

// One pass of the row gather: every 16-lane group takes up to R rows (t0, t0 + GROUPS, ...),
// all R row streams in flight together.  R is the same for the whole workgroup, so a pass
// over fewer rows than 4 * GROUPS issues no loads for rows that do not exist.
template <int WDT, int R, int NT>
__device__ __forceinline__ void gather_pass(const void* __restrict__ W, const float* __restrict__ bias,
                                            int d, const float* xs, const int32_t* list, int t0, int count,
                                            int act, float* dst) {
  constexpr int ELEMS = (WDT == SLONN_F32) ? 4 : 8;
  constexpr int ESZ = (WDT == SLONN_F32) ? 4 : 2;
  constexpr int GROUPS = NT / 16;          // 16-lane row groups
  const int l = threadIdx.x & 15;
  const int nv = d / ELEMS;
  int t[R], j[R];
  float acc[R];
  const uint4* w[R];
#pragma unroll
  for (int k = 0; k < R; ++k) {
    t[k] = t0 + k * GROUPS;
    const int tt = t[k] < count ? t[k] : t0;
    j[k] = list ? list[tt] : tt;
    acc[k] = 0.f;
    w[k] = reinterpret_cast<const uint4*>(static_cast<const char*>(W) + (size_t)j[k] * d * ESZ);
  }
#pragma unroll 2
  for (int i = l; i < nv; i += 16) {
    uint4 v[R];
#pragma unroll
    for (int k = 0; k < R; ++k) v[k] = w[k][i];
    const float* xp = xs + i * ELEMS;
#pragma unroll
    for (int k = 0; k < R; ++k) acc[k] = dot16<WDT>(v[k], xp, acc[k]);
  }
#pragma unroll
  for (int k = 0; k < R; ++k) acc[k] = reduce16(acc[k]);
#pragma unroll
  for (int k = 0; k < R; ++k)
    if (l == k && t[k] < count) {
      float z = acc[k] + bias[j[k]];
      if (act == SLONN_ACT_RELU) z = z > 0.0f ? z : 0.0f;
      dst[j[k]] = z;
    }
}

// rows listed in LDS (list == nullptr: rows 0..count-1) -> dst[j] = act(w_j . x + b_j)
template <int WDT, int NT>
__device__ __forceinline__ void gather_rows(const void* __restrict__ W, const float* __restrict__ bias,
                                            int d, const float* xs, const int32_t* list, int count,
                                            int act, float* dst) {
  constexpr int NW = NT / 64, GROUPS = NT / 16;
  if (count <= 2 * NW) {
    gather_few_rows<WDT, NT>(W, bias, d, xs, list, count, act, dst);
    return;
  }
  const int g = threadIdx.x >> 4;
  for (int base = 0; base < count; base += 4 * GROUPS) {
    const int left = count - base;                       // same for every thread
    const int t0 = base + g;
    if (left > 3 * GROUPS) {
      if (t0 < count) gather_pass<WDT, 4, NT>(W, bias, d, xs, list, t0, count, act, dst);
    } else if (left > 2 * GROUPS) {
      if (t0 < count) gather_pass<WDT, 3, NT>(W, bias, d, xs, list, t0, count, act, dst);
    } else if (left > GROUPS) {
      if (t0 < count) gather_pass<WDT, 2, NT>(W, bias, d, xs, list, t0, count, act, dst);
    } else {
      if (t0 < count) gather_pass<WDT, 1, NT>(W, bias, d, xs, list, t0, count, act, dst);
    }
  }
}

// LDS needed without the staging area of the in-kernel choice of k (a multiple of 16 bytes)
__host__ __device__ inline size_t fused_lds_base(const FusedArgs& a) {
  const size_t bytes = HASH_PART_BYTES + (size_t)(2 * a.max_dim + a.max_H) * 4 + (size_t)a.max_na * 8 +
                       SelectShared<NT_MAX>::words_besides_prio * 4 + (64 + 4) * 4 + (size_t)a.max_na * 2;
  return (bytes + 15) & ~(size_t)15;
}

template <bool POLICY, int NT>
__global__ __launch_bounds__(NT) void fused_forward_kernel(FusedArgs a) {
  constexpr int NW = NT / 64;
  constexpr int MU = SelectMu<NT>::value;
  extern __shared__ __align__(16) unsigned char smem[];
  double* hpart = reinterpret_cast<double*>(smem);                // [NT / (Hp / 4)][Hp] partial projections
  float* xbuf0 = reinterpret_cast<float*>(smem + HASH_PART_BYTES);
  float* xbuf1 = xbuf0 + a.max_dim;
  float* zs = xbuf1 + a.max_dim;
  uint32_t* prio = reinterpret_cast<uint32_t*>(zs + a.max_H);
  int32_t* alist = reinterpret_cast<int32_t*>(prio + a.max_na);
  SelectShared<NT, MU> sh;
  sh.prio = prio;
  sh.s_off = reinterpret_cast<uint32_t*>(alist + a.max_na);
  sh.s_len = sh.s_off + 64;
  sh.wave_cnt = reinterpret_cast<int*>(sh.s_len + 64);
  sh.s_misc = reinterpret_cast<uint32_t*>(sh.wave_cnt + MU * NW);
  static_assert(MU * NW == SELECT_MU * (NT_MAX / 64), "LDS carve-up assumes the counts of the largest workgroup");
  uint32_t* pkey = sh.s_misc + 4;                                 // [64] keys for the choice of k
  float* s_keep = reinterpret_cast<float*>(pkey + 64);            // [4] keep fraction chosen in the kernel
  int16_t* hmap = reinterpret_cast<int16_t*>(s_keep + 4);         // [max_na] node -> hash row or -1
  // only with the choice of k inside the kernel: staged bucket sums [L][G] and counts [L]
  double* pstage = reinterpret_cast<double*>(smem + fused_lds_base(a));
  uint32_t* pcount = reinterpret_cast<uint32_t*>(pstage + SLONN_MAX_L * SLONN_MAX_GRID);

  const int q = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  float* xs = xbuf0;
  float* xn = xbuf1;
  {
    const float4* x = reinterpret_cast<const float4*>(a.X + (size_t)q * a.ldx);
    for (int i = tid; i < (a.layer[0].d_in >> 2); i += NT) reinterpret_cast<float4*>(xs)[i] = x[i];
  }
  __syncthreads();

  for (int li = 0; li < a.n_layers; ++li) {
    const FusedLayer& Ly = a.layer[li];
    const int d = Ly.d_in, n = Ly.d_out;
    const bool last = (li == a.n_layers - 1);
    const bool activated = Ly.K > 0;
    int m = n;
    const int32_t* list = nullptr;
    // the caller's keep fraction is fetched now so that its latency hides behind the hash
    float kq = 1.0f;
    if (activated && !(POLICY && li >= a.pol.layer))
      kq = a.keep[(size_t)q * a.keep_qstride + (size_t)li * a.keep_lstride];

    if (activated) {
      // ---- hash: z_h = w_h . x + b_h in fp64, over the non-zero inputs only ----
      // (the input of a deeper layer is the sparse output of the layer before: at keep fraction k
      // only k of the hash rows' bytes are read; a zero input adds nothing to an fp64 sum)
      const int H = Ly.K * Ly.L;
      const int Hp = (H + 3) & ~3;
      int32_t* nz = reinterpret_cast<int32_t*>(xn);      // indices of the non-zero inputs, ascending
      int nnz = 0;
      {
        const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
        int it = 0;
        for (int base = 0; base < d; base += NT, ++it) {
          const int i = base + tid;
          const bool is_nz = i < d && xs[i] != 0.0f;
          const unsigned long long votes = __ballot(is_nz);
          int* cnt = sh.wave_cnt + (it & 1) * NW;          // two sets of counts: one barrier per round
          if (lane == 0) cnt[wave] = __popcll(votes);
          __syncthreads();
          int before = 0, total = 0;
#pragma unroll
          for (int w = 0; w < NW; ++w) {
            const int c = cnt[w];
            before += (w < wave) ? c : 0;
            total += c;
          }
          if (is_nz) nz[nnz + before + __popcll(votes & below)] = i;
          nnz += total;
        }
        __syncthreads();
      }
      {
        // thread (r, c): inputs r, r + R, ... of the list against hash columns 4c .. 4c + 3; a
        // wavefront's loads cover whole rows of WhT, and all of a thread's loads are in flight
        // together (up to eight).  Partial sums meet in LDS and are added in a fixed order.
        const int CG = Hp >> 2, R = NT / CG;
        const int r = tid / CG, c = tid - r * CG;
        const float bias_h = tid < H ? Ly.bh[tid] : 0.0f;   // on its way while the rows are read
        if (r < R) {
          double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
          const float* wt = Ly.WhT + 4 * c;
          auto rows = [&](auto uc) {
            constexpr int U = decltype(uc)::value;
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
          };
          if (nnz > 4 * R) rows(std::integral_constant<int, 8>{});
          else rows(std::integral_constant<int, 4>{});
          double* p = hpart + (size_t)r * Hp + 4 * c;
          p[0] = a0; p[1] = a1; p[2] = a2; p[3] = a3;
        }
        __syncthreads();
        // R partial sums per projection, added in a fixed order: where the workgroup has several
        // threads per projection, P of them take R / P consecutive sums each and one adds the results
        const int P = NT / Hp > 8 ? 8 : NT / Hp;
        int nsum = R;
        if (P > 1) {
          const int per = (R + P - 1) / P;
          const int h = tid % Hp, pp = tid / Hp;
          double part = 0.0;
          if (pp < P)
            for (int rr = pp * per; rr < (pp + 1) * per && rr < R; ++rr) part += hpart[(size_t)rr * Hp + h];
          __syncthreads();
          if (pp < P) hpart[(size_t)pp * Hp + h] = part;
          __syncthreads();
          nsum = P;
        }
        for (int h = tid; h < H; h += NT) {
          double acc = 0.0;
          for (int k = 0; k < nsum; ++k) acc += hpart[(size_t)k * Hp + h];
          const float z = (float)(acc + (double)(h == tid ? bias_h : Ly.bh[h]));
          zs[h] = z;
          if (Ly.tap_z) Ly.tap_z[(size_t)q * H + h] = z;
        }
      }
      // clear the next activation buffer (it held the list of non-zero inputs) and the
      // first-occurrence map
      for (int i = tid; i < n; i += NT) { xn[i] = 0.0f; prio[i] = 0xFFFFFFFFu; hmap[i] = Ly.hslot[i]; }
      __syncthreads();

      // ---- budget: from the caller, or chosen here from the Confidence LSH tables (ACLO,
      //      Section 2.2 / Eq. 4) with this layer's keys; the choice serves all later layers ----
      if (POLICY && li >= a.pol.layer) {
        if (li == a.pol.layer) {
          if (wave == 0 && lane < Ly.L) {
            uint32_t key = 0;
            for (int j = 0; j < Ly.K; ++j) key |= (zs[lane * Ly.K + j] > 0.0f ? 1u : 0u) << j;
            pkey[lane] = key;
          }
          __syncthreads();
          // all L*G bucket sums (<= 1024) are fetched at once ...
          const int G = a.pol.G, nb = 1 << Ly.K;
          for (int t = tid; t < Ly.L * G; t += NT) {
            const int b = t / G, g = t - b * G;
            const size_t bk = (size_t)b * nb + pkey[b];
            pstage[t] = a.pol.sum[bk * G + g];
            if (g == 0) pcount[b] = a.pol.cnt[bk];
          }
          __syncthreads();
          if (wave == 0) {
            // ... and pooled by lane g in table order (reproducible double sums; an empty
            // bucket holds the sum +0 and the count 0)
            bool ok = false;
            if (lane < G) {
              double sacc = 0.0;
              unsigned long long c = 0;
              for (int b = 0; b < Ly.L; ++b) { sacc += pstage[b * G + lane]; c += pcount[b]; }
              const double chat = c > 0 ? sacc / (double)c : a.pol.total[lane] / (double)a.pol.N;
              ok = chat >= (double)a.pol.thr[(size_t)q * a.pol.thr_stride];
            }
            const unsigned long long votes = __ballot(ok);
            if (lane == 0) {
              const int pick = votes ? (__ffsll((long long)votes) - 1) : a.pol.G - 1;
              const float kk = a.pol.grid[pick];
              s_keep[0] = kk;
              a.pol.keep_out[q] = kk;
            }
          }
          __syncthreads();
        }
        kq = s_keep[0];
      }
      m = budget_of(kq, n);

      // Section 3.4 variant: the H hash nodes head the active list and are never selected
      const int Hf = (a.hash_first && m < n) ? H : 0;
      const int msel = m > Hf ? m - Hf : 0;
      if (wave == 0 && lane == 0 && Ly.tap_cnt) Ly.tap_cnt[q] = Hf + msel;
      if (m < n) {
        // ---- keys, bucket lookup, merge: first msel distinct nodes in slot order ----
        if (Ly.ids_narrow)
          select_block<NT, MU, uint16_t>(zs, Ly.K, Ly.L, n, msel, Ly.dir, static_cast<const uint16_t*>(Ly.ids),
                                                Ly.global_rank, sh,
                                                Ly.tap_codes ? Ly.tap_codes + (size_t)q * Ly.L : nullptr, alist,
                                                Hf ? hmap : nullptr);
        else
          select_block<NT, MU, int32_t>(zs, Ly.K, Ly.L, n, msel, Ly.dir, static_cast<const int32_t*>(Ly.ids),
                                               Ly.global_rank, sh,
                                               Ly.tap_codes ? Ly.tap_codes + (size_t)q * Ly.L : nullptr, alist,
                                               Hf ? hmap : nullptr);
        list = alist;
        if (Ly.tap_idx) {
          for (int i = tid; i < Hf; i += NT) Ly.tap_idx[(size_t)q * n + i] = Ly.hnodes[i];
          for (int i = tid; i < msel; i += NT) Ly.tap_idx[(size_t)q * n + Hf + i] = alist[i];
        }
        if (Hf) {
          // every hash node's output comes from its projection; the list holds none of them
          for (int i = tid; i < n; i += NT) {
            const int hs = hmap[i];
            if (hs >= 0) {
              const float z = zs[hs];
              xn[i] = (Ly.act == SLONN_ACT_RELU && !(z > 0.0f)) ? 0.0f : z;
            }
          }
        }
        m = msel;
      } else {
        if (Ly.tap_codes && tid < Ly.L) {
          uint32_t key = 0;
          for (int j = 0; j < Ly.K; ++j) key |= (zs[tid * Ly.K + j] > 0.0f ? 1u : 0u) << j;
          Ly.tap_codes[(size_t)q * Ly.L + tid] = key;
        }
        if (Ly.tap_idx)
          for (int i = tid; i < n; i += NT) Ly.tap_idx[(size_t)q * n + i] = i;
      }

      // ---- reuse: active hash nodes take their output from the projections; the others
      //      are compacted in place (a round writes below what the next round reads) ----
      const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
      int kept = 0;
      for (int base = 0; base < (Hf ? 0 : m); base += NT) {
        const int i = base + tid;
        const int node = i < m ? (list ? alist[i] : i) : -1;
        const int hs = node >= 0 ? (int)hmap[node] : -1;
        if (hs >= 0) {
          const float z = zs[hs];
          xn[node] = (Ly.act == SLONN_ACT_RELU && !(z > 0.0f)) ? 0.0f : z;
        }
        const bool stays = node >= 0 && hs < 0;
        const unsigned long long votes = __ballot(stays);
        if (lane == 0) sh.wave_cnt[wave] = __popcll(votes);
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
          const int c = sh.wave_cnt[w];
          before += (w < wave) ? c : 0;
          total += c;
        }
        if (stays) alist[kept + before + __popcll(votes & below)] = node;
        kept += total;
        __syncthreads();
      }
      if (!Hf) { list = alist; m = kept; }
    }

    // ---- evaluate the active rows into the next layer's input ----
    const int act = (Ly.act == SLONN_ACT_RELU) ? SLONN_ACT_RELU : SLONN_ACT_NONE;
    if (Ly.w_dtype == SLONN_F32)
      gather_rows<SLONN_F32, NT>(Ly.W, Ly.bias, d, xs, list, m, act, xn);
    else
      gather_rows<SLONN_BF16, NT>(Ly.W, Ly.bias, d, xs, list, m, act, xn);
    __syncthreads();

    if (last) {
      // every node of the last layer was computed (it carries no Node Activator here)
      if (wave == 0) {
        float best = -INFINITY;
        int besti = 0x7FFFFFFF;
        for (int j = lane; j < n; j += 64) {
          const float v = xn[j];
          if (v > best || (v == best && j < besti)) { best = v; besti = j; }
        }
        for (int o = 32; o > 0; o >>= 1) {
          const float ob = __shfl_xor(best, o);
          const int oi = __shfl_xor(besti, o);
          if (ob > best || (ob == best && oi < besti)) { best = ob; besti = oi; }
        }
        if (a.argmax && lane == 0) a.argmax[q] = besti;
        if (Ly.act == SLONN_ACT_SOFTMAX) {
          float sum = 0.0f;
          for (int j = lane; j < n; j += 64) sum += expf(xn[j] - best);
          for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
          const float inv = 1.0f / sum;
          for (int j = lane; j < n; j += 64) xn[j] = expf(xn[j] - best) * inv;
        }
      }
      __syncthreads();
      if (a.Y)
        for (int j = tid; j < n; j += NT) a.Y[(size_t)q * n + j] = xn[j];
    }
    if (Ly.tap_out)
      for (int j = tid; j < n; j += NT) Ly.tap_out[(size_t)q * n + j] = xn[j];
    float* t = xs; xs = xn; xn = t;
    __syncthreads();
  }
}

__global__ __launch_bounds__(256) void transpose_hash_rows_kernel(const float* __restrict__ Wh, int H, int d, int Hp,
                                                                  float* __restrict__ WhT) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)d * Hp) return;
  const int j = (int)(i / Hp), h = (int)(i - (size_t)j * Hp);
  WhT[i] = h < H ? Wh[(size_t)h * d + j] : 0.0f;
}

}  // namespace

int launch_transpose_hash_rows(const float* Wh, int H, int d, int Hp, float* WhT, hipStream_t s) {
  const size_t total = (size_t)d * Hp;
  hipLaunchKernelGGL(transpose_hash_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, Wh, H, d, Hp,
                     WhT);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

size_t fused_lds_bytes(const FusedArgs& a) {
  size_t bytes = fused_lds_base(a);
  if (a.pol.sum) bytes += (size_t)SLONN_MAX_L * SLONN_MAX_GRID * 8 + SLONN_MAX_L * 4;
  return bytes;
}

namespace {
template <bool POLICY, int NT>
int launch_fused_nt(const FusedArgs& a, int B, size_t lds, hipStream_t s) {
  if (lds > 65536)
    SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(fused_forward_kernel<POLICY, NT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  hipLaunchKernelGGL((fused_forward_kernel<POLICY, NT>), dim3(B), dim3(NT), lds, s, a);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}
}  // namespace

int launch_fused_forward(const FusedArgs& a, int B, int in_flight, int n_cu, int max_lds, hipStream_t s) {
  ProfScope prof_(SLONN_PROF_FUSED, s);
  const size_t lds = fused_lds_bytes(a);
  if (lds > (size_t)max_lds)
    SLONN_FAIL(SLONN_EUNSUPPORTED, "fused path needs %zu bytes of LDS, device grants %d", lds, max_lds);
  // 1024 threads per query while the queries in flight use at most half the compute units, 512
  // up to four queries per unit, 256 beyond: two to four queries then share a unit (from this
  // launch or from batches on other streams).  C2, batch 256: two batches in flight 9.7 (1024
  // threads) / 15.7 (512) / 14.4 (256) M queries/s at keep .05, four in flight 16.3 (512) / 19.9 (256)
  const long long in_flight_q = (long long)B * in_flight;
  const int nt = 2 * in_flight_q <= n_cu ? 1024 : (in_flight_q >= 4ll * n_cu ? 256 : 512);
  if (a.pol.sum) {
    if (nt == 1024) return launch_fused_nt<true, 1024>(a, B, lds, s);
    return nt == 512 ? launch_fused_nt<true, 512>(a, B, lds, s) : launch_fused_nt<true, 256>(a, B, lds, s);
  }
  if (nt == 1024) return launch_fused_nt<false, 1024>(a, B, lds, s);
  return nt == 512 ? launch_fused_nt<false, 512>(a, B, lds, s) : launch_fused_nt<false, 256>(a, B, lds, s);
}

}  // namespace slonn
