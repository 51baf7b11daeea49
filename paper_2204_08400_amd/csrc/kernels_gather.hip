// Sparse layer forward (Section 1 "avoiding computations for these nodes altogether";
// Fig. 2 step 4): for each query only the selected nodes' weight rows are read and
// evaluated, y_j = act(w_j . x + b_j); the select kernel has already written +0 for
// every other node.  The work is a gather of whole contiguous rows: 0.5 flop per byte
// in fp32, 1 flop per byte with bf16 weights -> bandwidth-bound, plain vector FMAs.
//
// Mapping: a 256-thread workgroup serves one query and a chunk of 64 entries of its
// active list.  The query vector is staged once in LDS.  A row is read by a group of
// 16 lanes (one DPP row), 16 bytes per lane per step, so every step of a group
// covers 256 contiguous bytes of one weight row; the four rows a group owns are
// streamed together so each LDS read of x is used four times and eight 16-byte loads
// per lane are in flight.
#include <algorithm>

#include "slonn_internal.h"

namespace slonn {
namespace {

constexpr int LANES_PER_ROW = 16;
constexpr int ROWS_PER_GROUP = 4;
constexpr int ROWS_PER_BLOCK = (256 / LANES_PER_ROW) * ROWS_PER_GROUP;   // 64

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

// 16 bytes of a weight row against the matching slice of x (in LDS)
template <int WDT>
struct Chunk;

template <>
struct Chunk<SLONN_F32> {
  static constexpr int ELEMS = 4;
  using vec_t = float4;
  static __device__ __forceinline__ float dot(const vec_t& w, const float* xs, float acc) {
    const float4 x = *reinterpret_cast<const float4*>(xs);
    acc = fmaf(w.x, x.x, acc);
    acc = fmaf(w.y, x.y, acc);
    acc = fmaf(w.z, x.z, acc);
    acc = fmaf(w.w, x.w, acc);
    return acc;
  }
  static __device__ __forceinline__ float elem(const void* W, size_t i) {
    return static_cast<const float*>(W)[i];
  }
};

template <>
struct Chunk<SLONN_BF16> {
  static constexpr int ELEMS = 8;
  using vec_t = uint4;
  static __device__ __forceinline__ float dot(const vec_t& w, const float* xs, float acc) {
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
  static __device__ __forceinline__ float elem(const void* W, size_t i) {
    return bf16_lo(static_cast<const uint16_t*>(W)[i]);
  }
};

__device__ __forceinline__ float reduce16(float v) {
  v += __shfl_xor(v, 8, 16);
  v += __shfl_xor(v, 4, 16);
  v += __shfl_xor(v, 2, 16);
  v += __shfl_xor(v, 1, 16);
  return v;
}

// VECTOR: rows and x are 16-byte aligned and d is a multiple of the chunk size.
template <int WDT, bool VECTOR>
__global__ __launch_bounds__(256) void gather_forward_kernel(
    const void* __restrict__ W, const float* __restrict__ bias, const float* __restrict__ X, int ldx,
    const int32_t* __restrict__ active, const int32_t* __restrict__ cnt, int idx_stride,
    float* __restrict__ Y, int ldy, float* __restrict__ yc, int ldc, int d, int n, int act,
    int ychunks) {             // ychunks = gridDim.y (an argument is quicker to reach than the dispatch packet)
  extern __shared__ __align__(16) float xs[];
  using C = Chunk<WDT>;
  const int q = blockIdx.x;              // queries on x (no 65535 limit), chunks on y
  const int c = active ? cnt[q] : n;
  if ((int)blockIdx.y * ROWS_PER_BLOCK >= c) return;
  const int tid = threadIdx.x;
  const float* x = X + (size_t)q * ldx;
  if (VECTOR) {
    for (int i = tid; i < (d >> 2); i += 256)
      reinterpret_cast<float4*>(xs)[i] = reinterpret_cast<const float4*>(x)[i];
  } else {
    for (int i = tid; i < d; i += 256) xs[i] = x[i];
  }
  __syncthreads();

  const int g = tid / LANES_PER_ROW, l = tid % LANES_PER_ROW;
  const int32_t* list = active ? active + (size_t)q * idx_stride : nullptr;
  // the grid holds a bounded number of chunks per query (the budget is only known on the
  // device); a workgroup walks its chunks with the grid's stride
  for (int row0 = blockIdx.y * ROWS_PER_BLOCK; row0 < c; row0 += ychunks * ROWS_PER_BLOCK) {
    int t[ROWS_PER_GROUP], j[ROWS_PER_GROUP];
    float acc[ROWS_PER_GROUP];
#pragma unroll
    for (int k = 0; k < ROWS_PER_GROUP; ++k) {
      t[k] = row0 + g + k * (256 / LANES_PER_ROW);
      const int tt = t[k] < c ? t[k] : row0;          // surplus slots redo the first row
      j[k] = list ? list[tt] : tt;
      acc[k] = 0.0f;
    }
    if (t[0] >= c) break;                               // whole group beyond the list

    if (VECTOR) {
      using vec_t = typename C::vec_t;
      const int nv = d / C::ELEMS;
      const vec_t* w0 = reinterpret_cast<const vec_t*>(static_cast<const char*>(W) +
                                                       (size_t)j[0] * d * (WDT == SLONN_F32 ? 4 : 2));
      const vec_t* w1 = reinterpret_cast<const vec_t*>(static_cast<const char*>(W) +
                                                       (size_t)j[1] * d * (WDT == SLONN_F32 ? 4 : 2));
      const vec_t* w2 = reinterpret_cast<const vec_t*>(static_cast<const char*>(W) +
                                                       (size_t)j[2] * d * (WDT == SLONN_F32 ? 4 : 2));
      const vec_t* w3 = reinterpret_cast<const vec_t*>(static_cast<const char*>(W) +
                                                       (size_t)j[3] * d * (WDT == SLONN_F32 ? 4 : 2));
#pragma unroll 2
      for (int i = l; i < nv; i += LANES_PER_ROW) {
        const vec_t a0 = w0[i], a1 = w1[i], a2 = w2[i], a3 = w3[i];
        const float* xp = xs + i * C::ELEMS;
        acc[0] = C::dot(a0, xp, acc[0]);
        acc[1] = C::dot(a1, xp, acc[1]);
        acc[2] = C::dot(a2, xp, acc[2]);
        acc[3] = C::dot(a3, xp, acc[3]);
      }
    } else {
      for (int i = l; i < d; i += LANES_PER_ROW) {
        const float xv = xs[i];
#pragma unroll
        for (int k = 0; k < ROWS_PER_GROUP; ++k)
          acc[k] = fmaf(C::elem(W, (size_t)j[k] * d + i), xv, acc[k]);
      }
    }
#pragma unroll
    for (int k = 0; k < ROWS_PER_GROUP; ++k) acc[k] = reduce16(acc[k]);
#pragma unroll
    for (int k = 0; k < ROWS_PER_GROUP; ++k) {
      if (l == k && t[k] < c) {
        float z = acc[k] + bias[j[k]];
        if (act == SLONN_ACT_RELU) z = z > 0.0f ? z : 0.0f;
        if (Y) Y[(size_t)q * ldy + j[k]] = z;
        if (yc) yc[(size_t)q * ldc + t[k]] = z;
      }
    }
  }
}

// Small batches: with only a few queries there are too few (query, 64-row chunk) pairs to
// occupy the chip, so a workgroup takes 8 list entries at a time, one wavefront per row
// (two rows in flight per wavefront), and the grid is eight times finer.
constexpr int ROWS_PER_WAVE_BLOCK = 8;

template <int WDT>
__global__ __launch_bounds__(256) void gather_wave_kernel(
    const void* __restrict__ W, const float* __restrict__ bias, const float* __restrict__ X, int ldx,
    const int32_t* __restrict__ active, const int32_t* __restrict__ cnt, int idx_stride,
    float* __restrict__ Y, int ldy, float* __restrict__ yc, int ldc, int d, int n, int act,
    int ychunks) {             // ychunks = gridDim.y (an argument is quicker to reach than the dispatch packet)
  extern __shared__ __align__(16) float xs[];
  using C = Chunk<WDT>;
  using vec_t = typename C::vec_t;
  const int q = blockIdx.x;
  const int c = active ? cnt[q] : n;
  if ((int)blockIdx.y * ROWS_PER_WAVE_BLOCK >= c) return;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float* x = X + (size_t)q * ldx;
  for (int i = tid; i < (d >> 2); i += 256)
    reinterpret_cast<float4*>(xs)[i] = reinterpret_cast<const float4*>(x)[i];
  __syncthreads();
  const int nv = d / C::ELEMS;
  const int32_t* list = active ? active + (size_t)q * idx_stride : nullptr;
  for (int t0 = blockIdx.y * ROWS_PER_WAVE_BLOCK + 2 * wave; t0 < c; t0 += ychunks * ROWS_PER_WAVE_BLOCK) {
    const bool two = t0 + 1 < c;
    const int j0 = list ? list[t0] : t0, j1 = two ? (list ? list[t0 + 1] : t0 + 1) : j0;
    const vec_t* w0 = reinterpret_cast<const vec_t*>(static_cast<const char*>(W) +
                                                     (size_t)j0 * d * (WDT == SLONN_F32 ? 4 : 2));
    const vec_t* w1 = reinterpret_cast<const vec_t*>(static_cast<const char*>(W) +
                                                     (size_t)j1 * d * (WDT == SLONN_F32 ? 4 : 2));
    float acc0 = 0.0f, acc1 = 0.0f;
#pragma unroll 4
    for (int i = lane; i < nv; i += 64) {
      const vec_t a0 = w0[i], a1 = w1[i];
      const float* xp = xs + i * C::ELEMS;
      acc0 = C::dot(a0, xp, acc0);
      acc1 = C::dot(a1, xp, acc1);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      acc0 += __shfl_xor(acc0, o);
      acc1 += __shfl_xor(acc1, o);
    }
    if (lane == 0 || (lane == 1 && two)) {
      const int j = lane == 0 ? j0 : j1;
      float z = (lane == 0 ? acc0 : acc1) + bias[j];
      if (act == SLONN_ACT_RELU) z = z > 0.0f ? z : 0.0f;
      if (Y) Y[(size_t)q * ldy + j] = z;
      if (yc) yc[(size_t)q * ldc + t0 + lane] = z;
    }
  }
}

// A handful of queries: one workgroup per (query, list entry).  Nothing is staged: a thread's
// pieces of the row and of the activations go from memory to registers with all loads in flight
// together (the list entry is fetched beside the list length, before either is known to be
// needed), so a 16 KB row costs about two memory round trips instead of the six of a
// wavefront walking it after the query vector has been staged in LDS.
template <int WDT>
__global__ __launch_bounds__(256) void gather_row_kernel(
    const void* __restrict__ W, const float* __restrict__ bias, const float* __restrict__ X, int ldx,
    const int32_t* __restrict__ active, const int32_t* __restrict__ cnt, int idx_stride,
    float* __restrict__ Y, int ldy, float* __restrict__ yc, int ldc, int d, int n, int act, int xstride) {
  __shared__ float part[4];
  using C = Chunk<WDT>;
  using vec_t = typename C::vec_t;
  constexpr int U = 4;                     // pieces per thread held at once
  const int q = blockIdx.y;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int32_t* list = active ? active + (size_t)q * idx_stride : nullptr;
  // (idx_stride >= n >= gridDim.x: the entry exists whatever the list's length)
  int j = list ? list[blockIdx.x] : (int)blockIdx.x;
  const int c = active ? cnt[q] : n;
  const float* x = X + (size_t)q * ldx;
  const int nv = d / C::ELEMS;
  for (int t = blockIdx.x; t < c; t += xstride) {
    if (t != (int)blockIdx.x) j = list ? list[t] : t;
    const vec_t* w = reinterpret_cast<const vec_t*>(static_cast<const char*>(W) +
                                                    (size_t)j * d * (WDT == SLONN_F32 ? 4 : 2));
    float acc = 0.0f;
    for (int i0 = tid; i0 < nv; i0 += 256 * U) {
      vec_t wv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = i0 + 256 * u;
        wv[u] = w[i < nv ? i : tid];        // a surplus piece repeats a valid one and is not used
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = i0 + 256 * u;
        if (i < nv) acc = C::dot(wv[u], x + (size_t)i * C::ELEMS, acc);
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) part[wave] = acc;
    __syncthreads();
    if (tid == 0) {
      float z = ((part[0] + part[1]) + (part[2] + part[3])) + bias[j];
      if (act == SLONN_ACT_RELU) z = z > 0.0f ? z : 0.0f;
      if (Y) Y[(size_t)q * ldy + j] = z;
      if (yc) yc[(size_t)q * ldc + t] = z;
    }
    __syncthreads();
  }
}

// Row-block variant for layers whose weight matrix is much larger than an L2 slice:
// workgroup (q, block) evaluates the rows of query q that lie in one block of consecutive
// weight rows (about a megabyte).  The grid runs over queries fastest, so the workgroups
// resident at any moment all read the same one or two row blocks and each XCD's L2
// serves a row to every query that selected it instead of fetching it again.
template <int WDT>
__global__ __launch_bounds__(256) void gather_blocked_kernel(
    const void* __restrict__ W, const float* __restrict__ bias, const float* __restrict__ X, int ldx,
    RowBlocking rb, float* __restrict__ Y, int ldy, float* __restrict__ yc, int ldc, int d, int act,
    const int32_t* __restrict__ skip_group, int B, int by_xcd) {
  extern __shared__ __align__(16) float xs[];
  using C = Chunk<WDT>;
  using vec_t = typename C::vec_t;
  // Workgroups are dealt to the eight XCDs in turn.  Small batches (by_xcd): all queries of one
  // row block go to the same XCD (block b to XCD b % 8, queries fastest), so a block's rows are
  // fetched into one L2 and served from there to every query instead of once per XCD (C3 batch
  // 32: 49 -> 25 us per layer).  Large batches keep every XCD busy on every block (queries
  // fastest over all XCDs): there the eightfold fetch is shared by enough queries, and binding
  // a block to one XCD costs balance (C3 batch 1024 keep .05: 8 % slower).
  int q, blk;
  if (by_xcd) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    q = slot % B;
    blk = (slot / B) * 8 + xcd;
  } else {
    q = blockIdx.x % B;
    blk = blockIdx.x / B;
  }
  if (blk >= rb.nblk) return;
  if (skip_group && skip_group[q >> 4]) return;      // served by the grouped evaluation
  const int32_t* off = rb.blk_off + (size_t)q * (rb.nblk + 1);
  const int c0 = off[blk], c1 = off[blk + 1];
  if (c0 >= c1) return;
  const int tid = threadIdx.x;
  const float* x = X + (size_t)q * ldx;
  for (int i = tid; i < (d >> 2); i += 256)
    reinterpret_cast<float4*>(xs)[i] = reinterpret_cast<const float4*>(x)[i];
  __syncthreads();
  // One wavefront per row, two rows in flight: a (query, block) pair often holds only a
  // dozen rows, which would leave most 16-lane groups idle; these rows are long (the
  // matrix is large), so 64 lanes x 16 bytes per step still means many steps per row.
  const int wave = tid >> 6, lane = tid & 63;
  const int nv = d / C::ELEMS;
  const int32_t* pidx = rb.part_idx + (size_t)q * rb.stride;
  const int32_t* ppos = rb.part_pos + (size_t)q * rb.stride;
  for (int t0 = c0 + 2 * wave; t0 < c1; t0 += 8) {
    const bool two = t0 + 1 < c1;
    const int j0 = pidx[t0], j1 = pidx[two ? t0 + 1 : t0];
    const vec_t* w0 = reinterpret_cast<const vec_t*>(static_cast<const char*>(W) +
                                                     (size_t)j0 * d * (WDT == SLONN_F32 ? 4 : 2));
    const vec_t* w1 = reinterpret_cast<const vec_t*>(static_cast<const char*>(W) +
                                                     (size_t)j1 * d * (WDT == SLONN_F32 ? 4 : 2));
    float acc0 = 0.0f, acc1 = 0.0f;
#pragma unroll 4
    for (int i = lane; i < nv; i += 64) {
      const vec_t a0 = w0[i], a1 = w1[i];
      const float* xp = xs + i * C::ELEMS;
      acc0 = C::dot(a0, xp, acc0);
      acc1 = C::dot(a1, xp, acc1);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      acc0 += __shfl_xor(acc0, o);
      acc1 += __shfl_xor(acc1, o);
    }
    if (lane == 0 || (lane == 1 && two)) {
      const int j = lane == 0 ? j0 : j1;
      float z = (lane == 0 ? acc0 : acc1) + bias[j];
      if (act == SLONN_ACT_RELU) z = z > 0.0f ? z : 0.0f;
      if (Y) Y[(size_t)q * ldy + j] = z;
      if (yc) yc[(size_t)q * ldc + ppos[t0 + lane]] = z;
    }
  }
}

// First layer on sparse (ELL) input.  With input-major storage every non-zero pulls one
// contiguous row of n weights: a workgroup owns 64 consecutive nodes of one query (one lane
// per node), its four wavefronts split the non-zeros (staged in LDS), eight row reads are in
// flight per lane, and the four partial sums are added in LDS in a fixed order.
template <int WDT>
__global__ __launch_bounds__(256) void ell_layer_kernel(
    const void* __restrict__ W, int w_layout, const float* __restrict__ bias,
    const int32_t* __restrict__ idx, const float* __restrict__ val, const int32_t* __restrict__ nnz,
    int ell_stride, float* __restrict__ Y, int ldy, int d, int n, int act) {
  extern __shared__ __align__(16) unsigned char ell_smem[];
  using C = Chunk<WDT>;
  const int q = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // the row's entry count and columns live in device memory the host cannot check: the count is
  // clamped to the row's slots, an entry whose column lies outside [0, d) contributes nothing
  const int c = min(max(nnz[q], 0), ell_stride);
  int32_t* s_idx = reinterpret_cast<int32_t*>(ell_smem);
  float* s_val = reinterpret_cast<float*>(s_idx + ell_stride);
  float* part = s_val + ell_stride;                       // [4][64]
  for (int t = tid; t < c; t += 256) {
    const int i = idx[(size_t)q * ell_stride + t];
    const bool ok = (unsigned)i < (unsigned)d;
    s_idx[t] = ok ? i : 0;
    s_val[t] = ok ? val[(size_t)q * ell_stride + t] : 0.0f;
  }
  __syncthreads();
  const int j = blockIdx.y * 64 + lane;
  const int jj = j < n ? j : n - 1;
  const int per = (c + 3) / 4;
  const int t0 = wave * per, t1 = min(c, t0 + per);
  float acc = 0.0f;
  for (int t = t0; t < t1; t += 8) {
    float w[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int tt = t + u < t1 ? t + u : t0;
      const int i = s_idx[tt];
      const size_t at = (w_layout == SLONN_ROWS_ARE_INPUTS) ? (size_t)i * n + jj : (size_t)jj * d + i;
      w[u] = C::elem(W, at);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (t + u < t1) acc = fmaf(w[u], s_val[t + u], acc);
  }
  part[wave * 64 + lane] = acc;
  __syncthreads();
  if (wave == 0 && j < n) {
    float z = part[lane] + part[64 + lane] + part[128 + lane] + part[192 + lane] + bias[j];
    if (act == SLONN_ACT_RELU) z = z > 0.0f ? z : 0.0f;
    Y[(size_t)q * ldy + j] = z;
  }
}

// Softmax over the computed nodes and/or argmax (lowest id among equal maxima).
// One wavefront per query.  Values are read from the dense row Y[q][id], or, when the
// caller only keeps the compact form (Y == nullptr), from yc[q][t] in list order.
__global__ __launch_bounds__(64) void finalize_kernel(float* __restrict__ Y, int ldy, int n,
                                                     const int32_t* __restrict__ active,
                                                     const int32_t* __restrict__ cnt, int idx_stride,
                                                     float* __restrict__ yc, int ldc, int do_softmax,
                                                     int32_t* __restrict__ argmax) {
  const int q = blockIdx.x, lane = threadIdx.x;
  const int c = active ? cnt[q] : n;
  const int32_t* list = active ? active + (size_t)q * idx_stride : nullptr;
  float* y = Y ? Y + (size_t)q * ldy : nullptr;
  float* yq = yc ? yc + (size_t)q * ldc : nullptr;
  float best = -INFINITY;
  int besti = 0x7FFFFFFF;
  for (int t = lane; t < c; t += 64) {
    const int j = list ? list[t] : t;
    const float v = y ? y[j] : yq[t];
    if (v > best || (v == best && j < besti)) { best = v; besti = j; }
  }
  for (int o = 32; o > 0; o >>= 1) {
    const float ob = __shfl_xor(best, o);
    const int oi = __shfl_xor(besti, o);
    if (ob > best || (ob == best && oi < besti)) { best = ob; besti = oi; }
  }
  if (argmax && lane == 0) argmax[q] = besti;
  if (!do_softmax) return;
  float sum = 0.0f;
  for (int t = lane; t < c; t += 64) {
    const int j = list ? list[t] : t;
    sum += expf((y ? y[j] : yq[t]) - best);
  }
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
  const float inv = 1.0f / sum;
  for (int t = lane; t < c; t += 64) {
    const int j = list ? list[t] : t;
    const float p = expf((y ? y[j] : yq[t]) - best) * inv;
    if (y) y[j] = p;
    if (yq) yq[t] = p;
  }
}

// entries a query's list buffer is sure to hold (no list: ids are the positions themselves)
inline int idx_stride_or(const int32_t* active, int idx_stride, int n) { return active ? idx_stride : n; }

}  // namespace

int launch_gather_forward(const void* W, int w_dtype, const float* bias, const float* X, int ldx,
                          const int32_t* active, const int32_t* cnt, int idx_stride, int max_rows,
                          float* Y, int ldy, float* yc, int ldc, int B, int d, int n, int act,
                          hipStream_t s) {
  ProfScope prof_(SLONN_PROF_GATHER, s);
  if (max_rows <= 0 || B <= 0) return SLONN_OK;
  const int esz = (w_dtype == SLONN_F32) ? 4 : 2;
  const int chunk = 16 / esz;
  const bool vec = (d % chunk == 0) && (ldx % 4 == 0) && (reinterpret_cast<uintptr_t>(W) % 16 == 0) &&
                   (reinterpret_cast<uintptr_t>(X) % 16 == 0);
  const size_t lds = ((size_t)d + 8) * sizeof(float);
  // rows too long for the query vector to be staged in LDS (beyond 40 952 inputs): the kernel that
  // reads the vector from global memory, whatever the batch
  const bool too_long = lds > ((size_t)160 << 10);
  const bool row_ok = vec && (size_t)d * esz >= 4096 && max_rows <= idx_stride_or(active, idx_stride, n);
  if (too_long && (!row_ok || B > 65535))
    SLONN_FAIL(SLONN_EUNSUPPORTED, "gather: d_in %d does not fit the LDS staging buffer%s", d,
               row_ok ? " and the batch is beyond 65535" : " and the rows are not 16-byte aligned");
  // beyond 64 KB a kernel has to be granted its dynamic LDS explicitly
  auto grant = [&](const void* fn) -> int {
    if (lds > 65536) SLONN_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    return SLONN_OK;
  };
  const int a = (act == SLONN_ACT_RELU) ? SLONN_ACT_RELU : SLONN_ACT_NONE;
  // few queries, or few rows each (a skinny layer computed in full): the 64-row chunks of the
  // general kernel would leave most of the chip idle; long rows: one wavefront per row
  const long coarse_wgs = (long)B * ((max_rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK);
  if (row_ok && (B <= GATHER_ROW_MAX_BATCH || too_long)) {
    // one workgroup per list entry (at most 2048 per query, strided beyond)
    dim3 grid(std::min(max_rows, 2048), B);
    if (w_dtype == SLONN_F32)
      hipLaunchKernelGGL((gather_row_kernel<SLONN_F32>), grid, dim3(256), 0, s, W, bias, X, ldx, active, cnt,
                         idx_stride, Y, ldy, yc, ldc, d, n, a, (int)grid.x);
    else
      hipLaunchKernelGGL((gather_row_kernel<SLONN_BF16>), grid, dim3(256), 0, s, W, bias, X, ldx, active, cnt,
                         idx_stride, Y, ldy, yc, ldc, d, n, a, (int)grid.x);
    SLONN_HIP(hipGetLastError());
    return SLONN_OK;
  }
  if (vec && (B <= 16 || coarse_wgs < 1024) && (size_t)d * esz >= 1024) {
    int chunks = (max_rows + ROWS_PER_WAVE_BLOCK - 1) / ROWS_PER_WAVE_BLOCK;
    chunks = std::min(chunks, std::max(4, 4096 / B));
    dim3 grid(B, chunks);
    if (int g = grant(w_dtype == SLONN_F32 ? reinterpret_cast<const void*>(gather_wave_kernel<SLONN_F32>)
                                           : reinterpret_cast<const void*>(gather_wave_kernel<SLONN_BF16>)))
      return g;
    if (w_dtype == SLONN_F32)
      hipLaunchKernelGGL((gather_wave_kernel<SLONN_F32>), grid, dim3(256), lds, s, W, bias, X, ldx, active,
                         cnt, idx_stride, Y, ldy, yc, ldc, d, n, a, (int)grid.y);
    else
      hipLaunchKernelGGL((gather_wave_kernel<SLONN_BF16>), grid, dim3(256), lds, s, W, bias, X, ldx, active,
                         cnt, idx_stride, Y, ldy, yc, ldc, d, n, a, (int)grid.y);
    SLONN_HIP(hipGetLastError());
    return SLONN_OK;
  }
  // enough chunks per query to fill the chip, never more than the list can have
  int chunks = (max_rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
  const int want = std::max(4, (4096 + B - 1) / B);
  if (chunks > want) chunks = want;
  dim3 grid(B, chunks);
#define SLONN_LAUNCH_GATHER(WDT, VEC)                                                              \
  if (int g = grant(reinterpret_cast<const void*>(gather_forward_kernel<WDT, VEC>))) return g;     \
  hipLaunchKernelGGL((gather_forward_kernel<WDT, VEC>), grid, dim3(256), lds, s, W, bias, X, ldx,  \
                     active, cnt, idx_stride, Y, ldy, yc, ldc, d, n, a, (int)grid.y)
  if (w_dtype == SLONN_F32) {
    if (vec) { SLONN_LAUNCH_GATHER(SLONN_F32, true); } else { SLONN_LAUNCH_GATHER(SLONN_F32, false); }
  } else {
    if (vec) { SLONN_LAUNCH_GATHER(SLONN_BF16, true); } else { SLONN_LAUNCH_GATHER(SLONN_BF16, false); }
  }
#undef SLONN_LAUNCH_GATHER
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

int launch_gather_blocked(const void* W, int w_dtype, const float* bias, const float* X, int ldx,
                          const RowBlocking& rb, float* Y, int ldy, float* yc, int ldc, int B, int d,
                          int n, int act, const int32_t* skip_group, hipStream_t s) {
  ProfScope prof_(SLONN_PROF_GATHER, s);
  if (B <= 0) return SLONN_OK;
  const size_t lds = ((size_t)d + 8) * sizeof(float);
  if (lds > ((size_t)160 << 10))
    SLONN_FAIL(SLONN_EUNSUPPORTED, "gather: d_in %d does not fit the LDS staging buffer", d);
  if (lds > 65536)
    SLONN_HIP(hipFuncSetAttribute(w_dtype == SLONN_F32 ? reinterpret_cast<const void*>(gather_blocked_kernel<SLONN_F32>)
                                                       : reinterpret_cast<const void*>(gather_blocked_kernel<SLONN_BF16>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  const int by_xcd = B <= 128;
  dim3 grid((unsigned)(by_xcd ? 8 * ((rb.nblk + 7) / 8) : rb.nblk) * B);
  const int a = (act == SLONN_ACT_RELU) ? SLONN_ACT_RELU : SLONN_ACT_NONE;
  if (w_dtype == SLONN_F32)
    hipLaunchKernelGGL((gather_blocked_kernel<SLONN_F32>), grid, dim3(256), lds, s, W, bias, X, ldx, rb, Y,
                       ldy, yc, ldc, d, a, skip_group, B, by_xcd);
  else
    hipLaunchKernelGGL((gather_blocked_kernel<SLONN_BF16>), grid, dim3(256), lds, s, W, bias, X, ldx, rb, Y,
                       ldy, yc, ldc, d, a, skip_group, B, by_xcd);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

int launch_ell_layer(const void* W, int w_dtype, int w_layout, const float* bias, const int32_t* idx,
                     const float* val, const int32_t* nnz, int ell_stride, float* Y, int ldy, int B,
                     int d, int n, int act, hipStream_t s) {
  ProfScope prof_(SLONN_PROF_ELL, s);
  if ((n + 63) / 64 > 65535) SLONN_FAIL(SLONN_EUNSUPPORTED, "sparse-input layer with %d nodes is too wide", n);
  dim3 grid(B, (n + 63) / 64);
  const int a = (act == SLONN_ACT_RELU) ? SLONN_ACT_RELU : SLONN_ACT_NONE;
  const size_t lds = (size_t)ell_stride * 8 + 4 * 64 * 4;
  if (lds > 65536) SLONN_FAIL(SLONN_EUNSUPPORTED, "ELL input with %d slots per row does not fit LDS", ell_stride);
  if (w_dtype == SLONN_F32)
    hipLaunchKernelGGL((ell_layer_kernel<SLONN_F32>), grid, dim3(256), lds, s, W, w_layout, bias, idx, val,
                       nnz, ell_stride, Y, ldy, d, n, a);
  else
    hipLaunchKernelGGL((ell_layer_kernel<SLONN_BF16>), grid, dim3(256), lds, s, W, w_layout, bias, idx,
                       val, nnz, ell_stride, Y, ldy, d, n, a);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

int launch_finalize(float* Y, int ldy, int n, const int32_t* active, const int32_t* cnt,
                    int idx_stride, float* yc, int ldc, int do_softmax, int32_t* argmax, int B,
                    hipStream_t s) {
  ProfScope prof_(SLONN_PROF_FINALIZE, s);
  if (!do_softmax && !argmax) return SLONN_OK;
  hipLaunchKernelGGL(finalize_kernel, dim3(B), dim3(64), 0, s, Y, ldy, n, active, cnt, idx_stride, yc,
                     ldc, do_softmax, argmax);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

// ---- measurement aid: what a compute unit draws from L2 with 16-byte loads ----
namespace {
// Every workgroup (1024 threads, one per compute unit when the grid is the unit count) reads the
// same 2 MiB window `passes` times, four 16-byte loads in flight per lane: after the first pass the
// window sits in the L2 of every XCD.
__global__ __launch_bounds__(1024) void l2_read_probe_kernel(const uint4* __restrict__ buf, int pieces, int passes,
                                                             uint32_t* __restrict__ out) {
  uint32_t acc = 0;
  for (int p = 0; p < passes; ++p)
    for (int i = threadIdx.x; i + 3 * 1024 < pieces; i += 4 * 1024) {
      const uint4 a = buf[i], b = buf[i + 1024], c = buf[i + 2048], d = buf[i + 3072];
      acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
  out[(size_t)blockIdx.x * 1024 + threadIdx.x] = acc;
}
}  // namespace

// buf: 2 MiB + workgroups * 4096 bytes of device memory (any contents).  Returns the bytes the launch reads.
double launch_l2_read_probe(void* buf, int workgroups, int passes, hipStream_t s) {
  const int pieces = (2 << 20) / 16;
  uint32_t* out = reinterpret_cast<uint32_t*>(static_cast<char*>(buf) + (2 << 20));
  hipLaunchKernelGGL(l2_read_probe_kernel, dim3(workgroups), dim3(1024), 0, s, static_cast<const uint4*>(buf), pieces,
                     passes, out);
  return (double)pieces * 16.0 * passes * workgroups;
}

}  // namespace slonn
