// Node Activator query for one layer (Fig. 2 steps 1, 3, 4; Section 3.3): sign bits of
// the FreeHash projections -> one key per table -> one ranked node list per table ->
// the first m distinct nodes in rank-major, table-minor order, continuing down the
// whole-set ranking if the lists run out.
//
// Two kernels, both one workgroup per query (select_block.h; 256 threads, 1024 for batches of at
// most one query per compute unit): select_block_kernel
// keeps a 4-byte first-occurrence entry per node in LDS; select_wide_kernel, for layers too
// wide for that (a 100 000-node output layer would need 400 KB), keeps one bit per node
// plus a small per-round table.  Both can also regroup the finished list by weight-row
// block for the row-block gather.
#include <algorithm>

#include "select_block.h"
#include "slonn_internal.h"

namespace slonn {
namespace {

__device__ __forceinline__ int budget_of(float keep, int n) {
  double m = floor((double)keep * (double)n + 0.5);
  if (!(m >= 1.0)) m = 1.0;        // also a keep fraction that is not a number
  if (m > (double)n) m = (double)n;
  return (int)m;
}

constexpr int SEL_NT = 256;      // workgroup size for real batches
constexpr int SEL_NT_BIG = 1024; // up to one query per compute unit: four times as many threads per query
// (select per step with 256- against 1024-thread workgroups: C3 batch 128 75 / 51 us, batch 256
// 98 / 76, batch 512 111 / 116; C5 batch 128 407 / 245, batch 256 424 / 309)
constexpr int SEL_BIG_MAX_BATCH = 256;
constexpr int WIDE_MU = 4;       // slots per thread per round of the kernel for very wide layers (1024 per round)

// Regroup a finished list by weight-row block (counting sort; the order inside a group does
// not matter: outputs are written by node id and by selection position).  Selected hash nodes
// get their output from the projections z here and join no group.  hist: at least nblk + 1
// free words of LDS.  Called by the whole workgroup after the list is complete (the list was
// written by other threads: the barrier at the top also orders those global stores).
template <int NT>
__device__ __forceinline__ void partition_rows(const int32_t* out, int m, const RowBlocking& rb, int q,
                                               const float* z, uint32_t* hist) {
  const int tid = threadIdx.x;
  __syncthreads();
  for (int b = tid; b <= rb.nblk; b += NT) hist[b] = 0;
  __syncthreads();
  // (a thread's first KEEP entries stay in registers for the second pass; rows_per_block is a
  // power of two)
  constexpr int KEEP = 4;
  const int shift = __ffs(rb.rows_per_block) - 1;
  int id_r[KEEP];
#pragma unroll
  for (int u = 0; u < KEEP; ++u) id_r[u] = -1;         // -1: no entry, or a hash node (joins no group)
  auto first_pass = [&](int t) {
    const int id = out[t];
    const int hs = rb.hslot ? (int)rb.hslot[id] : -1;
    if (hs >= 0) {          // a selected hash node: its output is its projection
      float v = z[hs];
      if (rb.relu && !(v > 0.0f)) v = 0.0f;
      if (rb.y) rb.y[(size_t)q * rb.ldy + id] = v;
      if (rb.yc) rb.yc[(size_t)q * rb.ldc + t] = v;
      return -1;
    }
    atomicAdd(&hist[id >> shift], 1u);
    return id;
  };
#pragma unroll
  for (int u = 0; u < KEEP; ++u)
    if (tid + NT * u < m) id_r[u] = first_pass(tid + NT * u);
  for (int t = tid + NT * KEEP; t < m; t += NT) (void)first_pass(t);
  __syncthreads();
  if (tid < 64) {         // exclusive prefix sum over the row blocks by one wavefront
    uint32_t carry = 0;
    for (int b0 = 0; b0 <= rb.nblk; b0 += 64) {
      const int b = b0 + tid;
      const uint32_t v = (b < rb.nblk) ? hist[b] : 0u;
      uint32_t incl = v;
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = __shfl_up(incl, o);
        if (tid >= o) incl += up;
      }
      if (b <= rb.nblk) {
        const uint32_t excl = carry + incl - v;
        hist[b] = excl;
        rb.blk_off[(size_t)q * (rb.nblk + 1) + b] = (int32_t)excl;
      }
      carry += __shfl(incl, 63);
    }
  }
  __syncthreads();
  auto place = [&](int id, int t) {
    const uint32_t p = atomicAdd(&hist[id >> shift], 1u);
    rb.part_idx[(size_t)q * rb.stride + p] = id;
    rb.part_pos[(size_t)q * rb.stride + p] = t;
  };
#pragma unroll
  for (int u = 0; u < KEEP; ++u)
    if (id_r[u] >= 0) place(id_r[u], tid + NT * u);
  for (int t = tid + NT * KEEP; t < m; t += NT) {
    const int id = out[t];
    if (rb.hslot && rb.hslot[id] >= 0) continue;
    place(id, t);
  }
}

// Will the masked tiles serve query q?  The sum of the list lengths of the 128 queries of q's
// tile against the threshold, formed from their keep fractions (a list is as long as its
// budget, or as the K*L hash nodes at its head if those are more).  Every wavefront forms the sum
// for itself (two keep fractions per lane, one reduction over the lanes): no barrier, the same
// answer in every thread of the workgroup.
__device__ __forceinline__ bool tile_served(const RowBlocking& rb, const float* __restrict__ keep, int keep_stride,
                                            int n, int H, int q) {
  if (rb.served_min_per_query <= 0) return false;
  const int q0 = q - q % 128, nq = min(128, rb.B - q0);
  const int lane = threadIdx.x & 63;
  uint32_t mine = 0;
  for (int i = lane; i < nq; i += 64) {
    const int m = budget_of(keep[(size_t)(q0 + i) * keep_stride], n);
    mine += (uint32_t)((m == n || m > H) ? m : H);
  }
  for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o);
  return (long long)mine >= rb.served_min_per_query * nq;
}

// What the tile kernel reads about query q (RowBlocking::mask): for a query of a served tile one
// bit per node of its finished list out[0 .. total) (all: the whole layer), and from the tile's
// first query the tile's decision for each of its eight groups of 16 queries.  bits: (n + 31) / 32
// free words of LDS.  Whole workgroup.
template <int NT>
__device__ __forceinline__ void write_pair_mask(const RowBlocking& rb, int q, bool served, const int32_t* out,
                                                int total, int n, bool all, uint32_t* bits) {
  const int tid = threadIdx.x, words = (n + 31) >> 5;
  if (q % 128 == 0 && tid < 8) rb.flags[q / 16 + tid] = served ? 1 : 0;
  if (!served) return;
  uint32_t* row = rb.mask + (size_t)q * words;
  if (all) {
    for (int i = tid; i < words; i += NT)
      row[i] = (i == words - 1 && (n & 31)) ? ((1u << (n & 31)) - 1u) : 0xFFFFFFFFu;
    return;
  }
  __syncthreads();        // the list is complete, the LDS words are free
  for (int i = tid; i < words; i += NT) bits[i] = 0u;
  __syncthreads();
  for (int t = tid; t < total; t += NT) {
    const int node = out[t];
    atomicOr(&bits[node >> 5], 1u << (node & 31));
  }
  __syncthreads();
  for (int i = tid; i < words; i += NT) row[i] = bits[i];
}

// A medium batch leaves the hash projection's reduction split in hs.S partial sums per
// (query, hash row).  Add them in split order, add the bias, and store the projections of
// query q for this kernel and for the later readers.  Whole workgroup; ends with a barrier.
template <int NT>
__device__ __forceinline__ void sum_split_projections(const HashSplit& hs, int q, int H) {
  if (!hs.part) return;
  const size_t plane = (size_t)hs.B * H;
  for (int h = threadIdx.x; h < H; h += NT) {
    double sum = 0.0;
    for (int z = 0; z < hs.S; ++z) sum += hs.part[z * plane + (size_t)q * H + h];
    hs.Z[(size_t)q * H + h] = (float)(sum + (double)hs.bh[h]);
  }
  __syncthreads();
}

// slots per thread per round: both workgroup sizes cover up to 4096 slots in one round
template <int NT>
struct BlockMU { static constexpr int value = 4096 / NT; };

// (second launch bound: eight wavefronts per SIMD for the 512-thread workgroups of large batches --
// the kernel waits on memory round trips, and with the 106 scalar registers it would otherwise take
// only seven fit, i.e. three workgroups per compute unit instead of four.  The other sizes run one
// workgroup per compute unit or are bound by their vector registers: no point in spilling scalars.)
template <int NT, typename IdT, int MU = BlockMU<NT>::value>
__global__ __launch_bounds__(NT, NT == 512 ? 8 : 4) void select_block_kernel(
    const float* Z, int K, int L, int n, const uint32_t* __restrict__ dir,
    const IdT* __restrict__ ids, const int32_t* __restrict__ global_rank,
    const float* __restrict__ keep, int keep_stride, uint32_t* __restrict__ codes,
    int32_t* __restrict__ active, int32_t* __restrict__ cnt, int idx_stride,
    float* __restrict__ yzero, int ldy, RowBlocking rb, HashFirst hf, HashSplit hsp,
    const int32_t* __restrict__ order) {
  extern __shared__ __align__(16) uint32_t smem32[];
  SelectShared<NT, MU> sh;
  sh.prio = smem32;
  sh.s_off = smem32 + n;
  sh.s_len = sh.s_off + 64;
  sh.wave_cnt = reinterpret_cast<int*>(sh.s_len + 64);
  sh.s_misc = reinterpret_cast<uint32_t*>(sh.wave_cnt + MU * (NT / 64));

  const int q = order ? order[blockIdx.x] : (int)blockIdx.x, tid = threadIdx.x;
  const float keep_q = keep[(size_t)q * keep_stride];      // on its way while the keys form
  int32_t* out = active + (size_t)q * idx_stride;
  const float* z = Z + (size_t)q * K * L;
  sum_split_projections<NT>(hsp, q, K * L);
  // The last wavefront forms the keys and fetches the bucket directory (two dependent memory
  // round trips) right away; the others find the budget, clear the output row and the maps.
  uint32_t* codes_row = codes ? codes + (size_t)q * L : nullptr;
  constexpr int NI = NT - 64;          // threads that clear
  if (tid >= NI) select_keys<NT, MU>(z, K, L, dir, sh, codes_row);
  const int m = budget_of(keep_q, n);
  float* y = yzero ? yzero + (size_t)q * ldy : nullptr;
  const int H = hf.hnodes ? K * L : 0;          // hash nodes in front of the list (Section 3.4 variant)
  const int total = (m == n || m > H) ? m : H;
  const int words = (n + 31) >> 5;
  if (tid == 0) cnt[q] = total;
  // (the tile kernel writes every element of the output rows of the queries it serves, zeros for the
  // nodes that were not selected: those rows are not cleared here)
  const bool served = tile_served(rb, keep, keep_stride, n, H, q);
  if (served && rb.mask) y = nullptr;
  if (m == n) {   // the layer is computed in full: ascending ids, no table access (the keys are written as codes)
    if (y)
      for (int i = tid; i < n; i += NT) y[i] = 0.0f;
    for (int i = tid; i < n; i += NT) out[i] = i;
    if (rb.mask) write_pair_mask<NT>(rb, q, served, out, n, n, true, sh.prio);
    if (rb.part_idx && !served) partition_rows<NT>(out, n, rb, q, z, sh.prio);
    return;
  }
  const int16_t* hskip = H ? hf.hslot : nullptr;
  // (with pair masks asked for, the merge sets one bit per chosen node as it goes)
  sh.bits = rb.mask ? sh.s_misc + 4 : nullptr;
  if (tid < NI) {
    if (y)
      for (int i = tid; i < n; i += NI) y[i] = 0.0f;
    for (int i = tid; i < n; i += NI) sh.prio[i] = 0xFFFFFFFFu;
    if (sh.bits)
      for (int i = tid; i < words; i += NI) sh.bits[i] = 0u;
    for (int h = tid; h < H; h += NI) out[h] = hf.hnodes[h];
  }
  __syncthreads();
  if (sh.bits)
    for (int h = tid; h < H; h += NT) atomicOr(&sh.bits[hf.hnodes[h] >> 5], 1u << (hf.hnodes[h] & 31));
  select_merge<NT, MU, IdT>(L, n, total - H, ids, global_rank, sh, out + H, hskip);

  if (rb.mask) {      // (select_merge ends with a barrier: every bit is set)
    if (q % 128 == 0 && tid < 8) rb.flags[q / 16 + tid] = served ? 1 : 0;
    if (served)
      for (int i = tid; i < words; i += NT) rb.mask[(size_t)q * words + i] = sh.bits[i];
  }
  if (rb.part_idx && !served) partition_rows<NT>(out, total, rb, q, z, sh.prio);
}

template <typename IdT>
__global__ __launch_bounds__(SEL_NT) void select_wide_kernel(
    const float* Z, int K, int L, int n, const uint32_t* __restrict__ dir,
    const IdT* __restrict__ ids, const int32_t* __restrict__ global_rank,
    const float* __restrict__ keep, int keep_stride, uint32_t* __restrict__ codes,
    int32_t* __restrict__ active, int32_t* __restrict__ cnt, int idx_stride,
    float* __restrict__ yzero, int ldy, RowBlocking rb, HashFirst hf, HashSplit hsp,
    const int32_t* __restrict__ order) {
  extern __shared__ __align__(16) uint32_t smem32[];
  const int words = (n + 31) >> 5;
  SelectSharedWide<SEL_NT, WIDE_MU> sh;
  sh.taken = smem32;
  sh.tkey = reinterpret_cast<int32_t*>(smem32 + words);
  sh.tval = smem32 + words + SelectWideTable<SEL_NT, WIDE_MU>::entries;
  sh.s_off = sh.tval + SelectWideTable<SEL_NT, WIDE_MU>::entries;
  sh.s_len = sh.s_off + 64;
  sh.wave_cnt = reinterpret_cast<int*>(sh.s_len + 64);
  sh.s_misc = reinterpret_cast<uint32_t*>(sh.wave_cnt + WIDE_MU * (SEL_NT / 64));

  const int q = order ? order[blockIdx.x] : (int)blockIdx.x, tid = threadIdx.x;
  const int m = budget_of(keep[(size_t)q * keep_stride], n);
  int32_t* out = active + (size_t)q * idx_stride;
  const float* z = Z + (size_t)q * K * L;
  sum_split_projections<SEL_NT>(hsp, q, K * L);
  const int H = hf.hnodes ? K * L : 0;
  // (the tile kernel writes every element of the output rows of the queries it serves: not cleared here)
  const bool served = tile_served(rb, keep, keep_stride, n, H, q);
  if (yzero && !(served && rb.mask)) {
    float* y = yzero + (size_t)q * ldy;
    for (int i = tid; i < n; i += SEL_NT) y[i] = 0.0f;
  }
  const int total = (m == n || m > H) ? m : H;
  if (tid == 0) cnt[q] = total;
  if (m == n) {
    if (codes && tid < L) {
      uint32_t key = 0;
      for (int j = 0; j < K; ++j) key |= (z[tid * K + j] > 0.0f ? 1u : 0u) << j;
      codes[(size_t)q * L + tid] = key;
    }
    for (int i = tid; i < n; i += SEL_NT) out[i] = i;
    if (rb.mask) write_pair_mask<SEL_NT>(rb, q, served, out, n, n, true, sh.taken);
    if (rb.part_idx && !served) partition_rows<SEL_NT>(out, n, rb, q, z, sh.tval);
    return;
  }
  for (int i = tid; i < words; i += SEL_NT) sh.taken[i] = 0u;
  for (int i = tid; i < SelectWideTable<SEL_NT, WIDE_MU>::entries; i += SEL_NT) { sh.tkey[i] = -1; sh.tval[i] = 0xFFFFFFFFu; }
  for (int h = tid; h < H; h += SEL_NT) out[h] = hf.hnodes[h];
  __syncthreads();
  select_block_wide<SEL_NT, WIDE_MU, IdT>(z, K, L, n, total - H, dir, ids, global_rank, sh,
                            codes ? codes + (size_t)q * L : nullptr, out + H, H ? hf.hslot : nullptr);
  if (rb.mask) write_pair_mask<SEL_NT>(rb, q, served, out, total, n, false, sh.taken);
  if (rb.part_idx && !served) partition_rows<SEL_NT>(out, total, rb, q, z, sh.tval);
}

// Queries in descending order of their budget (256 classes of the keep fraction; the order inside
// a class is whatever the atomics give: it only decides which workgroup starts first).
__global__ __launch_bounds__(1024) void order_by_budget_kernel(const float* __restrict__ keep, int keep_stride,
                                                              int B, int32_t* __restrict__ order) {
  __shared__ uint32_t hist[256];
  const int tid = threadIdx.x;
  auto klass = [&](int q) {
    float k = keep[(size_t)q * keep_stride];
    k = k > 0.0f ? (k < 1.0f ? k : 1.0f) : 0.0f;        // also a keep fraction that is not a number
    return 255 - (int)(k * 255.0f);
  };
  if (tid < 256) hist[tid] = 0;
  __syncthreads();
  for (int q = tid; q < B; q += 1024) atomicAdd(&hist[klass(q)], 1u);
  __syncthreads();
  if (tid < 64) {         // exclusive prefix over the classes: four per lane
    uint32_t c[4], sum = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) { c[j] = hist[4 * tid + j]; sum += c[j]; }
    uint32_t incl = sum;
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t up = __shfl_up(incl, o);
      if (tid >= o) incl += up;
    }
    uint32_t run = incl - sum;
#pragma unroll
    for (int j = 0; j < 4; ++j) { hist[4 * tid + j] = run; run += c[j]; }
  }
  __syncthreads();
  for (int q = tid; q < B; q += 1024) order[atomicAdd(&hist[klass(q)], 1u)] = q;
}

__global__ void fill_iota_kernel(int32_t* __restrict__ idx, int stride, int32_t* __restrict__ cnt,
                                 int n, int B) {
  const int q = blockIdx.x;          // the batch (up to 2^20) in the grid's x dimension, whose limit is 2^31 - 1
  const int i = blockIdx.y * blockDim.x + threadIdx.x;
  if (q >= B) return;
  if (idx && i < n) idx[(size_t)q * stride + i] = i;
  if (i == 0 && cnt) cnt[q] = n;
}

}  // namespace

namespace {
template <typename IdT>
int launch_select_t(const float* Z, int K, int L, int n, const uint32_t* dir, const IdT* ids,
                    const int32_t* global_rank, const float* keep, int keep_stride, int B,
                    uint32_t* codes, int32_t* active, int32_t* cnt, int idx_stride, float* yzero,
                    int ldy, int max_lds, const RowBlocking* rb, const HashFirst& hf, const HashSplit& hsp,
                    const int32_t* order, hipStream_t s) {
  const RowBlocking rbv = rb ? *rb : RowBlocking{};
  // (one more bit per node where the kernel also writes the tile kernel's pair masks)
  const size_t lds_block = ((size_t)n + SelectShared<SEL_NT, BlockMU<SEL_NT>::value>::words_besides_prio +
                            (rbv.mask ? (size_t)(n + 31) / 32 : 0)) * 4;
  if (lds_block <= (size_t)max_lds) {
    // Up to four queries on a layer with many tables (the lists of 64 tables overlap so much that a
    // chosen node costs almost thirty slots): rounds of 12 288 slots, a third of the trips to table
    // memory (C5 batch 1: 219 -> 212 us per query, batch 4: 335 -> 314; with C3's 32 tables the
    // deeper rounds fetch more than they save at keep .25 and win 4 % at keep .5)
    constexpr int MU_FEW = 12;
    const size_t lds_few = lds_block + (size_t)(MU_FEW - BlockMU<SEL_NT_BIG>::value) * (SEL_NT_BIG / 64) * 4;
    if (B <= 4 && L >= 48 && lds_few <= (size_t)max_lds) {
      if (lds_few > 65536)
        SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(select_block_kernel<SEL_NT_BIG, IdT, MU_FEW>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_few));
      hipLaunchKernelGGL((select_block_kernel<SEL_NT_BIG, IdT, MU_FEW>), dim3(B), dim3(SEL_NT_BIG), lds_few, s, Z, K, L, n,
                         dir, ids, global_rank, keep, keep_stride, codes, active, cnt, idx_stride, yzero, ldy, rbv, hf, hsp, order);
    } else if (B <= SEL_BIG_MAX_BATCH) {
      if (lds_block > 65536)
        SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(select_block_kernel<SEL_NT_BIG, IdT>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_block));
      hipLaunchKernelGGL((select_block_kernel<SEL_NT_BIG, IdT>), dim3(B), dim3(SEL_NT_BIG), lds_block, s, Z, K, L, n,
                         dir, ids, global_rank, keep, keep_stride, codes, active, cnt, idx_stride, yzero, ldy, rbv, hf, hsp, order);
    } else if (B <= 2 * SEL_BIG_MAX_BATCH || lds_block * 5 > ((size_t)160 << 10)) {
      // up to two queries per compute unit, or maps so large that at most four workgroups share a
      // unit: 512 threads (select per step with 256 / 512 threads: C3 batch 512 103 / 92 us, batch
      // 1024 131 / 137; C5 batch 2048 814 / 766)
      if (lds_block > 65536)
        SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(select_block_kernel<512, IdT>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_block));
      hipLaunchKernelGGL((select_block_kernel<512, IdT>), dim3(B), dim3(512), lds_block, s, Z, K, L, n, dir,
                         ids, global_rank, keep, keep_stride, codes, active, cnt, idx_stride, yzero, ldy, rbv, hf, hsp, order);
    } else {
      if (lds_block > 65536)
        SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(select_block_kernel<SEL_NT, IdT>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_block));
      hipLaunchKernelGGL((select_block_kernel<SEL_NT, IdT>), dim3(B), dim3(SEL_NT), lds_block, s, Z, K, L, n, dir,
                         ids, global_rank, keep, keep_stride, codes, active, cnt, idx_stride, yzero, ldy, rbv, hf, hsp, order);
    }
    SLONN_HIP(hipGetLastError());
    return SLONN_OK;
  }
  const size_t lds = ((size_t)((n + 31) >> 5) + SelectSharedWide<SEL_NT, WIDE_MU>::words_besides_bitmap) * 4;
  if (lds > (size_t)max_lds)
    SLONN_FAIL(SLONN_EUNSUPPORTED, "select: layer with %d nodes needs %zu bytes of LDS, device grants %d",
               n, lds, max_lds);
  if (lds > 65536)
    SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(select_wide_kernel<IdT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  hipLaunchKernelGGL(select_wide_kernel<IdT>, dim3(B), dim3(SEL_NT), lds, s, Z, K, L, n, dir, ids, global_rank,
                     keep, keep_stride, codes, active, cnt, idx_stride, yzero, ldy, rb ? *rb : RowBlocking{}, hf, hsp, order);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}
}  // namespace

int launch_select(const float* Z, int K, int L, int n, const uint32_t* dir, const void* ids, bool ids_narrow,
                  const int32_t* global_rank, const float* keep, int keep_stride, int B,
                  uint32_t* codes, int32_t* active, int32_t* cnt, int idx_stride, float* yzero,
                  int ldy, int max_lds, const RowBlocking* rb, const HashFirst* hash_first,
                  const HashSplit* split, const int32_t* order, hipStream_t s) {
  ProfScope prof_(SLONN_PROF_SELECT, s);
  const HashFirst hf = hash_first ? *hash_first : HashFirst{};
  const HashSplit hsp = split ? *split : HashSplit{};
  if (ids_narrow)
    return launch_select_t(Z, K, L, n, dir, static_cast<const uint16_t*>(ids), global_rank, keep, keep_stride, B, codes,
                           active, cnt, idx_stride, yzero, ldy, max_lds, rb, hf, hsp, order, s);
  return launch_select_t(Z, K, L, n, dir, static_cast<const int32_t*>(ids), global_rank, keep, keep_stride, B, codes,
                         active, cnt, idx_stride, yzero, ldy, max_lds, rb, hf, hsp, order, s);
}

// More queries than workgroups of the select kernel fit on the device at once: the queries with
// the largest budgets (the longest merges) should start first.
bool select_wants_order(int n, int B, int max_lds, int n_cu) {
  const size_t lds_block = ((size_t)n + SelectShared<SEL_NT, BlockMU<SEL_NT>::value>::words_besides_prio) * 4;
  if (lds_block > (size_t)max_lds || B <= SEL_BIG_MAX_BATCH) return false;
  const size_t per_cu = std::min<size_t>(8, std::max<size_t>(1, ((size_t)160 << 10) / lds_block));
  return (size_t)B > per_cu * (size_t)n_cu;
}

int launch_order_by_budget(const float* keep, int keep_stride, int B, int32_t* order, hipStream_t s) {
  ProfScope prof_(SLONN_PROF_SELECT, s);
  hipLaunchKernelGGL(order_by_budget_kernel, dim3(1), dim3(1024), 0, s, keep, keep_stride, B, order);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

bool select_fills_row_blocks(int n, int max_lds) {
  return ((size_t)((n + 31) >> 5) + SelectSharedWide<SEL_NT, WIDE_MU>::words_besides_bitmap) * 4 <= (size_t)max_lds;
}

int launch_fill_iota(int32_t* idx, int stride, int32_t* cnt, int n, int B, hipStream_t s) {
  const int chunks = idx ? (n + 255) / 256 : 1;
  if (chunks > 65535) SLONN_FAIL(SLONN_EUNSUPPORTED, "compact output of a layer with %d nodes is too wide", n);
  dim3 grid(B, chunks);
  hipLaunchKernelGGL(fill_iota_kernel, grid, dim3(256), 0, s, idx, stride, cnt, n, B);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

}  // namespace slonn
