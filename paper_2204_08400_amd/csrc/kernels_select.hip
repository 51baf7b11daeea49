// Node Activator query for one layer (Fig. 2 steps 1, 3, 4; Section 3.3): sign bits of
// the FreeHash projections -> one key per table -> one ranked node list per table ->
// the first m distinct nodes in rank-major, table-minor order, continuing down the
// whole-set ranking if the lists run out.
//
// Two kernels.  select_block_kernel: a 256-thread workgroup per query with a 4-byte
// first-occurrence entry per node in LDS (select_block.h); used whenever that map fits.
// select_wave_kernel: for very wide layers (a 100 000-node output layer needs 400 KB of
// 4-byte entries), one wavefront per query and ONE BYTE per node:
//
// One wavefront serves one query.  A step looks at 64 consecutive slots of the merged
// order (slot s = rank r * L + table b, one lane per slot).  A byte map in LDS, one
// byte per node of the layer, resolves duplicates without atomics:
//   0xFF  node not seen yet
//   1..64 (lane+1) node claimed in the current step by that lane
//   0     node taken in an earlier step
// Lanes holding the same node lower the byte until it equals the smallest claiming
// lane (+1); only that lane -- the first occurrence in merge order -- keeps the node.
// Survivors are compacted with a ballot and a prefix population count.
#include "select_block.h"
#include "slonn_internal.h"

namespace slonn {
namespace {

__device__ __forceinline__ int budget_of(float keep, int n) {
  double m = floor((double)keep * (double)n + 0.5);
  if (m < 1.0) m = 1.0;
  if (m > (double)n) m = (double)n;
  return (int)m;
}

__global__ __launch_bounds__(64) void select_wave_kernel(
    const float* __restrict__ Z, int K, int L, int n, const uint32_t* __restrict__ dir,
    const int32_t* __restrict__ ids, const int32_t* __restrict__ global_rank,
    const float* __restrict__ keep, int keep_stride, uint32_t* __restrict__ codes,
    int32_t* __restrict__ active, int32_t* __restrict__ cnt, int idx_stride,
    float* __restrict__ yzero, int ldy) {
  extern __shared__ __align__(16) unsigned char smem[];
  // layout: [0, 256) s_off, [256, 512) s_len, [512, 512 + n) stamps
  uint32_t* s_off = reinterpret_cast<uint32_t*>(smem);
  uint32_t* s_len = s_off + 64;
  volatile unsigned char* stamp = smem + 512;

  const int q = blockIdx.x;
  const int lane = threadIdx.x;
  const int m = budget_of(keep[(size_t)q * keep_stride], n);
  int32_t* out = active + (size_t)q * idx_stride;

  if (yzero) {
    float* y = yzero + (size_t)q * ldy;
    for (int i = lane; i < n; i += 64) y[i] = 0.0f;
  }

  // keys and bucket directory (one lane per table)
  const int nb1 = (1 << K) + 1;
  uint32_t my_len = 0;
  if (lane < L) {
    const float* z = Z + (size_t)q * K * L + lane * K;
    uint32_t key = 0;
    for (int j = 0; j < K; ++j) key |= (z[j] > 0.0f ? 1u : 0u) << j;
    if (codes) codes[(size_t)q * L + lane] = key;
    uint32_t lo = dir[(size_t)lane * nb1 + key], hi = dir[(size_t)lane * nb1 + key + 1];
    s_off[lane] = lo;
    my_len = hi - lo;
    s_len[lane] = my_len;
  }
  if (lane == 0) cnt[q] = m;

  if (m == n) {   // the layer is computed in full: ascending ids, no table access
    for (int i = lane; i < n; i += 64) out[i] = i;
    return;
  }

  // longest list of this query
  uint32_t maxlen = my_len;
  for (int o = 32; o > 0; o >>= 1) {
    uint32_t other = __shfl_xor(maxlen, o);
    maxlen = other > maxlen ? other : maxlen;
  }

  {  // clear the byte map (n bytes, rounded up to words inside the allocation)
    uint32_t* w = reinterpret_cast<uint32_t*>(smem + 512);
    const int words = (n + 3) >> 2;
    for (int i = lane; i < words; i += 64) w[i] = 0xFFFFFFFFu;
  }
  __syncthreads();   // single wave: orders the LDS writes above with the reads below

  int count = 0;
  const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  const long long nslots = (long long)maxlen * L;
  for (long long base = 0; base < nslots && count < m; base += 64) {
    const long long s = base + lane;
    const uint32_t r = (uint32_t)(s / L);
    const int b = (int)(s - (long long)r * L);
    const bool valid = s < nslots && r < s_len[b];
    int node = -1;
    if (valid) node = ids[s_off[b] + r];
    const unsigned char me = (unsigned char)(lane + 1);
    if (valid) {
      // lower the byte to the smallest claiming lane; ends after at most as many
      // rounds as there are lanes holding this node
      while (true) {
        unsigned char cur = stamp[node];
        if (cur <= me) break;
        stamp[node] = me;
      }
    }
    __builtin_amdgcn_wave_barrier();
    const bool mine = valid && stamp[node] == me;
    const unsigned long long votes = __ballot(mine);
    if (mine) {
      stamp[node] = 0;
      int pos = count + __popcll(votes & below);
      if (pos < m) out[pos] = node;
    }
    count += __popcll(votes);
    __builtin_amdgcn_wave_barrier();
  }

  // fallback: the ranking over the whole training set (a permutation: no duplicates)
  for (int base = 0; base < n && count < m; base += 64) {
    const int i = base + lane;
    int node = -1;
    bool mine = false;
    if (i < n) {
      node = global_rank[i];
      mine = stamp[node] != 0;
    }
    const unsigned long long votes = __ballot(mine);
    if (mine) {
      int pos = count + __popcll(votes & below);
      if (pos < m) out[pos] = node;
    }
    count += __popcll(votes);
  }
}

constexpr int SEL_NT = 256;

__global__ __launch_bounds__(SEL_NT) void select_block_kernel(
    const float* __restrict__ Z, int K, int L, int n, const uint32_t* __restrict__ dir,
    const int32_t* __restrict__ ids, const int32_t* __restrict__ global_rank,
    const float* __restrict__ keep, int keep_stride, uint32_t* __restrict__ codes,
    int32_t* __restrict__ active, int32_t* __restrict__ cnt, int idx_stride,
    float* __restrict__ yzero, int ldy, RowBlocking rb) {
  extern __shared__ __align__(16) uint32_t smem32[];
  SelectShared<SEL_NT> sh;
  sh.prio = smem32;
  sh.s_off = smem32 + n;
  sh.s_len = sh.s_off + 64;
  sh.wave_cnt = reinterpret_cast<int*>(sh.s_len + 64);
  sh.s_misc = reinterpret_cast<uint32_t*>(sh.wave_cnt + SELECT_MU * (SEL_NT / 64));

  const int q = blockIdx.x, tid = threadIdx.x;
  const int m = budget_of(keep[(size_t)q * keep_stride], n);
  int32_t* out = active + (size_t)q * idx_stride;
  const float* z = Z + (size_t)q * K * L;
  if (yzero) {
    float* y = yzero + (size_t)q * ldy;
    for (int i = tid; i < n; i += SEL_NT) y[i] = 0.0f;
  }
  if (tid == 0) cnt[q] = m;
  if (m == n) {   // the layer is computed in full: ascending ids, no table access
    if (codes && tid < L) {
      uint32_t key = 0;
      for (int j = 0; j < K; ++j) key |= (z[tid * K + j] > 0.0f ? 1u : 0u) << j;
      codes[(size_t)q * L + tid] = key;
    }
    for (int i = tid; i < n; i += SEL_NT) out[i] = i;
    if (rb.part_idx) {      // every row is active: the groups are the row blocks themselves
      for (int i = tid; i < n; i += SEL_NT) {
        rb.part_idx[(size_t)q * rb.stride + i] = i;
        rb.part_pos[(size_t)q * rb.stride + i] = i;
      }
      for (int b = tid; b <= rb.nblk; b += SEL_NT)
        rb.blk_off[(size_t)q * (rb.nblk + 1) + b] = min(b * rb.rows_per_block, n);
    }
    return;
  }
  for (int i = tid; i < n; i += SEL_NT) sh.prio[i] = 0xFFFFFFFFu;
  __syncthreads();
  select_block<SEL_NT>(z, K, L, n, m, dir, ids, global_rank, sh, codes ? codes + (size_t)q * L : nullptr, out);

  if (rb.part_idx) {
    // Regroup the list by weight-row block (counting sort; the order inside a group does not
    // matter: outputs are written by node id and by selection position).  The map's first
    // nblk+1 words are free again and serve as the histogram.
    uint32_t* hist = sh.prio;
    for (int b = tid; b <= rb.nblk; b += SEL_NT) hist[b] = 0;
    __syncthreads();
    for (int t = tid; t < m; t += SEL_NT) atomicAdd(&hist[out[t] / rb.rows_per_block], 1u);
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
    for (int t = tid; t < m; t += SEL_NT) {
      const int id = out[t];
      const uint32_t p = atomicAdd(&hist[id / rb.rows_per_block], 1u);
      rb.part_idx[(size_t)q * rb.stride + p] = id;
      rb.part_pos[(size_t)q * rb.stride + p] = t;
    }
  }
}

__global__ void fill_iota_kernel(int32_t* __restrict__ idx, int stride, int32_t* __restrict__ cnt,
                                 int n, int B) {
  const int q = blockIdx.y;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= B) return;
  if (idx && i < n) idx[(size_t)q * stride + i] = i;
  if (i == 0 && cnt) cnt[q] = n;
}

}  // namespace

int launch_select(const float* Z, int K, int L, int n, const uint32_t* dir, const int32_t* ids,
                  const int32_t* global_rank, const float* keep, int keep_stride, int B,
                  uint32_t* codes, int32_t* active, int32_t* cnt, int idx_stride, float* yzero,
                  int ldy, int max_lds, const RowBlocking* rb, hipStream_t s) {
  ProfScope prof_(SLONN_PROF_SELECT, s);
  const size_t lds_block = ((size_t)n + SelectShared<SEL_NT>::words_besides_prio) * 4;
  if (lds_block <= (size_t)max_lds) {
    if (lds_block > 65536)
      SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(select_block_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_block));
    hipLaunchKernelGGL(select_block_kernel, dim3(B), dim3(SEL_NT), lds_block, s, Z, K, L, n, dir, ids,
                       global_rank, keep, keep_stride, codes, active, cnt, idx_stride, yzero, ldy,
                       rb ? *rb : RowBlocking{});
    SLONN_HIP(hipGetLastError());
    return SLONN_OK;
  }
  const size_t lds = 512 + (((size_t)n + 3) & ~(size_t)3);
  if (lds > (size_t)max_lds)
    SLONN_FAIL(SLONN_EUNSUPPORTED, "select: layer with %d nodes needs %zu bytes of LDS, device grants %d",
               n, lds, max_lds);
  if (lds > 65536) {
    SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(select_wave_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  }
  hipLaunchKernelGGL(select_wave_kernel, dim3(B), dim3(64), lds, s, Z, K, L, n, dir, ids, global_rank, keep,
                     keep_stride, codes, active, cnt, idx_stride, yzero, ldy);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

bool select_fills_row_blocks(int n, int max_lds) {
  return ((size_t)n + SelectShared<SEL_NT>::words_besides_prio) * 4 <= (size_t)max_lds;
}

int launch_fill_iota(int32_t* idx, int stride, int32_t* cnt, int n, int B, hipStream_t s) {
  dim3 grid(idx ? (n + 255) / 256 : 1, B);
  hipLaunchKernelGGL(fill_iota_kernel, grid, dim3(256), 0, s, idx, stride, cnt, n, B);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

}  // namespace slonn
