// Bucket member lists for all L tables of one LSH at once (Alg. 1 hashes every training input
// into one bucket per table; everything summed per bucket afterwards is summed in input order so
// that the results do not depend on scheduling).  Used by the Node Importance table build and by
// the Confidence LSH tables.
//   bucket_hist_kernel     hist[b][key] = number of inputs of table b's bucket key
//   bucket_scan_kernel     start[b][0..nb] = exclusive prefix sums (one workgroup per table)
//   bucket_members_kernel  members[b][start .. ] = the bucket's inputs in ascending order
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace slonn {
namespace {

__global__ void bucket_hist_kernel(const uint32_t* __restrict__ keys, int64_t N, int L, int nb,
                                   uint32_t* __restrict__ hist) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;      // (input, table)
  if (e >= N * L) return;
  const int b = (int)(e % L);
  const uint32_t key = keys[e];
  if (key < (uint32_t)nb) atomicAdd(&hist[(size_t)b * nb + key], 1u);
}

// start[b][0..nb] = exclusive prefix sums of hist[b][0..nb); cursor = copy of start
__global__ __launch_bounds__(256) void bucket_scan_kernel(const uint32_t* __restrict__ hist, int nb,
                                                         uint32_t* __restrict__ start,
                                                         uint32_t* __restrict__ cursor) {
  __shared__ uint32_t wsum[4];
  __shared__ uint32_t carry_s;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint32_t* h = hist + (size_t)b * nb;
  uint32_t* st = start + (size_t)b * (nb + 1);
  uint32_t* cu = cursor + (size_t)b * nb;
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (int k0 = 0; k0 < nb; k0 += 256) {
    const int k = k0 + tid;
    const uint32_t v = k < nb ? h[k] : 0u;
    uint32_t incl = v;
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    uint32_t before = carry_s;
    for (int w = 0; w < wave; ++w) before += wsum[w];
    if (k < nb) { st[k] = before + incl - v; cu[k] = before + incl - v; }
    __syncthreads();
    if (tid == 0) carry_s += wsum[0] + wsum[1] + wsum[2] + wsum[3];
    __syncthreads();
  }
  if (tid == 0) st[nb] = carry_s;
}

// Members of every bucket in ascending input order: one wavefront per table walks the inputs
// 64 at a time; lanes with equal keys find each other with K ballots, the lowest of them
// reserves the run of slots at the bucket's cursor (an L2 atomic, so the next chunk sees it)
// and every lane stores its input at reserved base + its rank among the equal lanes.
__global__ __launch_bounds__(64) void bucket_members_kernel(const uint32_t* __restrict__ keys, int64_t N,
                                                           int L, int K, int nb,
                                                           uint32_t* __restrict__ cursor,
                                                           uint32_t* __restrict__ members) {
  const int b = blockIdx.x, lane = threadIdx.x;
  uint32_t* cu = cursor + (size_t)b * nb;
  uint32_t* mem = members + (size_t)b * N;
  const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  for (int64_t x0 = 0; x0 < N; x0 += 64) {
    const int64_t x = x0 + lane;
    const bool live = x < N;
    const uint32_t key = live ? keys[x * L + b] : 0u;
    unsigned long long same = __ballot(live);
    for (int j = 0; j < K; ++j) {
      const unsigned long long bit = __ballot((key >> j) & 1u);
      same &= ((key >> j) & 1u) ? bit : ~bit;
    }
    if (!live) same = 0ull;
    const int rank = __popcll(same & below);
    const int leader = same ? (__ffsll((long long)same) - 1) : lane;
    uint32_t base = 0;
    if (live && rank == 0) base = atomicAdd(&cu[key], (uint32_t)__popcll(same));
    base = __shfl(base, leader);
    if (live) mem[base + rank] = (uint32_t)x;
  }
}

}  // namespace
}  // namespace slonn
