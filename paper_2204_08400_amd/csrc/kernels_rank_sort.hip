// Ranking of whole buckets by a radix sort (table build, set-up work): used where the LDS sorts of
// kernels_build.hip do not reach -- lists longer than 8192 ids on layers wider than that, buckets
// whose sums are equal in masses, and the whole-set ranking of a wide layer (Alg. 1: Rank =
// argsort(NodeScore), highest first; equal sums in ascending id order).
//
// The sort itself is rocPRIM's segmented radix sort, a plain library primitive: keys are the
// fp64 sums in descending order, values the node ids fed in ascending order; a radix sort is
// stable, so equal sums keep ascending ids.  Segments are whole buckets of more than 8192 sums
// (rocPRIM sorts segments of that size by radix passes, never by its small-segment network sorts).
#include <cstring>

#include <rocprim/rocprim.hpp>

#include <algorithm>

#include "slonn_internal.h"

namespace slonn {
namespace {

__global__ void iota_mod_kernel(int32_t* __restrict__ ids, size_t total, int n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) ids[i] = (int32_t)(i % (size_t)n);
}

__global__ void segment_offsets_kernel(uint32_t* __restrict__ offs, int segs, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i <= segs) offs[i] = (uint32_t)i * (uint32_t)n;
}

// the heads of the sorted segments to their places in the id array
__global__ __launch_bounds__(256) void copy_heads_kernel(const int32_t* __restrict__ sorted, int n, int seg0,
                                                        const uint32_t* __restrict__ off,
                                                        const uint32_t* __restrict__ len,
                                                        const uint32_t* __restrict__ only,
                                                        int32_t* __restrict__ out) {
  const int seg = seg0 + blockIdx.x;
  if (only && only[seg] == only[seg + 1]) return;
  const uint32_t l = len[seg], to = off[seg];
  const int32_t* src = sorted + (size_t)blockIdx.x * n;
  for (uint32_t i = threadIdx.x; i < l; i += 256) out[to + i] = src[i];
}

template <class T>
struct Buf {
  T* p = nullptr;
  ~Buf() { if (p) (void)hipFree(p); }
  hipError_t alloc(size_t count) { return hipMalloc(&p, std::max<size_t>(count, 1) * sizeof(T)); }
};

}  // namespace

int rank_by_sort(const double* score, int n, int segs, const uint32_t* off, const uint32_t* len,
                 const uint32_t* only, int32_t* out, hipStream_t s) {
  if (segs <= 0 || n <= 0) return SLONN_OK;
  // chunks of segments of at most 2^27 sums: bounded temporary memory, 32-bit offsets
  const int chunk = (int)std::max<size_t>(1, std::min<size_t>((size_t)segs, ((size_t)1 << 27) / (size_t)n));
  const size_t total = (size_t)chunk * n;
  if (total > 0x7FFFFFFFull) SLONN_FAIL(SLONN_EUNSUPPORTED, "build: a layer of %d nodes is too wide to rank by sorting", n);
  Buf<double> keys_out;
  Buf<int32_t> ids_in, ids_out;
  Buf<uint32_t> offs;
  Buf<char> tmp;
  SLONN_HIP(keys_out.alloc(total));
  SLONN_HIP(ids_in.alloc(total));
  SLONN_HIP(ids_out.alloc(total));
  SLONN_HIP(offs.alloc((size_t)chunk + 1));
  hipLaunchKernelGGL(iota_mod_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, ids_in.p, total, n);
  SLONN_HIP(hipGetLastError());
  hipLaunchKernelGGL(segment_offsets_kernel, dim3((chunk + 256) / 256), dim3(256), 0, s, offs.p, chunk, n);
  SLONN_HIP(hipGetLastError());
  size_t tmp_bytes = 0;
  if (chunk == 1)
    SLONN_HIP(rocprim::radix_sort_pairs_desc(nullptr, tmp_bytes, score, keys_out.p, ids_in.p, ids_out.p, (size_t)n, 0, 64, s));
  else
    SLONN_HIP(rocprim::segmented_radix_sort_pairs_desc(nullptr, tmp_bytes, score, keys_out.p, ids_in.p, ids_out.p,
                                                       (unsigned int)total, (unsigned int)chunk, offs.p, offs.p + 1, 0, 64, s));
  SLONN_HIP(tmp.alloc(tmp_bytes));
  for (int seg0 = 0; seg0 < segs; seg0 += chunk) {
    const int ns = std::min(chunk, segs - seg0);
    const double* src = score + (size_t)seg0 * n;
    if (chunk == 1)
      SLONN_HIP(rocprim::radix_sort_pairs_desc(tmp.p, tmp_bytes, src, keys_out.p, ids_in.p, ids_out.p, (size_t)n, 0, 64, s));
    else
      SLONN_HIP(rocprim::segmented_radix_sort_pairs_desc(tmp.p, tmp_bytes, src, keys_out.p, ids_in.p, ids_out.p,
                                                         (unsigned int)((size_t)ns * n), (unsigned int)ns, offs.p,
                                                         offs.p + 1, 0, 64, s));
    hipLaunchKernelGGL(copy_heads_kernel, dim3(ns), dim3(256), 0, s, ids_out.p, n, seg0, off, len, only, out);
    SLONN_HIP(hipGetLastError());
  }
  // the temporaries are freed when this returns: wait for the work that uses them
  SLONN_HIP(hipStreamSynchronize(s));
  return SLONN_OK;
}

}  // namespace slonn
