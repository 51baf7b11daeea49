// Large batches of a large fp32 layer: evaluation of the selected (query, node) pairs as masked
// dense tiles on the bf16 matrix cores (the paper's Section 6 names batch inference as future
// work).  At batch 1024 every 128-node block of a layer is wanted by some of any 128 queries,
// and a per-query gather moves keep x batch times the bytes of the matrix; a tile kernel moves
// the matrix once per 128 queries and leaves the arithmetic to the matrix cores.
//
// Arithmetic: an fp32 number is the exact sum of three bf16 numbers (8 + 8 + 8 significand
// bits): w = w_hi + w_mid + w_lo, x = x_hi + x_mid + x_lo.  Of the nine partial products the six
// with at most 16 bits of combined offset are accumulated (each exact in fp32, smallest first);
// the three left out (mid x lo, lo x mid, lo x lo) are below 2^-24 of the product, the size of
// one fp32 rounding.  Six v_mfma_f32_16x16x32_bf16 replace sixteen fp32 MFMAs of the same
// 16 x 16 x 32 block at a sixteenth of the cost each.
//
//   split3_kernel        fp32 rows -> three bf16 parts, interleaved per eight elements: element k
//                        of part p of row i at i * 3 d + (k / 8) * 24 + 8 p + k % 8, so a row's
//                        chunk of 32 elements is 192 contiguous bytes.  Weights once at model
//                        creation, activations once per layer call.
//   (the select kernel)  per 128 queries the decision whether the tile kernel or the per-query
//                        gather serves them (the queries must list at least a threshold of
//                        (query, node) pairs per query together), once per 16 queries, the unit
//                        the other paths skip by; for served queries one bit per (query, node)
//                        pair of the active lists (RowBlocking::mask, kernels_select.hip).  A
//                        selected hash node has its bit too: inside a tile its pair costs
//                        nothing extra, so its projection is not reused there.
//   masked_tiles_kernel  128 x 128 (query x node) tiles per workgroup with eight wavefronts as 2
//                        query halves x 4 node strips (128 x 256 with one weight part), or 64 x
//                        64 (64 x 128) with four for batches that would not fill the chip with
//                        the large tiles; chunks of 32 elements double-
//                        buffered in LDS, the next chunks' global loads in flight during the
//                        MFMAs; only selected pairs are written.
#include <algorithm>

#include "slonn_internal.h"

namespace slonn {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // a 16-byte piece (native vector: stays in registers)

constexpr int TM = 128;           // queries per decision unit
constexpr int TN = 128;           // nodes per tile
constexpr int PIECES = 12;        // 16-byte pieces per row and chunk: 4 groups of 8 elements x 3 parts

__global__ void split3_kernel(const float* __restrict__ X, int64_t ldx, int d, uint16_t* __restrict__ out) {
  const int64_t row = blockIdx.x;
  const int i = blockIdx.y * blockDim.x + threadIdx.x;
  if (i >= d) return;
  const float x = X[row * ldx + i];
  const uint32_t hb = __float_as_uint(x) & 0xFFFF0000u;
  const float r1 = x - __uint_as_float(hb);             // exact: hi keeps the leading bits of x
  const uint32_t mb = __float_as_uint(r1) & 0xFFFF0000u;
  const float r2 = r1 - __uint_as_float(mb);            // exact, at most 8 significant bits left
  const size_t at = (size_t)row * 3 * d + (size_t)(i >> 3) * 24 + (i & 7);
  out[at] = (uint16_t)(hb >> 16);
  out[at + 8] = (uint16_t)(mb >> 16);
  out[at + 16] = (uint16_t)(__float_as_uint(r2) >> 16);
}

// Barrier that orders LDS traffic only: global loads issued before it stay in flight across it
// (__syncthreads would wait for them as well).
__device__ __forceinline__ void lds_only_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// Eight consecutive fp32 numbers (a, b: their bits) as three pieces of eight bf16 numbers each:
// the leading 8 significand bits, the next 8, the last 8 (the arithmetic of split3_kernel).
// Two neighbouring elements (their bits) -> one 32-bit word of each part.
__device__ __forceinline__ void split_pair(uint32_t x0, uint32_t x1, uint32_t& hi, uint32_t& mid, uint32_t& lo) {
  const uint32_t x[2] = {x0, x1};
  uint32_t r1[2], r2[2];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const float f1 = __uint_as_float(x[e]) - __uint_as_float(x[e] & 0xFFFF0000u);      // exact
    r1[e] = __float_as_uint(f1);
    const float f2 = f1 - __uint_as_float(r1[e] & 0xFFFF0000u);                         // exact, at most 8 bits left
    r2[e] = __float_as_uint(f2);
  }
  hi = (x[0] >> 16) | (x[1] & 0xFFFF0000u);
  mid = (r1[0] >> 16) | (r1[1] & 0xFFFF0000u);
  lo = (r2[0] >> 16) | (r2[1] & 0xFFFF0000u);
}
__device__ __forceinline__ void split8(u32x4 a, u32x4 b, u32x4& hi, u32x4& mid, u32x4& lo) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const u32x4 v = j < 2 ? a : b;
    uint32_t h, m, l;
    split_pair(v[(2 * j) & 3], v[(2 * j + 1) & 3], h, m, l);
    hi[j] = h; mid[j] = m; lo[j] = l;
  }
}

// X3: activation rows in three interleaved bf16 parts (see above).  Wp: weight rows, for WP = 3 in
// the same three-part layout, for WP = 1 plain bf16 rows (bf16 weights: w x_hi, w x_mid, w x_lo
// are each exact in fp32, three MFMAs per block).  d a multiple of 32.
// Lane layout of v_mfma_f32_16x16x32_bf16 (checked on gfx950): lane l feeds row l % 16 of its
// operand with the eight elements 8 (l / 16) .. + 7 of the step; register v of lane l holds
// D[4 (l / 16) + v][l % 16], rows from the first operand (here: nodes), columns from the second
// (queries).
// TQ queries x TNN nodes per tile; WP weight parts; NT threads (wavefronts in 2 x NT / 128: query halves x node strips).
// XF: the activations come as fp32 rows Xf (16-byte aligned, ldx a multiple of 4) and are split
// into their three parts on the way from registers to LDS (44 vector instructions per thread and
// chunk in the shadow of 48 or 96 MFMAs), so that no three-part copy of them passes through HBM;
// otherwise X3 holds that copy.
template <int TQ, int TNN, int WP, int NT, bool XF>
__global__ __launch_bounds__(NT) void masked_tiles_kernel(const uint16_t* __restrict__ X3,
                                                          const float* __restrict__ Xf, int ldx,
                                                          const uint16_t* __restrict__ Wp,
                                                          const float* __restrict__ bias,
                                                          const uint32_t* __restrict__ mask,
                                                          const int32_t* __restrict__ flags,
                                                          float* __restrict__ Y, int ldy, int B, int n, int d,
                                                          int act) {
  extern __shared__ u32x4 tiles_lds[];     // two buffers of [TQ rows of X | TNN rows of W]
  constexpr int PX = PIECES, PW = 4 * WP;  // 16-byte pieces per row and chunk of 32 elements
  // LDS rows padded by two pieces: 14 (6) pieces per row.  A wavefront's fragment read -- lane (r, kg) takes
  // piece r * ROW + kg * parts + p -- then costs 4 LDS cycles, the full 256 bytes per cycle; with one
  // piece of padding (odd row lengths) or none it costs 8, and the kernel was bound by its LDS
  // traffic (measured per wavefront instruction with every row length from 9 to 34: the lengths
  // that are 2 modulo 4 are the conflict-free ones).
  constexpr int ROWX = PX + 2, ROWW = PW + 2;
  constexpr int BUF16 = TQ * ROWX + TNN * ROWW;
  constexpr int QB = TQ / 32;              // 16-query blocks per wavefront
  constexpr int XG = TQ * 4 / NT;          // XF: groups of eight fp32 activations per thread and chunk
  constexpr int XP = XF ? 2 * XG : TQ * PX / NT;   // 16-byte pieces of activations loaded per thread and chunk
  constexpr int XSTEP = XF ? 8 : PX;       // pieces per row and chunk in global memory
  static_assert(TQ * 4 % NT == 0, "activation groups must divide evenly");
  constexpr int WT = TNN * PW / NT;         // W pieces per thread and chunk
  constexpr int WN = NT / 128;             // node strips (wavefronts along the nodes)
  constexpr int NB = TNN / (16 * WN);       // 16-node blocks per wavefront
  static_assert(TQ * PX % NT == 0 && TNN * PW % NT == 0, "loader pieces must divide evenly");
  const int m0 = blockIdx.y * TQ, n0 = blockIdx.x * TNN;
  if (flags && !flags[m0 / 16]) return;    // these queries are served another way (no flags: all are served here)
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wq = wave / WN, wn = wave % WN;
  const int r = lane & 15, kg = lane >> 4;

  // loader: rows beyond the batch or the layer repeat the last valid row (their results are dropped)
  const u32x4* xsrc[XP];
  const u32x4* wsrc[WT];
  int dstx[XP], dstw[WT];
  if constexpr (XF) {
#pragma unroll
    for (int g = 0; g < XG; ++g) {
      const int idx = tid + NT * g, row = idx / 4, grp = idx % 4;
      xsrc[2 * g] = reinterpret_cast<const u32x4*>(Xf + (size_t)min(m0 + row, B - 1) * ldx) + 2 * grp;
      xsrc[2 * g + 1] = xsrc[2 * g] + 1;
      dstx[2 * g] = row * ROWX + 3 * grp;
      dstx[2 * g + 1] = 0;               // (unused)
    }
  } else {
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      const int idx = tid + NT * i, row = idx / PX, piece = idx % PX;
      xsrc[i] = reinterpret_cast<const u32x4*>(X3 + (size_t)min(m0 + row, B - 1) * 3 * d) + piece;
      dstx[i] = row * ROWX + piece;
    }
  }
#pragma unroll
  for (int i = 0; i < WT; ++i) {
    const int idx = tid + NT * i, row = idx / PW, piece = idx % PW;
    wsrc[i] = reinterpret_cast<const u32x4*>(Wp + (size_t)min(n0 + row, n - 1) * WP * d) + piece;
    dstw[i] = TQ * ROWX + row * ROWW + piece;
  }
  // Chunk c is multiplied out of LDS buffer c % 2 while chunk c + 1 moves from registers into the
  // other buffer and chunks c + 2 and c + 3 are on their way from L2 (two register sets: a
  // load has two chunks' worth of MFMAs to arrive).  One barrier per chunk, and one that orders
  // LDS traffic only: the global loads stay in flight across it.  Chunks past the end repeat the
  // last one and are dropped.
  const int nchunks = d / 32;
  const int last = nchunks - 1;
  u32x4 r0x[XP], r0w[WT], r1x[XP], r1w[WT];
#define SLONN_TILES_LOAD(RX, RW, CHUNK)                                            \
  {                                                                               \
    const size_t c_ = (size_t)min((CHUNK), last);                                 \
    _Pragma("unroll") for (int i = 0; i < XP; ++i) RX[i] = xsrc[i][c_ * XSTEP];   \
    _Pragma("unroll") for (int i = 0; i < WT; ++i) RW[i] = wsrc[i][c_ * PW];      \
  }
#define SLONN_TILES_STORE(BUF, RX, RW, SP)                                         \
  {                                                                               \
    u32x4* buf_ = tiles_lds + (BUF) * BUF16;                                      \
    if constexpr (XF) {                                                           \
      _Pragma("unroll") for (int g = 0; g < XG; ++g)                              \
        _Pragma("unroll") for (int p = 0; p < 3; ++p) buf_[dstx[2 * g] + p] = SP[g][p]; \
    } else {                                                                      \
      _Pragma("unroll") for (int i = 0; i < XP; ++i) buf_[dstx[i]] = RX[i];       \
    }                                                                             \
    _Pragma("unroll") for (int i = 0; i < WT; ++i) buf_[dstw[i]] = RW[i];         \
  }
  u32x4 sp[XG][3];                         // XF: the three parts of the chunk that moves to LDS next
  SLONN_TILES_LOAD(r0x, r0w, 0);
  SLONN_TILES_LOAD(r1x, r1w, 1);
  if constexpr (XF) {
#pragma unroll
    for (int g = 0; g < XG; ++g) split8(r0x[2 * g], r0x[2 * g + 1], sp[g][0], sp[g][1], sp[g][2]);
  }
  SLONN_TILES_STORE(0, r0x, r0w, sp);
  SLONN_TILES_LOAD(r0x, r0w, 2);
  lds_only_barrier();
  // now: LDS buffer 0 holds chunk 0, r1 chunk 1, r0 chunk 2

  f32x4 acc[NB][QB];                       // [node block][query block]
#pragma unroll
  for (int a = 0; a < NB; ++a)
#pragma unroll
    for (int b = 0; b < QB; ++b) acc[a][b] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // (XF: between the MFMAs the registers RX of the chunk that moves to LDS next are split into
  // sp, a few instructions after every query block, so that the vector instructions run in the
  // shadow of the MFMAs instead of in one run between two chunks)
  auto multiply = [&](int buf, const u32x4 (&RX)[XP]) {
    const u32x4* Xs = tiles_lds + buf * BUF16;
    const u32x4* Ws = Xs + TQ * ROWX;
    bf16x8 xb[QB][3];
#pragma unroll
    for (int b = 0; b < QB; ++b)
#pragma unroll
      for (int p = 0; p < 3; ++p) xb[b][p] = as_bf16x8(Xs[(wq * (TQ / 2) + b * 16 + r) * ROWX + kg * 3 + p]);
    constexpr int PAIRS = 4 / NB;          // XF: pairs of elements split per node block (NB is 2 or 4)
    static_assert(!XF || ((NB == 2 || NB == 4) && (QB == 2 || QB == 4)), "the split is spread over the blocks");
    uint32_t f1[XG][PAIRS][2], f2[XG][PAIRS][2];
#pragma unroll
    for (int a = 0; a < NB; ++a) {
      bf16x8 wa[WP];
#pragma unroll
      for (int p = 0; p < WP; ++p) wa[p] = as_bf16x8(Ws[(wn * 16 * NB + a * 16 + r) * ROWW + kg * WP + p]);
#pragma unroll
      for (int b = 0; b < QB; ++b) {
        f32x4 v = acc[a][b];               // smallest partial products first
        if (WP == 3) {
          v = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[WP - 1], xb[b][0], v, 0, 0, 0);
          v = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[WP / 2], xb[b][1], v, 0, 0, 0);
          v = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[0], xb[b][2], v, 0, 0, 0);
          v = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[WP / 2], xb[b][0], v, 0, 0, 0);
          v = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[0], xb[b][1], v, 0, 0, 0);
          v = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[0], xb[b][0], v, 0, 0, 0);
        } else {
          v = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[0], xb[b][2], v, 0, 0, 0);
          v = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[0], xb[b][1], v, 0, 0, 0);
          v = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[0], xb[b][0], v, 0, 0, 0);
        }
        acc[a][b] = v;
        if constexpr (XF) {
          // a quarter (QB = 4) or a half (QB = 2) of the split of this node block's share of the
          // elements; the scheduler may not move vector instructions or MFMAs past this point, so
          // the split's instructions stay in the shadow of the MFMAs around them
          constexpr int SPB = 4 / QB;      // stages per query block
#pragma unroll
          for (int st = b * SPB; st < (b + 1) * SPB; ++st)
#pragma unroll
            for (int g = 0; g < XG; ++g)
#pragma unroll
              for (int jj = 0; jj < PAIRS; ++jj) {
                const int j = a * PAIRS + jj;      // elements 2 j, 2 j + 1 of the group of eight
                const uint32_t x0 = RX[2 * g + (j >> 1)][(2 * j) & 3], x1 = RX[2 * g + (j >> 1)][(2 * j + 1) & 3];
                uint32_t(&t1)[2] = f1[g][jj];
                uint32_t(&t2)[2] = f2[g][jj];
                if (st == 0) {
                  t1[0] = __float_as_uint(__uint_as_float(x0) - __uint_as_float(x0 & 0xFFFF0000u));   // exact
                  t1[1] = __float_as_uint(__uint_as_float(x1) - __uint_as_float(x1 & 0xFFFF0000u));
                } else if (st == 1) {
                  t2[0] = __float_as_uint(__uint_as_float(t1[0]) - __uint_as_float(t1[0] & 0xFFFF0000u));   // exact
                  t2[1] = __float_as_uint(__uint_as_float(t1[1]) - __uint_as_float(t1[1] & 0xFFFF0000u));
                } else if (st == 2) {
                  sp[g][0][j] = (x0 >> 16) | (x1 & 0xFFFF0000u);
                  sp[g][1][j] = (t1[0] >> 16) | (t1[1] & 0xFFFF0000u);
                } else {
                  sp[g][2][j] = (t2[0] >> 16) | (t2[1] & 0xFFFF0000u);
                }
              }
          __builtin_amdgcn_sched_barrier(0x0004 | 0x0010 | 0x0080);   // scalar, memory and LDS instructions may cross
        }
      }
    }
  };
  int c = 0;
  for (; c + 2 <= nchunks; c += 2) {       // chunks c (buffer 0) and c + 1 (buffer 1)
    multiply(0, r1x);
    SLONN_TILES_STORE(1, r1x, r1w, sp);    // chunk c + 1
    SLONN_TILES_LOAD(r1x, r1w, c + 3);
    lds_only_barrier();
    multiply(1, r0x);
    SLONN_TILES_STORE(0, r0x, r0w, sp);    // chunk c + 2
    SLONN_TILES_LOAD(r0x, r0w, c + 4);
    lds_only_barrier();
  }
  if (c < nchunks) multiply(0, r1x);       // an odd number of chunks
#undef SLONN_TILES_LOAD
#undef SLONN_TILES_STORE

  // register v of block (a, b): node n0 + 16 NB wn + 16 a + 4 kg + v, query m0 + (TQ / 2) wq + 16 b + r.
  // Every element of the tile is written: the result for a selected pair, zero for the others (the
  // select kernel does not clear the output rows of the queries the tiles serve) -- four nodes of
  // one query as one 16-byte store where the row allows it.
  const int words = (n + 31) >> 5;
  const bool vec_out = (ldy % 4 == 0) && (reinterpret_cast<uintptr_t>(Y) % 16 == 0);
#pragma unroll
  for (int b = 0; b < QB; ++b) {
    const int q = m0 + wq * (TQ / 2) + b * 16 + r;
    if (q >= B) continue;
#pragma unroll
    for (int a = 0; a < NB; ++a) {
      const int node = n0 + wn * 16 * NB + a * 16 + 4 * kg; // a multiple of 4: its four bits share a word
      if (node >= n) continue;
      // (no mask: a layer computed in full, every pair counts)
      const uint32_t four = mask ? (mask[(size_t)q * words + (node >> 5)] >> (node & 31)) & 0xFu : 0xFu;
      float zv[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        float z = 0.0f;
        if (((four >> v) & 1u) && node + v < n) {
          z = acc[a][b][v] + bias[node + v];
          if (act == SLONN_ACT_RELU) z = z > 0.0f ? z : 0.0f;
        }
        zv[v] = z;
      }
      float* yp = Y + (size_t)q * ldy + node;
      if (vec_out && node + 3 < n) {
        *reinterpret_cast<float4*>(yp) = make_float4(zv[0], zv[1], zv[2], zv[3]);
      } else {
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (node + v < n) yp[v] = zv[v];
      }
    }
  }
}

template <int TQ, int TNN, int WP>
constexpr size_t tiles_lds_bytes() { return (size_t)2 * (TQ * (PIECES + 2) + TNN * (4 * WP + 2)) * 16; }

}  // namespace

bool masked_tiles_supported(int d, int n, int max_lds) {
  return d % 32 == 0 && (size_t)((n + 31) / 32) * 4 <= (size_t)max_lds && tiles_lds_bytes<128, 128, 3>() <= (size_t)max_lds;
}

// (pair masks, flags, and room for a three-part copy of the activations, which launch_dense_tiles
// makes of rows that are not 16-byte aligned)
size_t masked_tiles_workspace_bytes(int B, int n, int d) {
  const size_t mask = ((size_t)B * ((n + 31) / 32) * 4 + 255) / 256 * 256;
  const size_t flags = ((size_t)(B / 16 + TM / 16 + 1) * 4 + 255) / 256 * 256;
  return mask + flags + (size_t)B * 3 * d * 2 + 256;
}

int launch_split3(const float* X, int64_t ldx, int64_t rows, int d, uint16_t* out, hipStream_t s) {
  hipLaunchKernelGGL(split3_kernel, dim3((unsigned)rows, (d + 255) / 256), dim3(256), 0, s, X, ldx, d, out);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

namespace {

// The tile shape for a batch and a layer, and the launch.  X3 == nullptr: the kernel splits the
// fp32 activations X itself.
template <int TQ_, int TN_, int WP_, int NT_>
int launch_tiles_shape(const uint16_t* X3, const float* X, int ldx, const uint16_t* Wp, const float* bias,
                       const uint32_t* mask, const int32_t* flags, float* Y, int ldy, int B, int n, int d, int a,
                       hipStream_t s) {
  constexpr size_t lds = tiles_lds_bytes<TQ_, TN_, WP_>();
  static_assert(lds <= 160 * 1024, "two tile buffers must fit the LDS of a compute unit");
  const dim3 grid((n + TN_ - 1) / TN_, (B + TQ_ - 1) / TQ_);
  if (X3) {
    SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(masked_tiles_kernel<TQ_, TN_, WP_, NT_, false>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL((masked_tiles_kernel<TQ_, TN_, WP_, NT_, false>), grid, dim3(NT_), lds, s, X3, X, ldx, Wp, bias,
                       mask, flags, Y, ldy, B, n, d, a);
  } else {
    SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(masked_tiles_kernel<TQ_, TN_, WP_, NT_, true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL((masked_tiles_kernel<TQ_, TN_, WP_, NT_, true>), grid, dim3(NT_), lds, s, X3, X, ldx, Wp, bias,
                       mask, flags, Y, ldy, B, n, d, a);
  }
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

int launch_tiles(const uint16_t* X3, const float* X, int ldx, const uint16_t* Wp, int w_parts, const float* bias,
                 const uint32_t* mask, const int32_t* flags, float* Y, int ldy, int B, int n, int d, int a,
                 hipStream_t s) {
  // 128 x 128 tiles with eight wavefronts once they fill the chip (each weight tile is fetched
  // half as often: C3 batch 1024 190 -> 160 us per layer)
  const bool big = (long)((B + 127) / 128) * ((n + TN - 1) / TN) >= 256;
  const bool wide = (long)((B + 127) / 128) * ((n + 255) / 256) >= 256;
  if (w_parts == 3) {
    // below that 64 x 64 tiles with four wavefronts: four times as many workgroups (C3 tiles per
    // step, 64 x 128 against 64 x 64: batch 256 348 -> 213 us, batch 512 351 -> 340, batch 768
    // 508 -> 456; at batch 1024 the 128 x 128 tiles take 458 us, 64 x 64 tiles 596)
    if (big) return launch_tiles_shape<128, 128, 3, 512>(X3, X, ldx, Wp, bias, mask, flags, Y, ldy, B, n, d, a, s);
    return launch_tiles_shape<64, 64, 3, 256>(X3, X, ldx, Wp, bias, mask, flags, Y, ldy, B, n, d, a, s);
  }
  // one weight part: twice the node strip per wavefront keeps the LDS reads per MFMA down
  if (wide) return launch_tiles_shape<128, 256, 1, 512>(X3, X, ldx, Wp, bias, mask, flags, Y, ldy, B, n, d, a, s);
  if (big) return launch_tiles_shape<128, 128, 1, 512>(X3, X, ldx, Wp, bias, mask, flags, Y, ldy, B, n, d, a, s);
  return launch_tiles_shape<64, 128, 1, 256>(X3, X, ldx, Wp, bias, mask, flags, Y, ldy, B, n, d, a, s);
}

// fp32 rows the tile kernel can fetch in 16-byte pieces
bool rows_aligned(const float* X, int ldx) { return ldx % 4 == 0 && reinterpret_cast<uintptr_t>(X) % 16 == 0; }

}  // namespace

void masked_tiles_buffers(void* scratch, int B, int n, uint32_t** mask, int32_t** flags) {
  const size_t mask_bytes = ((size_t)B * ((n + 31) / 32) * 4 + 255) / 256 * 256;
  *mask = static_cast<uint32_t*>(scratch);
  *flags = reinterpret_cast<int32_t*>(static_cast<char*>(scratch) + mask_bytes);
}

// The select kernel has written the pair masks and the per-tile decisions into scratch
// (masked_tiles_buffers).  X: fp32 rows the kernel fetches in 16-byte pieces (16-byte aligned, ldx a
// multiple of 4).
int launch_masked_tiles(const uint16_t* Wp, int w_parts, const float* bias, const float* X, int ldx, float* Y,
                        int ldy, int B, int d, int n, int act, void* scratch, int32_t** flags_out, hipStream_t s) {
  if (!rows_aligned(X, ldx)) SLONN_FAIL(SLONN_EINVAL, "masked tiles: activations must be 16-byte aligned rows");
  uint32_t* mask = nullptr;
  int32_t* flags = nullptr;
  masked_tiles_buffers(scratch, B, n, &mask, &flags);
  *flags_out = flags;
  ProfScope prof_(SLONN_PROF_TILES, s);
  const int a = (act == SLONN_ACT_RELU) ? SLONN_ACT_RELU : SLONN_ACT_NONE;
  return launch_tiles(nullptr, X, ldx, Wp, w_parts, bias, mask, flags, Y, ldy, B, n, d, a, s);
}

// A layer computed in full for a large batch through the same tiles (no mask, every query
// served): bf16 weights as they are (w_parts 1) or fp32 weights in three parts (w_parts 3).
// scratch: 3 * B * d * 2 bytes (used for a three-part copy of activations that are not 16-byte aligned).
int launch_dense_tiles(const uint16_t* Wp, int w_parts, const float* bias, const float* X, int ldx, float* Y,
                       int ldy, int B, int d, int n, int act, void* scratch, hipStream_t s) {
  ProfScope prof_(SLONN_PROF_DENSE, s);
  uint16_t* X3 = nullptr;
  if (!rows_aligned(X, ldx)) {
    X3 = static_cast<uint16_t*>(scratch);
    const int rc = launch_split3(X, ldx, B, d, X3, s);
    if (rc) return rc;
  }
  const int a = (act == SLONN_ACT_RELU) ? SLONN_ACT_RELU : SLONN_ACT_NONE;
  return launch_tiles(X3, X, ldx, Wp, w_parts, bias, nullptr, nullptr, Y, ldy, B, n, d, a, s);
}

}  // namespace slonn
