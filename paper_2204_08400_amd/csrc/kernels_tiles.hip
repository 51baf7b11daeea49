// Large batches of a large layer: evaluation of the selected (query, node) pairs as masked dense
// tiles on the fp16 matrix cores (the paper's Section 6 names batch inference as future work).
// At batch 1024 every 128-node block of a layer is wanted by some of any 128 queries, and a
// per-query gather moves keep x batch times the bytes of the matrix; a tile kernel moves the
// matrix once per 128 queries and leaves the arithmetic to the matrix cores.
//
// Arithmetic: every row (a node's weights, a query's activations) is scaled by a power of two that
// brings its largest magnitude into [2^14, 2^15), and each scaled fp32 number v is written as the
// sum of two fp16 numbers, hi = v rounded to fp16 and lo = v - hi (exact in fp32) rounded to fp16:
// 11 + 11 significand bits, |v - hi - lo| <= 2^-22 |v| (on average 2^-24.5 |v|, the size of one
// fp32 rounding), and for the numbers below 2^-14 (2^-28 of the row's largest), where fp16 spaces
// its values 2^-24 apart, at most 2^-25, which is 2^-39 of the row's largest.  A bf16 weight (8
// significand bits) is one fp16 number, exactly.  Of the partial products hi x hi, hi x lo,
// lo x hi (lo x lo is below 2^-22 of the product and left out) each is exact in fp32; the matrix
// cores add them in fp32, smallest first, and the result is scaled back by the two rows' powers of
// two.  Three v_mfma_f32_16x16x32_f16 (two with bf16 weights) replace sixteen fp32 MFMAs of the
// same 16 x 16 x 32 block at a sixteenth of the cost each.  What this loses against an exact
// product is of the size of the rounding of the fp32 sums themselves (measured against the fp64
// reference the error is the same as that of a plain fp32 evaluation).
//
//   split_rows_kernel    rows -> fp16 parts, part-major per 32 elements: element k of part p of
//                        row i at i * P d + (k / 32) * 32 P + 32 p + k % 32, so a row's chunk of 32
//                        elements is 64 P contiguous bytes; and the row's exponent e (largest
//                        magnitude below 2^e).  Weights once at model creation.
//   row_exponent_kernel  the exponents of activation rows that no earlier kernel has supplied.
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
//                        MFMAs; whole output rows are written, zeros for pairs that are not selected.
#include <algorithm>
#include <climits>

#include "slonn_internal.h"

namespace slonn {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // a 16-byte piece (native vector: stays in registers)

constexpr int TM = 128;           // queries per decision unit
constexpr int TN = 128;           // nodes per tile
constexpr int XPARTS = 2;         // fp16 parts of an activation
constexpr int PIECES = 4 * XPARTS;   // 16-byte pieces per activation row and chunk of 32 elements
constexpr int SCALE_TOP = 15;     // a row with magnitudes below 2^e is scaled by 2^(SCALE_TOP - e)
constexpr int BAD_ROW = INT_MIN;  // exponent entry of a row with a non-finite element: not scaled

// exponent e of a row (largest magnitude in [2^(e-1), 2^e), 0 for a row of zeros) -> the power of two it is scaled by
__device__ __forceinline__ int tile_scale(int e) { return e == BAD_ROW ? 0 : SCALE_TOP - e; }

__device__ __forceinline__ float load_as_float(const float* p) { return *p; }
__device__ __forceinline__ float load_as_float(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }   // bf16
__device__ __forceinline__ uint16_t half_bits(_Float16 h) { return __builtin_bit_cast(uint16_t, h); }

// largest magnitude of a row over the workgroup's 256 threads -> its exponent
__device__ __forceinline__ int row_exponent_of(float mx, bool bad) {
  __shared__ float red[4];
  __shared__ int red_bad[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int b = bad ? 1 : 0;
  for (int o = 32; o > 0; o >>= 1) {
    mx = fmaxf(mx, __shfl_xor(mx, o));
    b |= __shfl_xor(b, o);
  }
  if (lane == 0) { red[wave] = mx; red_bad[wave] = b; }
  __syncthreads();
  const float m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  int e = 0;
  if (red_bad[0] | red_bad[1] | red_bad[2] | red_bad[3]) e = BAD_ROW;
  else if (m > 0.0f) (void)frexpf(m, &e);     // m = f * 2^e with f in [0.5, 1)
  return e;
}

// One workgroup of 256 threads per row.  expo_in (nullable): the rows' exponents where a kernel
// before this one has found them; otherwise they are found here (and stored in expo_out).
template <typename SRC, int PARTS>
__global__ __launch_bounds__(256) void split_rows_kernel(const SRC* __restrict__ V, int64_t ld, int d,
                                                        const int32_t* __restrict__ expo_in,
                                                        uint16_t* __restrict__ out, int32_t* __restrict__ expo_out) {
  const int64_t row = blockIdx.x;
  const SRC* v = V + row * ld;
  int e;
  if (expo_in) {
    e = expo_in[row];
  } else {
    float mx = 0.0f;
    bool bad = false;
    for (int k = threadIdx.x; k < d; k += 256) {
      const float a = fabsf(load_as_float(v + k));
      if (!(a <= 3.0e38f)) bad = true;            // infinity or NaN
      mx = fmaxf(mx, a);
    }
    e = row_exponent_of(mx, bad);
    if (threadIdx.x == 0 && expo_out) expo_out[row] = e;
  }
  const int sc = tile_scale(e);
  uint16_t* o = out + (size_t)row * PARTS * d;
  for (int k = threadIdx.x; k < d; k += 256) {
    const float x = ldexpf(load_as_float(v + k), sc);
    const _Float16 hi = (_Float16)x;
    const size_t at = (size_t)(k >> 5) * (32 * PARTS) + (k & 31);
    o[at] = half_bits(hi);
    if (PARTS == 2) o[at + 32] = half_bits((_Float16)(x - (float)hi));   // the difference is exact
  }
}

__global__ __launch_bounds__(256) void row_exponent_kernel(const float* __restrict__ X, int64_t ldx, int d,
                                                          int32_t* __restrict__ expo) {
  const int64_t row = blockIdx.x;
  const float* x = X + row * ldx;
  float mx = 0.0f;
  bool bad = false;
  if (ldx % 4 == 0 && reinterpret_cast<uintptr_t>(X) % 16 == 0) {
    for (int k = 4 * threadIdx.x; k + 3 < d; k += 1024) {
      const float4 v = *reinterpret_cast<const float4*>(x + k);
      const float a = fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w)));
      // (fmaxf drops a NaN operand: look at every element)
      if (!(fabsf(v.x) <= 3.0e38f) || !(fabsf(v.y) <= 3.0e38f) || !(fabsf(v.z) <= 3.0e38f) || !(fabsf(v.w) <= 3.0e38f)) bad = true;
      mx = fmaxf(mx, a);
    }
    for (int k = (d & ~3) + threadIdx.x; k < d; k += 256) {
      const float a = fabsf(x[k]);
      if (!(a <= 3.0e38f)) bad = true;
      mx = fmaxf(mx, a);
    }
  } else {
    for (int k = threadIdx.x; k < d; k += 256) {
      const float a = fabsf(x[k]);
      if (!(a <= 3.0e38f)) bad = true;
      mx = fmaxf(mx, a);
    }
  }
  const int e = row_exponent_of(mx, bad);
  if (threadIdx.x == 0) expo[row] = e;
}

// Barrier that orders LDS traffic only: global loads issued before it stay in flight across it
// (__syncthreads would wait for them as well).
__device__ __forceinline__ void lds_only_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ f16x8 as_f16x8(u32x4 v) { return __builtin_bit_cast(f16x8, v); }
__device__ __forceinline__ uint32_t pack_halves(_Float16 a, _Float16 b) { return __builtin_bit_cast(uint32_t, (f16x2){a, b}); }

// Eight consecutive fp32 numbers (a, b: their bits), scaled by 2^sc, as two pieces of eight fp16
// numbers each (the arithmetic of split_rows_kernel).
__device__ __forceinline__ void split8(u32x4 a, u32x4 b, int sc, u32x4& hi, u32x4& lo) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const u32x4 v = j < 2 ? a : b;
    const float x0 = ldexpf(__uint_as_float(v[(2 * j) & 3]), sc), x1 = ldexpf(__uint_as_float(v[(2 * j + 1) & 3]), sc);
    const _Float16 h0 = (_Float16)x0, h1 = (_Float16)x1;
    hi[j] = pack_halves(h0, h1);
    lo[j] = pack_halves((_Float16)(x0 - (float)h0), (_Float16)(x1 - (float)h1));
  }
}

// X2: activation rows in two fp16 parts (see above), xexp their exponents.  Wp: weight rows in WP
// fp16 parts, wexp their exponents (WP = 2: fp32 weights; WP = 1: bf16 weights, two MFMAs per
// block).  d a multiple of 32.
// Lane layout of v_mfma_f32_16x16x32_f16 (checked on gfx950): lane l feeds row l % 16 of its
// operand with the eight elements 8 (l / 16) .. + 7 of the step; register v of lane l holds
// D[4 (l / 16) + v][l % 16], rows from the first operand (here: nodes), columns from the second
// (queries).
// TQ queries x TNN nodes per tile; WP weight parts; NT threads (wavefronts in 2 x NT / 128: query halves x node strips).
// XF: the activations come as fp32 rows Xf (16-byte aligned, ldx a multiple of 4) and are scaled
// and split into their two parts on the way from registers to LDS (48 vector instructions per
// thread and chunk in the shadow of 32 or 48 MFMAs), so that no copy of them passes through HBM;
// otherwise X2 holds that copy.
template <int TQ, int TNN, int WP, int NT, bool XF>
__global__ __launch_bounds__(NT) void masked_tiles_kernel(const uint16_t* __restrict__ X2,
                                                          const float* __restrict__ Xf, int ldx,
                                                          const int32_t* __restrict__ xexp,
                                                          const uint16_t* __restrict__ Wp,
                                                          const int32_t* __restrict__ wexp,
                                                          const float* __restrict__ bias,
                                                          const uint32_t* __restrict__ mask,
                                                          const int32_t* __restrict__ flags,
                                                          float* __restrict__ Y, int ldy, int B, int n, int d,
                                                          int act) {
  extern __shared__ u32x4 tiles_lds[];     // two buffers of [TQ rows of X | TNN rows of W]
  constexpr int PX = PIECES, PW = 4 * WP;  // 16-byte pieces per row and chunk of 32 elements
  // LDS rows: the chunk's pieces part-major (piece 4 * part + group of eight elements) and two pieces
  // of padding, 10 (6) pieces per row.  A wavefront's fragment read -- lane (r, kg) takes piece
  // r * ROW + 4 * part + kg -- then costs 4 LDS cycles, the full 256 bytes per cycle; with the parts
  // of a group side by side (2 * kg + part) it costs 8 whatever the row length, and so it does with
  // one piece of padding or none (measured per wavefront instruction: the row lengths that are 2
  // modulo 4 are the conflict-free ones).
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
  int sxr[XG];                             // XF: the powers of two this thread's rows are scaled by
  if constexpr (XF) {
#pragma unroll
    for (int g = 0; g < XG; ++g) {
      const int idx = tid + NT * g, row = idx / 4, grp = idx % 4;
      const int q = min(m0 + row, B - 1);
      xsrc[2 * g] = reinterpret_cast<const u32x4*>(Xf + (size_t)q * ldx) + 2 * grp;
      xsrc[2 * g + 1] = xsrc[2 * g] + 1;
      dstx[2 * g] = row * ROWX + grp;
      dstx[2 * g + 1] = 0;               // (unused)
      sxr[g] = tile_scale(xexp[q]);
    }
  } else {
#pragma unroll
    for (int g = 0; g < XG; ++g) sxr[g] = 0;
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      const int idx = tid + NT * i, row = idx / PX, piece = idx % PX;
      xsrc[i] = reinterpret_cast<const u32x4*>(X2 + (size_t)min(m0 + row, B - 1) * XPARTS * d) + piece;
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
        _Pragma("unroll") for (int p = 0; p < XPARTS; ++p) buf_[dstx[2 * g] + 4 * p] = SP[g][p]; \
    } else {                                                                      \
      _Pragma("unroll") for (int i = 0; i < XP; ++i) buf_[dstx[i]] = RX[i];       \
    }                                                                             \
    _Pragma("unroll") for (int i = 0; i < WT; ++i) buf_[dstw[i]] = RW[i];         \
  }
  u32x4 sp[XG][XPARTS];                    // XF: the two parts of the chunk that moves to LDS next
  SLONN_TILES_LOAD(r0x, r0w, 0);
  SLONN_TILES_LOAD(r1x, r1w, 1);
  if constexpr (XF) {
#pragma unroll
    for (int g = 0; g < XG; ++g) split8(r0x[2 * g], r0x[2 * g + 1], sxr[g], sp[g][0], sp[g][1]);
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
    f16x8 xb[QB][XPARTS];
#pragma unroll
    for (int b = 0; b < QB; ++b)
#pragma unroll
      for (int p = 0; p < XPARTS; ++p) xb[b][p] = as_f16x8(Xs[(wq * (TQ / 2) + b * 16 + r) * ROWX + 4 * p + kg]);
    constexpr int PAIRS = 4 / NB;          // XF: pairs of elements split per node block (NB is 2 or 4)
    static_assert(!XF || ((NB == 2 || NB == 4) && (QB == 2 || QB == 4)), "the split is spread over the blocks");
    float xs[XG][PAIRS][2], rest[XG][PAIRS][2];
    _Float16 hi[XG][PAIRS][2];
#pragma unroll
    for (int a = 0; a < NB; ++a) {
      f16x8 wa[WP];
#pragma unroll
      for (int p = 0; p < WP; ++p) wa[p] = as_f16x8(Ws[(wn * 16 * NB + a * 16 + r) * ROWW + 4 * p + kg]);
#pragma unroll
      for (int b = 0; b < QB; ++b) {
        f32x4 v = acc[a][b];               // smallest partial products first
        if (WP == 2) {
          v = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa[WP - 1], xb[b][0], v, 0, 0, 0);
          v = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa[0], xb[b][1], v, 0, 0, 0);
          v = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa[0], xb[b][0], v, 0, 0, 0);
        } else {
          v = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa[0], xb[b][1], v, 0, 0, 0);
          v = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa[0], xb[b][0], v, 0, 0, 0);
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
                float(&t)[2] = xs[g][jj];
                float(&u)[2] = rest[g][jj];
                _Float16(&h)[2] = hi[g][jj];
                if (st == 0) {
                  t[0] = ldexpf(__uint_as_float(RX[2 * g + (j >> 1)][(2 * j) & 3]), sxr[g]);
                  t[1] = ldexpf(__uint_as_float(RX[2 * g + (j >> 1)][(2 * j + 1) & 3]), sxr[g]);
                } else if (st == 1) {
                  h[0] = (_Float16)t[0];
                  h[1] = (_Float16)t[1];
                } else if (st == 2) {
                  u[0] = t[0] - (float)h[0];       // exact
                  u[1] = t[1] - (float)h[1];
                } else {
                  sp[g][0][j] = pack_halves(h[0], h[1]);
                  sp[g][1][j] = pack_halves((_Float16)u[0], (_Float16)u[1]);
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
  // Every element of the tile is written: the result for a selected pair (the sum scaled back by
  // the two rows' powers of two, plus the bias), zero for the others (the select kernel does not
  // clear the output rows of the queries the tiles serve) -- four nodes of one query as one
  // 16-byte store where the row allows it.
  const int words = (n + 31) >> 5;
  const bool vec_out = (ldy % 4 == 0) && (reinterpret_cast<uintptr_t>(Y) % 16 == 0);
#pragma unroll
  for (int b = 0; b < QB; ++b) {
    const int q = m0 + wq * (TQ / 2) + b * 16 + r;
    if (q >= B) continue;
    const int back_q = -tile_scale(xexp[q]);
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
          z = ldexpf(acc[a][b][v], back_q - tile_scale(wexp[node + v])) + bias[node + v];
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

// scratch: pair masks | flags | exponents of the activation rows | their two-part copy (rows that are not 16-byte aligned)
struct TilesScratch {
  uint32_t* mask;
  int32_t* flags;
  int32_t* xexp;
  uint16_t* X2;
  size_t bytes;
};
TilesScratch tiles_scratch(void* scratch, int B, int n, int d) {
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  char* p = static_cast<char*>(scratch);
  TilesScratch t;
  t.mask = reinterpret_cast<uint32_t*>(p);  p += up((size_t)B * ((n + 31) / 32) * 4);
  t.flags = reinterpret_cast<int32_t*>(p);  p += up((size_t)(B / 16 + TM / 16 + 1) * 4);
  t.xexp = reinterpret_cast<int32_t*>(p);   p += up((size_t)B * 4);
  t.X2 = reinterpret_cast<uint16_t*>(p);    p += up((size_t)B * XPARTS * d * 2);
  t.bytes = (size_t)(p - static_cast<char*>(scratch));
  return t;
}

}  // namespace

bool masked_tiles_supported(int d, int n, int max_lds) {
  return d % 32 == 0 && (size_t)((n + 31) / 32) * 4 <= (size_t)max_lds && tiles_lds_bytes<128, 128, 2>() <= (size_t)max_lds;
}

size_t masked_tiles_workspace_bytes(int B, int n, int d) { return tiles_scratch(nullptr, B, n, d).bytes; }

size_t tile_weights_bytes(int w_dtype, int n, int d) { return (size_t)(w_dtype == SLONN_F32 ? 2 : 1) * n * d * 2; }

// Weight rows (fp32: two parts, bf16: one) for the tile kernel, with their exponents [n].
int launch_split_weights(const void* W, int w_dtype, int n, int d, uint16_t* out, int32_t* wexp, hipStream_t s) {
  if (w_dtype == SLONN_F32)
    hipLaunchKernelGGL((split_rows_kernel<float, 2>), dim3((unsigned)n), dim3(256), 0, s, static_cast<const float*>(W),
                       (int64_t)d, d, nullptr, out, wexp);
  else
    hipLaunchKernelGGL((split_rows_kernel<uint16_t, 1>), dim3((unsigned)n), dim3(256), 0, s,
                       static_cast<const uint16_t*>(W), (int64_t)d, d, nullptr, out, wexp);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

namespace {

// The tile shape for a batch and a layer, and the launch.  X2 == nullptr: the kernel splits the
// fp32 activations X itself.
template <int TQ_, int TN_, int WP_, int NT_>
int launch_tiles_shape(const uint16_t* X2, const float* X, int ldx, const int32_t* xexp, const uint16_t* Wp,
                       const int32_t* wexp, const float* bias, const uint32_t* mask, const int32_t* flags, float* Y,
                       int ldy, int B, int n, int d, int a, hipStream_t s) {
  constexpr size_t lds = tiles_lds_bytes<TQ_, TN_, WP_>();
  static_assert(lds <= 160 * 1024, "two tile buffers must fit the LDS of a compute unit");
  const dim3 grid((n + TN_ - 1) / TN_, (B + TQ_ - 1) / TQ_);
  if (X2) {
    SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(masked_tiles_kernel<TQ_, TN_, WP_, NT_, false>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL((masked_tiles_kernel<TQ_, TN_, WP_, NT_, false>), grid, dim3(NT_), lds, s, X2, X, ldx, xexp, Wp,
                       wexp, bias, mask, flags, Y, ldy, B, n, d, a);
  } else {
    SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(masked_tiles_kernel<TQ_, TN_, WP_, NT_, true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL((masked_tiles_kernel<TQ_, TN_, WP_, NT_, true>), grid, dim3(NT_), lds, s, X2, X, ldx, xexp, Wp,
                       wexp, bias, mask, flags, Y, ldy, B, n, d, a);
  }
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

int launch_tiles(const uint16_t* X2, const float* X, int ldx, const int32_t* xexp, const uint16_t* Wp, int w_parts,
                 const int32_t* wexp, const float* bias, const uint32_t* mask, const int32_t* flags, float* Y, int ldy,
                 int B, int n, int d, int a, hipStream_t s) {
  // 128 x 128 tiles with eight wavefronts once they fill the chip (each weight tile is fetched
  // half as often)
  const bool big = (long)((B + 127) / 128) * ((n + TN - 1) / TN) >= 256;
  const bool wide = (long)((B + 127) / 128) * ((n + 255) / 256) >= 256;
  if (w_parts == 2) {
    // below that 64 x 64 tiles with four wavefronts: four times as many workgroups
    if (big) return launch_tiles_shape<128, 128, 2, 512>(X2, X, ldx, xexp, Wp, wexp, bias, mask, flags, Y, ldy, B, n, d, a, s);
    return launch_tiles_shape<64, 64, 2, 256>(X2, X, ldx, xexp, Wp, wexp, bias, mask, flags, Y, ldy, B, n, d, a, s);
  }
  // one weight part: twice the node strip per wavefront keeps the LDS reads per MFMA down
  if (wide) return launch_tiles_shape<128, 256, 1, 512>(X2, X, ldx, xexp, Wp, wexp, bias, mask, flags, Y, ldy, B, n, d, a, s);
  if (big) return launch_tiles_shape<128, 128, 1, 512>(X2, X, ldx, xexp, Wp, wexp, bias, mask, flags, Y, ldy, B, n, d, a, s);
  return launch_tiles_shape<64, 128, 1, 256>(X2, X, ldx, xexp, Wp, wexp, bias, mask, flags, Y, ldy, B, n, d, a, s);
}

// fp32 rows the tile kernel can fetch in 16-byte pieces
bool rows_aligned(const float* X, int ldx) { return ldx % 4 == 0 && reinterpret_cast<uintptr_t>(X) % 16 == 0; }

int launch_row_exponents(const float* X, int ldx, int B, int d, int32_t* expo, hipStream_t s) {
  hipLaunchKernelGGL(row_exponent_kernel, dim3((unsigned)B), dim3(256), 0, s, X, (int64_t)ldx, d, expo);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

}  // namespace

void masked_tiles_buffers(void* scratch, int B, int n, uint32_t** mask, int32_t** flags) {
  const TilesScratch t = tiles_scratch(scratch, B, n, 32);
  *mask = t.mask;
  *flags = t.flags;
}

// The select kernel has written the pair masks and the per-tile decisions into scratch
// (masked_tiles_buffers).  X: fp32 rows the kernel fetches in 16-byte pieces (16-byte aligned, ldx a
// multiple of 4); xexp (nullable): their exponents (largest magnitude of row q below 2^xexp[q],
// INT_MIN for a row with a non-finite element) where a kernel before this one has found them.
int launch_masked_tiles(const uint16_t* Wp, int w_parts, const int32_t* wexp, const float* bias, const float* X, int ldx,
                        const int32_t* xexp, float* Y, int ldy, int B, int d, int n, int act, void* scratch,
                        int32_t** flags_out, hipStream_t s) {
  if (!rows_aligned(X, ldx)) SLONN_FAIL(SLONN_EINVAL, "masked tiles: activations must be 16-byte aligned rows");
  const TilesScratch t = tiles_scratch(scratch, B, n, d);
  *flags_out = t.flags;
  ProfScope prof_(SLONN_PROF_TILES, s);
  if (!xexp) {
    const int rc = launch_row_exponents(X, ldx, B, d, t.xexp, s);
    if (rc) return rc;
    xexp = t.xexp;
  }
  const int a = (act == SLONN_ACT_RELU) ? SLONN_ACT_RELU : SLONN_ACT_NONE;
  return launch_tiles(nullptr, X, ldx, xexp, Wp, w_parts, wexp, bias, t.mask, t.flags, Y, ldy, B, n, d, a, s);
}

// A layer computed in full for a large batch through the same tiles (no mask, every query
// served): weights through launch_split_weights.  scratch: masked_tiles_workspace_bytes(B, n, d)
// bytes (the rows' exponents, and a two-part copy of activations that are not 16-byte aligned).
int launch_dense_tiles(const uint16_t* Wp, int w_parts, const int32_t* wexp, const float* bias, const float* X, int ldx,
                       float* Y, int ldy, int B, int d, int n, int act, void* scratch, hipStream_t s) {
  ProfScope prof_(SLONN_PROF_DENSE, s);
  const TilesScratch t = tiles_scratch(scratch, B, n, d);
  int rc = launch_row_exponents(X, ldx, B, d, t.xexp, s);
  if (rc) return rc;
  const uint16_t* X2 = nullptr;
  if (!rows_aligned(X, ldx)) {
    hipLaunchKernelGGL((split_rows_kernel<float, 2>), dim3((unsigned)B), dim3(256), 0, s, X, (int64_t)ldx, d, t.xexp, t.X2,
                       nullptr);
    SLONN_HIP(hipGetLastError());
    X2 = t.X2;
  }
  const int a = (act == SLONN_ACT_RELU) ? SLONN_ACT_RELU : SLONN_ACT_NONE;
  return launch_tiles(X2, X, ldx, t.xexp, Wp, w_parts, wexp, bias, nullptr, nullptr, Y, ldy, B, n, d, a, s);
}

// ---- measurement aid: what the fp16 matrix cores deliver when nothing else is in the way ----
namespace {
// Eight wavefronts per workgroup, sixteen accumulators each, operands in registers: 32 MFMAs per
// iteration in the order the tile kernel issues them (two onto each accumulator, back to back).
__global__ __launch_bounds__(512) void mfma_rate_probe_kernel(float* __restrict__ out, int iters) {
  f16x8 a[4], b[8];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) a[i][j] = (_Float16)(0.001f * (float)((threadIdx.x + i + j) & 63));
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) b[i][j] = (_Float16)(0.002f * (float)((threadIdx.x + 3 * i + j) & 63));
  f32x4 acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
      for (int y = 0; y < 4; ++y) {
        acc[4 * x + y] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[x], b[2 * y + 1], acc[4 * x + y], 0, 0, 0);
        acc[4 * x + y] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[x], b[2 * y], acc[4 * x + y], 0, 0, 0);
      }
  }
  float sum = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; ++i) sum += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  out[(size_t)blockIdx.x * 512 + threadIdx.x] = sum;
}
}  // namespace

// out: workgroups * 512 floats of device memory (results nobody needs; they keep the loop alive).
// Returns the flops the launch executes.
double launch_mfma_rate_probe(float* out, int workgroups, int iters, hipStream_t s) {
  hipLaunchKernelGGL(mfma_rate_probe_kernel, dim3(workgroups), dim3(512), 0, s, out, iters);
  return 32.0 * 16384.0 * (double)iters * workgroups * 8;
}

}  // namespace slonn
