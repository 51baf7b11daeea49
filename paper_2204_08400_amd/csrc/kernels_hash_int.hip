// FreeHash projections of a large batch (Def. 2, Section 3.4) on the int8 matrix cores, with the
// sign of every projection certified.
//
// A hash bit is the sign of z = w . x + b, so z has to be right wherever it is close to zero.
// The fp64 matrix cores give that (hash_project_mfma_kernel) at 78 TFLOP/s; the int8 cores run
// at 5 POP/s, and integer dot products are exact.  Every row (a hash row of the layer, a query's
// activations) is written as a fixed-point number per element relative to a power of two above
// the row's largest magnitude, |v| < 2^e:  V = trunc(v * 2^(28 - e)), a signed 29-bit integer,
// cut into four signed 7-bit digits V = sum_s V_s 128^s.  Then
//     sum_k W[k] X[k] = sum_{s,t} 128^(s+t) sum_k W_s[k] X_t[k],
// every inner sum an exact int32 (|.| <= d * 127^2, at most four of them per accumulator:
// d <= 33 000).  The digit pairs with s + t >= 3 are kept (10 of 16).  What is lost is bounded
// rigorously, per element of the dot product and in units of 2^(e_w + e_x):
//   truncation of the operands   |w x - w' x'| < 2^-27 (1 + 2^-29)
//   the six dropped pairs        127^2 (1 + 2 * 128 + 3 * 128^2) 2^-56 < 2^-26.43
// together 1.86e-8 < 2^-25, and an element of x that is zero contributes no error at all (its digits
// are zero), so the projection is off by less than BOUND = nnz(x) * 2^(e_w + e_x - 25), nnz(x) <= d
// the number of non-zero activations of the query (the output of a sparse ReLU layer has few:
// C5 16 %, which takes the projections to recompute from 6 to 1 in 10^4).
// A projection with |z| > margin * BOUND has a certain sign; the others (about one in 10^4 on
// normal data of width 8192) and rows with non-finite entries are recomputed in fp64 like the
// fp64 kernel does.  The value itself is typically off by a few 10^-8 of its own size (the
// truncation errors and the dropped low digits have either sign and add up like a random walk):
// the size of the rounding error of an fp32 evaluation of the same dot product, which is the
// accuracy of every other node's output (Section 3.4 lets a selected hash node take its output
// from its projection).  A fifth digit and the pairs down to s + t = 3 of five (19 MFMAs per
// block instead of 10) tightened BOUND by 2^8 and took twice the time.
//
//   slice_digits_kernel   a row at a time per workgroup: row maximum -> e, four int8 digits per element,
//                         interleaved per 16 elements (element k, digit s of row i at
//                         i * 4 d + (k / 16) * 64 + 16 s + k % 16).
//   hash_int_tiles_kernel 128 queries x 64 hash rows per workgroup and slice of the reduction
//                         dimension, eight wavefronts (4 x 2) of 2 x 2 blocks, four int32
//                         accumulators per block (one per s + t), v_mfma_i32_16x16x64_i8,
//                         chunks of 64 elements double-buffered in LDS; writes the partial
//                         sums as fp64 integers.
//   hash_int_finish_kernel adds the partial sums, scales, adds the bias, certifies; the
//                         projections that are not certain are recomputed in fp64 by their
//                         workgroup, one after the other.
#include <algorithm>
#include <climits>

#include "slonn_internal.h"

namespace slonn {
namespace {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int DIGITS = 4;          // 7-bit digits per element
constexpr int FRAC_BITS = 7 * DIGITS;   // fixed point: 28 bits below 2^e
constexpr int MIN_PAIR = 3;        // digit pairs with s + t below it are dropped
constexpr int CLASSES = 2 * (DIGITS - 1) - MIN_PAIR + 1;   // s + t = 3 .. 6
constexpr int BOUND_EXP = -25;     // BOUND = nnz(x) * 2^(e_w + e_x + BOUND_EXP), derived above
constexpr int HQ = 128;            // queries per tile (hash rows per tile: 64 or 48, see the launcher)
constexpr int HPIECES = 4 * DIGITS;  // 16-byte pieces per row and chunk of 64 elements
// LDS row: 18 pieces, the chunk's pieces in digit-major order (piece 4 * digit + group): a wavefront's
// fragment read -- lane (r, kg) takes piece r * HROW + 4 * digit + kg -- then costs 4 LDS cycles, the full
// 256 bytes per cycle.  In the order of global memory (4 * group + digit) no row length from 16 to 40
// gets below 8 cycles, and the kernel was bound by its LDS traffic.
constexpr int HROW = HPIECES + 2;
__host__ __device__ constexpr int hash_lds_col(int piece) { return (piece % DIGITS) * 4 + piece / DIGITS; }
constexpr int BAD_ROW = INT_MIN;   // exponent entry of a row with a non-finite element

// Barrier that orders LDS traffic only: global loads issued before it stay in flight across it.
__device__ __forceinline__ void lds_only_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// A workgroup of 256 threads takes rows blockIdx.x, blockIdx.x + gridDim.x, ...; a thread holds
// up to MAXS slots of four consecutive elements of the row in registers (slot tid + 256 i: a
// wavefront's load is 1 KiB of consecutive bytes), so the row is read once: maximum, exponent,
// digits.  While one row is worked on the loads of the workgroup's next row are in flight (two
// register sets), so that over the whole grid the reads of later rows overlap the writes of
// earlier ones (one row per workgroup read everything first and wrote everything last: C5 45 us
// per layer for 131 MB).  The four lanes of a quad hold the sixteen elements of one group: after a
// 4 x 4 exchange inside the quad lane q holds digit q of all sixteen, one 16-byte store per lane,
// consecutive over the wavefront.
template <int MAXS>
__global__ __launch_bounds__(256) void slice_digits_kernel(const float* __restrict__ X, int64_t ldx, int d,
                                                    int8_t* __restrict__ out, int32_t* __restrict__ expo,
                                                    int32_t* __restrict__ nonzeros, int64_t rows) {
  static_assert(DIGITS == 4, "the quad exchange is written for four digits");
  __shared__ float red[2][4];
  __shared__ int red_nz[2][4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, q = tid & 3;
  const bool vec = (ldx % 4 == 0) && (reinterpret_cast<uintptr_t>(X) % 16 == 0);
  const int nslots = d >> 2;                   // d is a multiple of 64: whole quads
  auto load = [&](int64_t row, float4 (&xv)[MAXS]) {
    const float* x = X + row * ldx;
#pragma unroll
    for (int i = 0; i < MAXS; ++i) {
      const int slot = tid + 256 * i;
      if (slot < nslots) {
        if (vec) xv[i] = reinterpret_cast<const float4*>(x)[slot];
        else xv[i] = make_float4(x[4 * slot], x[4 * slot + 1], x[4 * slot + 2], x[4 * slot + 3]);
      } else {
        xv[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      }
    }
  };
  auto process = [&](int64_t row, const float4 (&xv)[MAXS], int par) {
    float mx = 0.0f;
    bool bad = false;
    int nz = 0;
#pragma unroll
    for (int i = 0; i < MAXS; ++i) {
      const float v4[4] = {xv[i].x, xv[i].y, xv[i].z, xv[i].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float v = fabsf(v4[j]);
        if (!(v <= 3.0e38f)) bad = true;          // infinity or NaN
        mx = fmaxf(mx, v);
        nz += v != 0.0f ? 1 : 0;
      }
    }
    if (bad) mx = __int_as_float(0x7f800000);
    for (int o = 32; o > 0; o >>= 1) {
      mx = fmaxf(mx, __shfl_xor(mx, o));
      nz += __shfl_xor(nz, o);
    }
    if (lane == 0) { red[par][wave] = mx; red_nz[par][wave] = nz; }
    lds_only_barrier();
    // (every thread forms the exponent from the four partial maxima; red[par] is written again two
    // rows on, with the next row's barrier in between)
    const float m = fmaxf(fmaxf(red[par][0], red[par][1]), fmaxf(red[par][2], red[par][3]));
    int e = 0;
    if (!(m <= 3.0e38f)) e = BAD_ROW;
    else if (m > 0.0f) (void)frexpf(m, &e);     // m = f * 2^e with f in [0.5, 1): |x| < 2^e
    if (tid == 0) {
      if (nonzeros) nonzeros[row] = (red_nz[par][0] + red_nz[par][1]) + (red_nz[par][2] + red_nz[par][3]);
      expo[row] = e;
    }
    u32x4* o = reinterpret_cast<u32x4*>(out + (size_t)row * DIGITS * d);
    const int sh = e == BAD_ROW ? 0 : FRAC_BITS - e;
#pragma unroll
    for (int i = 0; i < MAXS; ++i) {
      const int slot = tid + 256 * i;
      if (slot >= nslots) break;
      const float v4[4] = {xv[i].x, xv[i].y, xv[i].z, xv[i].w};
      uint32_t dg[DIGITS] = {0u, 0u, 0u, 0u};    // dg[s]: digit s of this slot's four elements, one byte each
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        // exact: a power of two times an fp32 number, below 2^28; then truncation towards zero
        const int V = e == BAD_ROW ? 0 : (int)ldexpf(v4[j], sh);
        const uint32_t a = (uint32_t)(V < 0 ? -V : V);
#pragma unroll
        for (int t = 0; t < DIGITS; ++t) {
          const int dig = (int)((a >> (7 * t)) & 127u);
          dg[t] |= (uint32_t)(uint8_t)(int8_t)(V < 0 ? -dig : dig) << (8 * j);
        }
      }
      // 4 x 4 exchange inside the quad: lane q ends with dg[q] of lanes 0 .. 3 of its quad, in lane order
      {
        const uint32_t s0 = (q & 1) ? dg[0] : dg[1], s1 = (q & 1) ? dg[2] : dg[3];
        const uint32_t r0 = __shfl_xor(s0, 1), r1 = __shfl_xor(s1, 1);
        if (q & 1) { dg[0] = r0; dg[2] = r1; } else { dg[1] = r0; dg[3] = r1; }
        // now lane q holds, for its pair of lanes (p, p + 1): dg[0], dg[1] = digit (q & 1) of p, p + 1; dg[2], dg[3] = digit 2 + (q & 1)
        const uint32_t t0 = (q & 2) ? dg[0] : dg[2], t1 = (q & 2) ? dg[1] : dg[3];
        const uint32_t u0 = __shfl_xor(t0, 2), u1 = __shfl_xor(t1, 2);
        if (q & 2) { dg[0] = u0; dg[1] = u1; } else { dg[2] = u0; dg[3] = u1; }
      }
      o[slot] = (u32x4){dg[0], dg[1], dg[2], dg[3]};
    }
  };
  float4 ra[MAXS], rb[MAXS];
  int64_t row = blockIdx.x;
  if (row >= rows) return;
  load(row, ra);
  while (true) {
    int64_t next = row + gridDim.x;
    if (next < rows) load(next, rb);
    process(row, ra, 0);
    if (next >= rows) break;
    row = next;
    next = row + gridDim.x;
    if (next < rows) load(next, ra);
    process(row, rb, 1);
    if (next >= rows) break;
    row = next;
  }
}

__device__ __forceinline__ i32x4 as_i32x4(u32x4 v) { return __builtin_bit_cast(i32x4, v); }

// Xd, Wd: rows in interleaved digits (see above); d a multiple of 64.  part[z][q][h]
// receives sum over the workgroup's chunks of sum_c 128^(c - 3) P_c (an integer below 2^52:
// exact in fp64).
// Lane layout of v_mfma_i32_16x16x64_i8 (checked on gfx950): lane l feeds row l % 16 of its
// operand with the sixteen elements 16 (l / 16) .. + 15 of the step; register v of lane l holds
// D[4 (l / 16) + v][l % 16], rows from the first operand (here: hash rows), columns from the
// second (queries).
// HH hash rows per tile, wavefronts as WQ query strips x WH hash-row strips (WQ * WH = 8)
template <int HH, int WQ, int WH>
__global__ __launch_bounds__(512) void hash_int_tiles_kernel(const int8_t* __restrict__ Xd,
                                                            const int8_t* __restrict__ Wd,
                                                            double* __restrict__ part, int B, int H, int d,
                                                            int nslices, int xcd_sx) {
  extern __shared__ u32x4 hash_lds[];       // two buffers of [HQ rows of X | HH rows of W][HROW]
  constexpr int BUF = (HQ + HH) * HROW;
  constexpr int TOTAL = (HQ + HH) * HPIECES;         // pieces per chunk
  constexpr int PER = (TOTAL + 511) / 512;           // per thread (the last one partly repeated)
  int tile_h, tile_q;                       // the workgroups of one XCD take a compact block of tiles
  xcd_tile(blockIdx.x, blockIdx.y, gridDim.x, gridDim.y, xcd_sx, tile_h, tile_q);
  const int q0 = tile_q * HQ, h0 = tile_h * HH;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  constexpr int NBQ = HQ / (16 * WQ), NBH = HH / (16 * WH);   // 16 x 16 blocks per wavefront
  static_assert(WQ * WH == 8 && HQ % (16 * WQ) == 0 && HH % (16 * WH) == 0, "wavefront grid must cover the tile");
  const int wq = wave / WH, wh = wave % WH;
  const int r = lane & 15, kg = lane >> 4;

  const u32x4* src[PER];
  int dst[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int idx = min(tid + 512 * i, TOTAL - 1);   // surplus slots repeat the last piece
    const bool isx = idx < HQ * HPIECES;
    const int j = isx ? idx : idx - HQ * HPIECES;
    const int row = j / HPIECES, piece = j % HPIECES;
    const int8_t* base = isx ? Xd + (size_t)min(q0 + row, B - 1) * DIGITS * d
                             : Wd + (size_t)min(h0 + row, H - 1) * DIGITS * d;
    src[i] = reinterpret_cast<const u32x4*>(base) + piece;
    dst[i] = (isx ? row : HQ + row) * HROW + hash_lds_col(piece);
  }
  // this workgroup's chunks of 64 elements
  const int nchunks = d / 64;
  const int per_z = (nchunks + nslices - 1) / nslices;      // nslices = gridDim.z, as an argument
  const int c_begin = min(nchunks, (int)blockIdx.z * per_z), c_end = min(nchunks, c_begin + per_z);
  const int last = max(c_end - 1, c_begin);

  i32x4 acc[NBH][NBQ][CLASSES];             // [hash block][query block][s + t - 3]
#pragma unroll
  for (int a = 0; a < NBH; ++a)
#pragma unroll
    for (int b = 0; b < NBQ; ++b)
#pragma unroll
      for (int c = 0; c < CLASSES; ++c) acc[a][b][c] = (i32x4){0, 0, 0, 0};

  u32x4 r0[PER];
#define SLONN_HASH_LOAD(R, CHUNK)                                                          \
  {                                                                                        \
    const size_t c_ = (size_t)min((CHUNK), last);                                          \
    _Pragma("unroll") for (int i = 0; i < PER; ++i) R[i] = src[i][c_ * HPIECES];           \
  }
#define SLONN_HASH_STORE(BUFI, R)                                                          \
  {                                                                                        \
    u32x4* b_ = hash_lds + (BUFI) * BUF;                                                   \
    _Pragma("unroll") for (int i = 0; i < PER; ++i) b_[dst[i]] = R[i];                     \
  }
  auto multiply = [&](int buf) {
    const u32x4* Xs = hash_lds + buf * BUF;
    const u32x4* Ws = Xs + HQ * HROW;
    // An MFMA consumes the whole chunk of 64 elements: lane (r, kg) supplies the 16 elements of
    // group kg, i.e. piece kg * DIGITS + digit of its row (at 4 * digit + kg of the LDS row).  One MFMA per
    // digit pair and block.
    i32x4 xd[NBQ][DIGITS];
#pragma unroll
    for (int b = 0; b < NBQ; ++b)
#pragma unroll
      for (int t = 0; t < DIGITS; ++t)
        xd[b][t] = as_i32x4(Xs[(wq * 16 * NBQ + b * 16 + r) * HROW + 4 * t + kg]);
#pragma unroll
    for (int s = 0; s < DIGITS; ++s) {
      i32x4 wd[NBH];
#pragma unroll
      for (int a = 0; a < NBH; ++a) wd[a] = as_i32x4(Ws[(wh * 16 * NBH + a * 16 + r) * HROW + 4 * s + kg]);
#pragma unroll
      for (int t = 0; t < DIGITS; ++t) {
        if (s + t < MIN_PAIR) continue;
#pragma unroll
        for (int a = 0; a < NBH; ++a)
#pragma unroll
          for (int b = 0; b < NBQ; ++b)
            acc[a][b][s + t - MIN_PAIR] =
                __builtin_amdgcn_mfma_i32_16x16x64_i8(wd[a], xd[b][t], acc[a][b][s + t - MIN_PAIR], 0, 0, 0);
      }
    }
  };

  // chunk c is multiplied out of buffer (c - c_begin) % 2 while chunk c + 1 moves from registers into
  // the other buffer and chunks c + 2 and c + 3 are on their way from L2 or HBM (two register sets: a
  // load has two chunks' worth of MFMAs to arrive); one LDS-only barrier per chunk
  if (c_begin < c_end) {
    u32x4 r1[PER];
    SLONN_HASH_LOAD(r0, c_begin);
    SLONN_HASH_LOAD(r1, c_begin + 1);
    SLONN_HASH_STORE(0, r0);
    SLONN_HASH_LOAD(r0, c_begin + 2);
    lds_only_barrier();
    int c = c_begin;
    for (; c + 2 <= c_end; c += 2) {
      multiply(0);
      SLONN_HASH_STORE(1, r1);             // chunk c + 1
      SLONN_HASH_LOAD(r1, c + 3);
      lds_only_barrier();
      multiply(1);
      SLONN_HASH_STORE(0, r0);             // chunk c + 2
      SLONN_HASH_LOAD(r0, c + 4);
      lds_only_barrier();
    }
    if (c < c_end) multiply(0);            // an odd number of chunks
  }
#undef SLONN_HASH_LOAD
#undef SLONN_HASH_STORE

  // register v of block (a, b): hash row h0 + 16 NBH wh + 16 a + 4 kg + v, query q0 + 16 NBQ wq + 16 b + r
  double* mine = part + (size_t)blockIdx.z * B * H;
#pragma unroll
  for (int b = 0; b < NBQ; ++b) {
    const int q = q0 + wq * 16 * NBQ + b * 16 + r;
    if (q >= B) continue;
#pragma unroll
    for (int a = 0; a < NBH; ++a)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int h = h0 + wh * 16 * NBH + a * 16 + 4 * kg + v;
        if (h >= H) continue;
        double sum = 0.0;
#pragma unroll
        for (int c = CLASSES - 1; c >= 0; --c) sum = sum * 128.0 + (double)acc[a][b][c][v];
        mine[(size_t)q * H + h] = sum;       // = sum_c 128^c P_c, in units of 128^3
      }
  }
}

// One lane per (query, hash row).  z = 128^3 * sum of the partial sums * 2^(e_w + e_x - 56) + bias.
// The projections that are not certain are listed in LDS and recomputed in fp64 by the whole
// workgroup, one after the other: every thread takes up to four 16-byte pieces of both rows at
// once (rows of a multiple of 64 elements), so a row of 4096 elements is one round trip to L2.
__global__ __launch_bounds__(256) void hash_int_finish_kernel(const double* __restrict__ part, int S,
                                                             const int32_t* __restrict__ ex,
                                                             const int32_t* __restrict__ nzx,
                                                             const int32_t* __restrict__ ew,
                                                             const float* __restrict__ X, int ldx,
                                                             const float* __restrict__ Wh,
                                                             const float* __restrict__ bh, float* __restrict__ Z,
                                                             int B, int H, int d, double margin) {
  __shared__ int s_n;
  __shared__ int s_list[256];
  __shared__ double s_part[4];
  const size_t total = (size_t)B * H;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const size_t i0 = (size_t)blockIdx.x * 256;
  const size_t i = i0 + tid;
  if (tid == 0) s_n = 0;
  __syncthreads();
  if (i < total) {
    const int q = (int)(i / H), h = (int)(i % H);
    const int eq = ex[q], eh = ew[h];
    bool redo = true;
    if (eq != BAD_ROW && eh != BAD_ROW) {
      double sum = 0.0;
      for (int z = 0; z < S; ++z) sum += part[(size_t)z * total + i];
      const double dot = ldexp(sum, 7 * MIN_PAIR + eq + eh - 2 * FRAC_BITS);
      const double zz = dot + (double)bh[h];
      const double bound = ldexp((double)min(d, nzx[q]), eq + eh + BOUND_EXP);
      if (fabs(zz) > margin * bound) {
        Z[i] = (float)zz;
        redo = false;
      }
    }
    if (redo) s_list[atomicAdd(&s_n, 1)] = tid;
  }
  __syncthreads();
  const int n_redo = s_n;
  for (int t = 0; t < n_redo; ++t) {        // (the order of the list does not enter any result)
    const size_t ii = i0 + s_list[t];
    const int qq = (int)(ii / H), hh = (int)(ii % H);
    const float* x = X + (size_t)qq * ldx;
    const float* w = Wh + (size_t)hh * d;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    if (((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w)) & 15) == 0) {
      const float4* x4 = reinterpret_cast<const float4*>(x);
      const float4* w4 = reinterpret_cast<const float4*>(w);
      const int n4 = d >> 2;
      for (int k0 = 0; k0 < n4; k0 += 1024) {
        float4 wv[4], xv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int k = k0 + 256 * j + tid;
          const bool in = k < n4;
          wv[j] = in ? w4[k] : make_float4(0.f, 0.f, 0.f, 0.f);
          xv[j] = in ? x4[k] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[j] = fma((double)wv[j].x, (double)xv[j].x, acc[j]);
          acc[j] = fma((double)wv[j].y, (double)xv[j].y, acc[j]);
          acc[j] = fma((double)wv[j].z, (double)xv[j].z, acc[j]);
          acc[j] = fma((double)wv[j].w, (double)xv[j].w, acc[j]);
        }
      }
    } else {
      for (int k0 = 0; k0 < d; k0 += 2048) {
        float wv[8], xv[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int k = k0 + 256 * j + tid;
          const bool in = k < d;
          wv[j] = in ? w[k] : 0.f;
          xv[j] = in ? x[k] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j & 3] = fma((double)wv[j], (double)xv[j], acc[j & 3]);
      }
    }
    double sum = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if (lane == 0) s_part[wave] = sum;
    __syncthreads();
    if (tid == s_list[t]) Z[ii] = (float)(((s_part[0] + s_part[1]) + (s_part[2] + s_part[3])) + (double)bh[hh]);
    __syncthreads();
  }
}

}  // namespace

int hash_int_digits() { return DIGITS; }

bool hash_int_supported(int d, int max_lds) {      // (d <= 16384: the slicing kernel holds a row in registers)
  return d % 64 == 0 && d <= 16384 && (size_t)2 * (HQ + 96) * HROW * 16 <= (size_t)max_lds;
}

// Tile height (96, 64 or 48 hash rows) and slices of the reduction dimension: the pair that fills one
// round of workgroups best (one workgroup per compute unit: the two tile buffers take most of
// its LDS), slices of at least 8 chunks.
void hash_int_plan(int B, int H, int d, int* hh_out, int* s_out) {
  const int nchunks = d / 64;
  int best_hh = 64, best_s = 1;
  long best_fill = -1;
  for (int hh : {96, 64, 48}) {
    // (the tall tile only where it wastes next to no rows: C5's 768 hash rows are 8 tiles of 96 - tiles
    // 107 -> 92 us; on C3's 320 rows it would pad to 384 and slice the reduction eightfold - 46.6 -> 48.6 us)
    if (hh == 96 && (long)((H + 95) / 96) * 96 * 100 > (long)H * 105) continue;
    const int tiles = ((B + HQ - 1) / HQ) * ((H + hh - 1) / hh);
    int S = 1;
    while (tiles * S * 2 <= 256 && S * 2 <= 8 && nchunks / (S * 2) >= 8) S *= 2;
    // useful work per slot of the rounds the grid takes (rows beyond H are wasted work), times how
    // far the tile's LDS traffic lets the matrix cores run: per chunk a 128 x 96 tile reads 20
    // operand fragments per wavefront for 60 MFMAs (the cores are the limit), 128 x 64 reads 16 for
    // 40 (about even), 128 x 48 with eight query strips reads 16 for 30 (LDS-bound at 0.7)
    const long rounds = (tiles * S + 255) / 256;
    const long eff = hh == 96 ? 100 : (hh == 64 ? 92 : 70);
    const long fill = (long)H * 1000 / ((H + hh - 1) / hh * hh) * (tiles * S) / (rounds * 256) * eff;
    if (fill > best_fill) { best_fill = fill; best_hh = hh; best_s = S; }
  }
  *hh_out = best_hh;
  *s_out = best_s;
}

size_t hash_int_workspace_bytes(int B, int H, int d) {
  const size_t x5 = ((size_t)B * DIGITS * d + 255) / 256 * 256;
  const size_t ex = ((size_t)B * 4 + 255) / 256 * 256;
  return x5 + 2 * ex + (size_t)8 * B * H * sizeof(double) + 256;      // digits | exponents | non-zero counts | partial sums
}

const int32_t* hash_int_row_exponents(const void* scratch, int B, int d) {
  const size_t x5_bytes = ((size_t)B * DIGITS * d + 255) / 256 * 256;
  return reinterpret_cast<const int32_t*>(static_cast<const char*>(scratch) + x5_bytes);
}

int launch_slice_digits(const float* X, int64_t ldx, int64_t rows, int d, int8_t* out, int32_t* expo,
                        int32_t* nonzeros, hipStream_t s) {
  // two rows per workgroup once every compute unit has several workgroups either way
  const unsigned grid = (unsigned)(rows >= 1024 ? (rows + 1) / 2 : rows);
  if (d <= 4096)
    hipLaunchKernelGGL(slice_digits_kernel<4>, dim3(grid), dim3(256), 0, s, X, ldx, d, out, expo, nonzeros, rows);
  else if (d <= 8192)
    hipLaunchKernelGGL(slice_digits_kernel<8>, dim3(grid), dim3(256), 0, s, X, ldx, d, out, expo, nonzeros, rows);
  else
    hipLaunchKernelGGL(slice_digits_kernel<16>, dim3(grid), dim3(256), 0, s, X, ldx, d, out, expo, nonzeros, rows);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

int launch_hash_project_int(const float* X, int ldx, const float* Wh, const int8_t* Wd, const int32_t* ew,
                            const float* bh, float* Z, int B, int H, int d, double margin, void* scratch,
                            hipStream_t s) {
  ProfScope prof_(SLONN_PROF_HASH, s);
  const size_t x5_bytes = ((size_t)B * DIGITS * d + 255) / 256 * 256;
  const size_t ex_bytes = ((size_t)B * 4 + 255) / 256 * 256;
  int8_t* Xd = static_cast<int8_t*>(scratch);
  int32_t* ex = reinterpret_cast<int32_t*>(static_cast<char*>(scratch) + x5_bytes);
  int32_t* nzx = reinterpret_cast<int32_t*>(static_cast<char*>(scratch) + x5_bytes + ex_bytes);
  double* part = reinterpret_cast<double*>(static_cast<char*>(scratch) + x5_bytes + 2 * ex_bytes);
  int rc = launch_slice_digits(X, ldx, B, d, Xd, ex, nzx, s);
  if (rc) return rc;
  int hh = 64, S = 1;
  hash_int_plan(B, H, d, &hh, &S);
  // XCD-aware tile order: per XCD the fewest bytes of digits (a tile of hash rows against a tile of queries)
  const int nx = (H + hh - 1) / hh, ny = (B + HQ - 1) / HQ;
  const int sx = xcd_split(nx, ny, (double)hh * DIGITS * d / S, (double)HQ * DIGITS * d / S);
  if (hh == 96) {
    constexpr size_t lds = (size_t)2 * (HQ + 96) * HROW * 16;
    static_assert(lds <= 160 * 1024, "two tile buffers must fit the LDS of a compute unit");
    SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(hash_int_tiles_kernel<96, 4, 2>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL((hash_int_tiles_kernel<96, 4, 2>), dim3((H + 95) / 96, (B + HQ - 1) / HQ, S), dim3(512), lds, s,
                       Xd, Wd, part, B, H, d, S, sx);
  } else if (hh == 64) {
    constexpr size_t lds = (size_t)2 * (HQ + 64) * HROW * 16;
    static_assert(lds <= 160 * 1024, "two tile buffers must fit the LDS of a compute unit");
    SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(hash_int_tiles_kernel<64, 4, 2>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL((hash_int_tiles_kernel<64, 4, 2>), dim3((H + 63) / 64, (B + HQ - 1) / HQ, S), dim3(512), lds, s,
                       Xd, Wd, part, B, H, d, S, sx);
  } else {
    constexpr size_t lds = (size_t)2 * (HQ + 48) * HROW * 16;
    SLONN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(hash_int_tiles_kernel<48, 8, 1>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL((hash_int_tiles_kernel<48, 8, 1>), dim3((H + 47) / 48, (B + HQ - 1) / HQ, S), dim3(512), lds, s,
                       Xd, Wd, part, B, H, d, S, sx);
  }
  SLONN_HIP(hipGetLastError());
  hipLaunchKernelGGL(hash_int_finish_kernel, dim3((unsigned)(((size_t)B * H + 255) / 256)), dim3(256), 0, s, part, S,
                     ex, nzx, ew, X, ldx, Wh, bh, Z, B, H, d, margin);
  SLONN_HIP(hipGetLastError());
  return SLONN_OK;
}

}  // namespace slonn
