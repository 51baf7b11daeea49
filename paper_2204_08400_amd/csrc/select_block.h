// Node Activator query by a whole workgroup (Fig. 2 steps 3-4; Section 3.3): keys ->
// one bucket per table -> the first m distinct nodes in rank-major, table-minor order,
// continuing down the whole-set ranking when the lists run out.  Shared by the
// whole-network kernel and the stand-alone select kernel.
//
// Slots are numbered s = rank * L + table.  Every thread takes up to MU consecutive slots per
// round; an LDS integer min over slot numbers finds each node's first occurrence (the result
// does not depend on the order the threads arrive in), survivors are compacted in slot
// order: one count per thread, a prefix over the lanes from one ballot per bit of the count,
// a prefix over the wavefronts from their totals in LDS -- no atomic counters.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace slonn {

constexpr int SELECT_MU = 4;     // default number of slots per thread per round

// MU: most slots a thread takes per round (a round covers up to MU * NT slots)
template <int NT, int MU = SELECT_MU>
struct SelectShared {            // LDS regions the caller carves out
  uint32_t* prio;                // [n]  first-occurrence map, 0xFFFFFFFF = node not seen
  uint32_t* s_off;               // [64] list offsets of this query
  uint32_t* s_len;               // [64] list lengths
  int* wave_cnt;                 // [MU * NT/64], the first NT/64 in use
  uint32_t* s_misc;              // [4]
  uint32_t* bits = nullptr;      // [(n + 31) / 32] optional: one bit per chosen node (select_merge)
  static constexpr int words_besides_prio = 64 + 64 + MU * (NT / 64) + 4;
};

// Keys and bucket directory of one query, by ONE wavefront (one lane per table): fills s_off,
// s_len and s_misc[0] (the longest list).  z: the query's K*L hash projections (LDS or global).
template <int NT, int MU = SELECT_MU>
__device__ __forceinline__ void select_keys(const float* z, int K, int L_, const uint32_t* __restrict__ dir,
                                            const SelectShared<NT, MU>& sh, uint32_t* codes_row) {
  const int lane = threadIdx.x & 63;
  const int nb1 = (1 << K) + 1;
  uint32_t len = 0;
  if (lane < L_) {
    uint32_t key = 0;
    for (int j = 0; j < K; ++j) key |= (z[lane * K + j] > 0.0f ? 1u : 0u) << j;
    if (codes_row) codes_row[lane] = key;
    const uint32_t lo = dir[(size_t)lane * nb1 + key], hi = dir[(size_t)lane * nb1 + key + 1];
    sh.s_off[lane] = lo;
    len = hi - lo;
    sh.s_len[lane] = len;
  }
  for (int o = 32; o > 0; o >>= 1) {
    const uint32_t other = __shfl_xor(len, o);
    len = other > len ? other : len;
  }
  if (lane == 0) sh.s_misc[0] = len;
}

// Barrier that orders LDS traffic only: global loads issued before it stay in flight across it
// (__syncthreads would wait for them as well).
__device__ __forceinline__ void select_lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// The merge, by the whole workgroup, after select_keys and a barrier.  prio[0..n) must hold
// 0xFFFFFFFF and be visible to all threads.  On return (all threads, after a barrier)
// out[0..m) holds the chosen ids in selection order.  0 <= m < n.
// hskip (nullable, LDS or global, [n]): nodes with an entry >= 0 are passed over wherever
// they turn up (the variant of Section 3.4 in which hash nodes are computed anyway and the
// Node Activator never selects them); the caller keeps m <= n minus their number.
// sh.bits (nullable, LDS, zeroed by the caller): receives one bit per chosen node.
// IdT: the type the lists are stored in (uint16_t for layers of up to 65 536 nodes, else int32_t)
template <int NT, int MU = SELECT_MU, typename IdT = int32_t>
__device__ __forceinline__ void select_merge(int L_, int n, int m, const IdT* __restrict__ ids,
                                             const int32_t* __restrict__ global_rank,
                                             const SelectShared<NT, MU>& sh, int32_t* out,
                                             const int16_t* hskip = nullptr) {
  constexpr int NW = NT / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));

  // A round covers per*NT slots with all their id loads in flight together.  Lists of
  // similar buckets overlap heavily, so a round is sized to about twelve slots per wanted
  // node: most queries then finish in one round, i.e. one table-memory latency.
  // A thread takes `per` consecutive slots (consecutive tables of one rank), so that positions
  // in slot order follow from one count per thread, and the lanes of a wavefront that read
  // the same table read consecutive ranks of it.
  // (Asking for the ids of round r + 1 before round r is worked through was tried: a query that
  // ends with round r has asked in vain, and most do -- slower on every workload.)
  const uint32_t L = (uint32_t)L_;
  const uint32_t nslots = sh.s_misc[0] * L;            // <= n * 64 < 2^32
  int per = (12 * m + NT - 1) / NT;
  per = per < 1 ? 1 : (per > MU ? MU : per);
  int count = 0;
  // slot / L without a division per thread: the round's first slot is divided once, the offset
  // inside the round (below 16384) by multiplication with ceil(2^20 / L)
  static_assert(MU * NT + 64 <= 16384, "round too large for the multiplicative division");
  static_assert(MU <= 32, "a thread's slots of a round are kept in 32-bit masks");
  const uint32_t magic = ((1u << 20) + L - 1) / L;
  // this thread's slots of the round that starts at slot `base`: ids requested, mask of the slots that exist
  auto request = [&](uint32_t base, int (&node)[MU]) -> uint32_t {
    uint32_t have = 0;
    if (base >= nslots) return have;
    const uint32_t r_base = base / L, rem_base = base - r_base * L;
    const uint32_t slot0 = base + tid * per;
    const uint32_t off = rem_base + tid * per;
    const uint32_t dr = (uint32_t)(((unsigned long long)off * magic) >> 20);
    uint32_t r = r_base + dr, b = off - dr * L;
#pragma unroll
    for (int u = 0; u < MU; ++u) {
      const bool v = u < per && slot0 + u < nslots && r < sh.s_len[b];
      node[u] = v ? (int)ids[sh.s_off[b] + r] : -1;
      have |= (v ? 1u : 0u) << u;
      if (++b == L) { b = 0; ++r; }
    }
    return have;
  };
  int node[MU];
  for (uint32_t base = 0; base < nslots && count < m; base += NT * per) {
    const uint32_t slot0 = base + tid * per;
    uint32_t valid = request(base, node);
    if (hskip) {
#pragma unroll
      for (int u = 0; u < MU; ++u)
        if (((valid >> u) & 1u) && hskip[node[u]] >= 0) valid &= ~(1u << u);
    }
#pragma unroll
    for (int u = 0; u < MU; ++u)
      if ((valid >> u) & 1u) atomicMin(&sh.prio[node[u]], slot0 + u);
    select_lds_barrier();
    uint32_t firsts = 0;
#pragma unroll
    for (int u = 0; u < MU; ++u)
      if (((valid >> u) & 1u) && sh.prio[node[u]] == slot0 + u) firsts |= 1u << u;
    // first occurrences in the lanes below this one and in the wavefront, from one ballot per
    // bit of the thread's count
    const int mine = __popc(firsts);
    int before = 0, in_wave = 0;
#pragma unroll
    for (int bit = 0; (1 << bit) <= MU; ++bit) {
      const unsigned long long has = __ballot((mine >> bit) & 1);
      before += __popcll(has & below) << bit;
      in_wave += __popcll(has) << bit;
    }
    if (lane == 0) sh.wave_cnt[wave] = in_wave;
    select_lds_barrier();
    // (the next write of wave_cnt comes after the next round's first barrier: no barrier here)
    int total = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const int c = sh.wave_cnt[w];
      before += (w < wave) ? c : 0;
      total += c;
    }
    int pos = count + before;
#pragma unroll
    for (int u = 0; u < MU; ++u) {
      if ((firsts >> u) & 1u) {
        if (pos < m) {
          out[pos] = node[u];
          if (sh.bits) atomicOr(&sh.bits[node[u] >> 5], 1u << (node[u] & 31));
        }
        ++pos;
      }
    }
    count += total;
  }
  __syncthreads();        // the last round's counts have been read; the list so far is visible
  // the lists ran out: continue down the whole-set ranking (a permutation: no duplicates)
  for (int base = 0; base < n && count < m; base += NT) {
    const int i = base + tid;
    int cand = -1;
    bool first = false;
    if (i < n) {
      cand = global_rank[i];
      first = sh.prio[cand] == 0xFFFFFFFFu && !(hskip && hskip[cand] >= 0);
    }
    const unsigned long long votes = __ballot(first);
    if (lane == 0) sh.wave_cnt[wave] = __popcll(votes);
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const int c = sh.wave_cnt[w];
      before += (w < wave) ? c : 0;
      total += c;
    }
    if (first) {
      const int pos = count + before + __popcll(votes & below);
      if (pos < m) {
        out[pos] = cand;
        if (sh.bits) atomicOr(&sh.bits[cand >> 5], 1u << (cand & 31));
      }
    }
    count += total;
    __syncthreads();
  }
}

// Keys by the first wavefront, then the merge: for callers whose projections are only ready
// now.  prio[0..n) must hold 0xFFFFFFFF and be visible to all threads (caller clears it and
// synchronises).
template <int NT, int MU = SELECT_MU, typename IdT = int32_t>
__device__ __forceinline__ void select_block(const float* z, int K, int L_, int n, int m,
                                             const uint32_t* __restrict__ dir,
                                             const IdT* __restrict__ ids,
                                             const int32_t* __restrict__ global_rank,
                                             const SelectShared<NT, MU>& sh, uint32_t* codes_row,
                                             int32_t* out, const int16_t* hskip = nullptr) {
  if (threadIdx.x < 64) select_keys<NT, MU>(z, K, L_, dir, sh, codes_row);
  __syncthreads();
  select_merge<NT, MU, IdT>(L_, n, m, ids, global_rank, sh, out, hskip);
}

// Same query for layers too wide for a 4-byte map entry per node (hundreds of thousands of
// output nodes): one BIT per node records the nodes taken in earlier rounds, and the nodes of
// the current round meet in a small open-addressing table in LDS (node id -> smallest slot
// number of the round), which is emptied again after each round.
// Round table: a power of two of entries, at least twice the MU * NT slots of a round.
template <int NT, int MU = SELECT_MU>
struct SelectWideTable {
  static constexpr int bits = (MU * NT * 2 <= 4096) ? 12 : 13;
  static constexpr int entries = 1 << bits;
  static_assert(MU * NT * 2 <= entries, "round table too small");
};

template <int NT, int MU = SELECT_MU>
struct SelectSharedWide {
  uint32_t* taken;               // [(n + 31) / 32] bitmap
  int32_t* tkey;                 // [SelectWideTable<NT, MU>::entries] node id or -1
  uint32_t* tval;                // [SelectWideTable<NT, MU>::entries] smallest slot of the round
  uint32_t* s_off;               // [64]
  uint32_t* s_len;               // [64]
  int* wave_cnt;                 // [MU * NT/64], the first NT/64 in use
  uint32_t* s_misc;              // [4]
  static constexpr int words_besides_bitmap =
      2 * SelectWideTable<NT, MU>::entries + 64 + 64 + MU * (NT / 64) + 4;
};

// taken[] must be zero and tkey[] = -1, tval[] = 0xFFFFFFFF on entry (caller + barrier).
// Slots, rounds and compaction as in select_merge (a thread takes consecutive slots; positions
// from one count per thread); a third barrier per round lets the round table be emptied.
template <int NT, int MU = SELECT_MU, typename IdT = int32_t>
__device__ __forceinline__ void select_block_wide(const float* z, int K, int L_, int n, int m,
                                                  const uint32_t* __restrict__ dir,
                                                  const IdT* __restrict__ ids,
                                                  const int32_t* __restrict__ global_rank,
                                                  const SelectSharedWide<NT, MU>& sh, uint32_t* codes_row,
                                                  int32_t* out, const int16_t* hskip = nullptr) {
  constexpr int TABLE = SelectWideTable<NT, MU>::entries;
  constexpr int TBITS = SelectWideTable<NT, MU>::bits;
  constexpr int NW = NT / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));

  if (wave == 0) {
    const int nb1 = (1 << K) + 1;
    uint32_t len = 0;
    if (lane < L_) {
      uint32_t key = 0;
      for (int j = 0; j < K; ++j) key |= (z[lane * K + j] > 0.0f ? 1u : 0u) << j;
      if (codes_row) codes_row[lane] = key;
      const uint32_t lo = dir[(size_t)lane * nb1 + key], hi = dir[(size_t)lane * nb1 + key + 1];
      sh.s_off[lane] = lo;
      len = hi - lo;
      sh.s_len[lane] = len;
    }
    for (int o = 32; o > 0; o >>= 1) {
      const uint32_t other = __shfl_xor(len, o);
      len = other > len ? other : len;
    }
    if (lane == 0) sh.s_misc[0] = len;
  }
  __syncthreads();

  const uint32_t L = (uint32_t)L_;
  const unsigned long long nslots = (unsigned long long)sh.s_misc[0] * L;
  int per = (12 * m + NT - 1) / NT;
  per = per < 1 ? 1 : (per > MU ? MU : per);
  int count = 0;
  static_assert(MU * NT + 64 <= 16384, "round too large for the multiplicative division");
  static_assert(MU <= 32, "a thread's first occurrences are kept in a 32-bit mask");
  const uint32_t magic = ((1u << 20) + L - 1) / L;      // see select_merge
  for (unsigned long long base = 0; base < nslots && count < m; base += (unsigned long long)NT * per) {
    const uint32_t r_base = (uint32_t)(base / L), rem_base = (uint32_t)(base - (unsigned long long)r_base * L);
    const uint32_t rel0 = tid * per;                     // slot numbers relative to the round
    const uint32_t off = rem_base + rel0;
    const uint32_t dr = (uint32_t)(((unsigned long long)off * magic) >> 20);
    uint32_t r = r_base + dr, b = off - dr * L;
    int node[MU], cell[MU];
    bool valid[MU];
#pragma unroll
    for (int u = 0; u < MU; ++u) {
      valid[u] = u < per && base + rel0 + u < nslots && r < sh.s_len[b];
      node[u] = valid[u] ? (int)ids[sh.s_off[b] + r] : -1;
      cell[u] = 0;
      if (++b == L) { b = 0; ++r; }
    }
    if (hskip) {
#pragma unroll
      for (int u = 0; u < MU; ++u)
        if (valid[u] && hskip[node[u]] >= 0) valid[u] = false;
    }
#pragma unroll
    for (int u = 0; u < MU; ++u) {
      if (valid[u] && ((sh.taken[node[u] >> 5] >> (node[u] & 31)) & 1u)) valid[u] = false;   // earlier round
      if (valid[u]) {
        uint32_t h = ((uint32_t)node[u] * 2654435761u) >> (32 - TBITS);
        while (true) {
          const int k = atomicCAS(&sh.tkey[h], -1, node[u]);
          if (k == -1 || k == node[u]) break;
          h = (h + 1) & (TABLE - 1);
        }
        atomicMin(&sh.tval[h], rel0 + u);
        cell[u] = (int)h;
      }
    }
    __syncthreads();
    uint32_t firsts = 0;
#pragma unroll
    for (int u = 0; u < MU; ++u)
      if (valid[u] && sh.tval[cell[u]] == rel0 + u) firsts |= 1u << u;
    const int mine = __popc(firsts);
    int before = 0, in_wave = 0;
#pragma unroll
    for (int bit = 0; (1 << bit) <= MU; ++bit) {
      const unsigned long long has = __ballot((mine >> bit) & 1);
      before += __popcll(has & below) << bit;
      in_wave += __popcll(has) << bit;
    }
    if (lane == 0) sh.wave_cnt[wave] = in_wave;
    __syncthreads();
    int total = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const int c = sh.wave_cnt[w];
      before += (w < wave) ? c : 0;
      total += c;
    }
    int pos = count + before;
#pragma unroll
    for (int u = 0; u < MU; ++u) {
      if ((firsts >> u) & 1u) {
        if (pos < m) out[pos] = node[u];
        ++pos;
        atomicOr(&sh.taken[node[u] >> 5], 1u << (node[u] & 31));
      }
    }
    count += total;
#pragma unroll
    for (int u = 0; u < MU; ++u)
      if (valid[u]) { sh.tkey[cell[u]] = -1; sh.tval[cell[u]] = 0xFFFFFFFFu; }
    __syncthreads();
  }
  for (int base = 0; base < n && count < m; base += NT) {
    const int i = base + tid;
    int node = -1;
    bool first = false;
    if (i < n) {
      node = global_rank[i];
      first = ((sh.taken[node >> 5] >> (node & 31)) & 1u) == 0 && !(hskip && hskip[node] >= 0);
    }
    const unsigned long long votes = __ballot(first);
    if (lane == 0) sh.wave_cnt[wave] = __popcll(votes);
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const int c = sh.wave_cnt[w];
      before += (w < wave) ? c : 0;
      total += c;
    }
    if (first) {
      const int pos = count + before + __popcll(votes & below);
      if (pos < m) out[pos] = node;
    }
    count += total;
    __syncthreads();
  }
}

}  // namespace slonn
