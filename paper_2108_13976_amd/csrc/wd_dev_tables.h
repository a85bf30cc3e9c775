// wd_dev_tables.h — keys, the bucket-sorted list of live agents, a team's LDS tables, the counting sort and the exact K-nearest search.
// Device-side helpers of libwd (gfx950); included by wd_kernels.hip only.
#ifndef WD_DEV_TABLES_H
#define WD_DEV_TABLES_H

#include "wd_dev_common.h"

namespace wd {
namespace dev {

// ----------------------------------------------------------------------------------
// Keys and the bucket-sorted list.  A key is (squared distance << idx_bits) | agent index,
// so unsigned comparison orders by distance first and index second.  The sorted list holds
// position and index of the live agents, grouped by bucket.
//   NARROW (32-bit keys): positions x | y << 16 in one array, 16-bit indices in another; the
//     squared distance of a candidate is one packed 16-bit subtract and one two-element dot
//     product.  A runner tagged in this step is marked by adding `dead_dx` to its y: that
//     puts its squared distance from any agent on the grid into the band whose key has bit
//     31 set, above every live key, so it sorts last and reads as "no neighbour" (its x stays
//     what it was: the strip-sorted list is ordered by it).
//   WIDE = 1 (64-bit keys): entries (x | y << 16 | dead bit, index).
//   WIDE = 2 (32-bit keys that need all 32 bits, so that no band is left for the dead mark):
//     arrays as in the narrow form; a tagged runner is marked in bit 15 of its index, which
//     costs two instructions per candidate.
// ----------------------------------------------------------------------------------
constexpr int kKeys31 = 0, kKeys64 = 1, kKeys32 = 2;
typedef short short2v __attribute__((ext_vector_type(2)));

struct Ent {
  uint32_t pos;  // x | y << 16 (plus the dead mark of the representation)
  uint32_t id;   // agent index
};

template <int WIDE>
struct SortedList;

template <>
struct SortedList<kKeys31> {
  using Key = uint32_t;
  uint32_t* pos;
  uint16_t* id;
  int dead_dx;
  __device__ __forceinline__ Ent get(uint32_t q) const { return Ent{pos[q], uint32_t(id[q])}; }
  __device__ __forceinline__ void put(uint32_t q, int x, int y, int i) const {
    pos[q] = uint32_t(x) | (uint32_t(y) << 16);
    id[q] = uint16_t(i);
  }
  __device__ __forceinline__ void mark_dead(uint32_t q) const { pos[q] += uint32_t(dead_dx) << 16; }
  __device__ __forceinline__ bool dead(const Ent& e) const { return int(e.pos >> 16) >= dead_dx; }
  static __device__ __forceinline__ int x(const Ent& e) { return int(e.pos & 0xFFFFu); }
  static __device__ __forceinline__ int y(const Ent& e) { return int(e.pos >> 16); }
};

template <>
struct SortedList<kKeys64> {
  using Key = unsigned long long;
  uint2* ent;
  __device__ __forceinline__ Ent get(uint32_t q) const {
    const uint2 v = ent[q];
    return Ent{v.x, v.y};
  }
  __device__ __forceinline__ void put(uint32_t q, int x, int y, int i) const {
    ent[q] = make_uint2(uint32_t(x) | (uint32_t(y) << 16), uint32_t(i));
  }
  __device__ __forceinline__ void mark_dead(uint32_t q) const { ent[q].x |= kDeadBit; }
  __device__ __forceinline__ bool dead(const Ent& e) const { return (e.pos & kDeadBit) != 0; }
  static __device__ __forceinline__ int x(const Ent& e) { return int(e.pos & 0x7FFFu); }
  static __device__ __forceinline__ int y(const Ent& e) { return int((e.pos >> 16) & 0x7FFFu); }
};

constexpr uint32_t kDeadIdFlag = 0x8000u;

template <>
struct SortedList<kKeys32> {
  using Key = uint32_t;
  uint32_t* pos;
  uint16_t* id;
  __device__ __forceinline__ Ent get(uint32_t q) const { return Ent{pos[q], uint32_t(id[q])}; }
  __device__ __forceinline__ void put(uint32_t q, int x, int y, int i) const {
    pos[q] = uint32_t(x) | (uint32_t(y) << 16);
    id[q] = uint16_t(i);
  }
  __device__ __forceinline__ void mark_dead(uint32_t q) const { id[q] = uint16_t(id[q] | kDeadIdFlag); }
  __device__ __forceinline__ bool dead(const Ent& e) const { return (e.id & kDeadIdFlag) != 0; }
  static __device__ __forceinline__ int x(const Ent& e) { return int(e.pos & 0xFFFFu); }
  static __device__ __forceinline__ int y(const Ent& e) { return int(e.pos >> 16); }
};

template <typename Key>
__device__ __forceinline__ Key key_none() {
  return ~Key(0);
}
// An empty list slot holds the initial value; in the narrow form also a dead candidate's key.
template <int WIDE, typename Key>
__device__ __forceinline__ bool key_is_none(Key k) {
  if constexpr (WIDE == kKeys31) return (k & kDeadBit) != 0;
  return k == ~Key(0);
}

// Positions by agent index: x | y << 16 | dead bit.
__device__ __forceinline__ uint32_t pack_pos(int x, int y, bool is_live) {
  return uint32_t(x) | (uint32_t(y) << 16) | (is_live ? 0u : kDeadBit);
}
__device__ __forceinline__ int pos_x_of(uint32_t pl) { return int(pl & 0x7FFFu); }
__device__ __forceinline__ int pos_y_of(uint32_t pl) { return int((pl >> 16) & 0x7FFFu); }

// ----------------------------------------------------------------------------------
// Team helpers
// ----------------------------------------------------------------------------------

// Exclusive prefix sum of one value per thread across a team of (1 << ts_log2) threads.
// Teams of up to one wave use lane shuffles; larger teams add per-wave totals through LDS
// (wave_totals: one int per wave of the team).  Contains a workgroup barrier when the team
// spans several waves, so every thread of the workgroup must call it.
__device__ __forceinline__ int team_exclusive_scan(int v, int lt, int ts_log2, int* wave_totals, int* total) {
  const int lane = lt & (kWaveSize - 1);  // teams of a wave or more start on wave boundaries
  const int width = ts_log2 >= 6 ? kWaveSize : (1 << ts_log2);
  const int sub = lane & (width - 1);
  int incl = v;
  for (int d = 1; d < width; d <<= 1) {
    const int up = __shfl_up(incl, d, width);
    if (sub >= d) incl += up;
  }
  if (ts_log2 <= 6) {
    *total = __shfl(incl, width - 1, width);
    return incl - v;
  }
  const int waves = 1 << (ts_log2 - 6);
  const int my_wave = lt >> 6;
  if (lane == kWaveSize - 1) wave_totals[my_wave] = incl;
  __syncthreads();
  int before = 0, all = 0;
  for (int w = 0; w < waves; ++w) {
    const int wt = wave_totals[w];
    all += wt;
    if (w < my_wave) before += wt;
  }
  *total = all;
  return before + incl - v;
}

struct Buckets {
  uint32_t mul;  // bucket coordinate of cell x is (x * mul) >> 16: buckets are 65536 / mul cells wide
  int nbx;       // buckets per grid side
  int bmin;      // width in cells of the narrowest bucket = floor(65536 / mul)
};

// Bucket width for n_live agents on the grid: about sqrt(lambda / density) cells, so that a
// bucket holds about lambda live agents, limited by the size of the bucket table.  lambda
// falls with the number of agents (lambda_c / sqrt(n), clamped): a crowded env is bound by the
// candidates each search visits, a sparse one by the per-ring overhead.  Any choice gives
// the same results; it only trades search rings against candidates per ring.
__device__ __forceinline__ Buckets choose_buckets(const Params& p, int n_live) {
  const float n = static_cast<float>(max(n_live, 1));
  const float lambda = fminf(fmaxf(p.lambda_c * rsqrtf(n), p.lambda_min), p.lambda_max);
  const float want = p.bucket_scale * sqrtf(n / lambda);
  uint32_t mul = static_cast<uint32_t>(fminf(want, 65536.0f) + 0.5f);
  mul = min(max(mul, 2u), p.bucket_mul_max);
  Buckets b;
  b.mul = mul;
  b.nbx = int((uint32_t(p.G - 1) * mul) >> 16) + 1;
  uint32_t w = static_cast<uint32_t>(65536.0f / static_cast<float>(mul));
  if (w * mul > 65536u) --w;
  if ((w + 1) * mul <= 65536u) ++w;
  b.bmin = int(w);
  return b;
}

__device__ __forceinline__ int bucket_coord(int x, const Buckets bk) { return int(__umul24(uint32_t(x), bk.mul) >> 16); }

// First cell of bucket coordinate b: the smallest x with (x * mul) >> 16 == b.
__device__ __forceinline__ int bucket_first_cell(int b, const Buckets bk) {
  return int((uint32_t(b) * 65536u + bk.mul - 1u) / bk.mul);
}

__device__ __forceinline__ int bucket_of(int x, int y, const Buckets bk) {
  return bucket_coord(y, bk) * bk.nbx + bucket_coord(x, bk);
}

// Views of one team's tables: in LDS, except that a large env (BIG) keeps slots, tag keys and
// credits in device memory unless they fit LDS too (and has no neighbour lists: its rows come
// from big_obs_kernel).
template <int WIDE, bool BIG>
struct TeamLds {
  using Key = typename SortedList<WIDE>::Key;
  uint32_t* pl;      // [NPAD] packed position + dead bit, by agent index
  uint16_t* nbr;     // [NPAD][K] neighbour indices; overlays the tail of slot/best/credits/counts
  uint32_t* nbr_lo;  // compact form for K = 4, N < 1024: ids 0..2 and two bits of id 3 per agent,
  uint8_t* nbr_hi;   // and the other eight bits of id 3 (same memory as nbr)
  int32_t* misc;     // [0] tags this step, [1] t after the call, [2] rows to be written, [3] length of retry[], [4..19] scan scratch (strip variant, during the search: slots waiting for the block search), [20..21] of the first team: workgroup votes, [22..23] bucket geometry for big_obs_kernel, [24] length of that waiting list
  uint16_t* edges;   // [nbx + 1] first cell of each bucket coordinate; edges[nbx] = G
  SortedList<WIDE> sorted;  // [NPAD + pad] the live agents, grouped by bucket
  uint16_t* slot;    // [NPAD] where agent i sits in `sorted`
  uint16_t* retry;   // [NPAD] slots whose neighbour search needs wider rings (reuses slot[] when that is in LDS)
  Key* best;         // [NPAD] per runner: smallest (distance, tagger) key in range
  int32_t* credits;  // [N_tag]
  uint32_t* counts;  // [nb_cap] bucket counts, then scatter cursors
  uint16_t* starts;  // [nb_cap + 1] bucket start offsets in `sorted`
  __device__ __forceinline__ TeamLds(unsigned char* smem, int team, const Params& p, int env) {
    unsigned char* keep = smem + team * p.keep_stride;
    unsigned char* xr = smem + p.x_base + team * p.x_stride;
    unsigned char* yr = smem + p.y_base + team * p.y_stride;
    pl = reinterpret_cast<uint32_t*>(keep + p.off_pl);
    misc = reinterpret_cast<int32_t*>(keep + p.off_misc);
    edges = reinterpret_cast<uint16_t*>(keep + p.off_edges);
    if constexpr (WIDE == kKeys64) {
      sorted.ent = reinterpret_cast<uint2*>(xr + p.off_sorted);
    } else {
      sorted.pos = reinterpret_cast<uint32_t*>(xr + p.off_sorted);
      sorted.id = reinterpret_cast<uint16_t*>(xr + p.off_sorted_id);
      if constexpr (WIDE == kKeys31) sorted.dead_dx = p.dead_dx;
    }
    starts = reinterpret_cast<uint16_t*>(xr + p.off_starts);
    counts = reinterpret_cast<uint32_t*>(yr + p.off_counts);
    retry = reinterpret_cast<uint16_t*>(yr + p.off_retry);
    if constexpr (BIG) {
      nbr = nullptr;  // no neighbour lists: big_obs_kernel writes rows straight from the search
      nbr_lo = nullptr;
      nbr_hi = nullptr;
      if (p.big_lds_tables) {  // (the pointers are generic then: either address space)
        slot = reinterpret_cast<uint16_t*>(yr + p.off_slot);
        best = reinterpret_cast<Key*>(yr + p.off_best);
        credits = reinterpret_cast<int32_t*>(yr + p.off_credits);
      } else {
        slot = p.g_slot + env * p.g_stride_agents;
        best = reinterpret_cast<Key*>(p.g_best) + env * p.g_stride_agents;
        credits = p.g_credits + env * p.g_stride_credits;
      }
    } else {
      nbr = reinterpret_cast<uint16_t*>(yr + p.off_nbr);
      nbr_lo = reinterpret_cast<uint32_t*>(yr + p.off_nbr);
      nbr_hi = reinterpret_cast<uint8_t*>(yr + p.off_nbr) + 4 * p.NPAD;
      slot = reinterpret_cast<uint16_t*>(yr + p.off_slot);
      best = reinterpret_cast<Key*>(yr + p.off_best);
      credits = reinterpret_cast<int32_t*>(yr + p.off_credits);
    }
  }
};

// Second half of the counting sort: bucket counts -> start offsets -> entries in bucket
// order.  `act` marks teams that take part; every thread of the workgroup must call
// (barriers inside).  Requires pl[] written and counts[] filled, and a barrier after that.
template <int WIDE, typename Tables>
__device__ __forceinline__ void scan_and_scatter(const Params& p, const Tables& L, bool act, int lt, int ts,
                                                 const Buckets bk) {
  int part = 0;
  const int j0 = lt * p.scan_chunk;
  if (act)
    for (int c = 0; c < p.scan_chunk; ++c) part += int(L.counts[j0 + c]);
  int total = 0;
  int run = team_exclusive_scan(part, lt, p.ts_log2, L.misc + 4, &total);
  if (act) {
    for (int c = 0; c < p.scan_chunk; ++c) {
      const int v = int(L.counts[j0 + c]);
      L.starts[j0 + c] = uint16_t(run);
      L.counts[j0 + c] = uint32_t(run);
      run += v;
    }
    if (lt == ts - 1) L.starts[p.nb_cap] = uint16_t(total);
  }
  __syncthreads();
  if (act) {
    for (int k = 0; k < p.gpt; ++k) {
      const int i0 = 4 * (lt + k * ts);
      if (i0 < p.N) {
        const uint4 v4 = *reinterpret_cast<const uint4*>(L.pl + i0);
        const uint32_t v[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (!(v[j] & kDeadBit)) {
            const int x = pos_x_of(v[j]), y = pos_y_of(v[j]);
            const uint32_t at = atomicAdd(&L.counts[bucket_of(x, y, bk)], 1u);
            L.sorted.put(at, x, y, i0 + j);
            L.slot[i0 + j] = uint16_t(at);
          }
        }
      }
    }
  }
  __syncthreads();
}

__device__ __forceinline__ uint32_t med3(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t r;
  asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Sorted insertion of `key` into an ascending list of KT keys (the largest falls off).
template <int KT>
__device__ __forceinline__ void insert_key(uint32_t (&keys)[KT], uint32_t key) {
#pragma unroll
  for (int k = KT - 1; k >= 1; --k) keys[k] = med3(keys[k - 1], keys[k], key);  // clamp key into [k-1, k]
  keys[0] = keys[0] < key ? keys[0] : key;
}

template <int KT>
__device__ __forceinline__ void insert_key(unsigned long long (&keys)[KT], unsigned long long key) {
#pragma unroll
  for (int k = KT - 1; k >= 1; --k) {
    const unsigned long long hi = keys[k - 1] > key ? keys[k - 1] : key;
    keys[k] = keys[k] < hi ? keys[k] : hi;
  }
  keys[0] = keys[0] < key ? keys[0] : key;
}

// dx*dx + dy*dy of a packed pair of 16-bit differences, in one instruction (the form without
// an accumulator register, which the compiler otherwise zeroes for every candidate)
__device__ __forceinline__ uint32_t squared_length(short2v d) {
  uint32_t r;
  asm("v_dot2_i32_i16 %0, %1, %1, 0" : "=v"(r) : "v"(d));
  return r;
}

// The agents in slots [qb, qe) of the bucket-sorted list as candidates for the key list of the agent
// at (x, y); one overload per key form.  ABOVE: only keys greater than `floor` count (the search
// for neighbours beyond those already found).
template <int KT, bool ABOVE = false>
__device__ __forceinline__ void scan_range(unsigned long long (&keys)[KT], uint32_t qb, uint32_t qe, int x, int y,
                                           int ib, const SortedList<kKeys64>& sorted, unsigned long long floor = 0) {
  for (uint32_t q = qb; q < qe; ++q) {
    const Ent ent = sorted.get(q);
    const int dx = SortedList<kKeys64>::x(ent) - x, dy = SortedList<kKeys64>::y(ent) - y;
    const uint32_t d2 = uint32_t(__mul24(dx, dx)) + uint32_t(__mul24(dy, dy));
    unsigned long long key = ((unsigned long long)(d2) << ib) | (unsigned long long)(ent.id);
    if (sorted.dead(ent)) key = key_none<unsigned long long>();
    if (ABOVE && key <= floor) key = key_none<unsigned long long>();
    insert_key<KT>(keys, key);
  }
}

template <int KT, bool ABOVE = false>
__device__ __forceinline__ void scan_range(uint32_t (&keys)[KT], uint32_t qb, uint32_t qe, int x, int y, int ib,
                                           const SortedList<kKeys31>& sorted, uint32_t floor = 0) {
  const short2v me = __builtin_bit_cast(short2v, uint32_t(x) | (uint32_t(y) << 16));
  // one running pointer per array, the loop ends on the first: three instructions of loop
  // overhead per candidate
  const uint32_t* pos = sorted.pos + qb;
  const uint32_t* const pos_end = sorted.pos + qe;
  const uint16_t* id = sorted.id + qb;
  for (; pos < pos_end; ++pos, ++id) {
    const short2v d = __builtin_bit_cast(short2v, *pos) - me;  // (dx, dy), one packed subtract
    uint32_t key = (squared_length(d) << ib) | uint32_t(*id);
    if (ABOVE && key <= floor) key = ~0u;
    insert_key<KT>(keys, key);
  }
}

template <int KT, bool ABOVE = false>
__device__ __forceinline__ void scan_range(uint32_t (&keys)[KT], uint32_t qb, uint32_t qe, int x, int y, int ib,
                                           const SortedList<kKeys32>& sorted, uint32_t floor = 0) {
  const short2v me = __builtin_bit_cast(short2v, uint32_t(x) | (uint32_t(y) << 16));
  for (uint32_t q = qb; q < qe; ++q) {
    const short2v d = __builtin_bit_cast(short2v, sorted.pos[q]) - me;
    const uint32_t d2 = squared_length(d);
    const uint32_t idv = sorted.id[q];
    // a marked entry becomes the empty key (all ones): sign-extend the flag bit over the key
    const uint32_t dead_mask = uint32_t(int32_t(idv << 16) >> 31);
    uint32_t key = ((d2 << ib) | idv) | dead_mask;
    if (ABOVE && key <= floor) key = ~0u;
    insert_key<KT>(keys, key);
  }
}

// The K smallest (squared distance, index) keys among the other live agents, exactly.
// Scans the (2r+1)^2 buckets around the agent's own; every agent outside that block is
// beyond a side of the block, so once the K-th key is nearer than the nearest cell beyond any
// side (or the block covers the grid) no unseen agent can enter the list; otherwise r doubles
// and only the buckets that the wider block adds, and that are near enough to matter, are
// scanned.  The agent's own entry is left out by splitting its bucket row at its slot.  FIRST: give
// up (return false) when the first ring does not settle the list; the caller queues the agent.
// ABOVE: the K smallest keys greater than `floor` (the next K neighbours after those up to `floor`).
template <int WIDE, int KT, bool FIRST, bool ABOVE = false>
__device__ __forceinline__ bool nearest_keys(typename SortedList<WIDE>::Key (&keys)[KT], int K, int x, int y,
                                             uint32_t self_slot, const Buckets bk, int ib,
                                             const SortedList<WIDE>& sorted, const uint16_t* starts,
                                             const uint16_t* edges, typename SortedList<WIDE>::Key floor = 0) {
  using Key = typename SortedList<WIDE>::Key;
  const int bx = bucket_coord(x, bk), by = bucket_coord(y, bk), last = bk.nbx - 1;
#pragma unroll
  for (int k = 0; k < KT; ++k) keys[k] = key_none<Key>();
  int px0 = 1, px1 = 0, py0 = 1, py1 = 0;  // block already scanned (empty)
  uint32_t kth_d2 = ~0u;                   // squared distance of the K-th key so far
  for (int r = 1;; r *= 2) {
    const int x0 = max(bx - r, 0), x1 = min(bx + r, last);
    const int y0 = max(by - r, 0), y1 = min(by + r, last);
    for (int row = y0; row <= y1; ++row) {
      const uint16_t* rs = starts + row * bk.nbx;
      if (row < py0 || row > py1) {
        // A row the earlier block did not touch.  It cannot improve the list if even its
        // nearest cell is farther than the K-th key (equal distance could still win on index).
        const int gap = row > by ? int(edges[row]) - y : y - (int(edges[row + 1]) - 1);
        if (r > 1 && uint32_t(gap * gap) > kth_d2) continue;
        // the agent's own row (first ring only) is split at its slot so that it does not meet itself
        const uint32_t qb = rs[x0], qe = rs[x1 + 1];
        const uint32_t split = row == by ? self_slot : qe;
        scan_range<KT, ABOVE>(keys, qb, split, x, y, ib, sorted, floor);
        scan_range<KT, ABOVE>(keys, split + 1, qe, x, y, ib, sorted, floor);
      } else {
        // only the buckets left and right of the earlier block are new
        if (x0 < px0) {
          const int gap = x - (int(edges[px0]) - 1);
          if (uint32_t(gap * gap) <= kth_d2) scan_range<KT, ABOVE>(keys, rs[x0], rs[px0], x, y, ib, sorted, floor);
        }
        if (x1 > px1) {
          const int gap = int(edges[px1 + 1]) - x;
          if (uint32_t(gap * gap) <= kth_d2)
            scan_range<KT, ABOVE>(keys, rs[px1 + 1], rs[x1 + 1], x, y, ib, sorted, floor);
        }
      }
      if (!key_is_none<WIDE>(keys[K - 1])) kth_d2 = uint32_t(keys[K - 1] >> ib);
    }
    // Every agent not scanned yet lies beyond a side of the block that is not the grid's
    // edge; `reach` is the distance to the nearest cell beyond such a side.
    int reach = 65535;
    if (x0 > 0) reach = min(reach, x - int(edges[x0]) + 1);
    if (x1 < last) reach = min(reach, int(edges[x1 + 1]) - x);
    if (y0 > 0) reach = min(reach, y - int(edges[y0]) + 1);
    if (y1 < last) reach = min(reach, int(edges[y1 + 1]) - y);
    if (reach == 65535) break;  // the block covers the grid
    if (kth_d2 < uint32_t(reach * reach)) break;
    if constexpr (FIRST) return false;  // the first ring did not settle it
    px0 = x0;
    px1 = x1;
    py0 = y0;
    py1 = y1;
  }
  return true;
}

// The same search by two neighbouring lanes (side 0 and 1 of one agent): each scans half of
// every range of slots, and at the end of a ring the two lists are merged through lane shuffles, so
// that both lanes decide alike whether the list is settled.  Inside a ring a lane prunes rows with
// the smaller of the pair's K-th distance after the ring before and the K-th of its own list, an
// upper bound of the pair's.  A search is a chain of
// dependent LDS reads whose length is the number of candidates: two lanes halve it.  Both lanes of
// a pair must call together, and both get the whole list.
template <int WIDE, int KT>
__device__ __forceinline__ void nearest_keys_pair(typename SortedList<WIDE>::Key (&keys)[KT], int K, int x, int y,
                                                  uint32_t self_slot, int side, const Buckets bk, int ib,
                                                  const SortedList<WIDE>& sorted, const uint16_t* starts,
                                                  const uint16_t* edges) {
  using Key = typename SortedList<WIDE>::Key;
  const int bx = bucket_coord(x, bk), by = bucket_coord(y, bk), last = bk.nbx - 1;
#pragma unroll
  for (int k = 0; k < KT; ++k) keys[k] = key_none<Key>();
  // this lane's half of the slots [qb, qe), without the agent's own slot
  const auto scan_half = [&](uint32_t qb, uint32_t qe) {
    const uint32_t mid = (qb + qe) >> 1;
    const uint32_t a = side ? mid : qb, b = side ? qe : mid;
    scan_range<KT>(keys, a, min(b, max(self_slot, a)), x, y, ib, sorted);
    scan_range<KT>(keys, max(a, min(self_slot + 1, b)), b, x, y, ib, sorted);
  };
  int px0 = 1, px1 = 0, py0 = 1, py1 = 0;  // block already scanned (empty)
  uint32_t kth_d2 = ~0u;                   // squared distance of the K-th key so far
  for (int r = 1;; r *= 2) {
    const int x0 = max(bx - r, 0), x1 = min(bx + r, last);
    const int y0 = max(by - r, 0), y1 = min(by + r, last);
    for (int row = y0; row <= y1; ++row) {
      const uint16_t* rs = starts + row * bk.nbx;
      if (row < py0 || row > py1) {
        const int gap = row > by ? int(edges[row]) - y : y - (int(edges[row + 1]) - 1);
        if (r > 1 && uint32_t(gap * gap) > kth_d2) continue;
        scan_half(rs[x0], rs[x1 + 1]);
      } else {
        if (x0 < px0) {
          const int gap = x - (int(edges[px0]) - 1);
          if (uint32_t(gap * gap) <= kth_d2) scan_half(rs[x0], rs[px0]);
        }
        if (x1 > px1) {
          const int gap = int(edges[px1 + 1]) - x;
          if (uint32_t(gap * gap) <= kth_d2) scan_half(rs[px1 + 1], rs[x1 + 1]);
        }
      }
      if (!key_is_none<WIDE>(keys[K - 1])) kth_d2 = min(kth_d2, uint32_t(keys[K - 1] >> ib));
    }
    {  // the other lane's list joins this one
      Key other[KT];
#pragma unroll
      for (int k = 0; k < KT; ++k) {
        if constexpr (sizeof(Key) == 8) {
          const uint32_t lo = uint32_t(__shfl_xor(int(uint32_t(keys[k])), 1));
          const uint32_t hi = uint32_t(__shfl_xor(int(uint32_t(keys[k] >> 32)), 1));
          other[k] = (Key(hi) << 32) | Key(lo);
        } else {
          other[k] = Key(uint32_t(__shfl_xor(int(keys[k]), 1)));
        }
      }
#pragma unroll
      for (int k = 0; k < KT; ++k) insert_key<KT>(keys, other[k]);
      kth_d2 = key_is_none<WIDE>(keys[K - 1]) ? ~0u : uint32_t(keys[K - 1] >> ib);
    }
    int reach = 65535;
    if (x0 > 0) reach = min(reach, x - int(edges[x0]) + 1);
    if (x1 < last) reach = min(reach, int(edges[x1 + 1]) - x);
    if (y0 > 0) reach = min(reach, y - int(edges[y0]) + 1);
    if (y1 < last) reach = min(reach, int(edges[y1 + 1]) - y);
    if (reach == 65535) break;  // the block covers the grid
    if (kth_d2 < uint32_t(reach * reach)) break;
    // Another ring: side 0 goes on with the merged list, side 1 with an empty one (and the merged
    // K-th distance as its bound), so that the next merge meets no key twice.
    if (side) {
#pragma unroll
      for (int k = 0; k < KT; ++k) keys[k] = key_none<Key>();
    }
    px0 = x0;
    px1 = x1;
    py0 = y0;
    py1 = y1;
  }
}

}  // namespace dev
}  // namespace wd
#endif  // WD_DEV_TABLES_H
