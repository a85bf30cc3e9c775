// wd_dev_strips.h — the strip-sorted list of live agents and the window search over it.
// Device-side helpers of libwd (gfx950); included by wd_kernels.hip only.
//
// The K-nearest search of the observation phase (arXiv 2108.13976, Sec. 5.1: an agent sees its
// K closest agents; Sec. 5.5: that keeps the step close to O(N)) is a chain of dependent LDS
// reads when it walks bucket ranges of data-dependent length, and a wave then waits for its
// longest lane.  Here the live agents are sorted by (strip, column): strips are horizontal bands
// of the grid about one K-th-neighbour distance tall, columns are 2^cshift cells wide, so inside a
// strip the list is ordered by x.  An agent then looks at FIXED windows of that list: the HO
// entries on either side of its own slot, and 2 HA entries around its column in the strip above
// and in the strip below.  Every lane does the same number of independent loads at constant
// offsets, the loop is fully unrolled, and the result is exact whenever the K-th key found is
// nearer than anything the windows cannot have seen: an agent of a scanned strip that lies
// beyond a window is at least as far in x as that window's last entry, and an agent of any other
// strip is beyond the far edge of the neighbouring strip.  Agents whose windows do not settle it
// (a few per cent) are queued for an exact block search over the same list.
//
// Positions in this list are kept scaled: x << h | (y << h) << 16 with 2 h = key_shift >= idx_bits.
// The packed difference to the agent's own entry is then (dx << h, dy << h), and its dot product
// with itself, accumulated onto the candidate's index, IS the key (d^2 << key_shift) + index: two
// vector instructions per candidate in front of the insertion instead of three.  An entry out of
// play (tagged in this step, or a pad) has y field 0x7FFF: its keys are at least
// Params.dead_key_min, above every key of a live pair (the host checks that the grid is small
// enough for that: (G - 1) << h at most about 13 500).
#ifndef WD_DEV_STRIPS_H
#define WD_DEV_STRIPS_H

#include <utility>

#include "wd_dev_tables.h"

namespace wd {
namespace dev {

constexpr uint32_t kStripDeadY = 0x7FFFu;     // y field of a list entry that is out of play
constexpr int kFar = 32767;                  // "no bound on this side", in cells
constexpr uint32_t kFarSq = 32767u * 32767u;  // its square: above every squared distance of 32-bit keys

struct Strips {
  uint32_t mul;  // strip of cell y: (y * mul) >> 16
  int R;         // strips
  int C;         // columns per strip
  int cshift;    // column of cell x: x >> cshift
  int hu;        // cells in the shortest strip
  int h;         // list positions are scaled by 2^h per axis
  uint32_t dead_min;  // keys from here on belong to entries out of play (or are empty)
};

// Strips for n_live agents: about strip_scale * sqrt(n) of them (the expected distance of the
// K-th neighbour shrinks with the square root of the density), as many as the table holds at most.
// Any choice gives the same results.
__device__ __forceinline__ Strips choose_strips(const Params& p, int n_live) {
  const float want = p.strip_scale * sqrtf(static_cast<float>(max(n_live, 1)));
  const int rw = min(max(int(want + 0.5f), 1), p.strip_rmax);
  Strips s;
  s.mul = (uint32_t(rw) << 16) / uint32_t(p.G);  // floor: the last cell lands in strip rw - 1 at most
  s.R = int((uint32_t(p.G - 1) * s.mul) >> 16) + 1;
  s.C = p.strip_C;
  s.cshift = p.cshift;
  uint32_t w = 65536u / s.mul;
  s.hu = int(max(w, 1u));
  s.h = p.pos_shift;
  s.dead_min = p.dead_key_min;
  return s;
}

// The geometry again from the multiplier and the strip count that choose_strips picked.
__device__ __forceinline__ Strips strips_of_env(const Params& p, uint32_t mul, int rows) {
  Strips s;
  s.mul = mul;
  s.R = rows;
  s.C = p.strip_C;
  s.cshift = p.cshift;
  s.hu = int(max(65536u / max(mul, 1u), 1u));
  s.h = p.pos_shift;
  s.dead_min = p.dead_key_min;
  return s;
}

__device__ __forceinline__ int strip_of(int y, const Strips sg) { return int(__umul24(uint32_t(y), sg.mul) >> 16); }
// first cell of strip r: the smallest y with (y * mul) >> 16 == r
__device__ __forceinline__ int strip_first_cell(int r, const Strips sg) {
  return int((uint32_t(r) * 65536u + sg.mul - 1u) / sg.mul);
}
__device__ __forceinline__ int strip_bin(int x, int y, const Strips sg) {
  return strip_of(y, sg) * sg.C + (x >> sg.cshift);
}

// The table T: 16-bit entries, two to a word so that LDS atomics can count in them.  While the
// list is built entry b + 1 is the counter, then the cursor, of bin b; after the scatter entry
// b is where bin b starts, and entry R * C the number of agents in the list.
__device__ __forceinline__ void strip_count(uint32_t* tw, int bin) {
  const uint32_t e = uint32_t(bin) + 1u;
  atomicAdd(&tw[e >> 1], (e & 1u) ? 0x10000u : 1u);
}
__device__ __forceinline__ uint32_t strip_take_slot(uint32_t* tw, int bin) {
  const uint32_t e = uint32_t(bin) + 1u;
  const uint32_t sh = (e & 1u) << 4;
  return (atomicAdd(&tw[e >> 1], 1u << sh) >> sh) & 0xFFFFu;
}

// Words of T in use for a geometry (entries 0 .. R * C).
__device__ __forceinline__ int strip_words(const Strips sg) { return (sg.R * sg.C + 2) >> 1; }

// Clears the table and writes the strip edges.
template <typename Tables>
__device__ __forceinline__ void strip_prepare(const Params& p, const Tables& L, const Strips sg, int lt, int ts) {
  uint32_t* tw = reinterpret_cast<uint32_t*>(L.starts);
  const int words = strip_words(sg);
  for (int j = lt; j < words; j += ts) tw[j] = 0u;
  for (int j = lt; j <= sg.R; j += ts) L.edges[j] = uint16_t(min(strip_first_cell(j, sg), p.G));
}

// Second half of the counting sort: counts -> start offsets -> entries in (strip, column) order,
// and the pads of the list: pad_l entries in front of slot 0 and pad_r behind the last slot that
// read as "no agent" from anywhere on the grid (the windows of the search run into them).
// `act` marks teams that take part; every thread of the workgroup must call (barriers inside).
// Requires pl[] written and the counts in T, and a barrier after that.
template <typename Tables>
__device__ __forceinline__ void strip_scan_and_scatter(const Params& p, const Tables& L, bool act, int lt, int ts,
                                                       const Strips sg) {
  uint32_t* tw = reinterpret_cast<uint32_t*>(L.starts);
  const int words = strip_words(sg);
  const int chunk = (words + ts - 1) >> p.ts_log2;
  const int j0 = lt * chunk, j1 = min(j0 + chunk, words);
  int part = 0;
  if (act)
    for (int j = j0; j < j1; ++j) {
      const uint32_t w = tw[j];
      part += int(w & 0xFFFFu) + int(w >> 16);
    }
  int total = 0;
  int run = team_exclusive_scan(part, lt, p.ts_log2, L.misc + 4, &total);
  if (act)
    for (int j = j0; j < j1; ++j) {
      const uint32_t w = tw[j];
      const uint32_t lo = uint32_t(run);
      run += int(w & 0xFFFFu);
      const uint32_t hi = uint32_t(run);
      run += int(w >> 16);
      tw[j] = lo | (hi << 16);
    }
  __syncthreads();
  if (act) {
    const uint32_t pad = kStripDeadY << 16;
    const int h = p.pos_shift;
    for (int j = lt; j < p.pad_l + p.pad_r; j += ts) {
      const int at = j < p.pad_l ? -1 - j : total + (j - p.pad_l);
      L.sorted.pos[at] = pad;
      L.sorted.id[at] = 0;
    }
    for (int k = 0; k < p.gpt; ++k) {
      const int i0 = 4 * (lt + k * ts);
      if (i0 < p.N) {
        const uint4 v4 = *reinterpret_cast<const uint4*>(L.pl + i0);
        const uint32_t v[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (!(v[j] & kDeadBit)) {
            const int x = pos_x_of(v[j]), y = pos_y_of(v[j]);
            const uint32_t at = strip_take_slot(tw, strip_bin(x, y, sg));
            L.sorted.put(at, x << h, y << h, i0 + j);
            L.slot[i0 + j] = uint16_t(at);
          }
        }
      }
    }
  }
  __syncthreads();
}

// Tag check from the tagger's side: the runners within the tag radius of tagger i get the
// smallest (distance, tagger) key.
template <typename Tables>
__device__ __forceinline__ void strip_tag_scan(const Params& p, const Tables& L, const Strips sg, int i) {
  const uint32_t me = L.pl[i];
  const int x = pos_x_of(me), y = pos_y_of(me);
  const int c0 = max(x - p.tag_rad, 0) >> sg.cshift, c1 = min(x + p.tag_rad, p.G - 1) >> sg.cshift;
  const int r0 = strip_of(max(y - p.tag_rad, 0), sg), r1 = strip_of(min(y + p.tag_rad, p.G - 1), sg);
  for (int row = r0; row <= r1; ++row) {
    const uint32_t q_end = L.starts[row * sg.C + c1 + 1];
    for (uint32_t q = L.starts[row * sg.C + c0]; q < q_end; ++q) {
      const uint32_t pv = L.sorted.pos[q];
      const int j = int(L.sorted.id[q]);
      if (j < p.N_tag) continue;
      const int dx = int((pv & 0xFFFFu) >> p.pos_shift) - x, dy = int(pv >> (16 + p.pos_shift)) - y;
      const uint32_t d2 = uint32_t(__mul24(dx, dx)) + uint32_t(__mul24(dy, dy));
      if (d2 <= uint32_t(p.tag_r2)) atomicMin(&L.best[j], (d2 << p.idx_bits) | uint32_t(i));
    }
  }
}

// One side of a window as a bound on x: `done` = the window reaches the end of the strip on that
// side (nothing unseen there), else every unseen agent of the strip on that side is at least
// `dist` columns-rounded cells away in x.
__device__ __forceinline__ int side_bound(bool done, int dist) { return done ? kFar : max(dist, 0); }

// A 2-byte LDS load at a constant offset from `base`, zero-extended.  Written out: left to the
// compiler, neighbouring index loads are merged into wide loads at 2-byte alignment (several LDS
// passes per access) and unpacked again, one more instruction per candidate.  The result must not
// be used before lds_wait().
template <int kByteOffset>
__device__ __forceinline__ uint32_t lds_read_u16(const uint16_t* base) {
  uint32_t v;
  // (the low word of a pointer into LDS is its LDS address)
  asm volatile("ds_read_u16 %0, %1 offset:%2" : "=v"(v) : "v"(uint32_t(reinterpret_cast<uintptr_t>(base))), "n"(kByteOffset));
  return v;
}
__device__ __forceinline__ void lds_wait() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
// ties a value loaded by lds_read_u16 to the lds_wait() in front of it
__device__ __forceinline__ void lds_loaded(uint32_t& v) { asm volatile("" : "+v"(v)); }

// Key of a candidate: squared length of the packed, scaled difference plus the candidate's index.
__device__ __forceinline__ uint32_t strip_key(short2v d, uint32_t index) {
  uint32_t r;
  asm("v_dot2_i32_i16 %0, %1, %1, %2" : "=v"(r) : "v"(d), "v"(index));
  return r;
}

// kN consecutive slots from slot kFirst of `wp` / `wi` on as candidates (one chunk of a window).
template <int K, int kFirst, int... J>
__device__ __forceinline__ void scan_chunk(uint32_t (&keys)[K], const uint32_t* __restrict__ wp, const uint16_t* wi,
                                           short2v mev, int ib, uint32_t& first, uint32_t& last,
                                           std::integer_sequence<int, J...>) {
  constexpr int kN = sizeof...(J);
  uint32_t pv[kN], iv[kN];
  ((pv[J] = wp[kFirst + J]), ...);
  ((iv[J] = lds_read_u16<2 * (kFirst + J)>(wi)), ...);
  lds_wait();
  (lds_loaded(iv[J]), ...);
  (insert_key<K>(keys, strip_key(__builtin_bit_cast(short2v, pv[J]) - mev, iv[J])), ...);
  first = pv[0];
  last = pv[kN - 1];
}

// N consecutive slots from `wp` / `wi` as candidates; x | y << 16 of the first and the last slot come
// back.  In chunks of eight: eight position and eight index loads are in flight before their
// candidates are inserted (all loads of a long window up front cost more registers than there are).
template <int K, int N, int kFirst = 0>
__device__ __forceinline__ void scan_slots(uint32_t (&keys)[K], const uint32_t* __restrict__ wp, const uint16_t* wi,
                                           short2v mev, int ib, uint32_t& first, uint32_t& last) {
  constexpr int kChunk = 8;
  constexpr int kN = N - kFirst < kChunk ? N - kFirst : kChunk;
  uint32_t f, l;
  scan_chunk<K, kFirst>(keys, wp, wi, mev, ib, f, l, std::make_integer_sequence<int, kN>{});
  if constexpr (kFirst == 0) first = f;
  if constexpr (kFirst + kN >= N)
    last = l;
  else
    scan_slots<K, N, kFirst + kN>(keys, wp, wi, mev, ib, first, last);
}

// The windows of the agent in slot q: HO slots on either side of it in its own strip, 2 HA slots
// around its column in the strips below and above, and (HF > 0) 2 HF slots in the strips beyond
// those.  Returns true if keys[] then holds its K nearest exactly.
//
// The list is one array, strip after strip, so a window may run past the ends of its strip into
// entries of other strips: that only adds candidates, as long as no entry is met twice.  So each
// window below ends where the window (or the strip) after it begins, and each window above begins
// where the window (or the strip) before it ends.
//
// PAIR: two neighbouring lanes share the agent, lane `side` 0 takes everything below the agent's
// slot, lane 1 everything above, and they merge their lists at the end (both return the same).
// The second try runs this way: it serves a few dozen agents per env, so the length of one lane's
// chain of loads is what it costs.
template <int K, int HO, int HA, int HF, bool PAIR>
__device__ __forceinline__ bool strip_window_search(uint32_t (&keys)[K], uint32_t me, int q, int side, const Strips sg,
                                                    int ib, int n_sorted, int pad, const uint32_t* __restrict__ pos,
                                                    const uint16_t* id, const uint16_t* __restrict__ T,
                                                    const uint16_t* __restrict__ edges) {
  constexpr int kLevels = HF > 0 ? 2 : 1;
  const short2v mev = __builtin_bit_cast(short2v, me);
  const int X = int((me & 0xFFFFu) >> sg.h), Y = int(me >> (16 + sg.h));
  const int r = strip_of(Y, sg);
  const uint32_t cm = (1u << sg.cshift) - 1u;
  const int C = sg.C;
  const int row0 = int(__umul24(uint32_t(r), uint32_t(C)));  // T index of the strip's first bin
  const int bin = row0 + (X >> sg.cshift);
#pragma unroll
  for (int k = 0; k < K; ++k) keys[k] = ~0u;
  const bool below = !PAIR || side == 0, above = !PAIR || side != 0;  // which halves this lane scans

  // own strip
  const int s_own = T[row0], e_own = T[row0 + C];
  uint32_t reach2;
  int lo_edge, hi_edge;  // slots that the windows so far cover, as far as the next window is concerned
  {
    uint32_t first = 0, last = 0, unused;
    if constexpr (PAIR) {
      const int a = side ? q + 1 : q - HO;
      scan_slots<K, HO>(keys, pos + a, id + a, mev, ib, first, last);
    } else {
      scan_slots<K, HO>(keys, pos + (q - HO), id + (q - HO), mev, ib, first, unused);
      scan_slots<K, HO>(keys, pos + (q + 1), id + (q + 1), mev, ib, unused, last);
    }
    const int bl = side_bound(!below || q - HO <= s_own, X - int(((first & 0xFFFFu) >> sg.h) | cm));
    const int br = side_bound(!above || q + HO >= e_own - 1, int(((last & 0xFFFFu) >> sg.h) & ~cm) - X);
    const int b = min(bl, br);
    reach2 = uint32_t(__mul24(b, b));
    lo_edge = min(s_own, q - HO);
    hi_edge = max(e_own, q + HO + 1);
  }
#pragma unroll
  for (int lv = 1; lv <= kLevels; ++lv) {
    constexpr int kNone = 1;  // (window length of a level that does not exist, to keep the template well formed)
    const int H = lv == 1 ? HA : HF;
    const bool has_dn = r >= lv, has_up = r + lv <= sg.R - 1;
    // one pass of this block per direction; a pair runs it once, with the direction in `up`
#pragma unroll
    for (int dir = 0; dir < (PAIR ? 1 : 2); ++dir) {
      const bool up = PAIR ? side != 0 : dir != 0;
      const bool has = up ? has_up : has_dn;
      const int bb = has ? (up ? bin + lv * C : bin - lv * C) : bin;
      const int pc = (int(T[bb]) + int(T[bb + 1]) + 1) >> 1;
      // the far end of that strip: its start (below) or its end (above)
      const int far_end = T[has ? (up ? row0 + (lv + 1) * C : row0 - lv * C) : (up ? row0 + C : row0)];
      const int gap = up ? int(edges[min(r + lv, sg.R)]) - Y : Y - int(edges[max(r - lv + 1, 0)]) + 1;
      const int near_end = up ? hi_edge : lo_edge;
      int a = up ? max(pc - H, near_end) : min(pc - H, near_end - 2 * H);
      // a window that would leave the pads is given up: nothing is known about that strip then
      const bool lost = up ? a + 2 * H > n_sorted + pad : a < -pad;
      if (!has || lost) a = n_sorted;  // the pad behind the list
      uint32_t first, last;
      if (lv == 1)
        scan_slots<K, 2 * HA>(keys, pos + a, id + a, mev, ib, first, last);
      else
        scan_slots<K, 2 * (HF > 0 ? HF : kNone)>(keys, pos + a, id + a, mev, ib, first, last);
      const bool done_l = up ? a <= near_end : a <= far_end;
      const bool done_r = up ? a + 2 * H >= far_end : a + 2 * H >= near_end;
      const int bl = side_bound(done_l, X - int(((first & 0xFFFFu) >> sg.h) | cm));
      const int br = side_bound(done_r, int(((last & 0xFFFFu) >> sg.h) & ~cm) - X);
      const int b = lost ? 0 : min(bl, br);
      const uint32_t bound = uint32_t(__mul24(b, b)) + uint32_t(__mul24(gap, gap));
      reach2 = min(reach2, has ? bound : kFarSq);
      if (has && !lost) {
        if (up)
          hi_edge = max(far_end, a + 2 * H);
        else
          lo_edge = min(far_end, a);
      }
    }
  }
  // strips farther away than the windows went
  const int far_dn = (below && r >= kLevels + 1) ? Y - int(edges[max(r - kLevels, 0)]) + 1 : kFar;
  const int far_up = (above && r + kLevels + 1 <= sg.R - 1) ? int(edges[min(r + kLevels + 1, sg.R)]) - Y : kFar;
  const int fb = min(far_dn, far_up);
  reach2 = min(reach2, uint32_t(__mul24(fb, fb)));
  if constexpr (PAIR) {
    // the other half of the agent's surroundings, from the neighbouring lane
    uint32_t other[K];
#pragma unroll
    for (int k = 0; k < K; ++k) other[k] = uint32_t(__shfl_xor(int(keys[k]), 1));
    reach2 = min(reach2, uint32_t(__shfl_xor(int(reach2), 1)));
#pragma unroll
    for (int k = 0; k < K; ++k) insert_key<K>(keys, other[k]);
  }
  const uint32_t kth = keys[K - 1];
  // (nothing unseen anywhere: the list is complete even if it holds fewer than K agents)
  return reach2 >= kFarSq || (kth < sg.dead_min && (kth >> ib) < reach2);
}

// A list of a few dozen agents: every entry is a candidate (exact without any bound; every lane
// reads the same entries, and 8 instructions per entry undercut the fixed windows).  Eight entries
// per round at constant offsets; the last round may run into the pad behind the list, whose
// entries are as far away as agents out of play.  The agent meets itself too: the list holds one
// key more than wanted, and the agent's own key (distance 0, its index) is taken out at the end,
// which is cheaper than a test per entry.
template <int K1, int... J>
__device__ __forceinline__ void scan_all_chunk(uint32_t (&keys)[K1], const uint32_t* __restrict__ wp,
                                               const uint16_t* wi, short2v mev, int ib,
                                               std::integer_sequence<int, J...>) {
  constexpr int kN = sizeof...(J);
  uint32_t pv[kN], iv[kN];
  ((pv[J] = wp[J]), ...);
  ((iv[J] = lds_read_u16<2 * J>(wi)), ...);
  lds_wait();
  (lds_loaded(iv[J]), ...);
  (insert_key<K1>(keys, strip_key(__builtin_bit_cast(short2v, pv[J]) - mev, iv[J])), ...);
}

template <int K>
__device__ __forceinline__ void strip_scan_all(uint32_t (&keys)[K], uint32_t me, uint32_t q, uint32_t n_sorted, int ib,
                                               const uint32_t* __restrict__ pos, const uint16_t* __restrict__ id) {
  const short2v mev = __builtin_bit_cast(short2v, me);
  uint32_t all[K + 1];
#pragma unroll
  for (int k = 0; k <= K; ++k) all[k] = ~0u;
  for (uint32_t s0 = 0; s0 < n_sorted; s0 += 8)
    scan_all_chunk<K + 1>(all, pos + s0, id + s0, mev, ib, std::make_integer_sequence<int, 8>{});
  const uint32_t own = id[q];  // squared distance 0
  bool passed = false;
#pragma unroll
  for (int k = 0; k < K; ++k) {
    passed |= all[k] == own;
    keys[k] = passed ? all[k + 1] : all[k];
  }
}

// Exact search for the agents that the windows did not settle: all bins within m strip heights
// of the agent, m doubling until the K-th key is nearer than the nearest cell outside the block
// (or the block covers the grid).
template <int K>
__device__ __forceinline__ void strip_block_search(uint32_t (&keys)[K], uint32_t me, uint32_t q, const Strips sg, int ib,
                                                   int G, const uint32_t* __restrict__ pos,
                                                   const uint16_t* __restrict__ id, const uint16_t* __restrict__ T,
                                                   const uint16_t* __restrict__ edges) {
  const short2v mev = __builtin_bit_cast(short2v, me);
  const int X = int((me & 0xFFFFu) >> sg.h), Y = int(me >> (16 + sg.h));
  for (int m = 2;; m *= 2) {
    const int half = min(m * sg.hu, kFar);
    const int c0 = max(X - half, 0) >> sg.cshift, c1 = min(X + half, G - 1) >> sg.cshift;
    const int r0 = strip_of(max(Y - half, 0), sg), r1 = strip_of(min(Y + half, G - 1), sg);
#pragma unroll
    for (int k = 0; k < K; ++k) keys[k] = ~0u;
    for (int row = r0; row <= r1; ++row) {
      const uint32_t qe = T[row * sg.C + c1 + 1];
      for (uint32_t s = T[row * sg.C + c0]; s < qe; ++s) {
        const uint32_t key = strip_key(__builtin_bit_cast(short2v, pos[s]) - mev, uint32_t(id[s]));
        insert_key<K>(keys, s == q ? ~0u : key);
      }
    }
    int reach = kFar;
    if (c0 > 0) reach = min(reach, X - ((c0 << sg.cshift) - 1));
    if (c1 < sg.C - 1) reach = min(reach, ((c1 + 1) << sg.cshift) - X);
    if (r0 > 0) reach = min(reach, Y - int(edges[r0]) + 1);
    if (r1 < sg.R - 1) reach = min(reach, int(edges[r1 + 1]) - Y);
    if (reach == kFar) return;  // the block covers the grid
    const uint32_t kth = keys[K - 1];
    if (kth < sg.dead_min && (kth >> ib) < uint32_t(__mul24(reach, reach))) return;
  }
}

}  // namespace dev
}  // namespace wd
#endif  // WD_DEV_STRIPS_H
