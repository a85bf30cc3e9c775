// wd_dev_rows.h — observation rows: partial (K nearest) and full, from a team's tables or from search keys.
// Device-side helpers of libwd (gfx950); included by wd_kernels.hip only.
#ifndef WD_DEV_ROWS_H
#define WD_DEV_ROWS_H

#include "wd_dev_tables.h"

namespace wd {
namespace dev {

constexpr int kMiscBucketMul = 22, kMiscBucketSide = 23;  // misc[] slots that carry the bucket geometry to big_obs_kernel
constexpr int kMiscQueue2 = 24;  // misc[] slot: agents waiting for the block search of the strip variant
constexpr int kMiscStripMul = 25, kMiscStripRows = 26;  // misc[] slots: strip geometry of the list the env's search runs on
constexpr uint32_t kCompactNone = 1023u;  // "no neighbour" in the compact 10-bit form

// One observation row (own features + K neighbour slots) written to `row` (registers, LDS
// or global).  KC > 0 fixes K at compile time so that the row can live in registers.  CN:
// the neighbour ids of agent i come from the compact form (K = 4).
template <int KC, bool CN, typename Tables, typename Ptr>
__device__ __forceinline__ void write_row(Ptr row, const Params& p, const Tables& L, int i, int k_runtime,
                                          float t_frac) {
  const int K = KC > 0 ? KC : k_runtime;
  const uint32_t me = L.pl[i];
  const int x = pos_x_of(me), y = pos_y_of(me);
  const bool lv = !(me & kDeadBit);
  row[0] = static_cast<float>(x) * p.inv_G;
  row[1] = static_cast<float>(y) * p.inv_G;
  row[2] = i < p.N_tag ? 1.0f : 0.0f;
  row[3] = lv ? 1.0f : 0.0f;
  row[4] = t_frac;
  uint32_t lo = 0, hi = 0;
  if constexpr (CN) {
    lo = L.nbr_lo[i];
    hi = L.nbr_hi[i];
  }
#pragma unroll
  for (int kk = 0; kk < K; ++kk) {
    uint32_t j;
    bool none;
    if constexpr (CN) {
      j = kk < 3 ? ((lo >> (10 * kk)) & 1023u) : ((lo >> 30) | (hi << 2));
      none = !lv || j == kCompactNone;
    } else {
      j = lv ? uint32_t(L.nbr[i * K + kk]) : kNoNeighbour;
      none = j == kNoNeighbour;
    }
    // no branch: an empty slot looks up the agent itself, whose offsets are zero, so only
    // the two flags need the mask
    const uint32_t jj = none ? uint32_t(i) : j;
    const uint32_t other = L.pl[jj];
    row[5 + 4 * kk + 0] = static_cast<float>(pos_x_of(other) - x) * p.inv_G;
    row[5 + 4 * kk + 1] = static_cast<float>(pos_y_of(other) - y) * p.inv_G;
    row[5 + 4 * kk + 2] = (!none && int(jj) < p.N_tag) ? 1.0f : 0.0f;
    row[5 + 4 * kk + 3] = none ? 0.0f : 1.0f;
  }
}

// Slot j of agent i's full observation row: zeros unless both are in play.
struct FullSlot {
  float a, b, c, d;
};

__device__ __forceinline__ FullSlot full_slot(uint32_t me, uint32_t other, bool other_is_tagger, float inv_G) {
  const bool both = !((me | other) & kDeadBit);
  FullSlot s;
  s.a = both ? static_cast<float>(pos_x_of(other) - pos_x_of(me)) * inv_G : 0.0f;
  s.b = both ? static_cast<float>(pos_y_of(other) - pos_y_of(me)) * inv_G : 0.0f;
  s.c = (both && other_is_tagger) ? 1.0f : 0.0f;
  s.d = both ? 1.0f : 0.0f;
  return s;
}

// Four floats of one neighbour slot; rows of 5 + 4N floats put slots on 4-byte boundaries only.
struct __attribute__((packed, aligned(4))) Slot4 {
  float a, b, c, d;
};

__device__ __forceinline__ void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}


// One partial-observation row written to memory straight from an agent's search keys (the
// large-env observation kernel; rows of agents out of the game pass lv = false).
template <int WIDE, int KT>
__device__ __forceinline__ void store_row(float* __restrict__ row, const Params& p, const uint32_t* pl, int i, int K,
                                          float t_frac, const typename SortedList<WIDE>::Key (&keys)[KT], bool lv) {
  using Key = typename SortedList<WIDE>::Key;
  const Key idx_mask = (Key(1) << p.idx_bits) - 1;
  const uint32_t me = pl[i];
  const int x = pos_x_of(me), y = pos_y_of(me);
  row[0] = static_cast<float>(x) * p.inv_G;
  row[1] = static_cast<float>(y) * p.inv_G;
  row[2] = i < p.N_tag ? 1.0f : 0.0f;
  row[3] = lv ? 1.0f : 0.0f;
  row[4] = t_frac;
#pragma unroll
  for (int kk = 0; kk < KT; ++kk) {
    if (kk < K) {
      const bool none = !lv || key_is_none<WIDE>(keys[kk]);
      const uint32_t j = none ? uint32_t(i) : uint32_t(keys[kk] & idx_mask);
      const uint32_t other = pl[j];
      row[5 + 4 * kk + 0] = static_cast<float>(pos_x_of(other) - x) * p.inv_G;
      row[5 + 4 * kk + 1] = static_cast<float>(pos_y_of(other) - y) * p.inv_G;
      row[5 + 4 * kk + 2] = (!none && int(j) < p.N_tag) ? 1.0f : 0.0f;
      row[5 + 4 * kk + 3] = none ? 0.0f : 1.0f;
    }
  }
}

// Half of such a row, for the two lanes that searched for one agent together: side 0 writes the
// agent's own features and the even neighbour slots, side 1 the odd ones.
template <int WIDE, int KT>
__device__ __forceinline__ void store_row_half(float* __restrict__ row, const Params& p, const uint32_t* pl, int i,
                                               int K, float t_frac, const typename SortedList<WIDE>::Key (&keys)[KT],
                                               int side) {
  using Key = typename SortedList<WIDE>::Key;
  const Key idx_mask = (Key(1) << p.idx_bits) - 1;
  const uint32_t me = pl[i];
  const int x = pos_x_of(me), y = pos_y_of(me);
  if (side == 0) {
    row[0] = static_cast<float>(x) * p.inv_G;
    row[1] = static_cast<float>(y) * p.inv_G;
    row[2] = i < p.N_tag ? 1.0f : 0.0f;
    row[3] = 1.0f;
    row[4] = t_frac;
  }
#pragma unroll
  for (int kk = 0; kk < KT; ++kk) {
    if (kk < K && (kk & 1) == side) {
      const bool none = key_is_none<WIDE>(keys[kk]);
      const uint32_t j = none ? uint32_t(i) : uint32_t(keys[kk] & idx_mask);
      const uint32_t other = pl[j];
      row[5 + 4 * kk + 0] = static_cast<float>(pos_x_of(other) - x) * p.inv_G;
      row[5 + 4 * kk + 1] = static_cast<float>(pos_y_of(other) - y) * p.inv_G;
      row[5 + 4 * kk + 2] = (!none && int(j) < p.N_tag) ? 1.0f : 0.0f;
      row[5 + 4 * kk + 3] = none ? 0.0f : 1.0f;
    }
  }
}

}  // namespace dev
}  // namespace wd
#endif  // WD_DEV_ROWS_H
