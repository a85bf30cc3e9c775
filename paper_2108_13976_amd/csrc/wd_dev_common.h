// wd_dev_common.h — random numbers (Philox4x32-10), the inverse-CDF sampler, four-wide loads and stores.
// Device-side helpers of libwd (gfx950); included by wd_kernels.hip only.
#ifndef WD_DEV_COMMON_H
#define WD_DEV_COMMON_H

#include "wd_internal.h"

namespace wd {
namespace dev {

constexpr uint32_t kDeadBit = 0x80000000u;  // in a packed position or entry: agent is out of play
constexpr uint32_t kStaleBit = 0x8000u;  // in a packed position: out of play since before this step began
constexpr uint32_t kNoNeighbour = 0xFFFFu;

// ----------------------------------------------------------------------------------
// Random numbers: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).  Ten rounds of
// two 32x32->64 multiplies and a word permutation, the key bumped by Weyl constants.
// ----------------------------------------------------------------------------------
struct Block4 {
  uint32_t w[4];
};

__device__ __forceinline__ Block4 philox_block(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint32_t hi_a = __umulhi(0xD2511F53u, c0), lo_a = 0xD2511F53u * c0;
    const uint32_t hi_b = __umulhi(0xCD9E8D57u, c2), lo_b = 0xCD9E8D57u * c2;
    c0 = hi_b ^ c1 ^ k0;
    c1 = lo_b;
    c2 = hi_a ^ c3 ^ k1;
    c3 = lo_a;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Block4{{c0, c1, c2, c3}};
}

// Counter layout: (global env id, index, g low word, stream | g high word << 8).  For
// sampling the index is the group (agent / 4) and agent i takes word i mod 4; for start
// positions the index is the agent and words 0, 1 give x, y.
__device__ __forceinline__ Block4 random_block(const Params& p, uint32_t env_local, uint32_t index,
                                               uint32_t g_lo, uint32_t g_hi, uint32_t stream) {
  return philox_block(p.env_offset + env_local, index, g_lo, stream | (g_hi << 8), p.seed_lo, p.seed_hi);
}

__device__ __forceinline__ uint32_t fastdiv(uint32_t a, const FastDiv& f) {
  const uint32_t t = __umulhi(a, f.mul);
  return (t + ((a - t) >> f.sh1)) >> f.sh2;
}

// Inverse-CDF draw: float32 running sum left to right, strict "<", last action as fall-through.
__device__ __forceinline__ int32_t sample_action(float p0, float p1, float p2, float p3, uint32_t word) {
  const float u = static_cast<float>(word >> 8) * (1.0f / 16777216.0f);
  const float c0 = 0.0f + p0;
  const float c1 = c0 + p1;
  const float c2 = c1 + p2;
  const float c3 = c2 + p3;
  return (u < c0) ? 0 : (u < c1) ? 1 : (u < c2) ? 2 : (u < c3) ? 3 : 4;
}

// Sixteen bytes at a 4-byte aligned address, which global memory takes in one access: a
// group's slices are 16-byte aligned only when the agent count is a multiple of four.
struct __attribute__((packed, aligned(4))) Quad32 {
  uint32_t a, b, c, d;
};

// Actions of the four agents of a group from their 20 probabilities and one random block.
// a0 = flat index of the group's first agent, n = how many of the four agents exist.
__device__ __forceinline__ void sample_group(const float* __restrict__ probs, int64_t a0, int n, bool vec,
                                             const Block4& r, int act[4]) {
  float f[20];
  if (vec) {
    const float4* src = reinterpret_cast<const float4*>(probs + a0 * kNumActions);
#pragma unroll
    for (int q = 0; q < 5; ++q) {
      const float4 v = src[q];
      f[4 * q + 0] = v.x;
      f[4 * q + 1] = v.y;
      f[4 * q + 2] = v.z;
      f[4 * q + 3] = v.w;
    }
  } else {
    // whole quads of the group's 5 n floats in one access each, the rest one by one
    const int quads = (n * kNumActions) >> 2;
    const Quad32* src = reinterpret_cast<const Quad32*>(probs + a0 * kNumActions);
#pragma unroll
    for (int q = 0; q < 5; ++q) {
      if (q < quads) {
        const Quad32 v = src[q];
        f[4 * q + 0] = __uint_as_float(v.a);
        f[4 * q + 1] = __uint_as_float(v.b);
        f[4 * q + 2] = __uint_as_float(v.c);
        f[4 * q + 3] = __uint_as_float(v.d);
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          f[4 * q + c] = (4 * q + c < n * kNumActions) ? probs[a0 * kNumActions + 4 * q + c] : 0.0f;
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) act[j] = sample_action(f[5 * j], f[5 * j + 1], f[5 * j + 2], f[5 * j + 3], r.w[j]);
}

// The same in two parts, for code that has other loads to issue before it waits for these: the
// group's 20 probabilities (zeros beyond agent n), then the draws.
__device__ __forceinline__ void load_group_probs(const float* __restrict__ probs, int64_t a0, int n, bool vec,
                                                 float f[20]) {
  if (vec) {
    const float4* src = reinterpret_cast<const float4*>(probs + a0 * kNumActions);
#pragma unroll
    for (int q = 0; q < 5; ++q) {
      const float4 v = src[q];
      f[4 * q + 0] = v.x;
      f[4 * q + 1] = v.y;
      f[4 * q + 2] = v.z;
      f[4 * q + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int c = 0; c < 20; ++c) f[c] = c < n * kNumActions ? probs[a0 * kNumActions + c] : 0.0f;
  }
}
__device__ __forceinline__ void draw_group(const float f[20], const Block4& r, int act[4]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) act[j] = sample_action(f[5 * j], f[5 * j + 1], f[5 * j + 2], f[5 * j + 3], r.w[j]);
}

__device__ __forceinline__ void load4(const int32_t* __restrict__ src, int64_t a0, int n, bool vec, int v[4]) {
  if (vec) {
    const int4 q = *reinterpret_cast<const int4*>(src + a0);
    v[0] = q.x;
    v[1] = q.y;
    v[2] = q.z;
    v[3] = q.w;
  } else if (n == 4) {
    const Quad32 q = *reinterpret_cast<const Quad32*>(src + a0);
    v[0] = int(q.a);
    v[1] = int(q.b);
    v[2] = int(q.c);
    v[3] = int(q.d);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = j < n ? src[a0 + j] : 0;
  }
}

__device__ __forceinline__ void store4(int32_t* __restrict__ dst, int64_t a0, int n, bool vec, const int v[4]) {
  if (vec) {
    *reinterpret_cast<int4*>(dst + a0) = make_int4(v[0], v[1], v[2], v[3]);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (j < n) dst[a0 + j] = v[j];
  }
}

__device__ __forceinline__ void store4(float* __restrict__ dst, int64_t a0, int n, bool vec, const float v[4]) {
  if (vec) {
    *reinterpret_cast<float4*>(dst + a0) = make_float4(v[0], v[1], v[2], v[3]);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (j < n) dst[a0 + j] = v[j];
  }
}

}  // namespace dev
}  // namespace wd
#endif  // WD_DEV_COMMON_H
