// Device-side view of the pools and handle translation (Fig. 1: the handle's
// pool tag selects the store, its page id indexes the table, the table entry
// is the physical slot).  Shared by every kernel; passed by value at launch.
// Everything in it is fixed when the pools are created: what rebalancing changes
// (table entries, pool capacities) lives in device memory behind its pointers, so
// a launch recorded in a graph still sees the current values when replayed.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace avmp {

struct DevPools {
  uint8_t* arena;                 // 128-byte aligned base
  uint64_t usable;                // SSM slots count down from arena + usable
  const uint32_t* table;          // [max_vid[0] + max_vid[1]]: vid -> slot, 0xFFFFFFFF unmapped
  const uint32_t* capacity;       // [2]: slots each pool holds now (two words behind the table)
  unsigned long long* faults;     // handles that did not translate
  uint64_t unit[2];
  uint32_t vid_base[2];
  uint32_t max_vid[2];
};

constexpr uint32_t kDevUnmapped = 0xFFFFFFFFu;

// handle -> byte offset from the arena base, or ~0 if the handle does not name a
// live unit of `want_pool`.  Every check is on values, so a bad handle can never
// produce an address outside the arena.
__device__ __forceinline__ uint64_t translate_offset(const DevPools& P, uint32_t h,
                                                     uint32_t want_pool) {
  const uint32_t cap = P.capacity[want_pool];            // does not depend on the handle: goes out first
  const uint32_t pool = h >> 30, vid = h & 0x3FFFFFFFu;
  if (pool != want_pool || vid >= P.max_vid[want_pool]) return ~0ull;
  const uint32_t slot = P.table[P.vid_base[want_pool] + vid];
  if (slot >= cap) return ~0ull;                         // also catches 0xFFFFFFFF
  return want_pool == 0 ? uint64_t(slot) * P.unit[0]
                        : P.usable - (uint64_t(slot) + 1) * P.unit[1];
}

__device__ __forceinline__ void count_fault(const DevPools& P) { atomicAdd(P.faults, 1ull); }

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) {
  return __uint_as_float(b << 16);
}

// Sums and maxima over the lanes of a row of 16 without going through LDS: data-parallel-primitive
// moves (quad permutes, then mirrors of 8 and of 16 lanes: after each step every lane holds the
// result of a group twice as large).
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_moved(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
// every lane of a 16-lane row ends up with the row's sum
__device__ __forceinline__ float sum_row16(float v) {
  v += dpp_moved<0xB1>(v);      // quad_perm [1,0,3,2]
  v += dpp_moved<0x4E>(v);      // quad_perm [2,3,0,1]
  v += dpp_moved<0x141>(v);     // row_half_mirror
  v += dpp_moved<0x140>(v);     // row_mirror
  return v;
}
// every lane of a 16-lane row ends up with the row's maximum
__device__ __forceinline__ float max_row16(float v) {
  v = fmaxf(v, dpp_moved<0xB1>(v));
  v = fmaxf(v, dpp_moved<0x4E>(v));
  v = fmaxf(v, dpp_moved<0x141>(v));
  v = fmaxf(v, dpp_moved<0x140>(v));
  return v;
}

template <typename E>
__device__ __forceinline__ float load_elem(const E* p);
template <>
__device__ __forceinline__ float load_elem<float>(const float* p) {
  return *p;
}
template <>
__device__ __forceinline__ float load_elem<uint16_t>(const uint16_t* p) {
  return bf16_bits_to_float(*p);
}

// Tokens a request attends over: its resident tokens, plus the one the step appends.
__device__ __forceinline__ uint32_t attended_tokens(const uint32_t* ctx, uint32_t r, uint32_t append) {
  const uint32_t n = ctx[r];
  return n > 0xFFFFFFFFu - append ? n : n + append;
}

// Split of a request's pages into chunks processed by different wavefronts and
// merged afterwards.  It depends on the request's page count only, never on
// physical placement, so results are identical under any placement and across
// migrations.  Short requests use kChunkPages-page chunks; long ones use larger
// chunks so that no request has more than kMaxChunks of them.
constexpr uint32_t kChunkPages = 8;
constexpr uint32_t kMaxChunks = 64;

__host__ __device__ __forceinline__ uint32_t chunk_pages_for(uint32_t n_pages) {
  const uint32_t span = kChunkPages * kMaxChunks;
  return kChunkPages * ((n_pages + span - 1) / span);
}
__host__ __device__ __forceinline__ uint32_t chunk_count_for(uint32_t n_pages) {
  if (n_pages == 0) return 0;
  const uint32_t cp = chunk_pages_for(n_pages);
  return (n_pages + cp - 1) / cp;
}

}  // namespace avmp
