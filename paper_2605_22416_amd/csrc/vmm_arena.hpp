// Arena whose physical memory is attached through the HIP virtual-memory API:
// one reserved address range, backed chunk by chunk, every chunk an allocation
// of its own.  Two chunk-aligned ranges can then exchange their backing without
// moving a byte, which is the physical-remap style of migration the paper names
// as the follow-up to its prototype (Method, "Dynamic Pool Rebalancing";
// Limitations).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

namespace avmp {

class VmmArena {
 public:
  VmmArena() = default;
  VmmArena(const VmmArena&) = delete;
  VmmArena& operator=(const VmmArena&) = delete;
  ~VmmArena() { destroy(); }

  // Smallest chunk the current device maps, 0 when it has no virtual-memory support.
  static uint64_t min_chunk();

  // `bytes` and `chunk` must be positive multiples of min_chunk(), bytes of chunk.
  hipError_t create(uint64_t bytes, uint64_t chunk);
  void destroy();

  // Exchange the backing of [off_a, off_a+bytes) and [off_b, off_b+bytes): both
  // chunk-aligned, disjoint, inside the arena.  Host-synchronous; no work that
  // touches either range may be in flight.  A failure part-way leaves a range
  // unmapped: broken() is then true for good and the arena must not be used.
  hipError_t exchange(uint64_t off_a, uint64_t off_b, uint64_t bytes);

  uint8_t* base() const { return base_; }
  uint64_t bytes() const { return bytes_; }
  uint64_t chunk() const { return chunk_; }
  bool broken() const { return broken_; }
  uint64_t exchanges() const { return exchanges_; }

 private:
  int device_ = 0;
  uint8_t* base_ = nullptr;
  uint64_t bytes_ = 0, chunk_ = 0;
  uint64_t mapped_chunks_ = 0;          // chunks [0, mapped_chunks_) are mapped (during create)
  std::vector<hipMemGenericAllocationHandle_t> backing_;   // by chunk index
  bool broken_ = false;
  uint64_t exchanges_ = 0;
};

}  // namespace avmp
