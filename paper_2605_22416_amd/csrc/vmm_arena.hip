#include "vmm_arena.hpp"

#include <utility>

namespace avmp {

namespace {

hipMemAllocationProp device_memory(int device) {
  hipMemAllocationProp prop = {};
  prop.type = hipMemAllocationTypePinned;
  prop.location.type = hipMemLocationTypeDevice;
  prop.location.id = device;
  return prop;
}

hipMemAccessDesc read_write(int device) {
  hipMemAccessDesc acc = {};
  acc.location.type = hipMemLocationTypeDevice;
  acc.location.id = device;
  acc.flags = hipMemAccessFlagsProtReadWrite;
  return acc;
}

}  // namespace

uint64_t VmmArena::min_chunk() {
  int device = 0, supported = 0;
  if (hipGetDevice(&device) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&supported, hipDeviceAttributeVirtualMemoryManagementSupported,
                            device) != hipSuccess || !supported)
    return 0;
  const hipMemAllocationProp prop = device_memory(device);
  size_t g = 0;
  if (hipMemGetAllocationGranularity(&g, &prop, hipMemAllocationGranularityMinimum) != hipSuccess)
    return 0;
  return g;
}

hipError_t VmmArena::create(uint64_t bytes, uint64_t chunk) {
  if (base_ != nullptr) return hipErrorInvalidValue;
  const uint64_t g = min_chunk();
  if (g == 0) return hipErrorNotSupported;
  if (bytes == 0 || chunk == 0 || chunk % g != 0 || bytes % chunk != 0) return hipErrorInvalidValue;
  hipError_t e = hipGetDevice(&device_);
  if (e != hipSuccess) return e;
  void* va = nullptr;
  e = hipMemAddressReserve(&va, bytes, 0, nullptr, 0);
  if (e != hipSuccess) return e;
  base_ = static_cast<uint8_t*>(va);
  bytes_ = bytes;
  chunk_ = chunk;
  const uint64_t n = bytes / chunk;
  backing_.reserve(n);
  const hipMemAllocationProp prop = device_memory(device_);
  for (uint64_t i = 0; i < n && e == hipSuccess; ++i) {
    hipMemGenericAllocationHandle_t h;
    e = hipMemCreate(&h, chunk, &prop, 0);
    if (e != hipSuccess) break;
    backing_.push_back(h);                       // owned from here on, mapped or not
    e = hipMemMap(base_ + i * chunk, chunk, 0, h, 0);
    if (e == hipSuccess) mapped_chunks_ = i + 1;
  }
  if (e == hipSuccess) {
    const hipMemAccessDesc acc = read_write(device_);
    e = hipMemSetAccess(base_, bytes, &acc, 1);
  }
  if (e != hipSuccess) destroy();
  return e;
}

void VmmArena::destroy() {
  if (base_ == nullptr) return;
  (void)hipDeviceSynchronize();
  if (!broken_) {
    if (mapped_chunks_) (void)hipMemUnmap(base_, mapped_chunks_ * chunk_);
  } else {
    // some chunk is unmapped: take them one by one and ignore the ones that are
    for (uint64_t i = 0; i < mapped_chunks_; ++i) (void)hipMemUnmap(base_ + i * chunk_, chunk_);
  }
  for (auto h : backing_) (void)hipMemRelease(h);
  (void)hipMemAddressFree(base_, bytes_);
  backing_.clear();
  base_ = nullptr;
  bytes_ = chunk_ = mapped_chunks_ = 0;
}

hipError_t VmmArena::exchange(uint64_t off_a, uint64_t off_b, uint64_t bytes) {
  if (base_ == nullptr || broken_) return hipErrorInvalidValue;
  if (bytes == 0 || bytes % chunk_ != 0 || off_a % chunk_ != 0 || off_b % chunk_ != 0)
    return hipErrorInvalidValue;
  if (off_a > bytes_ || bytes > bytes_ - off_a || off_b > bytes_ || bytes > bytes_ - off_b)
    return hipErrorInvalidValue;
  const uint64_t lo = off_a < off_b ? off_a : off_b, hi = off_a < off_b ? off_b : off_a;
  if (hi - lo < bytes) return hipErrorInvalidValue;      // overlapping
  const uint64_t ia = off_a / chunk_, ib = off_b / chunk_, k = bytes / chunk_;
  uint8_t* va = base_ + off_a;
  uint8_t* vb = base_ + off_b;
  // from the first unmap to the last set-access a failure leaves holes in the range
  hipError_t e = hipMemUnmap(va, bytes);
  if (e == hipSuccess) e = hipMemUnmap(vb, bytes);
  for (uint64_t c = 0; c < k && e == hipSuccess; ++c) {
    e = hipMemMap(va + c * chunk_, chunk_, 0, backing_[ib + c], 0);
    if (e == hipSuccess) e = hipMemMap(vb + c * chunk_, chunk_, 0, backing_[ia + c], 0);
  }
  const hipMemAccessDesc acc = read_write(device_);
  if (e == hipSuccess) e = hipMemSetAccess(va, bytes, &acc, 1);
  if (e == hipSuccess) e = hipMemSetAccess(vb, bytes, &acc, 1);
  if (e != hipSuccess) {
    broken_ = true;
    return e;
  }
  for (uint64_t c = 0; c < k; ++c) std::swap(backing_[ia + c], backing_[ib + c]);
  ++exchanges_;
  return hipSuccess;
}

}  // namespace avmp
