// In-place SSM single-token state update for gfx950 (Background, "KV Cache and
// SSM State Management": one contiguous block per layer per sequence, updated in
// place with contiguous reads and writes).
#include "conv_window.hpp"
#include "kernels.hpp"

#include <cmath>

namespace avmp {

namespace {

// ---------------------------------------------------------------------------
// SSM single-token state update, in place.  One workgroup per (head, request):
// the head's [P][N] fp32 tile (32 KiB at 64 x 128) is streamed once in and once
// out with 16-byte accesses; a row's N values sit in N/4 adjacent lanes, which
// also reduce y = sum_n S*C.  The state is touched exactly once per step, so
// its loads and stores are non-temporal (policy below).  A workgroup moves a whole
// tile in one burst of loads followed by one burst of stores: workgroups of 256
// threads that walk their tile in four passes measured 5.2 TB/s on MI355X, one-burst
// workgroups of 512 or 1024 threads 6.3 - 6.7 TB/s (which of the two: see the kernel
// for the Mamba-2 head shape below).
// ---------------------------------------------------------------------------
// The state tile goes through buffer accesses so that its cache policy can be
// named: non-temporal (touched once per step) and sc1 scope on top of it.  Against
// the plain non-temporal hint of global accesses the sc1 stores measured 1.5 - 2 %
// more bandwidth on MI355X with a working set far beyond the caches.  The
// descriptor covers exactly one head's tile, so no offset can leave it.
typedef uint32_t u32x4s __attribute__((ext_vector_type(4)));
constexpr int kStreamPolicy = 2 | 16;          // nt | sc1
constexpr int kBufferWord3 = 0x00020000;       // raw buffer of dwords, no swizzle

__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_descriptor(void* tile, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(tile, 0, int(bytes), kBufferWord3);
}
__device__ __forceinline__ u32x4s load_tile(__amdgpu_buffer_rsrc_t rsrc, uint32_t byte_off) {
  return __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_off, 0, kStreamPolicy);
}
__device__ __forceinline__ void store_tile(__amdgpu_buffer_rsrc_t rsrc, uint32_t byte_off, u32x4s v) {
  __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, byte_off, 0, kStreamPolicy);
}
__device__ __forceinline__ float4 as_float4(u32x4s v) {
  return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}
__device__ __forceinline__ u32x4s as_words(float4 v) {
  const u32x4s w = {__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
  return w;
}

// lanes 16..31 and 48..63 end up with the sum of their 32-lane half of the wavefront
__device__ __forceinline__ float sum_half32_into_upper_row(float v) {
  v = sum_row16(v);
  v += dpp_moved<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
  return v;
}

template <typename E>
__device__ __forceinline__ float4 load4(const E* p);
template <>
__device__ __forceinline__ float4 load4<float>(const float* p) {
  return *reinterpret_cast<const float4*>(p);
}
template <>
__device__ __forceinline__ float4 load4<uint16_t>(const uint16_t* p) {
  const uint2 u = *reinterpret_cast<const uint2*>(p);
  return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u),
                     __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xFFFF0000u));
}

// NS: compile-time dstate (0 = read it from the launch); EXACT: headdim is a
// multiple of the rows one pass covers, so no row needs a bounds test.
template <typename E, int THREADS, int ROWS, int NS, bool EXACT>
__global__ __launch_bounds__(THREADS) void ssm_update_kernel(SsmLaunch a) {
  const uint32_t h = blockIdx.x, r = blockIdx.y, tid = threadIdx.x;
  const uint32_t H = a.heads, Pd = a.headdim;
  const uint32_t N = NS ? uint32_t(NS) : a.dstate;
  const uint32_t lpr = N / 4;                  // lanes per row (power of two, <= 64)
  const uint32_t col = tid & (lpr - 1);
  const uint32_t row0 = tid / lpr;
  const uint32_t rpi = THREADS / lpr;          // rows per pass of the workgroup
  // the step's own inputs are requested before the handle -> table -> block chain is waited for
  const uint32_t handle = a.handles[r];
  const float dt = a.dt[size_t(r) * H + h];
  const float Ah = a.A[h];
  const float4 Bv = load4<E>(static_cast<const E*>(a.B) + size_t(r) * N + 4 * col);
  const float4 Cv = load4<E>(static_cast<const E*>(a.C) + size_t(r) * N + 4 * col);
  const uint64_t off = translate_offset(a.P, handle, 1);
  float* yrow = a.y + (size_t(r) * H + h) * Pd;
  if (off == ~0ull) {
    if (tid == 0) count_fault(a.P);
    for (uint32_t p = tid; p < Pd; p += THREADS) yrow[p] = 0.f;
    return;
  }
  const float decay = expf(dt * Ah);
  const E* xrow = static_cast<const E*>(a.x) + (size_t(r) * H + h) * Pd;
  float* tile = reinterpret_cast<float*>(a.P.arena + off) + size_t(h) * Pd * N;
  const __amdgpu_buffer_rsrc_t rsrc = tile_descriptor(tile, Pd * N * 4);

  for (uint32_t pbase = row0; pbase < Pd; pbase += rpi * ROWS) {
    float4 s[ROWS];
    float xs[ROWS];
#pragma unroll
    for (int k = 0; k < ROWS; ++k) {
      const uint32_t p = pbase + k * rpi;
      if (EXACT || p < Pd) {
        s[k] = as_float4(load_tile(rsrc, (p * N + 4 * col) * 4));
        xs[k] = load_elem<E>(xrow + p);
      }
    }
#pragma unroll
    for (int k = 0; k < ROWS; ++k) {
      const uint32_t p = pbase + k * rpi;
      // p < Pd is uniform over the lanes of a row and rows never straddle a
      // wavefront, but the shuffles below run on all lanes and only the
      // memory accesses are masked
      float part = 0.f;
      if (EXACT || p < Pd) {
        const float dtx = dt * xs[k];
        float4 v = s[k];
        v.x = decay * v.x + dtx * Bv.x;
        v.y = decay * v.y + dtx * Bv.y;
        v.z = decay * v.z + dtx * Bv.z;
        v.w = decay * v.w + dtx * Bv.w;
        store_tile(rsrc, (p * N + 4 * col) * 4, as_words(v));
        part = v.x * Cv.x + v.y * Cv.y + v.z * Cv.z + v.w * Cv.w;
      }
#pragma unroll
      for (uint32_t o = 32; o; o >>= 1)
        if (o < lpr) part += __shfl_xor(part, int(o));
      if ((EXACT || p < Pd) && col == 0) yrow[p] = part;
    }
  }
}

// ---------------------------------------------------------------------------
// The layer's short convolution done by the recurrence workgroup itself, at the Mamba-2 head
// shape: a launch of its own costs about 8 us per layer for 1.7 MB of traffic, most of it the
// launch.  A workgroup needs the convolution's outputs for the 2 x 128 channels of B and C,
// which every workgroup of the request needs, and for the x channels of its own head(s) (XCH
// of them, touched by nobody else).  Thread t < 256 takes channel t of [B | C], the XCH threads
// behind them one x channel each; outputs go through LDS to the lanes that use them.  (Sixteen
// bytes of channels per lane, as in the stand-alone kernel, leave the whole workgroup waiting at
// its barrier for two wavefronts that compute eight channels each: 93.8 us per layer against
// 86.0 us without the convolution.)  The x rows of the window move on at once.  The B and C rows
// are read by every workgroup of the request, so they move on only after all of them have
// read: behind the barrier, which every read of the workgroup has passed, the workgroup
// takes a ticket from the request's arrival counter, and the one that draws the last ticket
// reads the rows again at the end of the kernel, writes them one place on and clears the
// counter.  No workgroup waits for another.
// ---------------------------------------------------------------------------
// An element as loaded, one to a register (16-bit elements held two to a register would be
// packed the moment they arrive, and the loads behind them would wait for that).
template <typename E>
struct Held;
template <>
struct Held<float> {
  static __device__ __forceinline__ uint32_t load(const float* p) { return __float_as_uint(*p); }
  static __device__ __forceinline__ void store(float* p, uint32_t bits) { *p = __uint_as_float(bits); }
  static __device__ __forceinline__ float value(uint32_t bits) { return __uint_as_float(bits); }
};
template <>
struct Held<uint16_t> {
  static __device__ __forceinline__ uint32_t load(const uint16_t* p) { return *p; }
  static __device__ __forceinline__ void store(uint16_t* p, uint32_t bits) { *p = uint16_t(bits); }
  static __device__ __forceinline__ float value(uint32_t bits) { return bf16_bits_to_float(bits); }
};

template <typename E, int K, int XCH>
struct FusedConv {
  static constexpr int V = Vec<E>::N;
  static constexpr uint32_t kPd = 64, kN = 128, kShared = 2 * kN;
  static constexpr int kStaged = int(kShared) + XCH;     // floats of LDS: B, C, x of the workgroup's heads
  uint32_t in[K], taps[K], bias;   // as stored (Held); in[K-1] is the new token
  E* win;                   // this thread's channel in row 0 of the window
  uint32_t conv_dim, channel, ticket;
  bool mine;                // the thread has a channel

  // asks for the new token's input, the taps and the bias: nothing here waits for the handle
  __device__ __forceinline__ void request_token(const SsmLaunch& a, uint32_t r, uint32_t first_head) {
    const uint32_t t = threadIdx.x, hp = a.heads * kPd;
    conv_dim = hp + kShared;
    mine = t < kShared + uint32_t(XCH);
    channel = t < kShared ? hp + t : first_head * kPd + (t - kShared);
    ticket = 0;
    if (mine) {
#pragma unroll
      for (int k = 0; k < K; ++k)
        taps[k] = Held<E>::load(static_cast<const E*>(a.conv_taps) + size_t(k) * conv_dim + channel);
      bias = Held<E>::load(static_cast<const E*>(a.conv_bias) + channel);
      in[K - 1] = Held<E>::load(static_cast<const E*>(a.conv_u) + size_t(r) * conv_dim + channel);
    }
  }
  // asks for the channel's window rows behind the block's state
  __device__ __forceinline__ void request_window(uint8_t* block, uint64_t state_bytes) {
    win = reinterpret_cast<E*>(block + state_bytes) + channel;
    if (mine) {
#pragma unroll
      for (int k = 0; k < K - 1; ++k) in[k] = Held<E>::load(win + size_t(k) * conv_dim);
    }
  }
  // the channel's output to LDS, the workgroup's own rows moved on; the caller's barrier follows
  __device__ __forceinline__ void finish(float* staged) {
    if (!mine) return;
    // what was asked for above is first looked at here (widening a value where it was loaded
    // would wait for it there, in front of the state loads)
#pragma unroll
    for (int k = 0; k < K; ++k) asm volatile("" : "+v"(in[k]), "+v"(taps[k]));
    asm volatile("" : "+v"(bias));
    float x[K], w[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      x[k] = Held<E>::value(in[k]);
      w[k] = Held<E>::value(taps[k]);
    }
    staged[threadIdx.x] = conv_channel<K>(Held<E>::value(bias), w, x);
    if (threadIdx.x >= kShared) {
#pragma unroll
      for (int k = 0; k < K - 1; ++k) Held<E>::store(win + size_t(k) * conv_dim, in[k + 1]);
    }
  }
  // behind the barrier: every read of B's and C's rows by this workgroup has returned
  __device__ __forceinline__ void arrive(const SsmLaunch& a, uint32_t r) {
    // (the zero the compiler cannot see through keeps the address a per-lane value: with an
    // address it knows to be the same in every lane it would combine the lanes' additions and
    // hand the result out again at once, waiting for it here)
    uint32_t zero = 0;
    asm volatile("" : "+v"(zero) :: "memory");
    if (threadIdx.x == 0)
      ticket = __hip_atomic_fetch_add(a.conv_arrivals + size_t(r) * kArrivalStride + zero, 1u, __ATOMIC_RELAXED,
                                      __HIP_MEMORY_SCOPE_AGENT);
  }
  // at the end of the kernel: the last workgroup of the request to have read B's and C's rows
  // moves them on, sixteen bytes of channels per lane of the first wavefront
  __device__ __forceinline__ void close(const SsmLaunch& a, uint32_t r) {
    if ((threadIdx.x >> 6) != 0) return;
    // the ticket is looked at here and no earlier: the wavefront must not wait for it above
    asm volatile("" : "+v"(ticket) :: "memory");
    const uint32_t drawn = __builtin_amdgcn_readfirstlane(ticket);
    if (drawn != gridDim.x - 1 || threadIdx.x * V >= kShared) return;
    const size_t row_bytes = size_t(conv_dim) * sizeof(E);
    // thread 0's channel is the first of [B | C]
    const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(reinterpret_cast<uintptr_t>(win)));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(uint32_t(reinterpret_cast<uintptr_t>(win) >> 32));
    uint8_t* rows = reinterpret_cast<uint8_t*>((uint64_t(hi) << 32) | lo) + size_t(threadIdx.x) * 16;
    const uint8_t* token = static_cast<const uint8_t*>(a.conv_u) +
                           (size_t(r) * conv_dim + (conv_dim - kShared)) * sizeof(E) + size_t(threadIdx.x) * 16;
    Vec<E> next[K - 1];
#pragma unroll
    for (int k = 0; k < K - 2; ++k) next[k] = load_vec<E>(rows + (k + 1) * row_bytes);
    next[K - 2] = load_vec<E>(token);
#pragma unroll
    for (int k = 0; k < K - 1; ++k) store_vec<E>(rows + k * row_bytes, next[k]);
    if (threadIdx.x == 0)
      __hip_atomic_store(a.conv_arrivals + size_t(r) * kArrivalStride, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
};

// The same update at the Mamba-2 head shape, headdim 64 x dstate 128, with everything the shape
// fixes folded in at compile time: a row's 128 values in 32 adjacent lanes, THREADS / 32 rows per
// pass, one pass.  What the general kernel computes at run time (row geometry, loop bounds) sits
// in front of the first state load of every workgroup, and 8192 workgroups per launch pay for
// it: 86.1 against 87.2 us per layer at the Jamba-shaped batch of 64 with 1024 threads.
//
// Two shapes of it are used, by the length of the launch (measured on the decode step at
// batches of 32 ... 512 requests of 128 heads; us per layer):
//   * 512 threads, four rows per lane, state asked for as early as possible and the arithmetic
//     on B, C and the decay done while the loads are in flight: quickest to start and to drain,
//     sustains 6.2 - 6.4 TB/s however long the launch (45.4 / 85.8 / 127.8 / 170.2 / 257.1 /
//     714.0 at batch 32 / 64 / 96 / 128 / 192 / 512);
//   * 1024 threads, two rows per lane, that arithmetic finished BEFORE the state is asked for,
//     so that a row is stored the moment it arrives: slower off the mark, but 6.4 - 6.7 TB/s
//     once the launch is long enough (46.1 / 86.2 / 127.3 / 168.5 / 247.0 / 649.0; the general
//     kernel, which orders its work the same way, 87.1 / 128.9 / 171.2 / 248.0 / 652.6 from
//     batch 64 on).  With 512 threads this order is the slowest of all (87.0 at batch 64).
// The step is 2574 us at batch 64 with the first shape, 2581 us with the second.
constexpr uint64_t kShortLaunchTiles = 80 * 128;        // fp32 state: below this many (head, request) tiles, 512 threads
constexpr uint64_t kSmallLaunchTiles16 = 128 * 128;     // bf16 state: below, 512 threads and state first;
constexpr uint64_t kLongLaunchTiles16 = 224 * 128;      // from here on two heads per 1024 threads, arithmetic first
constexpr uint64_t kConvLongLaunchTiles16 = 160 * 128;  // with the convolution inside: two heads per 1024 threads from here on
// CONVK: taps of the layer's convolution done here (FusedConv), 0: x, B and C are read as given.
template <typename E, int THREADS, bool ARITHMETIC_FIRST, int CONVK = 0>
__global__ __launch_bounds__(THREADS) void ssm_update_mamba2_kernel(SsmLaunch a) {
  constexpr uint32_t N = 128, Pd = 64, kLanesPerRow = 32, kRowsPerPass = THREADS / kLanesPerRow;
  constexpr int kRows = Pd / kRowsPerPass;
  const uint32_t h = blockIdx.x, r = blockIdx.y, tid = threadIdx.x;
  const uint32_t H = a.heads;
  const uint32_t col = tid & (kLanesPerRow - 1), row0 = tid / kLanesPerRow;
  // the step's own inputs are requested before the handle -> table -> block chain is waited for
  const uint32_t handle = a.handles[r];
  const float dt = a.dt[size_t(r) * H + h];
  const float Ah = a.A[h];
  float4 Bv, Cv;
  [[maybe_unused]] FusedConv<E, CONVK ? CONVK : 2, 64> conv;
  if constexpr (CONVK == 0) {
    Bv = load4<E>(static_cast<const E*>(a.B) + size_t(r) * N + 4 * col);
    Cv = load4<E>(static_cast<const E*>(a.C) + size_t(r) * N + 4 * col);
  } else {
    conv.request_token(a, r, h);
  }
  const uint64_t off = translate_offset(a.P, handle, 1);
  float* yrow = a.y + (size_t(r) * H + h) * Pd;
  if (off == ~0ull) {
    if (tid == 0) count_fault(a.P);
    if (tid < Pd) yrow[tid] = 0.f;
    return;
  }
  if constexpr (CONVK != 0) conv.request_window(a.P.arena + off, uint64_t(H) * Pd * N * 4);
  float* tile = reinterpret_cast<float*>(a.P.arena + off) + size_t(h) * Pd * N;
  const __amdgpu_buffer_rsrc_t rsrc = tile_descriptor(tile, Pd * N * 4);
  const E* xrow = static_cast<const E*>(a.x) + (size_t(r) * H + h) * Pd;
  float decay = 0.f;
  if (ARITHMETIC_FIRST && CONVK == 0) {
    // nothing below may move above this point: B, C and the decay are in registers before the
    // first state load goes out
    decay = expf(dt * Ah);
    asm volatile("" :: "v"(decay), "v"(Bv.x), "v"(Bv.y), "v"(Bv.z), "v"(Bv.w), "v"(Cv.x), "v"(Cv.y),
                 "v"(Cv.z), "v"(Cv.w) : "memory");
  }
  float4 s[kRows];
  float xs[kRows];
#pragma unroll
  for (int k = 0; k < kRows; ++k) {
    const uint32_t p = row0 + k * kRowsPerPass;
    s[k] = as_float4(load_tile(rsrc, (p * N + 4 * col) * 4));
    if constexpr (CONVK == 0) xs[k] = load_elem<E>(xrow + p);
  }
  if constexpr (CONVK != 0) {
    __shared__ __align__(16) float staged[decltype(conv)::kStaged];
    conv.finish(staged);
    __syncthreads();
    conv.arrive(a, r);
    Bv = *reinterpret_cast<const float4*>(staged + 4 * col);
    Cv = *reinterpret_cast<const float4*>(staged + N + 4 * col);
#pragma unroll
    for (int k = 0; k < kRows; ++k) xs[k] = staged[2 * N + row0 + k * kRowsPerPass];
  }
  if (!ARITHMETIC_FIRST || CONVK != 0) decay = expf(dt * Ah);
#pragma unroll
  for (int k = 0; k < kRows; ++k) {
    const uint32_t p = row0 + k * kRowsPerPass;
    const float dtx = dt * xs[k];
    float4 v = s[k];
    v.x = decay * v.x + dtx * Bv.x;
    v.y = decay * v.y + dtx * Bv.y;
    v.z = decay * v.z + dtx * Bv.z;
    v.w = decay * v.w + dtx * Bv.w;
    store_tile(rsrc, (p * N + 4 * col) * 4, as_words(v));
    const float part = sum_half32_into_upper_row(v.x * Cv.x + v.y * Cv.y + v.z * Cv.z + v.w * Cv.w);
    if (col == kLanesPerRow - 1) yrow[p] = part;
  }
  if constexpr (CONVK != 0) conv.close(a, r);
}

// ---------------------------------------------------------------------------
// Same update with the state stored as bf16 (half the state traffic).  A lane
// moves 16 bytes = 8 state elements, so a row's N values sit in N/8 adjacent
// lanes.  Arithmetic is fp32: the stored bf16 is widened exactly, updated,
// reduced into y un-rounded, then rounded to nearest even for the store.
// ---------------------------------------------------------------------------
template <typename E>
__device__ __forceinline__ void load8(const E* p, float (&v)[8]);
template <>
__device__ __forceinline__ void load8<float>(const float* p, float (&v)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
  v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
template <>
__device__ __forceinline__ void load8<uint16_t>(const uint16_t* p, float (&v)[8]) {
  const uint4 u = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    v[2 * j] = __uint_as_float(w[j] << 16);
    v[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
  }
}

// Two fp32 values rounded to bf16 (to nearest, ties to even) and packed, `lo` in the low half:
// the conversion instruction of this chip, one operation for what takes nine on the integer side.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16_pair(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ uint64_t same_in_every_lane(uint64_t v) {
  const uint32_t lo = uint32_t(__builtin_amdgcn_readfirstlane(int(uint32_t(v))));
  const uint32_t hi = uint32_t(__builtin_amdgcn_readfirstlane(int(uint32_t(v >> 32))));
  return (uint64_t(hi) << 32) | lo;
}

// HPB heads share one workgroup (THREADS / HPB threads each), so that a workgroup of 1024
// threads still moves a 32 KiB burst.  At headdim 64 x dstate 128 three forms are used, by the
// length of the launch (us per layer on the decode step at 64 / 96 / 128 / 192 / 256 requests
// of 128 heads):
//   * a head per workgroup of 512 threads, state asked for first   48.8 / 70.8 / 93.3 / 142.4 / 189.3
//   * the same with B, C and the decay in registers before that    49.5 / 71.2 / 93.2 / 139.5 / 182.0
//   * two heads per workgroup of 1024 threads, arithmetic first    50.8 / 72.9 / 95.2 / 141.4 / 179.8
//   (two heads in 1024 threads, state first                        50.3 / 72.2 / 93.7 / 140.3 / 186.4)
// as with the fp32 state: short launches are mostly ramp-up and drain and want their loads out
// at once; long ones want a row stored the moment it arrives.
// PS: compile-time headdim (0 = read it from the launch), as NS for dstate.
// CONVK: taps of the layer's convolution done here (FusedConv; headdim 64 x dstate 128 only), 0: x, B
// and C are read as given.
template <typename E, int THREADS, int ROWS, int NS, bool EXACT, int HPB = 1, int PS = 0, int CONVK = 0,
          bool ARITHMETIC_FIRST = false>
__global__ __launch_bounds__(THREADS) void ssm_update_bf16state_kernel(SsmLaunch a) {
  static_assert(CONVK == 0 || (NS == 128 && PS == 64 && EXACT), "the convolution is fused at the Mamba-2 head shape only");
  constexpr uint32_t TPH = THREADS / HPB;            // threads per head
  // which of the workgroup's heads: the same for a whole wavefront, and said so, or the tile's
  // buffer descriptor counts as a per-lane value and every access to it is wrapped in a loop
  // over the distinct descriptors of the wavefront
  const uint32_t head_in_wg = HPB == 1 ? 0u : uint32_t(__builtin_amdgcn_readfirstlane(int(threadIdx.x / TPH)));
  const uint32_t h = blockIdx.x * HPB + head_in_wg, r = blockIdx.y, tid = threadIdx.x % TPH;
  const uint32_t H = a.heads, Pd = PS ? uint32_t(PS) : a.headdim;
  const uint32_t N = NS ? uint32_t(NS) : a.dstate;
  [[maybe_unused]] FusedConv<E, CONVK ? CONVK : 2, 64 * HPB> conv;
  if constexpr (CONVK != 0) conv.request_token(a, r, blockIdx.x * HPB);
  // (the block's offset is the same in every lane; behind the per-thread branches of the
  // convolution the compiler no longer sees that, and the descriptor built on it would be
  // taken for a per-lane value)
  const uint64_t off = same_in_every_lane(translate_offset(a.P, a.handles[r], 1));
  float* yrow = a.y + (size_t(r) * H + h) * Pd;
  if (off == ~0ull) {
    if (tid == 0) count_fault(a.P);
    for (uint32_t p = tid; p < Pd; p += TPH) yrow[p] = 0.f;
    return;
  }
  const uint32_t lpr = N / 8;                  // lanes per row (power of two, <= 32)
  const uint32_t col = tid & (lpr - 1);
  const uint32_t row0 = tid / lpr;
  const uint32_t rpi = TPH / lpr;
  const float dt = a.dt[size_t(r) * H + h];
  const float decay = expf(dt * a.A[h]);
  float Bv[8], Cv[8];
  if constexpr (CONVK == 0) {
    load8<E>(static_cast<const E*>(a.B) + size_t(r) * N + 8 * col, Bv);
    load8<E>(static_cast<const E*>(a.C) + size_t(r) * N + 8 * col, Cv);
    if constexpr (ARITHMETIC_FIRST) {
      // nothing below may move above this point: B, C and the decay are in registers before the
      // first state load goes out
      asm volatile("" :: "v"(decay), "v"(Bv[0]), "v"(Bv[1]), "v"(Bv[2]), "v"(Bv[3]), "v"(Bv[4]), "v"(Bv[5]),
                   "v"(Bv[6]), "v"(Bv[7]), "v"(Cv[0]), "v"(Cv[1]), "v"(Cv[2]), "v"(Cv[3]), "v"(Cv[4]),
                   "v"(Cv[5]), "v"(Cv[6]), "v"(Cv[7]) : "memory");
    }
  } else {
    conv.request_window(a.P.arena + off, uint64_t(H) * Pd * N * 2);
  }
  const E* xrow = static_cast<const E*>(a.x) + (size_t(r) * H + h) * Pd;
  uint16_t* tile = reinterpret_cast<uint16_t*>(a.P.arena + off) + size_t(h) * Pd * N;
  const __amdgpu_buffer_rsrc_t rsrc = tile_descriptor(tile, Pd * N * 2);
  [[maybe_unused]] const float* staged_x = nullptr;

  for (uint32_t pbase = row0; pbase < Pd; pbase += rpi * ROWS) {
    u32x4s raw[ROWS];
    float xs[ROWS];
#pragma unroll
    for (int k = 0; k < ROWS; ++k) {
      const uint32_t p = pbase + k * rpi;
      if (EXACT || p < Pd) {
        raw[k] = load_tile(rsrc, (p * N + 8 * col) * 2);
        if constexpr (CONVK == 0) xs[k] = load_elem<E>(xrow + p);
      }
    }
    if constexpr (CONVK != 0) {
      if (pbase == row0) {      // the first pass's state is on its way: now the convolution
        __shared__ __align__(16) float staged[decltype(conv)::kStaged];
        conv.finish(staged);
        __syncthreads();
        conv.arrive(a, r);
        load8<float>(staged + 8 * col, Bv);
        load8<float>(staged + 128 + 8 * col, Cv);
        staged_x = staged + 256 + head_in_wg * 64;
      }
#pragma unroll
      for (int k = 0; k < ROWS; ++k) xs[k] = staged_x[pbase + k * rpi];
    }
#pragma unroll
    for (int k = 0; k < ROWS; ++k) {
      const uint32_t p = pbase + k * rpi;
      float part = 0.f;
      if (EXACT || p < Pd) {
        const float dtx = dt * xs[k];
        const uint32_t w[4] = {raw[k].x, raw[k].y, raw[k].z, raw[k].w};
        uint32_t out[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float lo = decay * __uint_as_float(w[j] << 16) + dtx * Bv[2 * j];
          const float hi = decay * __uint_as_float(w[j] & 0xFFFF0000u) + dtx * Bv[2 * j + 1];
          part += lo * Cv[2 * j] + hi * Cv[2 * j + 1];
          out[j] = pack_bf16_pair(lo, hi);
        }
        const u32x4s packed = {out[0], out[1], out[2], out[3]};
        store_tile(rsrc, (p * N + 8 * col) * 2, packed);
      }
      if (NS == 128) {                         // a row is one 16-lane row of the wavefront
        part = sum_row16(part);
      } else {
#pragma unroll
        for (uint32_t o = 16; o; o >>= 1)
          if (o < lpr) part += __shfl_xor(part, int(o));
      }
      if ((EXACT || p < Pd) && col == 0) yrow[p] = part;
    }
  }
  if constexpr (CONVK != 0) conv.close(a, r);
}

}  // namespace

bool ssm_may_fuse_conv(uint32_t taps_k, uint32_t heads, uint32_t headdim, uint32_t dstate) {
  return taps_k == 4 && heads != 0 && headdim == 64 && dstate == 128;
}

bool ssm_fuses_conv(uint32_t taps_k, uint32_t heads, uint32_t headdim, uint32_t dstate,
                    uint32_t state_dtype, uint32_t batch) {
  return ssm_may_fuse_conv(taps_k, heads, headdim, dstate) &&
         (state_dtype == 1 || uint64_t(heads) * batch < kShortLaunchTiles);
}

namespace {

// the kernels that run the layer's four-tap convolution themselves (headdim 64 x dstate 128)
template <typename E>
hipError_t launch_with_conv(const SsmLaunch& a, hipStream_t s) {
  const dim3 grid(a.heads, a.batch);
  if (a.state_dtype == 1) {
    if (uint64_t(a.heads) * a.batch < kConvLongLaunchTiles16 || a.heads % 2 != 0)
      ssm_update_bf16state_kernel<E, 512, 2, 128, true, 1, 64, 4><<<grid, dim3(512), 0, s>>>(a);
    else
      ssm_update_bf16state_kernel<E, 1024, 2, 128, true, 2, 64, 4><<<dim3(a.heads / 2, a.batch), dim3(1024), 0, s>>>(a);
  } else {
    ssm_update_mamba2_kernel<E, 512, false, 4><<<grid, dim3(512), 0, s>>>(a);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_ssm(const SsmLaunch& a, hipStream_t s) {
  if (a.batch == 0) return hipSuccess;
  if (a.conv_k != 0) {
    if (!ssm_fuses_conv(a.conv_k, a.heads, a.headdim, a.dstate, a.state_dtype, a.batch) || !a.conv_u || !a.conv_taps ||
        !a.conv_bias || !a.conv_arrivals)
      return hipErrorInvalidValue;
    return a.dtype == 0 ? launch_with_conv<float>(a, s) : launch_with_conv<uint16_t>(a, s);
  }
  const dim3 grid(a.heads, a.batch);
  // a head's tile is headdim x dstate/4 16-byte accesses: big tiles get 1024 threads
  const bool big = uint64_t(a.headdim) * (a.dstate / 4) >= 1024;
  // the Mamba-2 shape (dstate 128, headdim a multiple of 64) gets a kernel with
  // compile-time row geometry and no bounds tests
  const bool exact128 = a.dstate == 128 && a.headdim % 64 == 0;
  if (a.state_dtype == 1) {
    const bool big16 = uint64_t(a.headdim) * (a.dstate / 8) >= 1024;
    const bool small16 = uint64_t(a.heads) * a.batch < kSmallLaunchTiles16;
    const bool long16 = uint64_t(a.heads) * a.batch >= kLongLaunchTiles16;
    if (a.dtype == 0) {
      if (exact128 && a.headdim == 64 && small16)     // the Mamba-2 shape
        ssm_update_bf16state_kernel<float, 512, 2, 128, true, 1, 64><<<grid, dim3(512), 0, s>>>(a);
      else if (exact128 && a.headdim == 64 && (!long16 || a.heads % 2 != 0))
        ssm_update_bf16state_kernel<float, 512, 2, 128, true, 1, 64, 0, true><<<grid, dim3(512), 0, s>>>(a);
      else if (exact128 && a.headdim == 64)
        ssm_update_bf16state_kernel<float, 1024, 2, 128, true, 2, 64, 0, true><<<dim3(a.heads / 2, a.batch), dim3(1024), 0, s>>>(a);
      else if (exact128 && a.heads % 2 == 0)
        ssm_update_bf16state_kernel<float, 1024, 2, 128, true, 2><<<dim3(a.heads / 2, a.batch), dim3(1024), 0, s>>>(a);
      else if (exact128) ssm_update_bf16state_kernel<float, 1024, 1, 128, true><<<grid, dim3(1024), 0, s>>>(a);
      else if (big16) ssm_update_bf16state_kernel<float, 1024, 1, 0, false><<<grid, dim3(1024), 0, s>>>(a);
      else ssm_update_bf16state_kernel<float, 256, 2, 0, false><<<grid, dim3(256), 0, s>>>(a);
    } else {
      if (exact128 && a.headdim == 64 && small16)
        ssm_update_bf16state_kernel<uint16_t, 512, 2, 128, true, 1, 64><<<grid, dim3(512), 0, s>>>(a);
      else if (exact128 && a.headdim == 64 && (!long16 || a.heads % 2 != 0))
        ssm_update_bf16state_kernel<uint16_t, 512, 2, 128, true, 1, 64, 0, true><<<grid, dim3(512), 0, s>>>(a);
      else if (exact128 && a.headdim == 64)
        ssm_update_bf16state_kernel<uint16_t, 1024, 2, 128, true, 2, 64, 0, true><<<dim3(a.heads / 2, a.batch), dim3(1024), 0, s>>>(a);
      else if (exact128 && a.heads % 2 == 0)
        ssm_update_bf16state_kernel<uint16_t, 1024, 2, 128, true, 2><<<dim3(a.heads / 2, a.batch), dim3(1024), 0, s>>>(a);
      else if (exact128) ssm_update_bf16state_kernel<uint16_t, 1024, 1, 128, true><<<grid, dim3(1024), 0, s>>>(a);
      else if (big16) ssm_update_bf16state_kernel<uint16_t, 1024, 1, 0, false><<<grid, dim3(1024), 0, s>>>(a);
      else ssm_update_bf16state_kernel<uint16_t, 256, 2, 0, false><<<grid, dim3(256), 0, s>>>(a);
    }
    return hipGetLastError();
  }
  if (a.dstate == 128 && a.headdim == 64) {
    const bool short_launch = uint64_t(a.heads) * a.batch < kShortLaunchTiles;
    if (a.dtype == 0) {
      if (short_launch) ssm_update_mamba2_kernel<float, 512, false><<<grid, dim3(512), 0, s>>>(a);
      else ssm_update_mamba2_kernel<float, 1024, true><<<grid, dim3(1024), 0, s>>>(a);
    } else {
      if (short_launch) ssm_update_mamba2_kernel<uint16_t, 512, false><<<grid, dim3(512), 0, s>>>(a);
      else ssm_update_mamba2_kernel<uint16_t, 1024, true><<<grid, dim3(1024), 0, s>>>(a);
    }
    return hipGetLastError();
  }
  if (a.dtype == 0) {
    if (exact128) ssm_update_kernel<float, 1024, 2, 128, true><<<grid, dim3(1024), 0, s>>>(a);
    else if (big) ssm_update_kernel<float, 1024, 2, 0, false><<<grid, dim3(1024), 0, s>>>(a);
    else ssm_update_kernel<float, 256, 4, 0, false><<<grid, dim3(256), 0, s>>>(a);
  } else {
    if (exact128) ssm_update_kernel<uint16_t, 1024, 2, 128, true><<<grid, dim3(1024), 0, s>>>(a);
    else if (big) ssm_update_kernel<uint16_t, 1024, 2, 0, false><<<grid, dim3(1024), 0, s>>>(a);
    else ssm_update_kernel<uint16_t, 256, 4, 0, false><<<grid, dim3(256), 0, s>>>(a);
  }
  return hipGetLastError();
}

}  // namespace avmp
