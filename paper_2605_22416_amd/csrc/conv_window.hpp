// One token of the short causal depthwise convolution in front of the SSM recurrence
// (the Mamba-2 layer of Background, "Hybrid Mamba-Transformer Architectures"), for the 16 bytes
// of consecutive channels a lane owns.  The block keeps, behind its recurrent state, the inputs
// of the previous K-1 tokens as [K-1][conv_dim] elements, oldest first.  Per channel c:
//     v = bias[c] + sum_k taps[k][c] * input_{t-(K-1)+k}[c],   out = v / (1 + exp(-v))
// Used by the stand-alone convolution kernel and by the recurrence kernels that do the
// convolution themselves, so that both compute the same bits.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace avmp {

template <typename E>
struct Vec;
template <>
struct Vec<float> {
  static constexpr int N = 4;
  float4 raw;
  __device__ float get(int i) const { return reinterpret_cast<const float*>(&raw)[i]; }
};
template <>
struct Vec<uint16_t> {
  static constexpr int N = 8;
  uint4 raw;
  __device__ float get(int i) const {
    const uint32_t w = reinterpret_cast<const uint32_t*>(&raw)[i >> 1];
    return (i & 1) ? __uint_as_float(w & 0xFFFF0000u) : __uint_as_float(w << 16);
  }
};

template <typename E>
__device__ __forceinline__ Vec<E> load_vec(const void* p) {
  Vec<E> v;
  v.raw = *static_cast<const decltype(v.raw)*>(p);
  return v;
}
template <typename E>
__device__ __forceinline__ void store_vec(void* p, const Vec<E>& v) {
  *static_cast<decltype(v.raw)*>(p) = v.raw;
}

// One channel: bias, taps and inputs oldest first.  Every kernel computes a channel through this
// one function, in this order of operations.
template <int K>
__device__ __forceinline__ float conv_channel(float bias, const float (&taps)[K], const float (&in)[K]) {
  float v = bias;
#pragma unroll
  for (int k = 0; k < K; ++k) v = fmaf(taps[k], in[k], v);
  return v / (1.f + expf(-v));
}

// What a lane needs for its channels: the window's K-1 rows and the new token, the K taps, the bias.
template <typename E, int K>
struct ConvInputs {
  Vec<E> in[K], w[K], b;
  // u, taps, bias: the lane's first channel in the new token's row, in tap row 0 and in the bias;
  // win: the same channel in row 0 of the window; row_bytes: conv_dim elements.  Two calls, because
  // only the window's address waits for the handle to be translated.
  __device__ __forceinline__ void load_token(const uint8_t* u, const uint8_t* taps, const uint8_t* bias,
                                             size_t row_bytes) {
#pragma unroll
    for (int k = 0; k < K; ++k) w[k] = load_vec<E>(taps + k * row_bytes);
    b = load_vec<E>(bias);
    in[K - 1] = load_vec<E>(u);
  }
  __device__ __forceinline__ void load_window(const uint8_t* win, size_t row_bytes) {
#pragma unroll
    for (int k = 0; k < K - 1; ++k) in[k] = load_vec<E>(win + k * row_bytes);
  }
  __device__ __forceinline__ void outputs(float (&out)[Vec<E>::N]) const {
#pragma unroll
    for (int i = 0; i < Vec<E>::N; ++i) {
      float x[K], t[K];
#pragma unroll
      for (int k = 0; k < K; ++k) {
        x[k] = in[k].get(i);
        t[k] = w[k].get(i);
      }
      out[i] = conv_channel<K>(b.get(i), t, x);
    }
  }
  // the window moves on: row k takes row k+1, the last row takes the new token
  __device__ __forceinline__ void advance(uint8_t* win, size_t row_bytes) const {
#pragma unroll
    for (int k = 0; k < K - 1; ++k) store_vec<E>(win + k * row_bytes, in[k + 1]);
  }
};

}  // namespace avmp
