// The short causal depthwise convolution in front of the SSM recurrence, one token
// per request (the Mamba-2 layer of Background, "Hybrid Mamba-Transformer
// Architectures").  The block behind the request's handle keeps, after its
// recurrent state, the inputs of the previous K-1 tokens as [K-1][conv_dim]
// elements, oldest first.  Per channel c:
//     v = bias[c] + sum_k taps[k][c] * input_{t-(K-1)+k}[c],   out = v / (1 + exp(-v))
// then the window moves on by one token.  A lane owns 16 bytes of consecutive
// channels of one request and is the only one to touch their window, so the
// update in place needs no ordering.  Outputs are fp32, split into the x, B and C
// arrays the recurrence kernel reads.
#include "conv_window.hpp"
#include "kernels.hpp"

namespace avmp {

namespace {

template <typename E, int K>
__global__ __launch_bounds__(256) void conv_update_kernel(ConvLaunch a) {
  constexpr int V = Vec<E>::N;
  const uint32_t r = blockIdx.y;
  const uint32_t c0 = (blockIdx.x * 256u + threadIdx.x) * V;
  if (c0 >= a.conv_dim) return;
  const size_t row = size_t(a.conv_dim) * sizeof(E);
  ConvInputs<E, K> cv;
  cv.load_token(static_cast<const uint8_t*>(a.u) + (size_t(r) * a.conv_dim + c0) * sizeof(E),
                static_cast<const uint8_t*>(a.taps) + size_t(c0) * sizeof(E),
                static_cast<const uint8_t*>(a.bias) + size_t(c0) * sizeof(E), row);
  // a handle that does not translate is counted by the recurrence kernel, which skips the request
  const uint64_t off = translate_offset(a.P, a.handles[r], 1);
  if (off == ~0ull) return;
  uint8_t* win = a.P.arena + off + a.state_bytes + size_t(c0) * sizeof(E);
  cv.load_window(win, row);
  float out[V];
  cv.outputs(out);
  cv.advance(win, row);
  // channels [0, HP) are x, then N of B, then N of C; a lane's channels never straddle two of them
  const uint32_t hp = a.heads * a.headdim;
  float* dst;
  if (c0 < hp) dst = a.x + size_t(r) * hp + c0;
  else if (c0 < hp + a.dstate) dst = a.B + size_t(r) * a.dstate + (c0 - hp);
  else dst = a.C + size_t(r) * a.dstate + (c0 - hp - a.dstate);
#pragma unroll
  for (int i = 0; i < V; i += 4)
    *reinterpret_cast<float4*>(dst + i) = make_float4(out[i], out[i + 1], out[i + 2], out[i + 3]);
}

template <typename E>
hipError_t launch_typed(const ConvLaunch& a, hipStream_t s) {
  constexpr int V = Vec<E>::N;
  const dim3 grid((a.conv_dim / V + 255) / 256, a.batch);
  switch (a.taps_k) {
    case 2: conv_update_kernel<E, 2><<<grid, dim3(256), 0, s>>>(a); break;
    case 3: conv_update_kernel<E, 3><<<grid, dim3(256), 0, s>>>(a); break;
    case 4: conv_update_kernel<E, 4><<<grid, dim3(256), 0, s>>>(a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

bool conv_supported(uint32_t dtype, uint32_t taps_k, uint32_t heads, uint32_t headdim,
                    uint32_t dstate) {
  const uint32_t v = dtype == 0 ? 4 : 8;      // channels in 16 bytes
  return taps_k >= 2 && taps_k <= 4 && (uint64_t(heads) * headdim) % v == 0 && dstate % v == 0;
}

hipError_t launch_conv_update(const ConvLaunch& a, hipStream_t s) {
  if (a.batch == 0) return hipSuccess;
  if (!conv_supported(a.dtype, a.taps_k, a.heads, a.headdim, a.dstate) ||
      a.conv_dim != a.heads * a.headdim + 2 * a.dstate)
    return hipErrorInvalidValue;
  return a.dtype == 0 ? launch_typed<float>(a, s) : launch_typed<uint16_t>(a, s);
}

}  // namespace avmp
