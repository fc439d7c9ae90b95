// Paged GQA decode attention on the CDNA4 matrix cores (bf16 in, fp32
// accumulate).  One wavefront per (KV head, chunk, request) serves the whole
// query group of that KV head, so K and V are read from HBM exactly once.
//
// The in-page layout is the matrix-core operand order, so operands go from
// global memory to registers to MFMA with no LDS staging and no conversion:
//   scores^T [16 tokens x 16 heads] = K [16 x D] . Q^T [D x 16]   (16x16x32 bf16,
//       A = K: lane l reads 16 bytes at  k_slab + kk*1024 + l*16  - linear)
//   out [16 heads x D] += P [16 x 16 tokens] . V [16 x D]         (16x16x16 bf16,
//       A = P is exactly the accumulator layout of scores^T; B = V: lane l
//       reads tokens 4*(l/16)..+3 of dim 16*nt + l%16, 8 bytes)
// Query heads beyond the group size are zero rows.  P is split into two bf16
// terms (hi + lo) so that the product keeps 16 mantissa bits; softmax statistics
// are fp32 in the log2 domain.
#include "kernels.hpp"

namespace avmp {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ uint32_t resident_tokens_m(const AttnLaunch& a, uint32_t r) {
  const uint32_t n = a.ctx[r];
  const uint64_t room = uint64_t(a.max_pages) * 16u;
  return n > room ? uint32_t(room) : n;
}

__device__ __forceinline__ uint64_t readlane64(uint64_t v, uint32_t lane) {
  const uint32_t lo = __builtin_amdgcn_readlane(uint32_t(v), lane);
  const uint32_t hi = __builtin_amdgcn_readlane(uint32_t(v >> 32), lane);
  return (uint64_t(hi) << 32) | lo;
}

template <int D>
struct PageRegs {
  uint4 k[D / 32];     // K operand tiles of one KV head
  uint2 v[D / 16];     // V operand tiles
};

template <int D>
__device__ __forceinline__ void load_page(PageRegs<D>& pr, const uint8_t* kslab, const uint8_t* vslab,
                                          uint32_t lane) {
#pragma unroll
  for (int kk = 0; kk < D / 32; ++kk)
    pr.k[kk] = *reinterpret_cast<const uint4*>(kslab + kk * 1024 + lane * 16);
  const uint32_t voff = (lane & 15) * 32 + (lane >> 4) * 8;
#pragma unroll
  for (int nt = 0; nt < D / 16; ++nt)
    pr.v[nt] = *reinterpret_cast<const uint2*>(vslab + nt * 512 + voff);
}

template <int D>
__global__ __launch_bounds__(64) void attn_mfma_kernel(AttnLaunch a) {
  constexpr int KK = D / 32;
  constexpr int NT = D / 16;
  const uint32_t g = blockIdx.x, c = blockIdx.y, r = blockIdx.z;
  const uint32_t lane = threadIdx.x, n = lane & 15, jg = lane >> 4;
  const uint32_t n_tok = resident_tokens_m(a, r);
  const uint32_t n_pages = (n_tok + 15) / 16;
  const uint32_t nch = chunk_count_for(n_pages);
  if (c >= nch) return;
  const uint32_t cp = chunk_pages_for(n_pages);
  const uint32_t p0 = c * cp;
  const uint32_t p1 = min(n_pages, p0 + cp);
  const uint32_t G = a.n_kv_heads, Hq = a.n_q_heads, Gq = Hq / G;

  // Q^T operand: lane (n = head in group, jg) holds dims 32*kk + 8*jg .. +7
  uint4 qreg[KK];
  {
    const uint16_t* qrow = static_cast<const uint16_t*>(a.q) + (size_t(r) * Hq + size_t(g) * Gq + n) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      qreg[kk] = n < Gq ? *reinterpret_cast<const uint4*>(qrow + 32 * kk + 8 * jg) : make_uint4(0, 0, 0, 0);
  }

  const float scale_log2 = kLog2e / sqrtf(float(D));
  float m = -INFINITY;        // running max of head n (log2 domain), same in all 4 lanes of the head
  float lsum = 0.f;           // this lane's share of the running sum of head n
  float4v acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = float4v{0.f, 0.f, 0.f, 0.f};

  const size_t kslab_off = size_t(g) * D * 32;                        // bytes: [D/8][16][8] bf16
  const size_t vslab_off = size_t(G) * D * 32 + size_t(g) * D * 32;   // bytes: [D][16] bf16

  auto process = [&](const PageRegs<D>& pr, uint32_t n_valid) {
    float4v s = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pr.k[kk]),
                                                  __builtin_bit_cast(bf16x8, qreg[kk]), s, 0, 0, 0);
    // s[i] = q_head(n) . k_token(4*jg + i)
    float sv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) sv[i] = (4 * jg + i < n_valid) ? s[i] * scale_log2 : -INFINITY;
    float pm = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
    pm = fmaxf(pm, __shfl_xor(pm, 16));
    pm = fmaxf(pm, __shfl_xor(pm, 32));
    const float m_new = fmaxf(m, pm);
    const float alpha = __builtin_amdgcn_exp2f(m - m_new);
    m = m_new;
    float p[4];
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      p[i] = __builtin_amdgcn_exp2f(sv[i] - m_new);
      hi[i] = __float_as_uint(p[i]) & 0xFFFF0000u;
      lo[i] = __float_as_uint(p[i] - __uint_as_float(hi[i]));
    }
    lsum = lsum * alpha + ((p[0] + p[1]) + (p[2] + p[3]));
    // two bf16 per register: low half = even token, high half = odd token
    const uint2 ahi = make_uint2((hi[0] >> 16) | hi[1], (hi[2] >> 16) | hi[3]);
    const uint2 alo = make_uint2((lo[0] >> 16) | (lo[1] & 0xFFFF0000u), (lo[2] >> 16) | (lo[3] & 0xFFFF0000u));
    const short4v a_hi = __builtin_bit_cast(short4v, ahi);
    const short4v a_lo = __builtin_bit_cast(short4v, alo);
    // accumulator row i of lane group jg belongs to head 4*jg + i, whose alpha sits in lane 4*jg + i
    float al[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) al[i] = __shfl(alpha, int(4 * jg + i));
    // tokens at or beyond n_valid hold arbitrary bits: clear them so 0 * x stays 0
    uint32_t mx = 0xFFFFFFFFu, my = 0xFFFFFFFFu;
    if (n_valid < 16) {
      mx = (4 * jg + 0 < n_valid ? 0x0000FFFFu : 0u) | (4 * jg + 1 < n_valid ? 0xFFFF0000u : 0u);
      my = (4 * jg + 2 < n_valid ? 0x0000FFFFu : 0u) | (4 * jg + 3 < n_valid ? 0xFFFF0000u : 0u);
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      float4v o = acc[nt];
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] *= al[i];
      const short4v vb = __builtin_bit_cast(short4v, make_uint2(pr.v[nt].x & mx, pr.v[nt].y & my));
      o = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_hi, vb, o, 0, 0, 0);
      o = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_lo, vb, o, 0, 0, 0);
      acc[nt] = o;
    }
  };

  // Pages are taken 64 at a time: each lane translates one handle, then the
  // wavefront walks them with one page of loads in flight ahead of the math.
  for (uint32_t base = p0; base < p1; base += 64) {
    const uint32_t cnt = min(64u, p1 - base);
    uint64_t my_off = ~0ull;
    if (lane < cnt) {
      my_off = translate_offset(a.P, a.handles[size_t(r) * a.max_pages + base + lane], 0);
      if (my_off == ~0ull) count_fault(a.P);
    }
    PageRegs<D> ra, rb;
    uint64_t off_a = readlane64(my_off, 0);
    if (off_a != ~0ull) load_page<D>(ra, a.P.arena + off_a + kslab_off, a.P.arena + off_a + vslab_off, lane);
    for (uint32_t i = 0; i < cnt; i += 2) {
      const uint64_t off_b = i + 1 < cnt ? readlane64(my_off, i + 1) : ~0ull;
      if (off_b != ~0ull) load_page<D>(rb, a.P.arena + off_b + kslab_off, a.P.arena + off_b + vslab_off, lane);
      if (off_a != ~0ull) process(ra, min(16u, n_tok - (base + i) * 16));
      off_a = i + 2 < cnt ? readlane64(my_off, i + 2) : ~0ull;
      if (off_a != ~0ull) load_page<D>(ra, a.P.arena + off_a + kslab_off, a.P.arena + off_a + vslab_off, lane);
      if (off_b != ~0ull) process(rb, min(16u, n_tok - (base + i + 1) * 16));
    }
  }

  // finish the row sums: head n's sum is spread over its 4 lanes
  lsum += __shfl_xor(lsum, 16);
  lsum += __shfl_xor(lsum, 32);
  float lh[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) lh[i] = __shfl(lsum, int(4 * jg + i));

  if (nch == 1) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t head = 4 * jg + i;
      if (head < Gq) {
        float* orow = a.o + (size_t(r) * Hq + size_t(g) * Gq + head) * D;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) orow[16 * nt + n] = lh[i] > 0.f ? acc[nt][i] / lh[i] : 0.f;
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t head = 4 * jg + i;
      if (head < Gq) {
        const size_t idx = (size_t(r) * a.max_chunks + c) * Hq + size_t(g) * Gq + head;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) a.part_o[idx * D + 16 * nt + n] = acc[nt][i];
      }
    }
    if (jg == 0 && n < Gq) {
      const size_t idx = (size_t(r) * a.max_chunks + c) * Hq + size_t(g) * Gq + n;
      a.part_ml[idx * 2] = m;
      a.part_ml[idx * 2 + 1] = lsum;
    }
  }
}

}  // namespace

bool attention_mfma_supported(const AttnLaunch& a) {
  if (a.dtype != 1) return false;
  if (a.head_dim != 64 && a.head_dim != 128 && a.head_dim != 256) return false;
  return a.n_q_heads / a.n_kv_heads <= 16;
}

hipError_t launch_attention_mfma(const AttnLaunch& a, hipStream_t s) {
  const dim3 grid(a.n_kv_heads, a.max_chunks, a.batch);
  switch (a.head_dim) {
    case 64: attn_mfma_kernel<64><<<grid, dim3(64), 0, s>>>(a); break;
    case 128: attn_mfma_kernel<128><<<grid, dim3(64), 0, s>>>(a); break;
    default: attn_mfma_kernel<256><<<grid, dim3(64), 0, s>>>(a); break;
  }
  return hipGetLastError();
}

}  // namespace avmp
