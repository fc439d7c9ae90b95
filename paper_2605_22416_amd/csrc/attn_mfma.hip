// Paged GQA decode attention on the CDNA4 matrix cores (bf16 in, fp32
// accumulate).  A wavefront serves the whole query group of one KV head, so K
// and V are read from HBM exactly once.
//
// Work split.  For each KV head the (request, page) pairs of the batch, in
// logical order, form one sequence of pages; it is cut into runs of equal cost
// (a page costs one, starting a request a few) and wavefront w walks run w,
// crossing request boundaries as it goes.  A run that covers a whole request
// writes the output row; otherwise it leaves a partial result (un-normalised
// sum, running max, running sum) that the merge kernel combines in logical
// order.  Every wavefront does about the same work, so the launch has no tail,
// and the split is a function of the context lengths alone: physical placement
// and migration cannot change one bit of the result.  A one-block plan kernel
// computes the page prefix sums and each run's stretch once per decode step.
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

template <int D>
struct PageRegs {
  uint4 k[D / 32];     // K operand tiles of one KV head
  uint2 v[D / 16];     // V operand tiles
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// K and V are read once per step: non-temporal loads keep them from displacing
// lines that will be reused (measured +12 % on the page walk).
__device__ __forceinline__ uint4 load16_stream(const uint8_t* p) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 load8_stream(const uint8_t* p) {
  const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
  return make_uint2(v.x, v.y);
}

template <int D>
__device__ __forceinline__ void load_page(PageRegs<D>& pr, const uint8_t* kslab, const uint8_t* vslab,
                                          uint32_t lane) {
#pragma unroll
  for (int kk = 0; kk < D / 32; ++kk) pr.k[kk] = load16_stream(kslab + kk * 1024 + lane * 16);
  const uint32_t voff = (lane & 15) * 32 + (lane >> 4) * 8;
#pragma unroll
  for (int nt = 0; nt < D / 16; ++nt) pr.v[nt] = load8_stream(vslab + nt * 512 + voff);
}

__device__ __forceinline__ uint32_t pages_of(uint32_t ctx, uint32_t max_pages) {
  const uint32_t n = (ctx >> 4) + ((ctx & 15u) ? 1u : 0u);
  return n > max_pages ? max_pages : n;      // a context beyond the handle row is clamped
}

constexpr uint32_t kMinRunPages = 4;
// What starting a request costs a wavefront, in pages' worth of time: the query load
// that waits on the request index, the refill of the page pipeline, the output row.
constexpr uint32_t kRequestCost = 5;

// One block: page prefix sums over the batch and the cut of the batch's pages into
// runs of equal COST.  Request r costs kRequestCost + its pages; on the cost axis it
// sits at prefix[r] + kRequestCost * r, its page p at that + kRequestCost + p.  Run w
// takes the pages whose position falls into [w * cpw, (w + 1) * cpw): as pages they
// are still one contiguous stretch of the batch's page sequence, so desc[w] =
// (first request, first page in it, first and one-past-last index in that sequence).
// plan[0] = total pages, plan[1] = cost per run (cpw).
__global__ __launch_bounds__(1024) void attn_plan_kernel(const uint32_t* __restrict__ ctx, uint32_t batch,
                                                         uint32_t max_pages, uint32_t runs,
                                                         uint32_t append,
                                                         uint32_t* __restrict__ plan,
                                                         uint32_t* __restrict__ prefix,
                                                         uint4* __restrict__ desc) {
  __shared__ uint32_t sums[1024];
  const uint32_t tid = threadIdx.x;
  const uint32_t seg = (batch + 1023) / 1024;
  const uint32_t lo = min(batch, tid * seg), hi = min(batch, lo + seg);
  uint32_t local = 0;
  for (uint32_t r = lo; r < hi; ++r) local += pages_of(attended_tokens(ctx, r, append), max_pages);
  sums[tid] = local;
  __syncthreads();
  for (uint32_t off = 1; off < 1024; off <<= 1) {          // inclusive scan
    const uint32_t add = tid >= off ? sums[tid - off] : 0;
    __syncthreads();
    sums[tid] += add;
    __syncthreads();
  }
  uint32_t run = sums[tid] - local;                         // exclusive start of this segment
  for (uint32_t r = lo; r < hi; ++r) {
    prefix[r] = run;
    run += pages_of(attended_tokens(ctx, r, append), max_pages);
  }
  const uint32_t total = sums[1023];
  const uint64_t total_cost = uint64_t(total) + uint64_t(kRequestCost) * batch;
  // equal shares, but room for at least kMinRunPages pages: with few pages in the batch,
  // shorter runs would only add partial results to merge
  const uint64_t cpw = max(uint64_t(kMinRunPages + kRequestCost), (total_cost + runs - 1) / runs);
  if (tid == 0) {
    prefix[batch] = total;
    plan[0] = total;
    plan[1] = uint32_t(cpw);
  }
  __syncthreads();                                          // prefix[] visible to the block
  // first page at or after cost position c: (request, page in it, index in the page sequence)
  auto first_page_at = [&](uint64_t c, uint32_t* rq, uint32_t* pg) -> uint32_t {
    if (c >= total_cost) {
      *rq = batch;
      *pg = 0;
      return total;
    }
    // last r whose cost position prefix[r] + kRequestCost * r is <= c
    uint32_t a = 0, b = batch;
    while (b - a > 1) {
      const uint32_t mid = (a + b) / 2;
      if (uint64_t(prefix[mid]) + uint64_t(kRequestCost) * mid <= c) a = mid; else b = mid;
    }
    const uint64_t at = uint64_t(prefix[a]) + uint64_t(kRequestCost) * a + kRequestCost;   // its page 0
    const uint32_t p = c > at ? uint32_t(c - at) : 0;       // c < position of request a + 1, so p < its pages
    *rq = a;                                                // (or p = 0 in a request without pages: the
    *pg = p;                                                //  walk skips it)
    return prefix[a] + p;
  };
  for (uint32_t w = tid; w < runs; w += 1024) {
    uint32_t r0, p0, r1, p1;
    const uint32_t first = first_page_at(uint64_t(w) * cpw, &r0, &p0);
    const uint32_t last = first_page_at(uint64_t(w + 1) * cpw, &r1, &p1);
    desc[w] = make_uint4(r0, p0, first, last);
  }
}

// Translation of every KV handle the step will touch, for all attention layers at
// once: slots[layer][prefix[r] + page] = physical slot (0xFFFFFFFF if the handle does
// not resolve).  The table cannot change inside a step, so the attention waves read
// their run's slots as one contiguous load instead of walking handle -> table per
// page batch, and the table is consulted once per page instead of once per KV head.
__global__ __launch_bounds__(256) void attn_translate_kernel(DevPools P, const uint32_t* __restrict__ handles,
                                                             const uint32_t* __restrict__ ctx,
                                                             const uint32_t* __restrict__ prefix,
                                                             uint32_t batch, uint32_t max_pages,
                                                             uint32_t append, uint32_t* __restrict__ slots) {
  const uint32_t page = blockIdx.x * 256 + threadIdx.x, r = blockIdx.y, la = blockIdx.z;
  if (page >= pages_of(attended_tokens(ctx, r, append), max_pages)) return;
  const size_t cap = size_t(batch) * max_pages;
  const uint32_t h = handles[la * cap + size_t(r) * max_pages + page];
  const uint64_t off = translate_offset(P, h, 0);
  uint32_t slot = kDevUnmapped;
  if (off == ~0ull) count_fault(P);
  else slot = uint32_t(off / P.unit[0]);
  slots[la * cap + prefix[r] + page] = slot;
}

// At least two wavefronts per SIMD for head_dim up to 128 (256 registers each).
template <int D>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(D <= 128 ? 2 : 1)))
void attn_mfma_kernel(AttnLaunch a) {
  constexpr int KK = D / 32;
  constexpr int NT = D / 16;
  const uint32_t g = blockIdx.x, w = blockIdx.y;
  const uint32_t lane = threadIdx.x, n = lane & 15, jg = lane >> 4;
  const uint4 start = a.desc[w];
  uint64_t item = start.z;                     // position in the batch's page sequence
  const uint64_t item_end = start.w;
  if (item >= item_end) return;
  uint32_t r = start.x, page = start.y;
  // the run's first 64 slots (for the usual run lengths: all of them), requested before
  // anything that depends on the context lengths
  const uint32_t item0 = uint32_t(item);
  const uint32_t win_n = uint32_t(min(uint64_t(64), item_end - item));
  const uint32_t my_win = lane < win_n ? a.slots[item0 + lane] : kDevUnmapped;
  const uint64_t unit_kv = a.P.unit[0];
  const uint32_t G = a.n_kv_heads, Hq = a.n_q_heads, Gq = Hq / G;
  const float scale_log2 = kLog2e / sqrtf(float(D));
  const size_t kslab_off = size_t(g) * D * 32;                        // bytes: [D/8][16][8] bf16
  const size_t vslab_off = size_t(G) * D * 32 + size_t(g) * D * 32;   // bytes: [D][16] bf16

  while (item < item_end && r < a.batch) {
    const uint32_t n_ctx = attended_tokens(a.ctx, r, a.append);
    const uint32_t n_pages = pages_of(n_ctx, a.max_pages);
    if (page >= n_pages) {             // request without pages (or exhausted): next one
      ++r;
      page = 0;
      continue;
    }
    const uint32_t n_tok = min(n_ctx, n_pages * 16u);
    const uint32_t p0 = page;
    const uint32_t p1 = uint32_t(min(uint64_t(n_pages), uint64_t(page) + (item_end - item)));

    // Q^T operand: lane (n = head in group, jg) holds dims 32*kk + 8*jg .. +7
    uint4 qreg[KK];
    {
      const uint16_t* qrow =
          static_cast<const uint16_t*>(a.q) + (size_t(r) * Hq + size_t(g) * Gq + n) * D;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
        qreg[kk] = n < Gq ? *reinterpret_cast<const uint4*>(qrow + 32 * kk + 8 * jg)
                          : make_uint4(0, 0, 0, 0);
    }
    float m = -INFINITY;   // running max of head n (log2 domain), same in the head's 4 lanes
    float lsum = 0.f;      // this lane's share of the running sum of head n
    float4v acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = float4v{0.f, 0.f, 0.f, 0.f};

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
      const uint2 alo = make_uint2((lo[0] >> 16) | (lo[1] & 0xFFFF0000u),
                                   (lo[2] >> 16) | (lo[3] & 0xFFFF0000u));
      const short4v a_hi = __builtin_bit_cast(short4v, ahi);
      const short4v a_lo = __builtin_bit_cast(short4v, alo);
      // accumulator row i of lane group jg is head 4*jg + i, whose alpha sits in lane 4*jg + i
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
        const short4v vb =
            __builtin_bit_cast(short4v, make_uint2(pr.v[nt].x & mx, pr.v[nt].y & my));
        o = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_hi, vb, o, 0, 0, 0);
        o = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_lo, vb, o, 0, 0, 0);
        acc[nt] = o;
      }
    };

    // Pages are taken 64 at a time (one slot per lane), then the wavefront walks
    // them with two pages of loads in flight ahead of the math.
    for (uint32_t base = p0; base < p1; base += 64) {
      const uint32_t cnt = min(64u, p1 - base);
      const uint32_t it0 = uint32_t(item) + (base - p0);       // flattened index of page `base`
      uint32_t my_slot;
      if (it0 - item0 + cnt <= 64)                             // inside the preloaded window
        my_slot = __shfl(my_win, int((lane + (it0 - item0)) & 63));
      else
        my_slot = lane < cnt ? a.slots[it0 + lane] : kDevUnmapped;
      PageRegs<D> ra, rb, rc;
      const uint8_t* arena = a.P.arena;
      if (__ballot(lane < cnt && my_slot == kDevUnmapped) == 0) {
        // every handle of the batch translated: straight-line pipeline, three page
        // buffers, two pages of loads in flight ahead of the math
        auto fetch = [&](PageRegs<D>& pr, uint32_t i) {
          if (i < cnt) {
            const uint64_t off = uint64_t(__builtin_amdgcn_readlane(my_slot, i)) * unit_kv;
            load_page<D>(pr, arena + off + kslab_off, arena + off + vslab_off, lane);
          }
        };
        fetch(ra, 0);
        fetch(rb, 1);
        for (uint32_t i = 0; i < cnt; i += 3) {
          fetch(rc, i + 2);
          process(ra, min(16u, n_tok - (base + i) * 16));
          fetch(ra, i + 3);
          if (i + 1 < cnt) process(rb, min(16u, n_tok - (base + i + 1) * 16));
          fetch(rb, i + 4);
          if (i + 2 < cnt) process(rc, min(16u, n_tok - (base + i + 2) * 16));
        }
      } else {
        // some handle did not translate (counted by the translation kernel): skip those pages
        for (uint32_t i = 0; i < cnt; ++i) {
          const uint32_t slot = __builtin_amdgcn_readlane(my_slot, i);
          if (slot == kDevUnmapped) continue;
          const uint64_t off = uint64_t(slot) * unit_kv;
          load_page<D>(ra, arena + off + kslab_off, arena + off + vslab_off, lane);
          process(ra, min(16u, n_tok - (base + i) * 16));
        }
      }
    }

    // finish the row sums: head n's sum is spread over its 4 lanes
    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);
    float lh[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) lh[i] = __shfl(lsum, int(4 * jg + i));

    if (p0 == 0 && p1 == n_pages) {          // the run covers the whole request: final row
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
      // a run leaves at most two partial results: slot 1 for the piece that starts its
      // request, slot 0 for the piece that continues one
      const size_t slot = (size_t(g) * a.runs + w) * 2 + (p0 == 0 ? 1 : 0);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t head = 4 * jg + i;
        if (head < Gq) {
          const size_t idx = slot * Gq + head;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) a.part_o[idx * D + 16 * nt + n] = acc[nt][i];
        }
      }
      if (jg == 0 && n < Gq) {
        const size_t idx = slot * Gq + n;
        a.part_ml[idx * 2] = m;
        a.part_ml[idx * 2 + 1] = lsum;
      }
    }
    item += p1 - p0;
    page = 0;
    ++r;
  }
}

// Combines the partial results of one (query head, request) in logical (run) order.
// Workgroup of four wavefronts: up to 64 pieces (every request of an ordinary
// batch) are handled by the first alone; a request spread over more runs (one long
// request in a small batch) gives every wavefront each fourth group of 64 pieces
// and the four partial sums are added in wavefront order.
__global__ __launch_bounds__(256) void attn_merge_runs_kernel(AttnLaunch a) {
  __shared__ float part_sum[3][256];        // wavefronts 1..3: partial output row (head_dim <= 256)
  __shared__ float part_l[3];
  const uint32_t j = blockIdx.x, r = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t D = a.head_dim, Hq = a.n_q_heads, Gq = Hq / a.n_kv_heads;
  const uint32_t g = j / Gq, head = j % Gq;
  float* orow = a.o + (size_t(r) * Hq + j) * D;
  if (j == 0 && threadIdx.x == 0 &&
      uint64_t(attended_tokens(a.ctx, r, a.append)) > uint64_t(a.max_pages) * 16u)
    count_fault(a.P);
  const uint32_t start = a.prefix[r], end = a.prefix[r + 1];
  if (start == end) {                       // no resident tokens: zero row
    for (uint32_t d = threadIdx.x; d < D; d += 256) orow[d] = 0.f;
    return;
  }
  // the runs that hold the request's first and last page (positions on the plan's cost axis)
  const uint64_t cpw = a.plan[1];
  const uint64_t at = uint64_t(start) + uint64_t(kRequestCost) * r + kRequestCost;
  const uint32_t wa = uint32_t(at / cpw), wb = uint32_t((at + (end - start) - 1) / cpw);
  if (wa == wb) return;                     // one run covered it and wrote the row
  const uint32_t np = wb - wa + 1;
  const bool wide = np > 64;                // the same for the whole workgroup
  if (!wide && wave != 0) return;
  auto piece = [&](uint32_t k) -> size_t {  // first piece starts the request (slot 1)
    return ((size_t(g) * a.runs + wa + k) * 2 + (k == 0 ? 1 : 0)) * Gq + head;
  };
  // the row maximum over all pieces
  float M = -INFINITY;
  for (uint32_t k = lane; k < np; k += 64) M = fmaxf(M, a.part_ml[piece(k) * 2]);
  for (int o = 32; o; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
  // groups of 64 pieces: lane k holds piece k's weight, which is broadcast while the
  // partial outputs are summed in piece order
  float L = 0.f;
  float sum[4] = {0.f, 0.f, 0.f, 0.f};      // output dims lane, lane + 64, ...
  for (uint32_t base = wide ? 64 * wave : 0; base < np; base += wide ? 256 : 64) {
    const uint32_t cnt = min(64u, np - base);
    float wgt = 0.f;
    if (lane < cnt) {
      const size_t idx = piece(base + lane);
      wgt = exp2f(a.part_ml[idx * 2] - M);
      L += a.part_ml[idx * 2 + 1] * wgt;
    }
#pragma unroll
    for (uint32_t q = 0; q < 4; ++q) {
      const uint32_t d = 64 * q + lane;
      if (64 * q >= D) break;
      uint32_t k = 0;
      for (; k + 4 <= cnt; k += 4) {
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = a.part_o[piece(base + k + u) * D + d];
#pragma unroll
        for (int u = 0; u < 4; ++u) sum[q] += v[u] * __shfl(wgt, int(k + u));
      }
      for (; k < cnt; ++k) sum[q] += a.part_o[piece(base + k) * D + d] * __shfl(wgt, int(k));
    }
  }
  for (int o = 32; o; o >>= 1) L += __shfl_xor(L, o);
  if (wide) {
    if (wave != 0) {
#pragma unroll
      for (uint32_t q = 0; q < 4; ++q) part_sum[wave - 1][64 * q + lane] = sum[q];
      if (lane == 0) part_l[wave - 1] = L;
    }
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (uint32_t w = 0; w < 3; ++w) {
      L += part_l[w];
#pragma unroll
      for (uint32_t q = 0; q < 4; ++q) sum[q] += part_sum[w][64 * q + lane];
    }
  }
#pragma unroll
  for (uint32_t q = 0; q < 4; ++q)
    if (64 * q < D) orow[64 * q + lane] = L > 0.f ? sum[q] / L : 0.f;
}

}  // namespace

bool attention_mfma_supported(uint32_t dtype, uint32_t n_q_heads, uint32_t n_kv_heads,
                              uint32_t head_dim) {
  if (dtype != 1) return false;
  if (head_dim != 64 && head_dim != 128 && head_dim != 256) return false;
  return n_q_heads / n_kv_heads <= 16;
}

uint32_t attention_runs_per_head(uint32_t n_kv_heads) {
  // about 2048 wavefronts per launch: one full set of resident waves on 256 CUs
  const uint32_t runs = 2048 / n_kv_heads;
  return runs ? runs : 1;
}

hipError_t launch_attention_plan(const AttnLaunch& a, hipStream_t s) {
  attn_plan_kernel<<<dim3(1), dim3(1024), 0, s>>>(a.ctx, a.batch, a.max_pages, a.runs, a.append,
                                                  const_cast<uint32_t*>(a.plan),
                                                  const_cast<uint32_t*>(a.prefix),
                                                  const_cast<uint4*>(a.desc));
  return hipGetLastError();
}

hipError_t launch_attention_translate(const AttnLaunch& a, const uint32_t* handles_all,
                                      uint32_t n_attn, uint32_t* slots_all, hipStream_t s) {
  const dim3 grid((a.max_pages + 255) / 256, a.batch, n_attn);
  attn_translate_kernel<<<grid, dim3(256), 0, s>>>(a.P, handles_all, a.ctx, a.prefix, a.batch,
                                                   a.max_pages, a.append, slots_all);
  return hipGetLastError();
}

hipError_t launch_attention_mfma(const AttnLaunch& a, hipStream_t s) {
  const dim3 grid(a.n_kv_heads, a.runs);
  switch (a.head_dim) {
    case 64: attn_mfma_kernel<64><<<grid, dim3(64), 0, s>>>(a); break;
    case 128: attn_mfma_kernel<128><<<grid, dim3(64), 0, s>>>(a); break;
    default: attn_mfma_kernel<256><<<grid, dim3(64), 0, s>>>(a); break;
  }
  return hipGetLastError();
}

hipError_t launch_attention_merge_runs(const AttnLaunch& a, hipStream_t s) {
  attn_merge_runs_kernel<<<dim3(a.n_q_heads, a.batch), dim3(256), 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace avmp
