// gfx950 kernels of the hybrid decode path: table maintenance, translation,
// shape-generic paged GQA decode attention (vector ALU), the chunk merge and the
// migration copy + remap.
#include "kernels.hpp"

#include <cmath>

namespace avmp {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

// ---------------------------------------------------------------------------
// table maintenance
// ---------------------------------------------------------------------------
__global__ void table_update_kernel(uint32_t* __restrict__ table,
                                    const TableUpdate* __restrict__ upd, uint32_t n) {
  // Updates are applied in list order per index: one thread walks nothing but
  // its own entry, and the host never queues two updates of one index in one
  // batch without ordering them (it coalesces to the last value first).
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) table[upd[i].index] = upd[i].slot;
}

// one workgroup's share of clearing a unit (the grid's x dimension shares the unit out)
__device__ __forceinline__ void zero_unit(const DevPools& P, int pool, uint32_t slot) {
  const uint64_t off = pool == 0 ? uint64_t(slot) * P.unit[0]
                                 : P.usable - (uint64_t(slot) + 1) * P.unit[1];
  uint4* dst = reinterpret_cast<uint4*>(P.arena + off);
  const uint64_t n16 = P.unit[pool] / 16;
  const uint4 z = make_uint4(0, 0, 0, 0);
  // plain stores: with the non-temporal hint this fill measured 24.5 us against 22.4 us
  for (uint64_t i = uint64_t(blockIdx.x) * 256 + threadIdx.x; i < n16; i += uint64_t(gridDim.x) * 256)
    dst[i] = z;
}

__global__ __launch_bounds__(256) void zero_units_kernel(DevPools P, int pool,
                                                         const uint32_t* __restrict__ slots) {
  const uint32_t slot = slots[blockIdx.y];
  if (slot >= P.capacity[pool]) return;     // freed and migrated away before the flush
  zero_unit(P, pool, slot);
}

// A flush whose lists fit the kernel arguments, one launch: rows 0 .. n_zero-1 of the grid
// clear one SSM block each, the row behind them writes the table entries.  The two do not
// touch the same memory; the capacity a slot is checked against is the host's (the device's
// copy may be among the entries being written).
__global__ __launch_bounds__(256) void flush_inline_kernel(InlineFlush f) {
  if (blockIdx.y == f.n_zero) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i < f.n_upd) f.table[f.upd[i].index] = f.upd[i].slot;
    return;
  }
  const uint32_t slot = f.zero[blockIdx.y];
  if (slot >= f.ssm_capacity) return;
  zero_unit(f.P, 1, slot);
}

__global__ void translate_kernel(DevPools P, const uint32_t* __restrict__ handles, uint32_t n,
                                 uint64_t* __restrict__ out) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const uint32_t h = handles[i];
  const uint32_t pool = h >> 30;
  out[i] = pool < 2 ? translate_offset(P, h, pool) : ~0ull;
}

// ---------------------------------------------------------------------------
// migration: copy each live unit out of the vacated range, then point its
// table entry at the new slot (Method, "Dynamic Pool Rebalancing"; the copy is
// what a single arena needs in place of the prototype's oversized tensors).
// Source slots lie at or above the new capacity and destinations below it, so
// no two copies overlap.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void copy_unit(const DevPools& P, uint32_t* __restrict__ table, int pool,
                                          const Move mv) {
  const uint64_t unit = P.unit[pool];
  const uint64_t so = pool == 0 ? uint64_t(mv.src_slot) * unit : P.usable - (uint64_t(mv.src_slot) + 1) * unit;
  const uint64_t dof = pool == 0 ? uint64_t(mv.dst_slot) * unit : P.usable - (uint64_t(mv.dst_slot) + 1) * unit;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4* __restrict__ src = reinterpret_cast<const u32x4*>(P.arena + so);
  u32x4* __restrict__ dst = reinterpret_cast<u32x4*>(P.arena + dof);
  const uint64_t n16 = unit / 16;
  const uint64_t stride = uint64_t(gridDim.x) * 256;
  uint64_t i = uint64_t(blockIdx.x) * 256 + threadIdx.x;
  // four independent 16-byte loads in flight per lane; every byte is touched once, so both
  // directions carry the non-temporal hint (16384 pages of 64 KiB: 351 us in these kernels;
  // with 1024-thread workgroups 371 us)
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride),
                c = __builtin_nontemporal_load(src + i + 2 * stride),
                d = __builtin_nontemporal_load(src + i + 3 * stride);
    __builtin_nontemporal_store(a, dst + i);
    __builtin_nontemporal_store(b, dst + i + stride);
    __builtin_nontemporal_store(c, dst + i + 2 * stride);
    __builtin_nontemporal_store(d, dst + i + 3 * stride);
  }
  for (; i < n16; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
  if (blockIdx.x == 0 && threadIdx.x == 0) table[P.vid_base[pool] + mv.vid] = mv.dst_slot;
}

__global__ __launch_bounds__(256) void migrate_copy_kernel(DevPools P, uint32_t* __restrict__ table,
                                                           int pool, const Move* __restrict__ moves) {
  copy_unit(P, table, pool, moves[blockIdx.y]);
}

// the same with the move list in the kernel arguments (short migrations)
__global__ __launch_bounds__(256) void migrate_copy_inline_kernel(InlineMoves m) {
  copy_unit(m.P, m.table, m.pool, m.mv[blockIdx.y]);
}

// ---------------------------------------------------------------------------
// KV append: the new token's K and V rows go into token slot ctx % 16 of page
// ctx / 16 (append-only KV behaviour: Background, "KV Cache and SSM State
// Management").  The caller has allocated that page; the in-page layout is the
// one the attention kernels read.  One workgroup per request.
// ---------------------------------------------------------------------------
template <typename E>
__global__ __launch_bounds__(256) void kv_append_kernel(AttnLaunch a) {
  const uint32_t r = blockIdx.x, tid = threadIdx.x;
  const uint32_t t = a.ctx[r];
  const uint32_t page = t / 16, slot = t % 16;
  if (page >= a.max_pages) {
    if (tid == 0) count_fault(a.P);
    return;
  }
  const uint64_t off = translate_offset(a.P, a.handles[size_t(r) * a.max_pages + page], 0);
  if (off == ~0ull) {
    if (tid == 0) count_fault(a.P);
    return;
  }
  const uint32_t D = a.head_dim, G = a.n_kv_heads;
  constexpr uint32_t X = 16 / sizeof(E);
  E* pg = reinterpret_cast<E*>(a.P.arena + off);
  const E* kn = static_cast<const E*>(a.k_new) + size_t(r) * G * D;
  const E* vn = static_cast<const E*>(a.v_new) + size_t(r) * G * D;
  for (uint32_t i = tid; i < G * D; i += 256) {
    const uint32_t g = i / D, d = i % D;
    pg[((size_t(g) * (D / X) + d / X) * 16 + slot) * X + d % X] = kn[i];
    pg[size_t(G) * 16 * D + (size_t(g) * D + d) * 16 + slot] = vn[i];
  }
}

// ---------------------------------------------------------------------------
// shape-generic paged GQA decode attention: one wavefront per (query head,
// chunk, request); the wavefronts of up to 16 query heads that share a KV head
// form one workgroup, so they walk the same pages at the same time on one
// compute unit and the group's K and V are fetched into its cache once, not once
// per query head.  Lane = (token t = lane%16, dim quarter = lane/16) for the
// scores; lane = dim for the weighted sum of V.  Online softmax in the log2
// domain, fp32 throughout.  Used for fp32 pools and for head shapes the
// matrix-core kernel does not take.
// ---------------------------------------------------------------------------
// Tokens of request r that the handle row can cover: a context longer than
// max_pages pages is the caller's mistake; it is clamped (and counted as a
// fault by the merge kernel) so that the handle row is never read past its end.
__device__ __forceinline__ uint32_t resident_tokens(const AttnLaunch& a, uint32_t r) {
  const uint32_t n = attended_tokens(a.ctx, r, a.append);
  const uint64_t room = uint64_t(a.max_pages) * 16u;
  return n > room ? uint32_t(room) : n;
}

constexpr uint32_t kGenericHeadsPerBlock = 16;

// one 16-byte group of elements as floats
template <typename E>
__device__ __forceinline__ void load_group(const E* p, float* out);
template <>
__device__ __forceinline__ void load_group<float>(const float* p, float* out) {
  const float4 v = *reinterpret_cast<const float4*>(p);
  out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}
template <>
__device__ __forceinline__ void load_group<uint16_t>(const uint16_t* p, float* out) {
  const uint4 v = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = __uint_as_float(w[i] << 16);
    out[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
  }
}

template <typename E>
__global__ __launch_bounds__(64 * kGenericHeadsPerBlock) void attn_generic_kernel(AttnLaunch a) {
  const uint32_t c = blockIdx.y, r = blockIdx.z;
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t n_tok = resident_tokens(a, r);
  const uint32_t n_pages = (n_tok + 15) / 16;
  const uint32_t nch = chunk_count_for(n_pages);
  if (c >= nch) return;
  const uint32_t cp = chunk_pages_for(n_pages);
  const uint32_t p0 = c * cp;
  const uint32_t p1 = min(n_pages, p0 + cp);
  const uint32_t D = a.head_dim, G = a.n_kv_heads, Hq = a.n_q_heads;
  // blockIdx.x = (KV head, slice of up to 16 heads of its query group)
  const uint32_t Gq = Hq / G, slices = (Gq + kGenericHeadsPerBlock - 1) / kGenericHeadsPerBlock;
  const uint32_t g = blockIdx.x / slices;
  const uint32_t in_group = (blockIdx.x % slices) * kGenericHeadsPerBlock + wave;
  const bool has_head = in_group < Gq;
  const uint32_t j = g * Gq + in_group;
  constexpr uint32_t X = 16 / sizeof(E);

  __shared__ float q_all[kGenericHeadsPerBlock][256];
  float* const qs = q_all[wave];
  if (has_head) {
    const E* qrow = static_cast<const E*>(a.q) + (size_t(r) * Hq + j) * D;
    for (uint32_t d = lane; d < D; d += 64) qs[d] = load_elem<E>(qrow + d);
  }
  __syncthreads();
  if (!has_head) return;

  const float scale_log2 = kLog2e / sqrtf(float(D));
  const uint32_t t = lane & 15, dq = lane >> 4;
  const uint32_t DQ = D / 4;
  float m = -INFINITY, l = 0.f;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};

  // the next page's handle is translated while this page is worked on
  auto offset_of = [&](uint32_t page) -> uint64_t {
    return translate_offset(a.P, a.handles[size_t(r) * a.max_pages + page], 0);
  };
  uint64_t off_next = offset_of(p0);
  for (uint32_t page = p0; page < p1; ++page) {
    const uint64_t off = off_next;
    if (page + 1 < p1) off_next = offset_of(page + 1);
    if (off == ~0ull) {                         // wave-uniform: skip the page, count it
      if (lane == 0) count_fault(a.P);
      continue;
    }
    const E* pg = reinterpret_cast<const E*>(a.P.arena + off);
    const uint32_t n_valid = min(16u, n_tok - page * 16);
    const E* kbase = pg + size_t(g) * D * 16;                       // [D/X][16][X]
    float s = 0.f;
    if (D % (4 * X) == 0) {
      // a lane's quarter of the dims is whole 16-byte groups: one load per group, and the
      // 16 token lanes of a group read 256 consecutive bytes
      for (uint32_t dg = dq * (DQ / X); dg < (dq + 1) * (DQ / X); ++dg) {
        float kf[X];
        load_group<E>(kbase + (size_t(dg) * 16 + t) * X, kf);
#pragma unroll
        for (uint32_t i = 0; i < X; ++i) s += qs[dg * X + i] * kf[i];
      }
    } else {                                    // head_dim is a multiple of X, so of four
      for (uint32_t d = dq * DQ; d < (dq + 1) * DQ; ++d)
        s += qs[d] * load_elem<E>(kbase + ((d / X) * 16 + t) * X + d % X);
    }
    s += __shfl_xor(s, 16);
    s += __shfl_xor(s, 32);
    s = (t < n_valid) ? s * scale_log2 : -INFINITY;                 // tail slots never count
    // the 16 token lanes of a row of the wavefront: maxima and sums by moves inside the row
    const float m_new = fmaxf(m, max_row16(s));
    const float alpha = exp2f(m - m_new);
    const float p = exp2f(s - m_new);
    l = l * alpha + sum_row16(p);
    m = m_new;
    const E* vbase = pg + size_t(G) * 16 * D + size_t(g) * D * 16;  // [D][16]
    float pt[16];
#pragma unroll
    for (int tt = 0; tt < 16; ++tt)         // every row of the wavefront holds the same 16 weights
      pt[tt] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(p), tt));
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t d = lane + 64 * i;
      if (d < D) {
        // the 16 tokens of one dim lie side by side; slots beyond the tail hold anything
        float vf[16];
#pragma unroll
        for (uint32_t x = 0; x < 16 / X; ++x) load_group<E>(vbase + size_t(d) * 16 + x * X, vf + x * X);
        float sum = acc[i] * alpha;
#pragma unroll
        for (int tt = 0; tt < 16; ++tt) sum += pt[tt] * (uint32_t(tt) < n_valid ? vf[tt] : 0.f);
        acc[i] = sum;
      }
    }
  }

  if (nch == 1) {
    float* orow = a.o + (size_t(r) * Hq + j) * D;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t d = lane + 64 * i;
      if (d < D) orow[d] = l > 0.f ? acc[i] / l : 0.f;
    }
  } else {
    const size_t idx = (size_t(r) * a.max_chunks + c) * Hq + j;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t d = lane + 64 * i;
      if (d < D) a.part_o[idx * D + d] = acc[i];
    }
    if (lane == 0) {
      a.part_ml[idx * 2] = m;
      a.part_ml[idx * 2 + 1] = l;
    }
  }
}

// Merge of per-chunk partial results in logical chunk order (so the result is a
// function of the logical batch alone).  One wavefront per (query head, request).
__global__ __launch_bounds__(64) void attn_merge_kernel(AttnLaunch a) {
  const uint32_t j = blockIdx.x, r = blockIdx.y, lane = threadIdx.x;
  if (j == 0 && lane == 0 && uint64_t(attended_tokens(a.ctx, r, a.append)) > uint64_t(a.max_pages) * 16u)
    count_fault(a.P);
  const uint32_t n_pages = (resident_tokens(a, r) + 15) / 16;
  const uint32_t nch = chunk_count_for(n_pages);
  const uint32_t D = a.head_dim, Hq = a.n_q_heads;
  float* orow = a.o + (size_t(r) * Hq + j) * D;
  if (nch == 0) {
    for (uint32_t d = lane; d < D; d += 64) orow[d] = 0.f;
    return;
  }
  if (nch == 1) return;            // written directly by the attention kernel
  const size_t base = (size_t(r) * a.max_chunks) * Hq + j;
  // lane c holds chunk c's statistics (nch <= 64); the weights are broadcast
  // while the partial outputs are summed in chunk order
  float mc = -INFINITY, lc = 0.f;
  if (lane < nch) {
    mc = a.part_ml[(base + size_t(lane) * Hq) * 2];
    lc = a.part_ml[(base + size_t(lane) * Hq) * 2 + 1];
  }
  float M = mc;
  for (int o = 32; o; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
  const float w = lane < nch ? exp2f(mc - M) : 0.f;
  float L = lc * w;
  for (int o = 32; o; o >>= 1) L += __shfl_xor(L, o);
  for (uint32_t d0 = 0; d0 < D; d0 += 64) {
    const uint32_t d = d0 + lane;
    float sum = 0.f;
    uint32_t c = 0;
    for (; c + 4 <= nch; c += 4) {
      float v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        v[u] = d < D ? a.part_o[(base + size_t(c + u) * Hq) * D + d] : 0.f;
#pragma unroll
      for (int u = 0; u < 4; ++u) sum += v[u] * __shfl(w, int(c + u));
    }
    for (; c < nch; ++c) {
      const float v = d < D ? a.part_o[(base + size_t(c) * Hq) * D + d] : 0.f;
      sum += v * __shfl(w, int(c));
    }
    if (d < D) orow[d] = L > 0.f ? sum / L : 0.f;
  }
}

}  // namespace

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
hipError_t launch_table_updates(uint32_t* table, const TableUpdate* upd, uint32_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  table_update_kernel<<<dim3((n + 255) / 256), dim3(256), 0, s>>>(table, upd, n);
  return hipGetLastError();
}

hipError_t launch_zero_units(const DevPools& P, int pool, const uint32_t* slots, uint32_t n,
                             hipStream_t s) {
  if (n == 0) return hipSuccess;
  const uint64_t n16 = P.unit[pool] / 16;
  uint32_t gx = uint32_t((n16 + 256 * 8 - 1) / (256 * 8));
  if (gx == 0) gx = 1;
  for (uint32_t done = 0; done < n; done += 65535) {
    const uint32_t cnt = n - done < 65535 ? n - done : 65535;
    zero_units_kernel<<<dim3(gx, cnt), dim3(256), 0, s>>>(P, pool, slots + done);
  }
  return hipGetLastError();
}

hipError_t launch_flush_inline(const InlineFlush& f, hipStream_t s) {
  if (f.n_upd == 0 && f.n_zero == 0) return hipSuccess;
  if (f.n_upd > kInlineUpdates || f.n_zero > kInlineZero) return hipErrorInvalidValue;
  const uint64_t n16 = f.P.unit[1] / 16;
  uint32_t gx = f.n_zero ? uint32_t((n16 + 256 * 8 - 1) / (256 * 8)) : 1;
  const uint32_t ux = (f.n_upd + 255) / 256;
  if (gx < ux) gx = ux;
  if (gx == 0) gx = 1;
  flush_inline_kernel<<<dim3(gx, f.n_zero + 1), dim3(256), 0, s>>>(f);
  return hipGetLastError();
}

hipError_t launch_migrate_copy_inline(const InlineMoves& m, hipStream_t s) {
  if (m.n == 0) return hipSuccess;
  if (m.n > kInlineMoves || (m.pool != 0 && m.pool != 1)) return hipErrorInvalidValue;
  const uint64_t n16 = m.P.unit[m.pool] / 16;
  uint32_t gx = uint32_t((n16 + 256 * 4 - 1) / (256 * 4));    // 16 KiB per workgroup
  if (gx == 0) gx = 1;
  migrate_copy_inline_kernel<<<dim3(gx, m.n), dim3(256), 0, s>>>(m);
  return hipGetLastError();
}

hipError_t launch_migrate_copy(const DevPools& P, uint32_t* table, int pool, const Move* moves,
                               uint32_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const uint64_t n16 = P.unit[pool] / 16;
  uint32_t gx = uint32_t((n16 + 256 * 4 - 1) / (256 * 4));    // 16 KiB per workgroup
  if (gx == 0) gx = 1;
  for (uint32_t done = 0; done < n; done += 65535) {
    const uint32_t cnt = n - done < 65535 ? n - done : 65535;
    migrate_copy_kernel<<<dim3(gx, cnt), dim3(256), 0, s>>>(P, table, pool, moves + done);
  }
  return hipGetLastError();
}

hipError_t launch_translate(const DevPools& P, const uint32_t* handles, uint32_t n, uint64_t* out,
                            hipStream_t s) {
  if (n == 0) return hipSuccess;
  translate_kernel<<<dim3((n + 255) / 256), dim3(256), 0, s>>>(P, handles, n, out);
  return hipGetLastError();
}

hipError_t launch_kv_append(const AttnLaunch& a, hipStream_t s) {
  if (a.batch == 0) return hipSuccess;
  if (a.dtype == 0)
    kv_append_kernel<float><<<dim3(a.batch), dim3(256), 0, s>>>(a);
  else
    kv_append_kernel<uint16_t><<<dim3(a.batch), dim3(256), 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_attention(const AttnLaunch& a, hipStream_t s) {
  if (a.batch == 0) return hipSuccess;
  if (a.plan != nullptr) return launch_attention_mfma(a, s);
  const uint32_t group = a.n_q_heads / a.n_kv_heads;
  const uint32_t slices = (group + kGenericHeadsPerBlock - 1) / kGenericHeadsPerBlock;
  const uint32_t waves = group < kGenericHeadsPerBlock ? group : kGenericHeadsPerBlock;
  const dim3 grid(a.n_kv_heads * slices, a.max_chunks, a.batch);
  if (a.dtype == 0)
    attn_generic_kernel<float><<<grid, dim3(64 * waves), 0, s>>>(a);
  else
    attn_generic_kernel<uint16_t><<<grid, dim3(64 * waves), 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_attention_merge(const AttnLaunch& a, hipStream_t s) {
  if (a.batch == 0) return hipSuccess;
  if (a.plan != nullptr) return launch_attention_merge_runs(a, s);
  attn_merge_kernel<<<dim3(a.n_q_heads, a.batch), dim3(64), 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace avmp
