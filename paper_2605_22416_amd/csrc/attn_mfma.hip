// Paged GQA decode attention on the CDNA4 matrix cores (bf16 in, fp32
// accumulate).  A wavefront serves the whole query group of one KV head, so K
// and V are read from HBM exactly once.
//
// Work split.  For each KV head the (request, page) pairs of the batch, in
// logical order, form one sequence of pages; it is cut into runs of equal cost
// (a page costs one, a request at least a few however short it is) and wavefront w
// walks run w, crossing request boundaries as it goes.  A run that covers a whole
// request writes the output row; otherwise it leaves a partial result
// (un-normalised sum, running max, running sum) that the merge kernel combines in
// logical (run) order, one workgroup per (request, KV head).  Every wavefront does
// about the same work, and the split is a function of the context lengths alone:
// physical placement and migration cannot change one bit of the result.  One
// preparation kernel per decode step holds a plan block (prefix sums of pages and
// costs, each run's stretch) and, beside it, the blocks that translate every KV
// handle of every attention layer to its slot.
//
// Why the merge is a launch of its own.  Letting the wavefront that completes a
// request (an arrival counter per request) merge inside the attention kernel was
// built and measured at the Jamba-shaped batch of 64: with device-scope fences around
// the counter the launch went from 46 to 165 us (on this chip such a fence writes
// back and invalidates a whole L2, and 2048 wavefronts do it at once); with
// device-scope loads and stores for the partial results and no fence, 59 us, against
// 46 + 4 us for the two launches.  All wavefronts end together, so the write-through
// stores, the counter round trip and the merge loads pile up at the end of the
// launch where nothing overlaps them.
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

// What a request costs the wavefronts that walk it, in pages' worth of time: its pages, but
// never less than kRequestFloor (a request of one page still waits for its query rows, fills
// the page pipeline and writes its output rows, and a wavefront that crosses many such
// requests is bound by those waits), plus kRequestCost for the start.  A request without
// pages costs nothing: no wavefront visits it.  Measured per layer (floor, start) = (6, 2) /
// (6, 1) / (8, 1) / (4, 2) / (8, 0), and pages + 5 for every request: 256 requests, half of
// them 1-4 pages long, 59.3 / 60.3 / 59.9 / 61.7 / 60.6, and 59.9 us; 64 requests of 8-128
// pages 48.2 / 48.5 / 48.7 / 48.6 / 49.9, and 49.1 us.
constexpr uint32_t kRequestFloor = 6;
constexpr uint32_t kRequestCost = 2;
__host__ __device__ __forceinline__ uint32_t request_cost(uint32_t pages) {
  if (pages == 0) return 0;
  return (pages < kRequestFloor ? kRequestFloor : pages) + kRequestCost;
}

// Preparation of a decode step's attention layers, one launch.
//
// Block 0 is the plan.  It computes, over the batch, the prefix sums of the requests' pages
// and of their costs (request_cost), and cuts the cost axis into runs of equal length cpw.
// Request r sits at pos[r] on that axis; what it costs beyond its pages comes first, then
// its pages, one unit each.  Run w takes the pages whose position falls into
// [w * cpw, (w + 1) * cpw): as pages they are still one contiguous stretch of the batch's
// page sequence, so desc[w] = (first request, first page in it, first and one-past-last
// index in that sequence).  plan[0] = total pages, plan[1] = cpw.  It also writes the zero
// output rows of requests without resident tokens and counts contexts that exceed the
// handle row.
//
// Every other block translates 256 entries of the handle tables of all attention
// layers: slots[layer][r][page] = physical slot (0xFFFFFFFF if the handle does not
// resolve, which is counted).  The table cannot change inside a step, so it is
// consulted once per page instead of once per page per KV head, and the attention
// waves read plain slots.  The two parts do not depend on each other.
struct PrepareArgs {
  DevPools P;
  const uint32_t* ctx;        // [batch]
  const uint32_t* handles;    // [n_attn][batch][max_pages]
  uint32_t* slots;            // [n_attn][batch][max_pages] out
  uint32_t* plan;             // [2] out
  uint32_t* prefix;           // [batch + 1] out: pages before each request
  uint32_t* pos;              // [batch + 1] out: cost before each request
  uint4* desc;                // [runs] out
  float* o;                   // [n_attn][batch][n_q_heads * head_dim]: rows of empty requests
  uint32_t batch, max_pages, runs, append, n_attn, row_floats;
  uint32_t pitch_log2, page_tiles, row_groups, n_tiles;   // translation blocks: see attn_prepare_kernel
};
constexpr uint32_t kPrepareBlocks = 2048;     // translating blocks of a launch, at most

__device__ void plan_block(const PrepareArgs& a) {
  // per thread: (cost << 32 | pages) summed over its segment of the batch, inclusive
  __shared__ uint64_t sums[1024];
  __shared__ uint64_t wave_sums[16];
  const uint32_t tid = threadIdx.x, batch = a.batch, runs = a.runs;
  const uint32_t seg = (batch + 1023) / 1024;
  const uint32_t lo = min(batch, tid * seg), hi = min(batch, lo + seg);
  auto packed = [&](uint32_t r) -> uint64_t {
    const uint32_t pg = pages_of(attended_tokens(a.ctx, r, a.append), a.max_pages);
    return (uint64_t(request_cost(pg)) << 32) | pg;
  };
  uint64_t local = 0;
  for (uint32_t r = lo; r < hi; ++r) local += packed(r);
  // inclusive scan over the 1024 threads: inside each wavefront, then over the 16 wavefronts
  uint64_t incl = local;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint64_t up = __shfl_up(incl, off);
    if ((tid & 63u) >= uint32_t(off)) incl += up;
  }
  if ((tid & 63u) == 63u) wave_sums[tid >> 6] = incl;
  __syncthreads();
  for (uint32_t wv = 0; wv < (tid >> 6); ++wv) incl += wave_sums[wv];
  sums[tid] = incl;
  uint64_t run = incl - local;                              // exclusive start of this segment
  for (uint32_t r = lo; r < hi; ++r) {
    a.prefix[r] = uint32_t(run);
    a.pos[r] = uint32_t(run >> 32);
    run += packed(r);
  }
  __syncthreads();                                          // sums[], prefix[], pos[] visible to the block
  const uint32_t total = uint32_t(sums[1023]);
  const uint64_t total_cost = sums[1023] >> 32;
  // equal shares, but never shorter than the least a request costs: with few pages in the
  // batch, shorter runs would only add partial results to merge
  const uint64_t cpw = max(uint64_t(kRequestFloor + kRequestCost), (total_cost + runs - 1) / runs);
  if (tid == 0) {
    a.prefix[batch] = total;
    a.pos[batch] = uint32_t(total_cost);
    a.plan[0] = total;
    a.plan[1] = uint32_t(cpw);
  }
  // pages and cost before request r: up to 1024 requests every thread's segment is one request
  // and the sums in shared memory answer; beyond that the arrays just written do
  auto before = [&](uint32_t r) -> uint64_t {
    if (seg == 1) return r == 0 ? 0ull : sums[r - 1];
    return (uint64_t(a.pos[r]) << 32) | a.prefix[r];
  };
  // first page at or after cost position c: (request, page in it, index in the page sequence)
  auto first_page_at = [&](uint64_t c, uint32_t* rq, uint32_t* pg) -> uint32_t {
    if (c >= total_cost) {
      *rq = batch;
      *pg = 0;
      return total;
    }
    // last r whose position is <= c; requests without pages have no width, so this is never
    // one of them (c < total_cost: a request with pages follows any such position)
    uint32_t lo_r = 0, hi_r = batch;
    while (hi_r - lo_r > 1) {
      const uint32_t mid = (lo_r + hi_r) / 2;
      if ((before(mid) >> 32) <= c) lo_r = mid; else hi_r = mid;
    }
    const uint64_t here = before(lo_r);
    const uint64_t next = lo_r + 1 < batch ? before(lo_r + 1) : sums[1023];
    const uint32_t pages = uint32_t(next) - uint32_t(here);
    // its page 0 sits behind what the request costs beyond its pages
    const uint64_t at = (here >> 32) + (request_cost(pages) - pages);
    const uint32_t p = c > at ? uint32_t(c - at) : 0;       // c < position of the next request, so p < pages
    *rq = lo_r;
    *pg = p;
    return uint32_t(here) + p;
  };
  for (uint32_t w = tid; w < runs; w += 1024) {
    uint32_t r0, p0, r1, p1;
    const uint32_t first = first_page_at(uint64_t(w) * cpw, &r0, &p0);
    const uint32_t last = first_page_at(uint64_t(w + 1) * cpw, &r1, &p1);
    a.desc[w] = make_uint4(r0, p0, first, last);
  }
  // requests without resident tokens get zero rows; a context beyond the handle row is counted
  __shared__ uint32_t n_empty;
  uint32_t* const empties = reinterpret_cast<uint32_t*>(sums);   // the scan is done with it (room for 2048)
  __syncthreads();
  if (tid == 0) n_empty = 0;
  __syncthreads();
  for (uint32_t r = tid; r < batch; r += 1024) {
    const uint32_t n = attended_tokens(a.ctx, r, a.append);
    if (uint64_t(n) > uint64_t(a.max_pages) * 16u)
      for (uint32_t la = 0; la < a.n_attn; ++la) count_fault(a.P);
    if (n != 0) continue;
    const uint32_t at = atomicAdd(&n_empty, 1u);
    if (at < 1024) {
      empties[at] = r;
    } else {                                                // more than the list holds: by this thread alone
      for (uint32_t la = 0; la < a.n_attn; ++la) {
        float* rows = a.o + (size_t(la) * batch + r) * a.row_floats;
        for (uint32_t d = 0; d < a.row_floats; ++d) rows[d] = 0.f;
      }
    }
  }
  __syncthreads();
  const uint32_t listed = min(n_empty, 1024u);
  for (uint32_t i = 0; i < listed; ++i) {
    const uint32_t r = empties[i];
    for (uint32_t la = 0; la < a.n_attn; ++la) {
      float* rows = a.o + (size_t(la) * batch + r) * a.row_floats;
      for (uint32_t d = tid; d < a.row_floats; d += 1024) rows[d] = 0.f;
    }
  }
}

__global__ __launch_bounds__(1024) void attn_prepare_kernel(PrepareArgs a) {
  if (blockIdx.x == 0) {
    plan_block(a);
    return;
  }
  // One entry per thread and tile.  Rows of up to 1024 pages: a tile is 1024 >> pitch_log2 whole
  // rows, each on a power-of-two pitch; longer rows: page_tiles tiles of 1024 entries per row.
  // Entries beyond the request's pages are left as they are.  The grid holds at most
  // kPrepareBlocks translating blocks, which walk the tiles between them: a batch of long rows
  // has far more tiles than pages to translate (516 requests with room for 16384 pages each,
  // four of them that long: 33 k tiles of which 2.3 k hold pages; one block per tile took 137 us,
  // nearly all of it the launching of blocks with nothing to do).
  for (uint32_t tile = blockIdx.x - 1; tile < a.n_tiles; tile += gridDim.x - 1) {
    // tiles are numbered page tile by page tile, so that the tiles of the rows' first 1024 pages,
    // which every row with pages has, are dealt out evenly over the blocks
    const uint32_t row_group = tile % a.row_groups, page_tile = tile / a.row_groups;
    if (a.page_tiles > 1) {
      // long rows: the tile lies within one row (row_group); beyond that row's pages there is
      // nothing to do, and no handle is asked for
      if (row_group >= a.n_attn * a.batch) continue;
      const uint32_t row_pages = pages_of(attended_tokens(a.ctx, row_group % a.batch, a.append), a.max_pages);
      if (page_tile * 1024u >= row_pages) continue;
    }
    const uint32_t row = (row_group << (10 - a.pitch_log2)) + (threadIdx.x >> a.pitch_log2);
    const uint32_t page = page_tile * 1024 + (threadIdx.x & ((1u << a.pitch_log2) - 1u));
    if (row >= a.n_attn * a.batch || page >= a.max_pages) continue;
    const uint32_t r = row % a.batch;
    const uint64_t e = uint64_t(row) * a.max_pages + page;
    // the handle is requested together with the context length, not after it
    const uint32_t n_ctx = attended_tokens(a.ctx, r, a.append);
    uint32_t h = a.handles[e];
    asm volatile("" : "+v"(h));
    if (page >= pages_of(n_ctx, a.max_pages)) continue;
    const uint64_t off = translate_offset(a.P, h, 0);
    uint32_t slot = kDevUnmapped;
    if (off == ~0ull) count_fault(a.P);
    else slot = uint32_t(off / a.P.unit[0]);
    a.slots[e] = slot;
  }
}

// Where run w of KV head g keeps a partial result: a run leaves at most two, slot 1 for
// the piece that starts its request, slot 0 for the piece that continues one.
__device__ __forceinline__ size_t partial_slot(uint32_t g, uint32_t runs, uint32_t w, bool starts_request) {
  return (size_t(g) * runs + w) * 2 + (starts_request ? 1 : 0);
}

// Combines the np partial results of (request r, KV head g), left by runs wa .. wa + np - 1,
// into the output rows of HS query heads of the group, head0 .. head0 + HS - 1.  One
// wavefront; the order of every sum depends on np alone.
//   statistics: lane (piece kk, head i) of a block of 64 / HS pieces holds that piece's running
//     max and sum; the row maximum M_i and the total L_i come from shuffles across the block;
//   rows: a partial row is D floats = D / 4 lanes of float4, so one load instruction fetches
//     64 / (D / 4) rows; lane group `sub` takes the pieces k = sub (mod that many), adds them
//     up in ascending k, and the groups are added in ascending order at the end.
// Row loads go out in chunks of up to 32 per lane, and in the usual case of a single block of
// statistics the first chunk is issued before anything is waited for.
template <int D, int HS>
__device__ void merge_pieces(const AttnLaunch& a, uint32_t g, uint32_t r, uint32_t wa, uint32_t np,
                             uint32_t lane, uint32_t head0) {
  constexpr uint32_t LPR = D / 4;            // lanes per partial row
  constexpr uint32_t RPL = 64 / LPR;         // rows per load instruction: 4, 2 or 1
  constexpr uint32_t PB = 64 / HS;           // pieces per block of statistics
  constexpr uint32_t ROUNDS = PB / RPL;      // load rounds that cover a block
  constexpr uint32_t CH = ROUNDS * HS <= 32 ? ROUNDS : 32 / HS;     // rounds per chunk of loads
  const uint32_t Hq = a.n_q_heads, Gq = Hq / a.n_kv_heads;
  const uint32_t kk = lane / HS, hi = head0 + lane % HS;     // statistics role
  const uint32_t sub = lane / LPR, c = lane % LPR;           // row role
  auto row_of = [&](uint32_t k, uint32_t head) -> size_t {
    return partial_slot(g, a.runs, wa + k, k == 0) * Gq + head;
  };
  float M = -INFINITY;                        // row maximum of head hi over all pieces
  float L = 0.f;                              // this lane's share of the total of head hi
  float4 acc[HS];
#pragma unroll
  for (int i = 0; i < HS; ++i) acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  const bool one_block = np <= PB;
  if (!one_block) {                           // the maxima need a pass of their own
    for (uint32_t base = 0; base < np; base += 4 * PB) {
      float m4[4];
#pragma unroll
      for (uint32_t u = 0; u < 4; ++u) {
        const uint32_t k = base + u * PB + kk;
        m4[u] = (k < np && hi < Gq) ? a.part_ml[row_of(k, hi) * 2] : -INFINITY;
      }
      M = fmaxf(fmaxf(M, fmaxf(m4[0], m4[1])), fmaxf(m4[2], m4[3]));
    }
#pragma unroll
    for (uint32_t o = HS; o < 64; o <<= 1) M = fmaxf(M, __shfl_xor(M, int(o)));
  }
  for (uint32_t base = 0; base < np; base += PB) {
    float2 ml = make_float2(-INFINITY, 0.f);
    if (base + kk < np && hi < Gq) ml = *reinterpret_cast<const float2*>(a.part_ml + row_of(base + kk, hi) * 2);
    const uint32_t rounds = (min(np - base, PB) + RPL - 1) / RPL;
    float wgt = 0.f;
    for (uint32_t t0 = 0; t0 < rounds; t0 += CH) {
      float4 v[CH][HS];
#pragma unroll
      for (uint32_t t = 0; t < CH; ++t) {
        const uint32_t k = base + (t0 + t) * RPL + sub;
#pragma unroll
        for (int i = 0; i < HS; ++i)
          v[t][i] = (t0 + t < rounds && k < np && head0 + i < Gq)
                        ? *reinterpret_cast<const float4*>(a.part_o + row_of(k, head0 + i) * D + 4 * c)
                        : make_float4(0.f, 0.f, 0.f, 0.f);
      }
      if (t0 == 0) {                          // the block's weights, once its statistics are in
        if (one_block) {
          M = ml.x;
#pragma unroll
          for (uint32_t o = HS; o < 64; o <<= 1) M = fmaxf(M, __shfl_xor(M, int(o)));
        }
        wgt = ml.x == -INFINITY ? 0.f : exp2f(ml.x - M);     // -inf: a piece whose pages were all skipped
        L += ml.y * wgt;
      }
#pragma unroll
      for (uint32_t t = 0; t < CH; ++t) {
        const uint32_t k2 = (t0 + t) * RPL + sub;            // piece within the block
#pragma unroll
        for (int i = 0; i < HS; ++i) {
          const float w = __shfl(wgt, int((k2 % PB) * HS + i));   // 0 where the piece does not exist
          acc[i].x += w * v[t][i].x;
          acc[i].y += w * v[t][i].y;
          acc[i].z += w * v[t][i].z;
          acc[i].w += w * v[t][i].w;
        }
      }
    }
  }
#pragma unroll
  for (uint32_t o = HS; o < 64; o <<= 1) L += __shfl_xor(L, int(o));
  // lane groups 1 .. RPL-1 hand their sums to group 0, which adds them in ascending order
#pragma unroll
  for (int i = 0; i < HS; ++i) {
    float4 sum = acc[i];
#pragma unroll
    for (uint32_t q = 1; q < RPL; ++q) {
      const int src = int(q * LPR + c);
      sum.x += __shfl(acc[i].x, src);
      sum.y += __shfl(acc[i].y, src);
      sum.z += __shfl(acc[i].z, src);
      sum.w += __shfl(acc[i].w, src);
    }
    const float Li = __shfl(L, i);            // lane i (piece 0 of the block, head head0 + i) holds the total
    if (sub == 0 && head0 + i < Gq) {
      float* orow = a.o + (size_t(r) * Hq + size_t(g) * Gq + head0 + i) * D;
      const float inv = Li > 0.f ? 1.f / Li : 0.f;
      *reinterpret_cast<float4*>(orow + 4 * c) =
          Li > 0.f ? make_float4(sum.x * inv, sum.y * inv, sum.z * inv, sum.w * inv)
                   : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
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
  const uint32_t max_pages = a.max_pages;
  // Slots come 64 at a time, one per lane: lane l of a fetch for (request rr, page bb) holds the
  // slot of page bb + l.  The fetch for the stretch after the one being walked is always in
  // flight (the same request's next 64 pages, or the next request's first), and the first is
  // requested before anything that depends on the context lengths.
  uint32_t pre_r = 0, pre_base = 0, pre_val = kDevUnmapped;
  auto fetch_slots = [&](uint32_t rr, uint32_t bb) -> uint32_t {
    return (rr < a.batch && uint64_t(bb) + lane < max_pages)
               ? a.slots[size_t(rr) * max_pages + bb + lane] : kDevUnmapped;
  };
  auto prefetch_slots = [&](uint32_t rr, uint32_t bb) {
    pre_r = rr;
    pre_base = bb;
    pre_val = fetch_slots(rr, bb);
  };
  prefetch_slots(r, page);
  const uint64_t unit_kv = a.P.unit[0];
  const uint32_t G = a.n_kv_heads, Hq = a.n_q_heads, Gq = Hq / G;
  const float scale_log2 = kLog2e / sqrtf(float(D));
  const size_t kslab_off = size_t(g) * D * 32;                        // bytes: [D/8][16][8] bf16
  const size_t vslab_off = size_t(G) * D * 32 + size_t(g) * D * 32;   // bytes: [D][16] bf16

  while (item < item_end && r < a.batch) {
    const uint32_t n_ctx = attended_tokens(a.ctx, r, a.append);
    const uint32_t n_pages = pages_of(n_ctx, max_pages);
    if (page >= n_pages) {             // request without pages (or exhausted): next one
      ++r;
      page = 0;
      continue;
    }
    const uint32_t n_tok = min(n_ctx, n_pages * 16u);
    const uint32_t p0 = page;
    const uint32_t p1 = uint32_t(min(uint64_t(n_pages), uint64_t(page) + (item_end - item)));
    const bool run_goes_on = item + (p1 - p0) < item_end;            // into the next request

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
      uint32_t my_slot = (pre_r == r && pre_base == base) ? pre_val : fetch_slots(r, base);
      if (lane >= cnt) my_slot = kDevUnmapped;
      if (base + 64 < p1) prefetch_slots(r, base + 64);
      else if (run_goes_on) prefetch_slots(r + 1, 0);
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
        // some handle did not translate (counted by the preparation kernel): skip those pages
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
      const size_t slot = partial_slot(g, a.runs, w, p0 == 0);
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

// Merge of the partial results that the runs left, one workgroup of four wavefronts (one in
// launches of a thousand or more workgroups) per (KV head, request).  A query group of up to four heads whose request was cut into at most 16
// pieces (every request of an ordinary batch) is one wavefront's work, all heads at once; a
// longer list of pieces, or a wider group, is taken head by head, the heads shared out over
// the wavefronts.  The runs that hold the request's first and last page follow from its
// position on the plan's cost axis.
template <int D>
__global__ __launch_bounds__(256) void attn_merge_runs_kernel(AttnLaunch a) {
  const uint32_t g = blockIdx.x, r = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t n_waves = blockDim.x >> 6;
  const uint32_t start = a.prefix[r], end = a.prefix[r + 1];
  const uint64_t pos = a.pos[r];
  if (start == end) return;                 // no resident tokens: the plan wrote the zero rows
  const uint64_t cpw = a.plan[1];
  const uint64_t at = pos + (request_cost(end - start) - (end - start));      // position of its page 0
  const uint32_t wa = uint32_t(at / cpw), wb = uint32_t((at + (end - start) - 1) / cpw);
  if (wa == wb) return;                     // one run covered it and wrote the rows
  const uint32_t np = wb - wa + 1, Gq = a.n_q_heads / a.n_kv_heads;
  if (Gq <= 4 && np <= 16) {
    if (wave == 0) merge_pieces<D, 4>(a, g, r, wa, np, lane, 0);
    return;
  }
  for (uint32_t head = wave; head < Gq; head += n_waves) merge_pieces<D, 1>(a, g, r, wa, np, lane, head);
}

}  // namespace

bool attention_mfma_supported(uint32_t dtype, uint32_t n_q_heads, uint32_t n_kv_heads,
                              uint32_t head_dim) {
  if (dtype != 1) return false;
  if (head_dim != 64 && head_dim != 128 && head_dim != 256) return false;
  return n_q_heads / n_kv_heads <= 16;
}

uint32_t attention_runs_per_head(uint32_t n_kv_heads) {
  // about 2048 wavefronts per launch: one full set of resident waves on 256 CUs (measured per
  // layer at the Jamba-shaped batch of 64 with 1024 / 1536 / 2048 / 3072 / 4096 / 8192 wavefronts:
  // 47.3 / 47.3 / 46.4 / 47.7 / 49.2 / 49.8 us; beyond one resident set the extra partial
  // results and request starts cost more than the finer balance gains)
  const uint32_t runs = 2048 / n_kv_heads;
  return runs ? runs : 1;
}

hipError_t launch_attention_prepare(const AttnLaunch& a, const uint32_t* handles_all, uint32_t n_attn,
                                    uint32_t* slots_all, float* o_all,
                                    hipStream_t s) {
  PrepareArgs p{};
  p.P = a.P;
  p.ctx = a.ctx;
  p.handles = handles_all;
  p.slots = slots_all;
  p.plan = const_cast<uint32_t*>(a.plan);
  p.prefix = const_cast<uint32_t*>(a.prefix);
  p.pos = const_cast<uint32_t*>(a.pos);
  p.desc = const_cast<uint4*>(a.desc);
  p.o = o_all;
  p.batch = a.batch;
  p.max_pages = a.max_pages;
  p.runs = a.runs;
  p.append = a.append;
  p.n_attn = n_attn;
  p.row_floats = a.n_q_heads * a.head_dim;
  uint32_t pitch_log2 = 0;
  while (pitch_log2 < 10 && (1u << pitch_log2) < a.max_pages) ++pitch_log2;
  p.pitch_log2 = pitch_log2;
  p.page_tiles = a.max_pages > 1024 ? (a.max_pages + 1023) / 1024 : 1;
  const uint64_t rows = uint64_t(n_attn) * a.batch;
  const uint32_t rows_per_block = 1024u >> pitch_log2;
  const uint64_t row_groups = (rows + rows_per_block - 1) / rows_per_block;
  const uint64_t tiles = row_groups * p.page_tiles;
  if (rows > 0xFFFFFFFFull || tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
  p.row_groups = uint32_t(row_groups);
  p.n_tiles = uint32_t(tiles);
  const uint32_t blocks = 1 + uint32_t(tiles < kPrepareBlocks ? tiles : kPrepareBlocks);
  attn_prepare_kernel<<<dim3(blocks), dim3(1024), 0, s>>>(p);
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
  const dim3 grid(a.n_kv_heads, a.batch);
  // Four wavefronts per (KV head, request) pay off where piece lists are long; with a thousand or
  // more workgroups most of them are short requests that wave 0 handles alone (or that need no
  // merge at all), and the three idle wavefronts only take a second round of residency
  // (batch 256, half of it 1-4 page requests: 10.9 -> 7.1 us per layer).
  const dim3 block(uint64_t(a.n_kv_heads) * a.batch >= 1024 ? 64 : 256);
  switch (a.head_dim) {
    case 64: attn_merge_runs_kernel<64><<<grid, block, 0, s>>>(a); break;
    case 128: attn_merge_runs_kernel<128><<<grid, block, 0, s>>>(a); break;
    default: attn_merge_runs_kernel<256><<<grid, block, 0, s>>>(a); break;
  }
  return hipGetLastError();
}

}  // namespace avmp
