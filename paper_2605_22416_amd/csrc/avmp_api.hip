// C ABI of the library: glue between the host-side pool state, the device
// table mirror and the kernels.  See include/avmp.h for the contract.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/avmp.h"
#include "kernels.hpp"
#include "pool_state.hpp"
#include "vmm_arena.hpp"

namespace {

thread_local std::string g_last_error;

constexpr const char* kDeadPools =
    "a device call failed half way through a migration: these pools can only be destroyed";

int fail(int code, const char* what) {
  g_last_error = what;
  return code;
}

int fail_hip(hipError_t e, const char* where) {
  g_last_error = std::string(where) + ": " + hipGetErrorString(e);
  return AVMP_ERR_DEVICE;
}

#define HIP_TRY(expr)                                \
  do {                                               \
    hipError_t e_ = (expr);                          \
    if (e_ != hipSuccess) return fail_hip(e_, #expr); \
  } while (0)

// Pinned host buffers that kernels read directly (lists of table updates, slots
// to clear, moves).  A buffer is reused only after the event recorded behind its
// last consumer has completed, so the host never overwrites a list in flight.
struct Staging {
  struct Buf {
    void* host = nullptr;
    size_t cap = 0;
    hipEvent_t ev = nullptr;
    bool busy = false;
  };
  std::vector<Buf> bufs;

  hipError_t acquire(size_t bytes, Buf** out) {
    for (auto& b : bufs) {
      if (b.busy && hipEventQuery(b.ev) == hipSuccess) b.busy = false;
      if (!b.busy && b.cap >= bytes) {
        *out = &b;
        return hipSuccess;
      }
    }
    Buf b;
    b.cap = bytes < (1u << 16) ? (1u << 16) : bytes;
    hipError_t e = hipHostMalloc(&b.host, b.cap, hipHostMallocDefault);
    if (e != hipSuccess) return e;
    e = hipEventCreateWithFlags(&b.ev, hipEventDisableTiming);
    if (e != hipSuccess) {
      (void)hipHostFree(b.host);
      return e;
    }
    bufs.push_back(b);
    *out = &bufs.back();
    return hipSuccess;
  }
  hipError_t release_after(Buf* b, hipStream_t s) {
    b->busy = true;
    return hipEventRecord(b->ev, s);
  }
  void destroy() {
    for (auto& b : bufs) {
      if (b.busy) (void)hipEventSynchronize(b.ev);
      (void)hipEventDestroy(b.ev);
      (void)hipHostFree(b.host);
    }
    bufs.clear();
  }
};

// Work buffer of avmp_decode_step_noalloc: one array per GPU, alive for the whole process.
// In host code its name is only a stand-in for the symbol; the memory's address on a
// device comes from hipGetSymbolAddress with that device current (scratch_on_device).
constexpr size_t kScratchBytes = size_t(AVMP_NOALLOC_WORKSPACE_BYTES);
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on device `dev` (looked up once per device); nullptr on failure,
// with the reason in *err.
void* scratch_on_device(int dev, hipError_t* err) {
  *err = hipSuccess;
  if (dev < 0 || dev >= kMaxDevices) {
    *err = hipErrorInvalidDevice;
    return nullptr;
  }
  if (g_scratch_ptr[dev] != nullptr) return g_scratch_ptr[dev];
  int current = -1;
  *err = hipGetDevice(&current);
  if (*err != hipSuccess) return nullptr;
  if (current != dev) {
    *err = hipSetDevice(dev);
    if (*err != hipSuccess) return nullptr;
  }
  void* ptr = nullptr;
  *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
  if (current != dev) {
    const hipError_t back = hipSetDevice(current);
    if (*err == hipSuccess) *err = back;
  }
  if (*err != hipSuccess) return nullptr;
  g_scratch_ptr[dev] = ptr;
  return ptr;
}

}  // namespace

struct avmp_vmm_arena {
  avmp::VmmArena impl;
};

constexpr uint32_t kMaxBatch = 65535;        // requests of one decode step (a grid dimension)

struct avmp_pools {
  avmp_config_t cfg{};
  avmp::PoolState st;
  bool has_device = false;
  int device = -1;                     // the GPU the arena lives on
  uint8_t* arena = nullptr;
  uint32_t* table_dev = nullptr;
  uint32_t* conv_arrivals_dev = nullptr;       // per request of a batch, zero between launches; only where
                                               // the recurrence kernel runs the convolution itself
  unsigned long long* faults_dev = nullptr;
  unsigned long long* faults_host = nullptr;   // pinned: where avmp_device_faults reads the counter to
  float* ws = nullptr;                 // work buffer of the decode step (see WorkLayout)
  size_t ws_bytes = 0;
  uint64_t ws_allocations = 0;
  std::vector<void*> ws_retired;       // outgrown work buffers: a step in flight (or a captured
                                       // graph) may still name them, so they live until destroy
  std::vector<avmp::TableUpdate> pending;
  bool pending_entries = false;        // `pending` holds table entries, not just the two capacities
  std::vector<uint32_t> pending_zero;  // SSM slots to clear
  Staging staging;
  avmp::Rebalancer rebalancer;
  avmp::VmmArena* remap = nullptr;     // non-null: migrate may exchange backing instead of copying
  bool remappable[2] = {false, false}; // per pool: every slot covers whole chunks of `remap`
  bool dead = false;                   // part of the arena lost its mapping: launch nothing

  // per-kernel timing: event pairs on the launch stream, summed at read time
  struct ProfRec {
    int kind;
    hipEvent_t a, b;
  };
  bool profiling = false;
  std::vector<ProfRec> prof;       // records in use since the last read
  std::vector<ProfRec> prof_free;  // event pairs ready for reuse

  int prof_start(int kind, hipStream_t s) {
    ProfRec r{};
    if (!prof_free.empty()) {
      r = prof_free.back();
      prof_free.pop_back();
    } else {
      if (hipEventCreate(&r.a) != hipSuccess) return -1;
      if (hipEventCreate(&r.b) != hipSuccess) {
        (void)hipEventDestroy(r.a);
        return -1;
      }
    }
    r.kind = kind;
    (void)hipEventRecord(r.a, s);
    prof.push_back(r);
    return int(prof.size()) - 1;
  }
  void prof_stop(int idx, hipStream_t s) { (void)hipEventRecord(prof[size_t(idx)].b, s); }

  // the device table is followed by the two pool capacities, updated like table entries
  size_t table_entries() const { return size_t(st.max_vid(0)) + st.max_vid(1); }
  void queue_capacities() {   // does not count as a pending table entry
    for (int pl = 0; pl < 2; ++pl)
      pending.push_back({uint32_t(table_entries()) + uint32_t(pl), st.capacity(pl)});
  }

  avmp::DevPools dev_view() const {
    avmp::DevPools P{};
    P.arena = arena;
    P.usable = st.geometry().usable;
    P.table = table_dev;
    P.capacity = table_dev + table_entries();
    P.faults = faults_dev;
    for (int p = 0; p < 2; ++p) {
      P.unit[p] = st.geometry().unit[p];
      P.vid_base[p] = st.vid_base(p);
      P.max_vid[p] = st.max_vid(p);
    }
    return P;
  }
};

namespace {

bool shape_from_config(const avmp_config_t* c, avmp::ShapeArgs* s) {
  if (c == nullptr) return false;
  if (c->dtype != AVMP_F32 && c->dtype != AVMP_BF16) return false;
  s->elem_bytes = c->dtype == AVMP_F32 ? 4 : 2;
  if (c->attention_page_tokens != 16) return false;
  if (c->n_kv_heads == 0 || c->n_q_heads == 0 || c->n_q_heads % c->n_kv_heads != 0) return false;
  const uint32_t x = 16 / s->elem_bytes;
  if (c->head_dim == 0 || c->head_dim % x != 0 || c->head_dim > 256) return false;
  const uint32_t n = c->ssm_dstate;
  if (n < 4 || n > 256 || (n & (n - 1)) != 0) return false;
  if (c->ssm_state_dtype != AVMP_F32 && c->ssm_state_dtype != AVMP_BF16) return false;
  s->state_bytes = c->ssm_state_dtype == AVMP_F32 ? 4 : 2;
  if (s->state_bytes == 2 && n < 8) return false;      // a lane moves 16 bytes = 8 bf16 of a row
  if (c->ssm_heads == 0 || c->ssm_headdim == 0) return false;
  if (c->ssm_heads > 65535 || c->n_q_heads > 65535) return false;
  // one head's state tile is addressed with 32-bit byte offsets
  if (uint64_t(c->ssm_headdim) * n * 4 >= (1ull << 31)) return false;
  if (c->ssm_conv_kernel != 0 &&
      !avmp::conv_supported(c->dtype, c->ssm_conv_kernel, c->ssm_heads, c->ssm_headdim, n))
    return false;
  s->conv_kernel = c->ssm_conv_kernel;
  if (c->ssm_pad_to_kv_page > 1) return false;
  s->pad_ssm_to_kv_page = c->ssm_pad_to_kv_page == 1;
  s->page_tokens = c->attention_page_tokens;
  s->n_q_heads = c->n_q_heads;
  s->n_kv_heads = c->n_kv_heads;
  s->head_dim = c->head_dim;
  s->ssm_heads = c->ssm_heads;
  s->ssm_headdim = c->ssm_headdim;
  s->ssm_dstate = c->ssm_dstate;
  return true;
}

struct ProfScope {
  avmp_pools* p;
  hipStream_t s;
  int idx = -1;
  ProfScope(avmp_pools* pools, bool on, int kind, hipStream_t stream) : p(pools), s(stream) {
    if (on) idx = p->prof_start(kind, s);
  }
  ~ProfScope() {
    if (idx >= 0) p->prof_stop(idx, s);
  }
};

// Queue -> device: table entries (coalesced to the last value per index, so the
// scatter has no ordering hazard) and zero fills of freshly allocated SSM blocks.
int flush_pending(avmp_pools* p, hipStream_t s) {
  if (p->dead) return fail(AVMP_ERR_DEVICE, kDeadPools);
  if (!p->has_device) return fail(AVMP_ERR_DEVICE, "pools have no device arena");
  if (p->pending.empty() && p->pending_zero.empty()) return AVMP_OK;
  std::vector<avmp::TableUpdate> upd;
  if (!p->pending.empty()) {
    std::unordered_map<uint32_t, uint32_t> last;
    last.reserve(p->pending.size() * 2);
    for (const auto& u : p->pending) last[u.index] = u.slot;
    upd.reserve(last.size());
    for (const auto& kv : last) upd.push_back({kv.first, kv.second});
  }
  if (upd.size() <= avmp::kInlineUpdates && p->pending_zero.size() <= avmp::kInlineZero) {
    // short lists (a decode step's churn) ride in the kernel arguments: one launch, no staging
    avmp::InlineFlush f{};
    f.P = p->dev_view();
    f.table = p->table_dev;
    f.n_upd = uint32_t(upd.size());
    f.n_zero = uint32_t(p->pending_zero.size());
    f.ssm_capacity = p->st.capacity(AVMP_POOL_SSM);
    if (f.n_upd) std::memcpy(f.upd, upd.data(), upd.size() * sizeof(avmp::TableUpdate));
    if (f.n_zero) std::memcpy(f.zero, p->pending_zero.data(), p->pending_zero.size() * sizeof(uint32_t));
    {
      ProfScope scope(p, p->profiling, AVMP_K_TABLE, s);
      HIP_TRY(avmp::launch_flush_inline(f, s));
    }
    p->pending.clear();
    p->pending_zero.clear();
    p->pending_entries = false;
    return AVMP_OK;
  }
  const size_t upd_bytes = upd.size() * sizeof(avmp::TableUpdate);
  const size_t zero_bytes = p->pending_zero.size() * sizeof(uint32_t);
  Staging::Buf* b = nullptr;
  HIP_TRY(p->staging.acquire(upd_bytes + zero_bytes, &b));
  char* host = static_cast<char*>(b->host);
  if (upd_bytes) std::memcpy(host, upd.data(), upd_bytes);
  if (zero_bytes) std::memcpy(host + upd_bytes, p->pending_zero.data(), zero_bytes);
  {
    ProfScope scope(p, p->profiling, AVMP_K_TABLE, s);
    HIP_TRY(avmp::launch_table_updates(p->table_dev,
                                       reinterpret_cast<const avmp::TableUpdate*>(host),
                                       uint32_t(upd.size()), s));
    HIP_TRY(avmp::launch_zero_units(p->dev_view(), AVMP_POOL_SSM,
                                    reinterpret_cast<const uint32_t*>(host + upd_bytes),
                                    uint32_t(p->pending_zero.size()), s));
  }
  HIP_TRY(p->staging.release_after(b, s));
  p->pending.clear();
  p->pending_zero.clear();
  p->pending_entries = false;
  return AVMP_OK;
}

// Where the decode step keeps what is neither input nor output: the fp32 outputs of one
// layer's short convolution, the split-K partial results of one attention layer, the run
// plan of the matrix-core path and the pre-translated slots of every attention layer.
struct WorkLayout {
  bool mfma = false;
  uint32_t runs = 0, max_chunks = 0;
  size_t conv_floats = 0, part_rows = 0, part_floats = 0, prefix_words = 0, plan_words = 0,
         slot_cap = 0, slot_words = 0;
  size_t bytes() const {
    return (conv_floats + part_floats + plan_words + slot_words) * sizeof(float);
  }
};

WorkLayout work_layout(const avmp_config_t& c, uint32_t n_attn, uint32_t n_ssm, uint32_t batch,
                       uint32_t max_pages) {
  WorkLayout L;
  if (batch == 0) return L;
  if (n_attn) {
    L.mfma = avmp::attention_mfma_supported(c.dtype, c.n_q_heads, c.n_kv_heads, c.head_dim);
    L.runs = avmp::attention_runs_per_head(c.n_kv_heads);
    const uint32_t worst = (max_pages + avmp::kChunkPages - 1) / avmp::kChunkPages;
    L.max_chunks = worst < avmp::kMaxChunks ? worst : avmp::kMaxChunks;
    L.part_rows = L.mfma ? size_t(L.runs) * 2 * c.n_q_heads
                         : size_t(batch) * L.max_chunks * c.n_q_heads;
    L.part_floats = (L.part_rows * (size_t(c.head_dim) + 2) + 3) / 4 * 4;   // keeps the plan 16-byte aligned
    L.prefix_words = (size_t(batch) + 4) / 4 * 4;                           // batch + 1 entries
    L.plan_words = 4 + 2 * L.prefix_words + size_t(L.runs) * 4;           // plan, page and cost prefix sums, runs
    L.slot_cap = size_t(batch) * max_pages;                                 // per attention layer
    L.slot_words = L.mfma ? size_t(n_attn) * L.slot_cap : 0;
  }
  if (c.ssm_conv_kernel != 0 && n_ssm) {
    const size_t conv_dim = size_t(c.ssm_heads) * c.ssm_headdim + 2 * size_t(c.ssm_dstate);
    L.conv_floats = (size_t(batch) * conv_dim + 3) / 4 * 4;
  }
  return L;
}

// The work buffer only ever grows, by at least a factor of two, and an outgrown buffer is
// kept until the pools are destroyed: growing neither waits for the device nor takes memory
// away from a step that is still in flight or recorded in a graph.
int grow_workspace(avmp_pools* p, size_t bytes) {
  if (bytes <= p->ws_bytes) return AVMP_OK;
  if (bytes < 2 * p->ws_bytes) bytes = 2 * p->ws_bytes;
  void* fresh = nullptr;
  HIP_TRY(hipMalloc(&fresh, bytes));
  if (p->ws) p->ws_retired.push_back(p->ws);
  p->ws = static_cast<float*>(fresh);
  p->ws_bytes = bytes;
  ++p->ws_allocations;
  return AVMP_OK;
}

// Pages per request that a growing work buffer is sized for: twice the row in hand and at
// least 1024 tokens, so that a decode loop whose handle rows widen page by page allocates
// once.
uint32_t roomy_pages(uint32_t max_pages) {
  const uint64_t twice = 2ull * max_pages;
  return uint32_t(twice < 64 ? 64 : (twice > 0xFFFFFFFFull ? 0xFFFFFFFFull : twice));
}

// Argument checks of a decode step; counts the layers of each kind.
int check_step(avmp_pools* p, const avmp_step_t* st, uint32_t* n_attn_out, uint32_t* n_ssm_out) {
  if (p == nullptr || st == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null argument");
  if (!p->has_device) return fail(AVMP_ERR_DEVICE, "pools have no device arena");
  if (p->dead) return fail(AVMP_ERR_DEVICE, kDeadPools);
  if (st->n_layers != 0 && st->layer_kind == nullptr) return fail(AVMP_ERR_INVALID_ARG, "layer_kind");
  uint32_t n_attn = 0, n_ssm = 0;
  for (uint32_t i = 0; i < st->n_layers; ++i) {
    if (st->layer_kind[i] == AVMP_LAYER_ATTENTION) ++n_attn;
    else if (st->layer_kind[i] == AVMP_LAYER_SSM) ++n_ssm;
    else return fail(AVMP_ERR_INVALID_ARG, "unknown layer kind");
  }
  if (st->batch > kMaxBatch) return fail(AVMP_ERR_INVALID_ARG, "batch above 65535");
  if (n_attn && uint64_t(st->batch) * st->max_pages > 0x7FFFFFFFull)      // page counts are summed in 32 bits
    return fail(AVMP_ERR_INVALID_ARG, "batch x max_pages above 2^31 - 1");
  if (n_attn && st->batch &&
      (!st->kv_handles || !st->ctx || !st->q || !st->o || st->max_pages == 0))
    return fail(AVMP_ERR_INVALID_ARG, "attention layers need kv_handles, ctx, q, o, max_pages");
  if (n_attn && st->batch &&
      ((reinterpret_cast<uintptr_t>(st->q) | reinterpret_cast<uintptr_t>(st->o)) & 15u))
    return fail(AVMP_ERR_INVALID_ARG, "q and o must be 16-byte aligned");
  if ((st->k_new == nullptr) != (st->v_new == nullptr))
    return fail(AVMP_ERR_INVALID_ARG, "k_new and v_new go together");
  const bool conv = p->cfg.ssm_conv_kernel != 0;
  if (n_ssm && st->batch && (!st->ssm_handles || !st->dt || !st->A || !st->y))
    return fail(AVMP_ERR_INVALID_ARG, "SSM layers need ssm_handles, dt, A, y");
  if (n_ssm && st->batch && !conv && (!st->x || !st->B || !st->C))
    return fail(AVMP_ERR_INVALID_ARG, "SSM layers need x, B, C");
  if (n_ssm && st->batch && conv) {
    if (!st->xbc || !st->conv_taps || !st->conv_bias)
      return fail(AVMP_ERR_INVALID_ARG,
                  "pools with a convolution window need xbc, conv_taps, conv_bias");
    if ((reinterpret_cast<uintptr_t>(st->xbc) | reinterpret_cast<uintptr_t>(st->conv_taps) |
         reinterpret_cast<uintptr_t>(st->conv_bias)) & 15u)
      return fail(AVMP_ERR_INVALID_ARG, "xbc, conv_taps, conv_bias must be 16-byte aligned");
  }
  *n_attn_out = n_attn;
  *n_ssm_out = n_ssm;
  return AVMP_OK;
}

// Enqueues the kernels of one decode step.  `ws` is a work buffer of at least L.bytes().
int run_step(avmp_pools* p, const avmp_step_t* st, hipStream_t s, uint32_t n_attn,
             const WorkLayout& L, float* ws, bool profile) {
  const avmp_config_t& c = p->cfg;
  const size_t eb = c.dtype == AVMP_F32 ? 4 : 2;
  const bool mfma = L.mfma;
  const bool append = st->k_new != nullptr;
  const bool conv = c.ssm_conv_kernel != 0;
  const size_t conv_dim = size_t(c.ssm_heads) * c.ssm_headdim + 2 * size_t(c.ssm_dstate);
  float* const conv_out = ws;
  float* const part_base = ws + L.conv_floats;
  uint32_t* plan_base = reinterpret_cast<uint32_t*>(part_base + L.part_floats);
  uint32_t* slots_base = plan_base + L.plan_words;
  const avmp::DevPools P = p->dev_view();
  uint32_t ia = 0, is = 0;
  bool planned = false;
  for (uint32_t i = 0; i < st->n_layers; ++i) {
    if (st->layer_kind[i] == AVMP_LAYER_ATTENTION) {
      avmp::AttnLaunch a{};
      a.P = P;
      if (mfma) {
        a.plan = plan_base;
        a.prefix = plan_base + 4;
        a.pos = plan_base + 4 + L.prefix_words;
        a.desc = reinterpret_cast<const uint4*>(plan_base + 4 + 2 * L.prefix_words);
        a.runs = L.runs;
        a.slots = slots_base + size_t(ia) * L.slot_cap;
      }
      a.handles = st->kv_handles + size_t(ia) * st->batch * st->max_pages;
      a.ctx = st->ctx;
      const size_t row = size_t(st->batch) * c.n_q_heads * c.head_dim;
      a.q = static_cast<const char*>(st->q) + size_t(ia) * row * eb;
      a.o = st->o + size_t(ia) * row;
      a.part_o = part_base;
      a.part_ml = part_base + L.part_rows * c.head_dim;
      a.batch = st->batch;
      a.max_pages = st->max_pages;
      a.max_chunks = L.max_chunks;
      a.n_q_heads = c.n_q_heads;
      a.n_kv_heads = c.n_kv_heads;
      a.head_dim = c.head_dim;
      a.dtype = c.dtype;
      if (append) {
        const size_t kvrow = size_t(st->batch) * c.n_kv_heads * c.head_dim * eb;
        a.append = 1;
        a.k_new = static_cast<const char*>(st->k_new) + size_t(ia) * kvrow;
        a.v_new = static_cast<const char*>(st->v_new) + size_t(ia) * kvrow;
        ProfScope scope(p, profile, AVMP_K_TABLE, s);
        HIP_TRY(avmp::launch_kv_append(a, s));
      }
      if (mfma && !planned) {            // context lengths are the same for every layer
        ProfScope scope(p, profile, AVMP_K_ATTENTION_PREPARE, s);
        HIP_TRY(avmp::launch_attention_prepare(a, st->kv_handles, n_attn, slots_base, st->o, s));
        planned = true;
      }
      {
        ProfScope scope(p, profile, AVMP_K_ATTENTION, s);
        HIP_TRY(avmp::launch_attention(a, s));
      }
      {
        ProfScope scope(p, profile, AVMP_K_ATTENTION_MERGE, s);
        HIP_TRY(avmp::launch_attention_merge(a, s));
      }
      ++ia;
    } else {
      avmp::SsmLaunch a{};
      a.P = P;
      a.handles = st->ssm_handles + size_t(is) * st->batch;
      const size_t xrow = size_t(st->batch) * c.ssm_heads * c.ssm_headdim;
      if (!conv) {
        a.x = static_cast<const char*>(st->x) + size_t(is) * xrow * eb;
        a.B = static_cast<const char*>(st->B) + size_t(is) * st->batch * c.ssm_dstate * eb;
        a.C = static_cast<const char*>(st->C) + size_t(is) * st->batch * c.ssm_dstate * eb;
      }
      a.dt = st->dt + size_t(is) * st->batch * c.ssm_heads;
      a.A = st->A + size_t(is) * c.ssm_heads;
      a.y = st->y + size_t(is) * xrow;
      a.batch = st->batch;
      a.heads = c.ssm_heads;
      a.headdim = c.ssm_headdim;
      a.dstate = c.ssm_dstate;
      a.dtype = c.dtype;
      a.state_dtype = c.ssm_state_dtype;
      if (conv && p->conv_arrivals_dev != nullptr &&
          avmp::ssm_fuses_conv(c.ssm_conv_kernel, c.ssm_heads, c.ssm_headdim, c.ssm_dstate, c.ssm_state_dtype, st->batch)) {
        // the recurrence kernel runs the convolution itself
        a.conv_u = static_cast<const char*>(st->xbc) + size_t(is) * st->batch * conv_dim * eb;
        a.conv_taps = static_cast<const char*>(st->conv_taps) + size_t(is) * c.ssm_conv_kernel * conv_dim * eb;
        a.conv_bias = static_cast<const char*>(st->conv_bias) + size_t(is) * conv_dim * eb;
        a.conv_arrivals = p->conv_arrivals_dev;
        a.conv_k = c.ssm_conv_kernel;
      } else if (conv) {
        // x, B and C of this layer come out of the convolution, as fp32
        avmp::ConvLaunch cv{};
        cv.P = P;
        cv.handles = a.handles;
        cv.u = static_cast<const char*>(st->xbc) + size_t(is) * st->batch * conv_dim * eb;
        cv.taps = static_cast<const char*>(st->conv_taps) + size_t(is) * c.ssm_conv_kernel * conv_dim * eb;
        cv.bias = static_cast<const char*>(st->conv_bias) + size_t(is) * conv_dim * eb;
        cv.x = conv_out;
        cv.B = conv_out + xrow;
        cv.C = cv.B + size_t(st->batch) * c.ssm_dstate;
        cv.state_bytes = uint64_t(c.ssm_heads) * c.ssm_headdim * c.ssm_dstate *
                         (c.ssm_state_dtype == AVMP_F32 ? 4 : 2);
        cv.batch = st->batch;
        cv.heads = c.ssm_heads;
        cv.headdim = c.ssm_headdim;
        cv.dstate = c.ssm_dstate;
        cv.conv_dim = uint32_t(conv_dim);
        cv.taps_k = c.ssm_conv_kernel;
        cv.dtype = c.dtype;
        {
          ProfScope scope(p, profile, AVMP_K_CONV, s);
          HIP_TRY(avmp::launch_conv_update(cv, s));
        }
        a.x = cv.x;
        a.B = cv.B;
        a.C = cv.C;
        a.dtype = AVMP_F32;
      }
      {
        ProfScope scope(p, profile, AVMP_K_SSM, s);
        HIP_TRY(avmp::launch_ssm(a, s));
      }
      ++is;
    }
  }
  return AVMP_OK;
}

}  // namespace

extern "C" {

const char* avmp_last_error(void) { return g_last_error.c_str(); }

int avmp_geometry(const avmp_config_t* cfg, size_t arena_bytes, avmp_geometry_t* out) {
  avmp::ShapeArgs s{};
  avmp::Geometry g{};
  if (out == nullptr || !shape_from_config(cfg, &s) || !avmp::compute_geometry(s, arena_bytes, &g))
    return fail(AVMP_ERR_INVALID_ARG, "unsupported shape or arena size");
  out->unit_bytes[0] = g.unit[0];
  out->unit_bytes[1] = g.unit[1];
  out->ssm_native_bytes = g.ssm_native;
  out->usable_bytes = g.usable;
  out->max_slots[0] = g.max_slots[0];
  out->max_slots[1] = g.max_slots[1];
  return AVMP_OK;
}

int avmp_pools_create(const avmp_config_t* cfg, void* arena_dev, size_t arena_bytes,
                      avmp_pools_t** out) {
  avmp::ShapeArgs s{};
  avmp::Geometry g{};
  if (out == nullptr || !shape_from_config(cfg, &s) || !avmp::compute_geometry(s, arena_bytes, &g))
    return fail(AVMP_ERR_INVALID_ARG, "unsupported shape or arena size");
  if (arena_dev != nullptr && (reinterpret_cast<uintptr_t>(arena_dev) & 127u) != 0)
    return fail(AVMP_ERR_INVALID_ARG, "arena must be 128-byte aligned");
  avmp_pools* p = new (std::nothrow) avmp_pools();
  if (p == nullptr) return fail(AVMP_ERR_INVALID_ARG, "out of host memory");
  p->cfg = *cfg;
  const uint32_t* ranks[2] = {cfg->slot_rank[0], cfg->slot_rank[1]};
  if (!p->st.init(g, cfg->kv_capacity, cfg->ssm_capacity, cfg->max_vid, ranks)) {
    delete p;
    return fail(AVMP_ERR_INVALID_ARG,
                "capacities do not fit the arena, or slot_rank is not a permutation");
  }
  p->cfg.slot_rank[0] = p->cfg.slot_rank[1] = nullptr;
  if (arena_dev != nullptr) {
    p->arena = static_cast<uint8_t*>(arena_dev);
    const size_t entries = size_t(p->st.max_vid(0)) + p->st.max_vid(1);
    // the GPU that holds the arena, and that GPU's copy of the static work buffer
    hipPointerAttribute_t attr{};
    hipError_t e = hipPointerGetAttributes(&attr, arena_dev);
    int current = -1;
    if (e == hipSuccess) {
      p->device = attr.device;
      e = hipGetDevice(&current);
    } else {
      (void)hipGetLastError();          // memory HIP does not track (a VA reservation): current device
      e = hipGetDevice(&current);
      p->device = current;
    }
    if (e == hipSuccess && current != p->device) {
      delete p;
      return fail(AVMP_ERR_INVALID_ARG, "the arena's GPU must be the current device");
    }
    if (e == hipSuccess) (void)scratch_on_device(p->device, &e);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&p->table_dev), (entries + 2) * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMemset(p->table_dev, 0xFF, entries * sizeof(uint32_t));
    const uint32_t caps[2] = {p->st.capacity(0), p->st.capacity(1)};
    if (e == hipSuccess) e = hipMemcpy(p->table_dev + entries, caps, sizeof caps, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&p->faults_dev), sizeof(unsigned long long));
    if (e == hipSuccess) e = hipMemset(p->faults_dev, 0, sizeof(unsigned long long));
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&p->faults_host), sizeof(unsigned long long), hipHostMallocDefault);
    if (e == hipSuccess && avmp::ssm_may_fuse_conv(cfg->ssm_conv_kernel, cfg->ssm_heads, cfg->ssm_headdim, cfg->ssm_dstate)) {
      const size_t bytes = size_t(kMaxBatch) * avmp::kArrivalStride * sizeof(uint32_t);
      e = hipMalloc(reinterpret_cast<void**>(&p->conv_arrivals_dev), bytes);
      if (e == hipSuccess) e = hipMemset(p->conv_arrivals_dev, 0, bytes);
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
      if (p->conv_arrivals_dev) (void)hipFree(p->conv_arrivals_dev);
      if (p->table_dev) (void)hipFree(p->table_dev);
      if (p->faults_dev) (void)hipFree(p->faults_dev);
      if (p->faults_host) (void)hipHostFree(p->faults_host);
      delete p;
      return fail_hip(e, "avmp_pools_create");
    }
    p->has_device = true;
  }
  *out = p;
  return AVMP_OK;
}

int avmp_pools_destroy(avmp_pools_t* p) {
  if (p == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null pools");
  if (p->has_device) {
    (void)hipDeviceSynchronize();
    p->staging.destroy();
    for (auto* v : {&p->prof, &p->prof_free})
      for (auto& r : *v) {
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
      }
    if (p->ws) (void)hipFree(p->ws);
    for (void* old : p->ws_retired) (void)hipFree(old);
    (void)hipFree(p->table_dev);
    if (p->conv_arrivals_dev) (void)hipFree(p->conv_arrivals_dev);
    (void)hipFree(p->faults_dev);
    (void)hipHostFree(p->faults_host);
  }
  delete p;
  return AVMP_OK;
}

int avmp_alloc(avmp_pools_t* p, int pool, uint32_t n, avmp_handle_t* out) {
  if (p == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null pools");
  // a request larger than the pool is refused before any handle is written
  const size_t room = (pool == 0 || pool == 1) ? p->st.capacity(pool) : 0;
  std::vector<uint32_t> tmp((n < room ? n : room) + 1);
  const size_t upd0 = p->pending.size(), zero0 = p->pending_zero.size();
  const int rc = p->st.alloc(pool, n, out ? tmp.data() : nullptr, &p->pending, &p->pending_zero);
  p->pending_entries = true;
  if (rc != AVMP_OK) {
    p->pending.resize(upd0);
    p->pending_zero.resize(zero0);
    return fail(rc, rc == AVMP_ERR_CAPACITY ? "pool is full" : "bad pool, n or out");
  }
  std::memcpy(out, tmp.data(), size_t(n) * sizeof(uint32_t));
  if (!p->has_device) {
    p->pending.clear();
    p->pending_zero.clear();
  }
  return AVMP_OK;
}

int avmp_free(avmp_pools_t* p, const avmp_handle_t* handles, uint32_t n) {
  if (p == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null pools");
  const int rc = p->st.free_units(handles, n, &p->pending);
  p->pending_entries = true;
  if (rc != AVMP_OK) return fail(rc, rc == AVMP_ERR_INVALID_HANDLE ? "stale or malformed handle" : "bad n");
  if (!p->has_device) p->pending.clear();
  return AVMP_OK;
}

int avmp_policy_set(avmp_pools_t* p, const avmp_policy_t* pol) {
  if (p == nullptr || pol == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null argument");
  if (!(pol->threshold_low >= 0.0 && pol->threshold_low < pol->threshold_high &&
        pol->threshold_high <= 1.0))
    return fail(AVMP_ERR_INVALID_ARG, "need 0 <= threshold_low < threshold_high <= 1");
  if (pol->migration_batch_size < 1) return fail(AVMP_ERR_INVALID_ARG, "migration_batch_size < 1");
  p->rebalancer = avmp::Rebalancer();
  p->rebalancer.policy.threshold_low = pol->threshold_low;
  p->rebalancer.policy.threshold_high = pol->threshold_high;
  p->rebalancer.policy.migration_batch_size = pol->migration_batch_size;
  p->rebalancer.policy.min_rebalance_interval_ops = pol->min_rebalance_interval_ops;
  return AVMP_OK;
}

int avmp_policy_state(const avmp_pools_t* p, avmp_policy_state_t* out) {
  if (p == nullptr || out == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null argument");
  out->state = uint32_t(p->rebalancer.state);
  out->has_rebalanced = p->rebalancer.has_rebalanced ? 1u : 0u;
  out->last_rebalance_op = p->rebalancer.last_rebalance_op;
  out->rebalance_count = p->rebalancer.rebalance_count;
  out->oom_events = p->rebalancer.oom_events;
  return AVMP_OK;
}

int avmp_alloc_auto(avmp_pools_t* p, int pool, uint32_t n, avmp_handle_t* out, void* stream,
                    uint32_t* donor_units_migrated) {
  if (donor_units_migrated) *donor_units_migrated = 0;
  int rc = avmp_alloc(p, pool, n, out);
  if (rc != AVMP_ERR_CAPACITY) return rc;
  // the capacity-error handler: the only place where the state machine runs
  uint32_t donate = 0;
  const avmp::PoolState::Step step = p->st.on_capacity_error(pool, &p->rebalancer, &donate);
  if (step == avmp::PoolState::kStepNone) {
    ++p->rebalancer.oom_events;
    return rc;
  }
  const int mrc = step == avmp::PoolState::kStepFromGap ? avmp_absorb_gap(p, pool, nullptr)
                                                        : avmp_migrate(p, 1 - pool, donate, stream, nullptr);
  if (mrc != AVMP_OK) return mrc;         // cannot happen for a planned step; device errors only
  p->st.rebalance_done(&p->rebalancer);
  if (donor_units_migrated) *donor_units_migrated = donate;
  rc = avmp_alloc(p, pool, n, out);
  if (rc == AVMP_ERR_CAPACITY) ++p->rebalancer.oom_events;
  return rc;
}

int avmp_absorb_gap(avmp_pools_t* p, int pool, avmp_migrate_result_t* out) {
  if (p == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null pools");
  if (p->dead) return fail(AVMP_ERR_DEVICE, kDeadPools);
  uint32_t gain = 0;
  uint64_t wasted = 0;
  const int rc = p->st.absorb_gap(pool, &gain, &wasted);
  if (rc != AVMP_OK)
    return fail(rc, rc == AVMP_ERR_CAPACITY ? "the gap holds less than one unit of this pool" : "bad pool");
  if (p->has_device) p->queue_capacities();
  if (out) {
    out->units_copied = 0;
    out->recipient_gain = gain;
    out->bytes_wasted = wasted;
  }
  return AVMP_OK;
}

int avmp_flush(avmp_pools_t* p, void* stream) {
  if (p == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null pools");
  return flush_pending(p, static_cast<hipStream_t>(stream));
}

int avmp_migrate(avmp_pools_t* p, int donor, uint32_t n, void* stream, avmp_migrate_result_t* out) {
  if (p == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null pools");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (p->dead) return fail(AVMP_ERR_DEVICE, kDeadPools);
  if (p->has_device && (donor == 0 || donor == 1) && n != 0 &&
      (p->pending_entries || !p->pending_zero.empty())) {
    // queued zero fills and table entries refer to the geometry before the move (the copy
    // kernel rewrites entries in stream order; queued capacities alone can wait)
    const int rc = flush_pending(p, s);
    if (rc != AVMP_OK) return rc;
  }
  const int rc = p->st.migrate_begin(donor, n);
  if (rc != AVMP_OK)
    return fail(rc, rc == AVMP_ERR_CAPACITY ? "donor has too few free units" : "bad donor or n");
  // from here on nothing can fail but a HIP call
  uint32_t moved = 0;
  const bool exchange = p->has_device && p->remap != nullptr && p->remappable[donor];
  if (p->has_device && !exchange && n <= avmp::kInlineMoves) {
    // a short migration (the policy's default batch): the whole move list rides in the
    // arguments of one copy launch
    avmp::InlineMoves im{};
    moved = p->st.migrate_moves(im.mv, n);          // at most n units move
    if (moved != 0) {
      im.P = p->dev_view();
      im.table = p->table_dev;
      im.pool = donor;
      im.n = moved;
      ProfScope scope(p, p->profiling, AVMP_K_MIGRATE_COPY, s);
      const hipError_t e = avmp::launch_migrate_copy_inline(im, s);
      if (e != hipSuccess) {
        p->dead = true;
        return fail_hip(e, "avmp_migrate: copy launch");
      }
    }
  } else if (p->has_device && !exchange) {
    // The moves are planned straight into pinned memory, a slice at a time, and each slice's
    // copy is launched before the next is planned: the device copies while the host plans.
    // The copy kernel rewrites the table entries of the units it moves.
    // Slices grow (1024, 2048, 4096, ... up to 8192 moves): the first copy starts early, the
    // later ones are long enough to run at full rate.
    uint32_t slice = 1024;
    Staging::Buf* b = nullptr;
    avmp::Move* list = nullptr;
    for (;;) {
      if (b == nullptr) {                     // at most n units move: one list for the whole call
        const hipError_t e = p->staging.acquire(size_t(n) * sizeof(avmp::Move), &b);
        if (e != hipSuccess) {
          p->dead = true;                     // the host tables are half way through a migration
          return fail_hip(e, "avmp_migrate: pinned memory for the move list");
        }
        list = static_cast<avmp::Move*>(b->host);
      }
      const uint32_t k = p->st.migrate_moves(list + moved, slice);
      if (k == 0) break;
      if (slice < 8192) slice *= 2;
      {
        ProfScope scope(p, p->profiling, AVMP_K_MIGRATE_COPY, s);
        const hipError_t e = avmp::launch_migrate_copy(p->dev_view(), p->table_dev, donor, list + moved, k, s);
        if (e != hipSuccess) {
          p->dead = true;
          return fail_hip(e, "avmp_migrate: copy launch");
        }
      }
      moved += k;
    }
    const hipError_t e = p->staging.release_after(b, s);
    if (e != hipSuccess) {
      p->dead = true;
      return fail_hip(e, "avmp_migrate: event behind the move list");
    }
  } else {
    std::vector<avmp::Move> moves(n);
    for (uint32_t k; (k = p->st.migrate_moves(moves.data() + moved, n - moved)) != 0;) moved += k;
    if (exchange && moved != 0) {
      // nothing may touch a range while its backing changes
      hipError_t e = hipDeviceSynchronize();
      const uint64_t unit = p->st.geometry().unit[donor];
      for (uint32_t i = 0; e == hipSuccess && i < moved; ++i)
        e = p->remap->exchange(p->st.byte_offset(donor, moves[i].src_slot),
                               p->st.byte_offset(donor, moves[i].dst_slot), unit);
      if (e != hipSuccess) {
        p->dead = true;
        return fail_hip(e, "avmp_migrate: exchanging the backing of two slots");
      }
      for (uint32_t i = 0; i < moved; ++i)
        p->pending.push_back({p->st.vid_base(donor) + moves[i].vid, moves[i].dst_slot});
      p->pending_entries = true;
    }
  }
  uint32_t gain = 0;
  uint64_t wasted = 0;
  p->st.migrate_end(&gain, &wasted);
  if (p->has_device) p->queue_capacities();   // reach the device with the next flush, before any kernel
  if (out) {
    out->units_copied = moved;
    out->recipient_gain = gain;
    out->bytes_wasted = wasted;
  }
  return AVMP_OK;
}

uint64_t avmp_vmm_min_chunk(void) { return avmp::VmmArena::min_chunk(); }

int avmp_vmm_arena_create(uint64_t bytes, uint64_t chunk_bytes, avmp_vmm_arena_t** out) {
  if (out == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null out");
  const uint64_t g = avmp::VmmArena::min_chunk();
  if (g == 0) return fail(AVMP_ERR_DEVICE, "device has no virtual-memory support");
  if (bytes == 0 || chunk_bytes == 0 || chunk_bytes % g != 0 || bytes % chunk_bytes != 0)
    return fail(AVMP_ERR_INVALID_ARG,
                "bytes must be a multiple of chunk_bytes, chunk_bytes of avmp_vmm_min_chunk()");
  avmp_vmm_arena* a = new (std::nothrow) avmp_vmm_arena();
  if (a == nullptr) return fail(AVMP_ERR_INVALID_ARG, "out of host memory");
  const hipError_t e = a->impl.create(bytes, chunk_bytes);
  if (e != hipSuccess) {
    delete a;
    return fail_hip(e, "avmp_vmm_arena_create");
  }
  *out = a;
  return AVMP_OK;
}

void* avmp_vmm_arena_base(const avmp_vmm_arena_t* a) { return a ? a->impl.base() : nullptr; }

int avmp_vmm_arena_destroy(avmp_vmm_arena_t* a) {
  if (a == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null arena");
  delete a;
  return AVMP_OK;
}

int avmp_migrate_by_remap(avmp_pools_t* p, avmp_vmm_arena_t* a) {
  if (p == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null pools");
  if (a == nullptr) {
    p->remap = nullptr;
    return AVMP_OK;
  }
  if (!p->has_device) return fail(AVMP_ERR_DEVICE, "pools have no device arena");
  const avmp::Geometry& g = p->st.geometry();
  const uint64_t chunk = a->impl.chunk();
  if (a->impl.broken() || p->arena != a->impl.base() || g.usable > a->impl.bytes())
    return fail(AVMP_ERR_INVALID_ARG, "the pools do not sit on this arena");
  // KV slots start at multiples of their unit, SSM slots at usable minus such multiples
  const bool kv_ok = g.unit[0] % chunk == 0;
  const bool ssm_ok = g.unit[1] % chunk == 0 && g.usable % chunk == 0;
  if (!kv_ok && !ssm_ok)
    return fail(AVMP_ERR_INVALID_ARG, "no pool's slots cover whole chunks of this arena");
  p->remap = &a->impl;
  p->remappable[0] = kv_ok;
  p->remappable[1] = ssm_ok;
  return AVMP_OK;
}

int avmp_decode_step(avmp_pools_t* p, const avmp_step_t* st, void* stream) {
  uint32_t n_attn = 0, n_ssm = 0;
  int rc = check_step(p, st, &n_attn, &n_ssm);
  if (rc != AVMP_OK) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  rc = flush_pending(p, s);
  if (rc != AVMP_OK) return rc;
  if (st->batch == 0) return AVMP_OK;
  const WorkLayout L = work_layout(p->cfg, n_attn, n_ssm, st->batch, st->max_pages);
  if (L.bytes() > p->ws_bytes) {
    const WorkLayout roomy = work_layout(p->cfg, n_attn, n_ssm, st->batch, roomy_pages(st->max_pages));
    rc = grow_workspace(p, roomy.bytes());
    if (rc != AVMP_OK) return rc;
  }
  return run_step(p, st, s, n_attn, L, p->ws, p->profiling);
}

int avmp_decode_step_noalloc(avmp_pools_t* p, const avmp_step_t* st, void* stream) {
  uint32_t n_attn = 0, n_ssm = 0;
  const int rc = check_step(p, st, &n_attn, &n_ssm);
  if (rc != AVMP_OK) return rc;
  // pushing queued table updates takes pinned staging memory and events: not in this call
  if (!p->pending.empty() || !p->pending_zero.empty())
    return fail(AVMP_ERR_INVALID_ARG,
                "table updates or zero fills are queued: call avmp_flush before avmp_decode_step_noalloc");
  if (st->batch == 0) return AVMP_OK;
  const WorkLayout L = work_layout(p->cfg, n_attn, n_ssm, st->batch, st->max_pages);
  if (L.bytes() > kScratchBytes) {
    char msg[160];
    std::snprintf(msg, sizeof msg,
                  "this step needs a work buffer of %zu bytes; the static one holds %zu "
                  "(AVMP_NOALLOC_WORKSPACE_BYTES)", L.bytes(), kScratchBytes);
    return fail(AVMP_ERR_INVALID_ARG, msg);
  }
  hipError_t e = hipSuccess;
  void* ws = scratch_on_device(p->device, &e);
  if (ws == nullptr) return fail_hip(e, "hipGetSymbolAddress(scratch)");
  // no per-kernel event pairs here: creating events allocates
  return run_step(p, st, static_cast<hipStream_t>(stream), n_attn, L, static_cast<float*>(ws), false);
}

int avmp_workspace_reserve(avmp_pools_t* p, uint32_t n_attention_layers, uint32_t n_ssm_layers,
                           uint32_t batch, uint32_t max_pages) {
  if (p == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null pools");
  if (!p->has_device) return fail(AVMP_ERR_DEVICE, "pools have no device arena");
  if (batch > 65535) return fail(AVMP_ERR_INVALID_ARG, "batch above 65535");
  return grow_workspace(p, work_layout(p->cfg, n_attention_layers, n_ssm_layers, batch, max_pages).bytes());
}

int avmp_workspace_info(const avmp_pools_t* p, uint64_t* bytes, uint64_t* allocations) {
  if (p == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null pools");
  if (bytes) *bytes = p->ws_bytes;
  if (allocations) *allocations = p->ws_allocations;
  return AVMP_OK;
}

int avmp_translate(avmp_pools_t* p, const avmp_handle_t* handles_dev, uint32_t n,
                   uint64_t* offsets_dev, void* stream) {
  if (p == nullptr || (n && (!handles_dev || !offsets_dev)))
    return fail(AVMP_ERR_INVALID_ARG, "null argument");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int rc = flush_pending(p, s);
  if (rc != AVMP_OK) return rc;
  HIP_TRY(avmp::launch_translate(p->dev_view(), handles_dev, n, offsets_dev, s));
  return AVMP_OK;
}

int avmp_resolve(const avmp_pools_t* p, avmp_handle_t h, uint32_t* pool, uint32_t* slot,
                 uint64_t* byte_off) {
  if (p == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null pools");
  uint32_t pl, sl;
  uint64_t off;
  if (!p->st.resolve(h, &pl, &sl, &off)) return fail(AVMP_ERR_INVALID_HANDLE, "not a live handle");
  if (pool) *pool = pl;
  if (slot) *slot = sl;
  if (byte_off) *byte_off = off;
  return AVMP_OK;
}

int avmp_stats(const avmp_pools_t* p, avmp_stats_t* out) {
  if (p == nullptr || out == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null argument");
  const avmp::Counters& c = p->st.counters();
  for (int i = 0; i < 2; ++i) {
    out->capacity[i] = p->st.capacity(i);
    out->live[i] = p->st.live(i);
    out->free_units[i] = p->st.capacity(i) - p->st.live(i);
  }
  out->gap_bytes = p->st.gap();
  out->ops = c.ops;
  out->capacity_errors = c.capacity_errors;
  out->migrations = c.migrations;
  out->units_copied = c.units_copied;
  out->bytes_migrated = c.bytes_migrated;
  out->bytes_wasted = c.bytes_wasted;
  return AVMP_OK;
}

int avmp_profile_enable(avmp_pools_t* p, int on) {
  if (p == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null pools");
  if (!p->has_device) return fail(AVMP_ERR_DEVICE, "pools have no device arena");
  p->profiling = on != 0;
  return AVMP_OK;
}

int avmp_profile_read(avmp_pools_t* p, void* stream, avmp_profile_t* out) {
  if (p == nullptr || out == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null argument");
  if (!p->has_device) return fail(AVMP_ERR_DEVICE, "pools have no device arena");
  HIP_TRY(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  std::memset(out, 0, sizeof(*out));
  hipError_t first_error = hipSuccess;
  for (const auto& r : p->prof) {           // every pair goes back to the free list, whatever happens
    float ms = 0.f;
    const hipError_t e = hipEventElapsedTime(&ms, r.a, r.b);
    if (e == hipSuccess) {
      out->ms[r.kind] += double(ms);
      out->launches[r.kind] += 1;
    } else if (first_error == hipSuccess) {
      first_error = e;
    }
    p->prof_free.push_back(r);
  }
  p->prof.clear();
  if (first_error != hipSuccess) return fail_hip(first_error, "hipEventElapsedTime");
  return AVMP_OK;
}

int avmp_device_faults(avmp_pools_t* p, void* stream, uint64_t* out) {
  if (p == nullptr || out == nullptr) return fail(AVMP_ERR_INVALID_ARG, "null argument");
  if (!p->has_device) return fail(AVMP_ERR_DEVICE, "pools have no device arena");
  // read and reset in stream order, behind the kernels already queued and ahead of later ones
  hipStream_t s = static_cast<hipStream_t>(stream);
  HIP_TRY(hipMemcpyAsync(p->faults_host, p->faults_dev, sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipMemsetAsync(p->faults_dev, 0, sizeof(unsigned long long), s));
  HIP_TRY(hipStreamSynchronize(s));
  *out = *p->faults_host;
  return AVMP_OK;
}

}  // extern "C"
