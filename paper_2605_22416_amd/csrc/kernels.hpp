// Launchers of the gfx950 kernels.  Each returns the hipError_t of its launch.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "device_common.hpp"
#include "pool_state.hpp"

namespace avmp {

struct AttnLaunch {
  DevPools P;
  const uint32_t* handles;   // device [batch][max_pages] of this layer
  const uint32_t* ctx;       // device [batch]
  const void* q;             // device [batch][Hq][D]
  float* o;                  // device [batch][Hq][D]
  float* part_o;             // device [batch][max_chunks][Hq][D]
  float* part_ml;            // device [batch][max_chunks][Hq][2]
  uint32_t batch, max_pages, max_chunks;
  uint32_t n_q_heads, n_kv_heads, head_dim;
  uint32_t dtype;            // 0 f32, 1 bf16
  uint32_t append;           // 1: the step appended one token, attend over ctx + 1 tokens
  const void* k_new;         // device [batch][Hkv][D] (append only)
  const void* v_new;         // device [batch][Hkv][D] (append only)
  // matrix-core path only: balanced runs (see attn_mfma.hip)
  const uint32_t* plan;      // device [2]: total pages, cost per run
  const uint32_t* prefix;    // device [batch + 1]: page prefix sums
  const uint32_t* pos;       // device [batch + 1]: cost prefix sums (the axis the runs are cut on)
  const uint4* desc;         // device [runs]: each run's first (request, page) and its stretch
                             // [first, last) of the batch's page sequence
  const uint32_t* slots;     // device [batch][max_pages]: this layer's pre-translated slots
  uint32_t runs;             // runs (wavefronts) per KV head
};

struct SsmLaunch {
  DevPools P;
  const uint32_t* handles;   // device [batch]
  const void* x;             // device [batch][H][P]
  const float* dt;           // device [batch][H]
  const float* A;            // device [H]
  const void* B;             // device [batch][N]
  const void* C;             // device [batch][N]
  float* y;                  // device [batch][H][P]
  uint32_t batch, heads, headdim, dstate;
  uint32_t dtype;            // x, B, C element type: 0 f32, 1 bf16
  uint32_t state_dtype;      // storage type of the state block: 0 f32, 1 bf16
  // Convolution done by the recurrence kernel itself (conv_k != 0; see ssm_fuses_conv): x, B and
  // C above are not read, they come out of the block's window and these; dtype is their type.
  const void* conv_u;        // device [batch][H*P + 2*N] elements: this token's inputs
  const void* conv_taps;     // device [K][H*P + 2*N] elements
  const void* conv_bias;     // device [H*P + 2*N] elements
  uint32_t* conv_arrivals;   // device [batch][kArrivalStride], zero between launches: workgroups of a request that
                             // have read its window
  uint32_t conv_k;           // taps, 0: no convolution
};

struct ConvLaunch {
  DevPools P;
  const uint32_t* handles;   // device [batch]: SSM blocks whose window is used and advanced
  const void* u;             // device [batch][conv_dim] elements: this token's inputs
  const void* taps;          // device [K][conv_dim] elements, tap K-1 meets the newest token
  const void* bias;          // device [conv_dim] elements
  float* x;                  // device [batch][H][P] out
  float* B;                  // device [batch][N] out
  float* C;                  // device [batch][N] out
  uint64_t state_bytes;      // bytes of recurrent state in front of the window
  uint32_t batch, heads, headdim, dstate, conv_dim, taps_k;
  uint32_t dtype;            // element type of u, taps, bias and the window: 0 f32, 1 bf16
};

// Short lists travel inside the kernel arguments instead of pinned staging memory: nothing to
// keep alive behind the launch, so no event, and one launch for a flush's table entries and
// zero fills.  Sized to stay under the 4 KiB a launch may carry.
constexpr uint32_t kInlineUpdates = 416, kInlineZero = 64, kInlineMoves = 300;

struct InlineFlush {
  DevPools P;
  uint32_t* table;
  uint32_t n_upd, n_zero;
  uint32_t ssm_capacity;            // the host's value at the flush: slots at or beyond it are not cleared
  uint32_t pad_;
  TableUpdate upd[kInlineUpdates];  // coalesced: one entry per index
  uint32_t zero[kInlineZero];       // SSM slots to clear
};
static_assert(sizeof(InlineFlush) <= 4096, "kernel arguments are limited to 4 KiB");

struct InlineMoves {
  DevPools P;
  uint32_t* table;
  int pool;
  uint32_t n;
  Move mv[kInlineMoves];
};
static_assert(sizeof(InlineMoves) <= 4096, "kernel arguments are limited to 4 KiB");

hipError_t launch_flush_inline(const InlineFlush& f, hipStream_t s);
hipError_t launch_migrate_copy_inline(const InlineMoves& m, hipStream_t s);

bool conv_supported(uint32_t dtype, uint32_t taps_k, uint32_t heads, uint32_t headdim,
                    uint32_t dstate);
hipError_t launch_conv_update(const ConvLaunch& a, hipStream_t s);
hipError_t launch_kv_append(const AttnLaunch& a, hipStream_t s);
hipError_t launch_attention(const AttnLaunch& a, hipStream_t s);
// matrix-core variant (attn_mfma.hip): bf16, head_dim 64/128/256, query group <= 16
bool attention_mfma_supported(uint32_t dtype, uint32_t n_q_heads, uint32_t n_kv_heads,
                              uint32_t head_dim);
uint32_t attention_runs_per_head(uint32_t n_kv_heads);
// once per decode step: run plan, zero rows of empty requests (o_all is
// [n_attn][batch][Hq][D]) and the handles of all attention layers -> slots
hipError_t launch_attention_prepare(const AttnLaunch& a, const uint32_t* handles_all, uint32_t n_attn,
                                    uint32_t* slots_all, float* o_all, hipStream_t s);
hipError_t launch_attention_mfma(const AttnLaunch& a, hipStream_t s);
hipError_t launch_attention_merge_runs(const AttnLaunch& a, hipStream_t s);
hipError_t launch_attention_merge(const AttnLaunch& a, hipStream_t s);
// Arrival counters sit a cache line apart: additions to one line are carried out one after the
// other, whichever word they go to (counters of 64 requests packed into two lines: 110 us per layer
// against 86 us without the convolution).
constexpr uint32_t kArrivalStride = 32;

// Whether the recurrence kernel runs the layer's convolution itself, so that no convolution
// launch is needed: at the Mamba-2 head shape (headdim 64 x dstate 128) with four taps, for
// every launch with a bf16 state and for the shorter launches with an fp32 state (measured, us
// per layer, convolution + recurrence as two launches against one: fp32 state 7.9 + 90.2
// against 92.5 at 64 requests of 128 heads, 15.2 + 333.7 against 361.8 at 256; bf16 state
// 8.0 + 49.8 against 52.3 and 15.1 + 190.7 against 191.9).  ssm_may_fuse_conv: for some batch.
bool ssm_may_fuse_conv(uint32_t taps_k, uint32_t heads, uint32_t headdim, uint32_t dstate);
bool ssm_fuses_conv(uint32_t taps_k, uint32_t heads, uint32_t headdim, uint32_t dstate,
                    uint32_t state_dtype, uint32_t batch);
hipError_t launch_ssm(const SsmLaunch& a, hipStream_t s);
hipError_t launch_table_updates(uint32_t* table, const TableUpdate* upd, uint32_t n, hipStream_t s);
hipError_t launch_zero_units(const DevPools& P, int pool, const uint32_t* slots, uint32_t n,
                             hipStream_t s);
hipError_t launch_migrate_copy(const DevPools& P, uint32_t* table, int pool, const Move* moves,
                               uint32_t n, hipStream_t s);
hipError_t launch_translate(const DevPools& P, const uint32_t* handles, uint32_t n, uint64_t* out,
                            hipStream_t s);

}  // namespace avmp
