/*
 * avmp.h - C ABI of the MI355X hybrid decode path over asymmetric pools.
 *
 * Two physically distinct pools, KV pages and SSM state blocks, live in ONE
 * caller-owned device arena behind one 32-bit virtual handle space (paper:
 * Method, "Asymmetric Virtual Page Table", Fig. 1).  The library keeps the
 * virtual page table on the host, mirrors it on the device, and runs the steps
 * that read through it as gfx950 kernels: handle translation, paged
 * grouped-query decode attention, the single-token SSM state update done in
 * place, and the capacity migration that copies units and rewrites the table
 * (Method, "Dynamic Pool Rebalancing").
 *
 * Conventions
 *  - plain C, int status returns, no callbacks; out-parameters are written
 *    only on AVMP_OK; a failing call leaves every observable unchanged except
 *    the logical operation counter where stated.
 *  - "host" / "device" on a pointer says where the memory must live.  The
 *    caller owns the arena, every input/output buffer and the stream; the
 *    library owns its metadata, the device table mirror and a work buffer.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    avmp_decode_step, avmp_migrate, avmp_flush and avmp_translate are
 *    asynchronous on it.  All device work of one pools object must be issued
 *    on one stream or be ordered by the caller.
 *  - AVMP_ERR_DEVICE from avmp_migrate, avmp_alloc_auto or avmp_decode_step means a
 *    HIP call failed after host metadata may already have changed: the pools
 *    object must then be destroyed.  Every other error is a clean no-op.
 *  - avmp_decode_step keeps split-K partial results, its run plan and the
 *    translated slots in a work buffer of the library's.  The buffer is
 *    allocated on first use (or by avmp_workspace_reserve) for twice the handle
 *    row in hand and at least 64 pages per request; it only ever grows, by a
 *    factor of two or more, without waiting for the device, and an outgrown
 *    buffer stays allocated until the pools are destroyed.  With the buffer in
 *    place and nothing queued, a step only launches kernels and can be captured
 *    in a HIP graph.
 *  - not thread-safe: one thread per pools object (the paper's allocator is
 *    single-process).
 *
 * Arena geometry.  usable = arena_bytes rounded down to 128.  KV slot s is at
 * arena + s*unit_kv (ascending from the base); SSM slot i is at
 * arena + usable - (i+1)*unit_ssm (descending from the top).  The high ends of
 * both slot ranges face one shared gap, so "the donor shrinks at the high end
 * of its address space and the recipient grows" holds in a single arena.
 * Slab anchors are 128-byte aligned, units 16-byte aligned (Method,
 * "Asymmetric Virtual Page Table").
 *
 * Layout inside a KV page (not fixed by the paper; chosen so that a wavefront's
 * 16-byte loads are contiguous AND already in matrix-core operand order).
 * With T = 16 tokens, G = KV heads, D = head_dim, x = 16 / element_bytes:
 *    K element (g, t, d) at element index ((g*(D/x) + d/x)*T + t)*x + d%x
 *    V element (g, t, d) at element index G*T*D + (g*D + d)*T + t
 * An SSM block is [ssm_heads][ssm_headdim][ssm_dstate], row-major, fp32 or bf16
 * (ssm_state_dtype), followed by the convolution window if ssm_conv_kernel is set.
 */
#ifndef AVMP_H
#define AVMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* 32-bit virtual handle: bits [31:30] pool tag, bits [29:0] virtual page id
 * (Fig. 1: pool_id | page_id).  All-ones is never a valid handle. */
typedef uint32_t avmp_handle_t;
#define AVMP_PAGE_ID_BITS 30u
#define AVMP_INVALID_HANDLE 0xFFFFFFFFu

enum {
  AVMP_OK = 0,
  AVMP_ERR_CAPACITY = 1,        /* the paper's CapacityError */
  AVMP_ERR_INVALID_HANDLE = 2,
  AVMP_ERR_INVALID_ARG = 3,
  AVMP_ERR_DEVICE = 4           /* a HIP call failed, or no device attached */
};
enum { AVMP_POOL_KV = 0, AVMP_POOL_SSM = 1 };
enum { AVMP_F32 = 0, AVMP_BF16 = 1 };
enum { AVMP_LAYER_ATTENTION = 0, AVMP_LAYER_SSM = 1 };

typedef struct avmp_pools avmp_pools_t;     /* opaque, owned by the library */

typedef struct avmp_config {
  uint32_t dtype;                  /* AVMP_F32 / AVMP_BF16: element type of K, V, q, x, B, C */
  uint32_t attention_page_tokens;  /* tokens per KV page; only 16 (the paper's default) */
  uint32_t n_q_heads;              /* multiple of n_kv_heads */
  uint32_t n_kv_heads;
  uint32_t head_dim;               /* multiple of 16/element_bytes */
  uint32_t ssm_heads;              /* H */
  uint32_t ssm_headdim;            /* P */
  uint32_t ssm_dstate;             /* N: power of two, 4..256 */
  uint32_t ssm_state_dtype;        /* AVMP_F32 (default, 0) or AVMP_BF16: storage type of the SSM
                                      state in its block (the paper's bytes_per_element).
                                      Arithmetic is fp32 either way; bf16 storage needs N >= 8 */
  uint32_t ssm_conv_kernel;        /* 0 (default): the block is the recurrent state alone.  2..4: K
                                      taps of the layer's short causal convolution; the block then
                                      also keeps, behind the state, the inputs of the last K-1 tokens
                                      as [K-1][H*P + 2*N] elements (oldest first), and a step takes
                                      xbc / conv_taps / conv_bias instead of x, B, C.  Needs H*P and
                                      N to be multiples of 16/element_bytes.  With K = 4, P = 64 and
                                      N = 128 the recurrence kernel runs the convolution itself and
                                      the pools hold 8 MiB more device memory (one arrival counter
                                      per request of the largest batch, a cache line apart) */
  uint32_t ssm_pad_to_kv_page;     /* 0 (default): the block has its native size.  1: the sizing of a
                                      unified pool (Background, "Existing Cache Management"; the
                                      padded_unified baseline of Evaluation, "Experimental Setup"):
                                      the block is padded up to a whole number of KV pages.  Only the
                                      unit size changes; avmp_geometry reports both sizes */
  uint32_t kv_capacity;            /* initial KV pool capacity in pages */
  uint32_t ssm_capacity;           /* initial SSM pool capacity in blocks */
  uint32_t max_vid[2];             /* virtual ids per pool; 0 = as many as slots could ever exist */
  const uint32_t* slot_rank[2];    /* host, or NULL = identity.  A permutation of
                                      [0, max_slots[pool]): allocation takes the free slot of
                                      LOWEST rank below the pool's capacity.  Copied at create. */
} avmp_config_t;

typedef struct avmp_geometry {
  uint64_t unit_bytes[2];          /* KV page bytes, SSM block bytes (rounded up to 16; with
                                      ssm_pad_to_kv_page to a multiple of the KV page) */
  uint64_t ssm_native_bytes;       /* SSM block bytes without that padding */
  uint64_t usable_bytes;
  uint32_t max_slots[2];           /* usable_bytes / unit_bytes[pool] */
} avmp_geometry_t;

typedef struct avmp_migrate_result {
  uint32_t units_copied;           /* live donor units moved out of the vacated range */
  uint32_t recipient_gain;         /* new recipient slots */
  uint64_t bytes_wasted;           /* (gap before + n*unit_donor) mod unit_recipient: the paper's
                                      wasted bytes; kept as the gap and reused next time */
} avmp_migrate_result_t;

typedef struct avmp_stats {
  uint32_t capacity[2];
  uint32_t live[2];
  uint32_t free_units[2];
  uint64_t gap_bytes;
  uint64_t ops;                    /* logical operation counter: alloc/free/migrate calls that
                                      passed argument validation, successful or not */
  uint64_t capacity_errors;        /* avmp_alloc calls refused with AVMP_ERR_CAPACITY */
  uint64_t migrations;
  uint64_t units_copied;
  uint64_t bytes_migrated;         /* sum of n*unit_donor over successful migrations */
  uint64_t bytes_wasted;           /* sum of per-migration bytes_wasted */
} avmp_stats_t;

/* One hybrid decode step: layers in model order; per-kind arrays are indexed by
 * the layer's ordinal among layers of its kind.  ctx counts tokens already
 * resident; the step appends the new token only if k_new / v_new are given.
 * Two requests of one batch must not name the same SSM handle. */
typedef struct avmp_step {
  uint32_t batch;                    /* at most 65535; with attention layers, batch x max_pages < 2^31 */
  uint32_t n_layers;
  const uint8_t* layer_kind;         /* host [n_layers]: AVMP_LAYER_* */
  uint32_t max_pages;                /* row stride of kv_handles; >= ceil(max ctx / 16) */
  const avmp_handle_t* kv_handles;   /* device [n_attn][batch][max_pages]; entries at or beyond
                                        ceil(ctx/16) are ignored */
  const uint32_t* ctx;               /* device [batch] tokens resident per request (may be 0) */
  const void* q;                     /* device [n_attn][batch][n_q_heads][head_dim] elements, 16-byte aligned */
  float* o;                          /* device [n_attn][batch][n_q_heads][head_dim] fp32 out, 16-byte aligned */
  const avmp_handle_t* ssm_handles;  /* device [n_ssm][batch] */
  const void* x;                     /* device [n_ssm][batch][H][P] elements */
  const float* dt;                   /* device [n_ssm][batch][H] fp32, already positive */
  const float* A;                    /* device [n_ssm][H] fp32 (negative decay rates) */
  const void* B;                     /* device [n_ssm][batch][N] elements */
  const void* C;                     /* device [n_ssm][batch][N] elements */
  float* y;                          /* device [n_ssm][batch][H][P] fp32 out */
  /* Optional append of the step's new token (both NULL: no append).  When given,
   * each attention layer first writes the token's K and V rows into token slot
   * ctx % 16 of page ctx / 16 of every request (the caller has allocated that
   * page and placed its handle in kv_handles), then attends over ctx + 1 tokens.
   * ctx itself is not modified. */
  const void* k_new;                 /* device [n_attn][batch][n_kv_heads][head_dim] elements */
  const void* v_new;                 /* device [n_attn][batch][n_kv_heads][head_dim] elements */
  /* Pools created with ssm_conv_kernel = K take these three instead of x, B and C
   * (which are then ignored; all three 16-byte aligned).  Each SSM layer first runs
   * its short convolution for the new token, per channel c of [x (H*P) | B (N) | C (N)]:
   *   v = conv_bias[c] + sum_k conv_taps[k][c] * input_{t-(K-1)+k}[c],  out = v / (1 + exp(-v)),
   * tap K-1 meeting xbc and the earlier taps the window kept in the block, which then
   * moves on by one token; the fp32 outputs feed the recurrence unrounded. */
  const void* xbc;                   /* device [n_ssm][batch][H*P + 2*N] elements */
  const void* conv_taps;             /* device [n_ssm][K][H*P + 2*N] elements */
  const void* conv_bias;             /* device [n_ssm][H*P + 2*N] elements */
} avmp_step_t;

/* Size arithmetic of Method, "Asymmetric Virtual Page Table": KV page =
 * attention_page_tokens x per_token_bytes (K and V of one attention layer, all
 * KV heads), SSM block = state_dim x bytes_per_element (4 or 2), plus the convolution
 * window if configured; both rounded up to 16.
 * Host only.  AVMP_ERR_INVALID_ARG on unsupported shapes. */
int avmp_geometry(const avmp_config_t* cfg, size_t arena_bytes, avmp_geometry_t* out);

/* Create the two pools over a caller-owned arena (Method, "Asymmetric Virtual
 * Page Table": KVPagesStore + SSMBlocksStore behind one VirtualPageTable).
 * arena_dev: device pointer, 128-byte aligned, arena_bytes long, must outlive
 * the pools.  arena_dev == NULL creates metadata-only pools (the paper's
 * prototype mode: tables and counters, no data movement); on such pools
 * avmp_migrate updates tables only and every device entry point returns
 * AVMP_ERR_DEVICE.  Initial capacities must fit: else AVMP_ERR_INVALID_ARG. */
int avmp_pools_create(const avmp_config_t* cfg, void* arena_dev, size_t arena_bytes,
                      avmp_pools_t** out);
int avmp_pools_destroy(avmp_pools_t* pools);

/* allocate() of Method, "Dynamic Pool Rebalancing": take n units of `pool`.
 * All-or-nothing.  Each unit gets the lowest free virtual id and the
 * best-ranked free slot below the pool's capacity; out[0..n) (host) receives
 * the handles.  AVMP_ERR_CAPACITY (counted) if fewer than n units are free.
 * New SSM blocks read as zero: the zero fill is queued and executed on the
 * stream of the next avmp_flush / avmp_decode_step / avmp_migrate, so a caller
 * that writes a block itself must call avmp_flush first. n == 0: INVALID_ARG. */
int avmp_alloc(avmp_pools_t* pools, int pool, uint32_t n, avmp_handle_t* out);

/* The inverse of allocate() (Method, "Dynamic Pool Rebalancing": units return to
 * the pool their handle's tag names; Fig. 1's table entry is unmapped).  Returns n
 * units (host array of handles, pools may be mixed).  Any stale, duplicate or
 * malformed handle: AVMP_ERR_INVALID_HANDLE, nothing freed. */
int avmp_free(avmp_pools_t* pools, const avmp_handle_t* handles, uint32_t n);

/* Capacity migration of Method, "Dynamic Pool Rebalancing": the donor pool
 * shrinks by n_donor_units at the high end of its slot range and the other
 * pool grows.  Live donor units in the vacated range are first copied on the
 * device to the best-ranked free slots below the new capacity and the table is
 * rewritten (handles stay valid).  All-or-nothing (the paper's rollback
 * clause): AVMP_ERR_CAPACITY if the donor has fewer than n free units.  The
 * moves are planned straight into pinned memory and copied in slices (1024 units,
 * then 2048, 4096 and 8192), each launched on `stream` while the host plans the next. */
int avmp_migrate(avmp_pools_t* pools, int donor_pool, uint32_t n_donor_units, void* stream,
                 avmp_migrate_result_t* out);

/* The bytes between the two pools belong to neither: what a migration left over
 * (its wasted bytes, Method, "Dynamic Pool Rebalancing") and whatever the arena
 * holds beyond the initial capacities.  avmp_absorb_gap gives `pool` every whole
 * unit that fits into them: its capacity grows by gap / unit slots just above the
 * old capacity, nothing is copied, nobody shrinks; the remainder stays in the gap
 * and is reported as bytes_wasted (units_copied = 0).  Counted as a migration of
 * zero donor bytes.  AVMP_ERR_CAPACITY, nothing changed, if the gap holds less than
 * one unit.  Host only: the new capacity reaches the device with the next flush. */
int avmp_absorb_gap(avmp_pools_t* pools, int pool, avmp_migrate_result_t* out);

/* One hybrid decode step over both caches (Background, "KV Cache and SSM State
 * Management": paged scatter-gather reads of the KV cache, in-place contiguous
 * update of one SSM block per layer per sequence; handles resolved as in Fig. 1):
 * translation + paged GQA attention + SSM update for every layer of `step`,
 * enqueued on `stream`.  Attention per (request r, query
 * head j, g = j / (n_q_heads/n_kv_heads)): o = softmax_t(q.K_t[g]/sqrt(D)) . V[g]
 * over the ctx[r] resident tokens; SSM per (r, h, p, n): a = exp(dt*A),
 * S <- a*S + dt*x*B[n] in place, y = sum_n S*C[n] with the updated S (before it is
 * rounded to a bf16 block, when the state is stored as bf16). */
int avmp_decode_step(avmp_pools_t* pools, const avmp_step_t* step, void* stream);

/* avmp_decode_step for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and same results as avmp_decode_step, but the work
 * buffer is a static device array of AVMP_NOALLOC_WORKSPACE_BYTES that each GPU the
 * library runs on holds from first use until the process ends, and the call
 * allocates nothing (no device, pinned or event allocation).
 *  - table updates and zero fills queued by avmp_alloc / avmp_free / avmp_migrate
 *    must have been pushed with avmp_flush: AVMP_ERR_INVALID_ARG otherwise;
 *  - a step whose work buffer would exceed the static array (large batch x handle
 *    row: 4 bytes per attention layer, request and page of row width, plus about
 *    8.5 MB of partial results at 32 query heads x 128) is refused with
 *    AVMP_ERR_INVALID_ARG and a message that names both sizes;
 *  - every call on one GPU uses that GPU's array, whatever the pools object: calls
 *    that overlap in time on one GPU (different streams) race.  Nothing in the
 *    array has to survive from one call to the next;
 *  - per-kernel timing (avmp_profile_enable) does not cover this call. */
#define AVMP_NOALLOC_WORKSPACE_BYTES (32u << 20)
int avmp_decode_step_noalloc(avmp_pools_t* pools, const avmp_step_t* step, void* stream);

/* Work buffer of avmp_decode_step (its size follows from the number of layers of
 * each kind, the batch and the handle-row width).  avmp_workspace_reserve sizes it
 * ahead of time for the largest step the caller will issue, so that no later step
 * allocates; avmp_workspace_info reports its size in bytes and how many times it
 * has been allocated so far (either pointer may be NULL). */
int avmp_workspace_reserve(avmp_pools_t* pools, uint32_t n_attention_layers, uint32_t n_ssm_layers,
                           uint32_t batch, uint32_t max_pages);
int avmp_workspace_info(const avmp_pools_t* pools, uint64_t* bytes, uint64_t* allocations);

/* Rebalancing policy of Method, "Dynamic Pool Rebalancing" and Fig. 2.  A
 * four-state machine (BALANCED, KV_PRESSURED / SSM_PRESSURED, REBALANCING) is
 * evaluated only inside the capacity-error handler of avmp_alloc_auto:
 * BALANCED -> X_PRESSURED when pool X's free fraction is below threshold_low;
 * X_PRESSURED -> REBALANCING when the other pool's free fraction exceeds
 * threshold_high and at least min_rebalance_interval_ops logical operations
 * have passed since the last rebalance; REBALANCING -> BALANCED when the
 * migration completes; X_PRESSURED -> BALANCED when X's free fraction recovers.
 * One rebalance gives the starving pool up to migration_batch_size units
 * (limited by the donor's free units).  When the gap between the pools already
 * holds that many units the step takes them from there (avmp_absorb_gap): no donor
 * is needed, so threshold_high is not consulted, but the step is throttled and
 * counted like any other.  Defaults: 0.05, 0.30, 128, 1000.
 * Where the paper's text and its Fig. 2 differ, Fig. 2 is followed: a failing
 * allocation rebalances only if its own pool's free fraction is below
 * threshold_low, and a failure in one pool is ignored while the machine waits in
 * the other pool's PRESSURED state. */
typedef struct avmp_policy {
  double threshold_low;
  double threshold_high;
  uint32_t migration_batch_size;
  uint32_t reserved;
  uint64_t min_rebalance_interval_ops;
} avmp_policy_t;

enum { AVMP_BALANCED = 0, AVMP_KV_PRESSURED = 1, AVMP_SSM_PRESSURED = 2, AVMP_REBALANCING = 3 };

typedef struct avmp_policy_state {
  uint32_t state;                /* AVMP_BALANCED ... */
  uint32_t has_rebalanced;
  uint64_t last_rebalance_op;    /* value of the operation counter at the last rebalance */
  uint64_t rebalance_count;
  uint64_t oom_events;           /* avmp_alloc_auto calls that finally failed */
} avmp_policy_state_t;

/* Set the policy and reset the state machine.  AVMP_ERR_INVALID_ARG unless
 * 0 <= threshold_low < threshold_high <= 1 and migration_batch_size >= 1 (the
 * paper's validation check: low >= high has no defined transition semantics). */
int avmp_policy_set(avmp_pools_t* pools, const avmp_policy_t* policy);
int avmp_policy_state(const avmp_pools_t* pools, avmp_policy_state_t* out);

/* allocate() with the capacity-error handler: like avmp_alloc, but when the pool
 * is full the state machine above may migrate capacity from the other pool (on
 * `stream`, as avmp_migrate) and the allocation is retried once.  With no donor
 * it behaves exactly as avmp_alloc (static partition).  *donor_units_migrated
 * (may be NULL) receives the number of units the other pool gave up (0 when
 * nothing moved or the step came out of the gap).  It is written on every return,
 * also when the retry still ends in AVMP_ERR_CAPACITY: the capacity has moved by
 * then, as avmp_stats shows.  This is the one exception to "a failing call leaves
 * every observable unchanged". */
int avmp_alloc_auto(avmp_pools_t* pools, int pool, uint32_t n, avmp_handle_t* out, void* stream,
                    uint32_t* donor_units_migrated);

/* Push queued table updates (Fig. 1's VirtualPageTable, mirrored on the device),
 * pool capacities and zero fills of new SSM blocks to the device on `stream`. */
int avmp_flush(avmp_pools_t* pools, void* stream);

/* Device-side translation (Fig. 1: pool tag selects the store, page id indexes
 * the table, the entry is the physical slot) of n handles (device array) to byte
 * offsets from the arena base (device array, UINT64_MAX for handles that do not
 * resolve). */
int avmp_translate(avmp_pools_t* pools, const avmp_handle_t* handles_dev, uint32_t n,
                   uint64_t* offsets_dev, void* stream);

/* Host-side resolve (Fig. 1's lookup): handle -> pool, physical slot, byte
 * offset from the arena base.  AVMP_ERR_INVALID_HANDLE if not live. */
int avmp_resolve(const avmp_pools_t* pools, avmp_handle_t h, uint32_t* pool, uint32_t* slot,
                 uint64_t* byte_off);

/* The allocator's counters (Method, "Dynamic Pool Rebalancing" and Evaluation:
 * per-pool capacity and free units behind the free fractions of Fig. 2, the logical
 * operation counter the throttle reads, capacity errors, migrations, migrated and
 * wasted bytes). */
int avmp_stats(const avmp_pools_t* pools, avmp_stats_t* out);

/* Report and reset, in the order of `stream` (behind the kernels already queued on
 * it), the number of handles that the kernels could not translate (such
 * pages/blocks are skipped, never touched); returns after `stream` has drained.
 * Not for use under graph capture. */
int avmp_device_faults(avmp_pools_t* pools, void* stream, uint64_t* out);

/* Per-kernel timing with HIP events on the launch stream.  While enabled, every
 * kernel the library launches is bracketed by an event pair; avmp_profile_read
 * synchronises `stream`, adds up elapsed milliseconds and launch counts per
 * kernel kind since the last read, writes them to *out and resets them. */
enum {
  AVMP_K_ATTENTION = 0,        /* paged GQA decode attention (per layer) */
  AVMP_K_ATTENTION_MERGE = 1,  /* merge of split-K partial results (per layer) */
  AVMP_K_SSM = 2,              /* SSM state update (per layer) */
  AVMP_K_MIGRATE_COPY = 3,     /* migration copy + remap */
  AVMP_K_TABLE = 4,            /* table scatter + zero fill of new SSM blocks */
  AVMP_K_CONV = 5,             /* short convolution in front of the recurrence (per layer); no
                                  launches where the recurrence kernel runs it itself: its time
                                  is then part of AVMP_K_SSM */
  AVMP_K_ATTENTION_PREPARE = 6,/* run plan + translation of all KV handles (once per step) */
  AVMP_K_COUNT = 7
};
typedef struct avmp_profile {
  double ms[AVMP_K_COUNT];
  uint64_t launches[AVMP_K_COUNT];
} avmp_profile_t;
int avmp_profile_enable(avmp_pools_t* pools, int on);
int avmp_profile_read(avmp_pools_t* pools, void* stream, avmp_profile_t* out);

/* Migration by physical remap instead of copy: what the paper leaves as the
 * step after its prototype (Method, "Dynamic Pool Rebalancing": on-demand
 * physical page remapping; Limitations: mapping virtual addresses to physical
 * pages dynamically).  An avmp_vmm_arena_t is a device address range reserved
 * through the HIP virtual-memory API and backed by separate physical chunks of
 * chunk_bytes each.  Pools created on avmp_vmm_arena_base() and then switched
 * with avmp_migrate_by_remap() move a live unit out of the vacated range by
 * exchanging the physical chunks behind its old and its new slot; tables,
 * capacities, gap and every resolved location come out exactly as with the
 * copying avmp_migrate (the content of free slots is unspecified in both).
 *
 * avmp_vmm_min_chunk: smallest chunk_bytes of the current device (0: no
 *   virtual-memory support).
 * avmp_vmm_arena_create: bytes a multiple of chunk_bytes, chunk_bytes a multiple
 *   of the minimum; AVMP_ERR_INVALID_ARG otherwise, AVMP_ERR_DEVICE when the
 *   device refuses.  The arena belongs to the current device and to the caller,
 *   who destroys it after the pools that sit on it.
 * avmp_migrate_by_remap: arena non-NULL switches remap on, NULL switches back to
 *   copy.  A pool takes part when each of its slots covers whole chunks: its
 *   unit size a multiple of chunk_bytes (and, for the SSM pool, whose slots are
 *   counted down from the top, the usable arena size too); a pool that does not
 *   keeps copying when it is the donor.  AVMP_ERR_INVALID_ARG (nothing changes)
 *   if neither pool qualifies or the pools' arena is not the arena's base.
 * With remap on, avmp_migrate from a qualifying donor first waits for the whole
 * device (no work that touches the arena may be in flight on any stream) and the
 * exchanges run on the host, a few driver calls per chunk; units_copied in the
 * result then counts exchanged units.  A failed exchange leaves part of the
 * arena unmapped: AVMP_ERR_DEVICE, and pools and arena must be destroyed without
 * launching anything more on them. */
typedef struct avmp_vmm_arena avmp_vmm_arena_t;
uint64_t avmp_vmm_min_chunk(void);
int avmp_vmm_arena_create(uint64_t bytes, uint64_t chunk_bytes, avmp_vmm_arena_t** out);
void* avmp_vmm_arena_base(const avmp_vmm_arena_t* arena);
int avmp_vmm_arena_destroy(avmp_vmm_arena_t* arena);
int avmp_migrate_by_remap(avmp_pools_t* pools, avmp_vmm_arena_t* arena);

/* Text of the last error raised on the calling thread ("" if none). */
const char* avmp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* AVMP_H */
