// Host-side state of the two pools and the virtual page table: integer logic
// only (no device calls), so it can be built and sanitised with a plain host
// compiler.  Follows Method, "Asymmetric Virtual Page Table" (handle, table,
// unit sizes, alignment) and "Dynamic Pool Rebalancing" (allocate, capacity
// error, migration with rollback, wasted bytes).
#pragma once

#include <cstdint>
#include <vector>

namespace avmp {

constexpr uint32_t kUnmapped = 0xFFFFFFFFu;
constexpr uint32_t kPageIdBits = 30;
constexpr uint32_t kPageIdMask = (1u << kPageIdBits) - 1;
constexpr int kPools = 2;

// Set of integers in [0, n) with O(log64 n) insert / erase / find-min: a
// 64-ary summary tree over a bitmap.  Used for "lowest free virtual id" and
// "free slot of lowest rank".
class MinBitset {
 public:
  void init(uint64_t n);
  void insert(uint64_t i);
  void erase(uint64_t i);
  bool contains(uint64_t i) const { return (lv_[0][i >> 6] >> (i & 63)) & 1; }
  int64_t min() const;               // -1 when empty
  int64_t next(uint64_t from) const; // smallest member >= from, -1 if none
  uint64_t size() const { return count_; }

 private:
  std::vector<std::vector<uint64_t>> lv_;   // lv_[0] = leaves
  uint64_t count_ = 0;
};

struct TableUpdate {       // device table entry to rewrite
  uint32_t index;          // vid_base[pool] + vid
  uint32_t slot;           // new slot, or kUnmapped
};

struct Move {              // one unit copy of a migration
  uint32_t src_slot, dst_slot, vid;
};

struct Geometry {
  uint64_t ssm_native;           // SSM block bytes before unified-pool padding (= unit[1] without it)
  uint64_t unit[kPools];
  uint64_t usable;
  uint32_t max_slots[kPools];
};

struct Counters {
  uint64_t ops = 0, capacity_errors = 0, migrations = 0, units_copied = 0, bytes_migrated = 0,
           bytes_wasted = 0;
};

struct ShapeArgs {
  uint32_t elem_bytes, page_tokens, n_q_heads, n_kv_heads, head_dim, ssm_heads, ssm_headdim,
      ssm_dstate, state_bytes;
  uint32_t conv_kernel = 0;   // taps of the short convolution; 0 = no window in the SSM block
  bool pad_ssm_to_kv_page = false;   // unified-pool sizing: the block padded to whole KV pages
};

// Returns false if the shape is unusable (zero sizes, more than 2^30 slots).
bool compute_geometry(const ShapeArgs& s, uint64_t arena_bytes, Geometry* g);

// Rebalancing policy of Method, "Dynamic Pool Rebalancing" / Fig. 2: thresholds
// on per-pool free fractions, a bound on the migration step and a throttle on the
// logical operation counter.  Defaults are the paper's.
struct Policy {
  double threshold_low = 0.05;
  double threshold_high = 0.30;
  uint32_t migration_batch_size = 128;        // units of the recipient pool per rebalance
  uint64_t min_rebalance_interval_ops = 1000;
};

enum PressureState { kBalanced = 0, kKvPressured = 1, kSsmPressured = 2, kRebalancing = 3 };

struct Rebalancer {
  Policy policy;
  int state = kBalanced;
  bool has_rebalanced = false;
  uint64_t last_rebalance_op = 0;
  uint64_t rebalance_count = 0;
  uint64_t oom_events = 0;                    // allocations that finally failed
};

class PoolState {
 public:
  // rank[p] may be empty (identity).  Returns false on invalid arguments.
  bool init(const Geometry& g, uint32_t kv_capacity, uint32_t ssm_capacity,
            const uint32_t max_vid[kPools], const uint32_t* const rank[kPools]);

  // Status codes are the C ABI's (0 ok, 1 capacity, 2 invalid handle, 3 invalid arg).
  int alloc(int pool, uint32_t n, uint32_t* out_handles, std::vector<TableUpdate>* upd,
            std::vector<uint32_t>* new_ssm_slots);
  int free_units(const uint32_t* handles, uint32_t n, std::vector<TableUpdate>* upd);
  int migrate(int donor, uint32_t n, std::vector<Move>* moves, std::vector<TableUpdate>* upd,
              uint32_t* gain, uint64_t* wasted);
  // The same migration in three steps, so that a caller can start copying the first moves
  // while the rest is still being planned.  migrate_begin validates (all-or-nothing: after
  // AVMP_OK nothing can fail) and takes the vacated range's free slots out of the free set;
  // migrate_moves writes up to `max` further moves (ascending source slot) and returns how
  // many, 0 once all live units of the vacated range have a new slot; migrate_end moves the
  // capacity and updates the counters.  No other call may come between begin and end.
  int migrate_begin(int donor, uint32_t n);
  uint32_t migrate_moves(Move* out, uint32_t max);
  void migrate_end(uint32_t* gain, uint64_t* wasted);
  // The whole units of `pool` that fit into the gap between the pools go to it: no donor,
  // no copy.  1 (capacity) if the gap holds less than one unit.
  int absorb_gap(int pool, uint32_t* gain, uint64_t* wasted);
  bool resolve(uint32_t h, uint32_t* pool, uint32_t* slot, uint64_t* off) const;

  // The CapacityError handler of allocate(): runs the state machine for a failed
  // allocation in `pool` and says what to do now.  kStepNone: nothing (not pressured,
  // no donor above threshold_high, throttled).  kStepMigrate: the OTHER pool donates
  // *donor_units.  kStepFromGap: the gap already holds the step's units, absorb it.
  // For the last two the state is kRebalancing; call rebalance_done() after the move.
  enum Step { kStepNone = 0, kStepMigrate = 1, kStepFromGap = 2 };
  Step on_capacity_error(int pool, Rebalancer* rb, uint32_t* donor_units) const;
  void rebalance_done(Rebalancer* rb) const;

  uint64_t byte_offset(int pool, uint32_t slot) const {
    return pool == 0 ? uint64_t(slot) * g_.unit[0] : g_.usable - (uint64_t(slot) + 1) * g_.unit[1];
  }
  const Geometry& geometry() const { return g_; }
  uint32_t capacity(int p) const { return capacity_[p]; }
  uint32_t live(int p) const { return live_[p]; }
  uint32_t max_vid(int p) const { return max_vid_[p]; }
  uint32_t vid_base(int p) const { return p == 0 ? 0 : max_vid_[0]; }
  uint64_t gap() const { return gap_; }
  const Counters& counters() const { return c_; }

 private:
  Geometry g_{};
  uint32_t capacity_[kPools]{}, live_[kPools]{}, max_vid_[kPools]{};
  uint64_t gap_ = 0;
  std::vector<uint32_t> slot_of_[kPools];     // vid -> slot (the virtual page table)
  std::vector<uint32_t> vid_of_[kPools];      // slot -> vid
  std::vector<uint32_t> rank_of_[kPools];     // slot -> rank
  std::vector<uint32_t> slot_at_[kPools];     // rank -> slot
  MinBitset free_rank_[kPools];               // ranks of free slots below capacity
  MinBitset free_vid_[kPools];
  Counters c_;
  struct {                                    // a migration between begin and end
    int donor = -1;
    uint32_t n = 0, next_src = 0, oldcap = 0, moved = 0;
    uint64_t rank_cursor = 0;                 // every free rank below it has been taken
  } mig_;
};

}  // namespace avmp
