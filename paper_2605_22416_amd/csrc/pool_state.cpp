#include "pool_state.hpp"

#include <algorithm>

namespace avmp {

// ---------------------------------------------------------------------------
// MinBitset
// ---------------------------------------------------------------------------
void MinBitset::init(uint64_t n) {
  lv_.clear();
  count_ = 0;
  uint64_t words = (n + 63) / 64;
  if (words == 0) words = 1;
  for (;;) {
    lv_.emplace_back(words, 0ull);
    if (words == 1) break;
    words = (words + 63) / 64;
  }
}

void MinBitset::insert(uint64_t i) {
  if (contains(i)) return;
  ++count_;
  for (auto& level : lv_) {
    uint64_t& w = level[i >> 6];
    bool was_empty = (w == 0);
    w |= 1ull << (i & 63);
    if (!was_empty) break;
    i >>= 6;
  }
}

void MinBitset::erase(uint64_t i) {
  if (!contains(i)) return;
  --count_;
  for (auto& level : lv_) {
    uint64_t& w = level[i >> 6];
    w &= ~(1ull << (i & 63));
    if (w != 0) break;
    i >>= 6;
  }
}

int64_t MinBitset::min() const {
  if (count_ == 0) return -1;
  uint64_t idx = 0;
  for (size_t l = lv_.size(); l-- > 0;) {
    uint64_t w = lv_[l][idx];
    idx = (idx << 6) | uint64_t(__builtin_ctzll(w));
  }
  return int64_t(idx);
}

int64_t MinBitset::next(uint64_t from) const {
  const uint64_t n_leaf_bits = uint64_t(lv_[0].size()) << 6;
  if (count_ == 0 || from >= n_leaf_bits) return -1;
  // climb while the rest of the current word (at and above `from`) is empty, then descend
  uint64_t idx = from;
  size_t l = 0;
  for (;;) {
    const uint64_t w = lv_[l][idx >> 6] & (~0ull << (idx & 63));
    if (w != 0) {
      idx = (idx & ~63ull) | uint64_t(__builtin_ctzll(w));
      break;
    }
    idx = (idx >> 6) + 1;                     // first word to the right, seen from the level above
    if (++l == lv_.size() || idx >= (uint64_t(lv_[l].size()) << 6)) return -1;
  }
  while (l > 0) {
    --l;
    idx = (idx << 6) | uint64_t(__builtin_ctzll(lv_[l][idx]));
  }
  return int64_t(idx);
}

// ---------------------------------------------------------------------------
// geometry
// ---------------------------------------------------------------------------
static uint64_t round_up(uint64_t v, uint64_t m) { return (v + m - 1) / m * m; }

bool compute_geometry(const ShapeArgs& s, uint64_t arena_bytes, Geometry* g) {
  if (s.elem_bytes == 0 || s.page_tokens == 0 || s.n_kv_heads == 0 || s.head_dim == 0 ||
      s.ssm_heads == 0 || s.ssm_headdim == 0 || s.ssm_dstate == 0 || s.state_bytes == 0)
    return false;
  // KV page = attention_page_tokens x per_token_bytes; per_token_bytes = K and V
  // of one layer for all KV heads.  SSM block = state_dim x bytes_per_element.
  uint64_t per_token = 2ull * s.n_kv_heads * s.head_dim * s.elem_bytes;
  g->unit[0] = round_up(uint64_t(s.page_tokens) * per_token, 16);
  uint64_t block = uint64_t(s.ssm_heads) * s.ssm_headdim * s.ssm_dstate * s.state_bytes;
  if (s.conv_kernel)   // + the inputs of the last K-1 tokens on the x, B and C channels
    block += uint64_t(s.conv_kernel - 1) *
             (uint64_t(s.ssm_heads) * s.ssm_headdim + 2ull * s.ssm_dstate) * s.elem_bytes;
  g->ssm_native = round_up(block, 16);
  // a unified pool hands out one page size: the block takes a whole number of KV pages
  g->unit[1] = s.pad_ssm_to_kv_page ? round_up(g->ssm_native, g->unit[0]) : g->ssm_native;
  g->usable = arena_bytes / 128 * 128;
  for (int p = 0; p < kPools; ++p) {
    uint64_t m = g->usable / g->unit[p];
    if (m > kPageIdMask) return false;      // slot and virtual ids must fit 30 bits
    g->max_slots[p] = uint32_t(m);
  }
  return true;
}

// ---------------------------------------------------------------------------
// PoolState
// ---------------------------------------------------------------------------
bool PoolState::init(const Geometry& g, uint32_t kv_capacity, uint32_t ssm_capacity,
                     const uint32_t max_vid[kPools], const uint32_t* const rank[kPools]) {
  g_ = g;
  uint64_t need = uint64_t(kv_capacity) * g.unit[0] + uint64_t(ssm_capacity) * g.unit[1];
  if (need > g.usable) return false;
  capacity_[0] = kv_capacity;
  capacity_[1] = ssm_capacity;
  gap_ = g.usable - need;
  for (int p = 0; p < kPools; ++p) {
    max_vid_[p] = max_vid[p] ? max_vid[p] : g.max_slots[p];
    if (max_vid_[p] > kPageIdMask) return false;
    live_[p] = 0;
    uint32_t ns = g.max_slots[p];
    slot_of_[p].assign(max_vid_[p], kUnmapped);
    vid_of_[p].assign(ns, kUnmapped);
    rank_of_[p].resize(ns);
    slot_at_[p].assign(ns, kUnmapped);
    for (uint32_t s = 0; s < ns; ++s) {
      uint32_t r = rank[p] ? rank[p][s] : s;
      if (r >= ns || slot_at_[p][r] != kUnmapped) return false;   // not a permutation
      rank_of_[p][s] = r;
      slot_at_[p][r] = s;
    }
    free_rank_[p].init(ns);
    for (uint32_t s = 0; s < capacity_[p]; ++s) free_rank_[p].insert(rank_of_[p][s]);
    free_vid_[p].init(max_vid_[p]);
    for (uint32_t v = 0; v < max_vid_[p]; ++v) free_vid_[p].insert(v);
  }
  uint64_t total_vid = uint64_t(max_vid_[0]) + max_vid_[1];
  return total_vid <= 0xFFFFFFFFull;
}

int PoolState::alloc(int pool, uint32_t n, uint32_t* out, std::vector<TableUpdate>* upd,
                     std::vector<uint32_t>* new_ssm_slots) {
  if ((pool != 0 && pool != 1) || n == 0 || out == nullptr) return 3;
  ++c_.ops;
  if (free_rank_[pool].size() < n || free_vid_[pool].size() < n) {
    ++c_.capacity_errors;
    return 1;
  }
  for (uint32_t i = 0; i < n; ++i) {
    uint32_t vid = uint32_t(free_vid_[pool].min());
    uint32_t r = uint32_t(free_rank_[pool].min());
    uint32_t slot = slot_at_[pool][r];
    free_vid_[pool].erase(vid);
    free_rank_[pool].erase(r);
    slot_of_[pool][vid] = slot;
    vid_of_[pool][slot] = vid;
    out[i] = (uint32_t(pool) << kPageIdBits) | vid;
    upd->push_back({vid_base(pool) + vid, slot});
    if (pool == 1) new_ssm_slots->push_back(slot);
  }
  live_[pool] += n;
  return 0;
}

bool PoolState::resolve(uint32_t h, uint32_t* pool, uint32_t* slot, uint64_t* off) const {
  uint32_t p = h >> kPageIdBits, vid = h & kPageIdMask;
  if (p >= uint32_t(kPools) || vid >= max_vid_[p]) return false;
  uint32_t s = slot_of_[p][vid];
  if (s == kUnmapped) return false;
  if (pool) *pool = p;
  if (slot) *slot = s;
  if (off) *off = byte_offset(int(p), s);
  return true;
}

int PoolState::free_units(const uint32_t* handles, uint32_t n, std::vector<TableUpdate>* upd) {
  if (n == 0 || handles == nullptr) return 3;
  ++c_.ops;
  for (uint32_t i = 0; i < n; ++i)
    if (!resolve(handles[i], nullptr, nullptr, nullptr)) return 2;
  std::vector<uint32_t> sorted(handles, handles + n);
  std::sort(sorted.begin(), sorted.end());
  if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end()) return 2;
  for (uint32_t i = 0; i < n; ++i) {
    uint32_t p = handles[i] >> kPageIdBits, vid = handles[i] & kPageIdMask;
    uint32_t slot = slot_of_[p][vid];
    slot_of_[p][vid] = kUnmapped;
    vid_of_[p][slot] = kUnmapped;
    free_vid_[p].insert(vid);
    free_rank_[p].insert(rank_of_[p][slot]);
    --live_[p];
    upd->push_back({vid_base(int(p)) + vid, kUnmapped});
  }
  return 0;
}

int PoolState::migrate_begin(int donor, uint32_t n) {
  if ((donor != 0 && donor != 1) || n == 0) return 3;
  ++c_.ops;
  // all-or-nothing: checked before anything is touched, so "rollback" is trivial
  if (n > capacity_[donor] || free_rank_[donor].size() < n) return 1;
  const uint32_t oldcap = capacity_[donor], newcap = oldcap - n;
  // free slots of the vacated high range leave the free set first ...
  for (uint32_t s = newcap; s < oldcap; ++s)
    if (vid_of_[donor][s] == kUnmapped) free_rank_[donor].erase(rank_of_[donor][s]);
  mig_.donor = donor;
  mig_.n = n;
  mig_.oldcap = oldcap;
  mig_.next_src = newcap;
  mig_.moved = 0;
  mig_.rank_cursor = 0;
  return 0;
}

uint32_t PoolState::migrate_moves(Move* out, uint32_t max) {
  const int donor = mig_.donor;
  uint32_t k = 0;
  // ... then each live unit there moves to the best-ranked free slot below the new capacity;
  // successive best ranks only grow, so the search resumes where the last one ended
  for (; mig_.next_src < mig_.oldcap && k < max; ++mig_.next_src) {
    const uint32_t s = mig_.next_src;
    const uint32_t vid = vid_of_[donor][s];
    if (vid == kUnmapped) continue;
    const uint32_t r = uint32_t(free_rank_[donor].next(mig_.rank_cursor));
    mig_.rank_cursor = uint64_t(r) + 1;
    const uint32_t dst = slot_at_[donor][r];
    free_rank_[donor].erase(r);
    vid_of_[donor][dst] = vid;
    vid_of_[donor][s] = kUnmapped;
    slot_of_[donor][vid] = dst;
    out[k++] = {s, dst, vid};
  }
  mig_.moved += k;
  return k;
}

void PoolState::migrate_end(uint32_t* gain_out, uint64_t* wasted_out) {
  const int donor = mig_.donor, recip = 1 - donor;
  capacity_[donor] = mig_.oldcap - mig_.n;
  uint64_t avail = gap_ + uint64_t(mig_.n) * g_.unit[donor];
  uint32_t gain = uint32_t(avail / g_.unit[recip]);
  gap_ = avail % g_.unit[recip];
  for (uint32_t s = capacity_[recip]; s < capacity_[recip] + gain; ++s)
    free_rank_[recip].insert(rank_of_[recip][s]);
  capacity_[recip] += gain;
  ++c_.migrations;
  c_.units_copied += mig_.moved;
  c_.bytes_migrated += uint64_t(mig_.n) * g_.unit[donor];
  c_.bytes_wasted += gap_;
  *gain_out = gain;
  *wasted_out = gap_;
  mig_.donor = -1;
}

int PoolState::migrate(int donor, uint32_t n, std::vector<Move>* moves,
                       std::vector<TableUpdate>* upd, uint32_t* gain_out, uint64_t* wasted_out) {
  const int rc = migrate_begin(donor, n);
  if (rc != 0) return rc;
  Move buf[256];
  for (uint32_t k; (k = migrate_moves(buf, 256)) != 0;)
    for (uint32_t i = 0; i < k; ++i) {
      moves->push_back(buf[i]);
      upd->push_back({vid_base(donor) + buf[i].vid, buf[i].dst_slot});
    }
  migrate_end(gain_out, wasted_out);
  return 0;
}

int PoolState::absorb_gap(int pool, uint32_t* gain_out, uint64_t* wasted_out) {
  if (pool != 0 && pool != 1) return 3;
  ++c_.ops;
  const uint64_t gain = gap_ / g_.unit[pool];
  if (gain == 0) return 1;
  for (uint64_t s = capacity_[pool]; s < capacity_[pool] + gain; ++s)
    free_rank_[pool].insert(rank_of_[pool][s]);
  capacity_[pool] += uint32_t(gain);
  gap_ -= gain * g_.unit[pool];
  ++c_.migrations;
  c_.bytes_wasted += gap_;
  *gain_out = uint32_t(gain);
  *wasted_out = gap_;
  return 0;
}

PoolState::Step PoolState::on_capacity_error(int pool, Rebalancer* rb, uint32_t* donor_units_out) const {
  const Policy& pol = rb->policy;
  const int other = 1 - pool;
  *donor_units_out = 0;
  auto free_fraction = [&](int p) {
    return capacity_[p] ? double(capacity_[p] - live_[p]) / double(capacity_[p]) : 0.0;
  };
  const int pressured = pool == 0 ? kKvPressured : kSsmPressured;
  // "free recovers"
  if (rb->state == kKvPressured && free_fraction(0) >= pol.threshold_low) rb->state = kBalanced;
  if (rb->state == kSsmPressured && free_fraction(1) >= pol.threshold_low) rb->state = kBalanced;
  if (rb->state == kBalanced && free_fraction(pool) < pol.threshold_low) rb->state = pressured;
  if (rb->state != pressured) return kStepNone;
  const uint64_t want = uint64_t(pol.migration_batch_size) * g_.unit[pool];
  const bool from_gap = want <= gap_;         // bytes nobody owns already hold the step's units
  if (!from_gap && !(free_fraction(other) > pol.threshold_high)) return kStepNone;   // no donor: static behaviour
  if (rb->has_rebalanced && c_.ops - rb->last_rebalance_op < pol.min_rebalance_interval_ops)
    return kStepNone;                                                // throttled
  if (from_gap) {
    rb->state = kRebalancing;
    return kStepFromGap;
  }
  uint64_t donor_units = (want - gap_ + g_.unit[other] - 1) / g_.unit[other];
  const uint64_t donor_free = capacity_[other] - live_[other];
  if (donor_units > donor_free) donor_units = donor_free;
  if (donor_units == 0) return kStepNone;
  rb->state = kRebalancing;
  *donor_units_out = uint32_t(donor_units);
  return kStepMigrate;
}

void PoolState::rebalance_done(Rebalancer* rb) const {
  ++rb->rebalance_count;
  rb->has_rebalanced = true;
  rb->last_rebalance_op = c_.ops;
  rb->state = kBalanced;                                             // migration complete
}

}  // namespace avmp
