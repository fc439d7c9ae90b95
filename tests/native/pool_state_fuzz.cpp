// Host-side pool logic under AddressSanitizer / UBSan: a long random trace of
// alloc / free / migrate / policy calls with structural invariants checked
// after every call.  Built and run by tests/test_host_sanitizers.py.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <set>
#include <vector>

#include "pool_state.hpp"

using namespace avmp;

#define REQUIRE(c) do { if (!(c)) { std::printf("FAILED %s line %d\n", #c, __LINE__); return 1; } } while (0)

int main(int argc, char** argv) {
  const unsigned seed = argc > 1 ? unsigned(std::atoi(argv[1])) : 1u;
  std::mt19937 rng(seed);
  ShapeArgs sh{4, 16, 4, 2, 64, 4, 32, 16, 4};
  Geometry g{};
  const uint64_t arena = 37 * 16384 + 11 * 8192 + 640;
  REQUIRE(compute_geometry(sh, arena, &g));
  REQUIRE(g.unit[0] == 16384 && g.unit[1] == 8192);
  std::vector<uint32_t> rank[2];
  for (int p = 0; p < 2; ++p) {
    rank[p].resize(g.max_slots[p]);
    for (uint32_t i = 0; i < g.max_slots[p]; ++i) rank[p][i] = i;
    std::shuffle(rank[p].begin(), rank[p].end(), rng);
  }
  const uint32_t max_vid[2] = {0, 0};
  const uint32_t* ranks[2] = {rank[0].data(), rank[1].data()};
  PoolState st;
  REQUIRE(st.init(g, 37, 11, max_vid, ranks));
  Rebalancer rb;
  rb.policy.migration_batch_size = 3;
  rb.policy.min_rebalance_interval_ops = 25;
  std::vector<uint32_t> live;
  std::vector<TableUpdate> upd;
  std::vector<uint32_t> zero;
  std::vector<Move> moves;
  for (int step = 0; step < 200000; ++step) {
    const unsigned u = rng() % 100;
    const int pool = int(rng() % 2);
    upd.clear(); zero.clear(); moves.clear();
    if (u < 50) {
      const uint32_t n = 1 + rng() % 5;
      uint32_t out[8];
      int rc = st.alloc(pool, n, out, &upd, &zero);
      if (rc == 1) {
        uint32_t donate = 0;
        const PoolState::Step step_kind = st.on_capacity_error(pool, &rb, &donate);
        if (step_kind != PoolState::kStepNone) {
          uint32_t gain; uint64_t wasted;
          if (step_kind == PoolState::kStepFromGap) {
            REQUIRE(st.absorb_gap(pool, &gain, &wasted) == 0);
          } else {
            // planned in slices, as the library does it
            REQUIRE(st.migrate_begin(1 - pool, donate) == 0);
            Move buf[3];
            for (uint32_t k; (k = st.migrate_moves(buf, 3)) != 0;) moves.insert(moves.end(), buf, buf + k);
            st.migrate_end(&gain, &wasted);
          }
          st.rebalance_done(&rb);
          rc = st.alloc(pool, n, out, &upd, &zero);
        }
      }
      REQUIRE(rc == 0 || rc == 1);
      if (rc == 0) live.insert(live.end(), out, out + n);
    } else if (u < 90) {
      if (live.empty()) continue;
      uint32_t hs[4];
      uint32_t k = 1 + rng() % 3;
      if (k > live.size()) k = uint32_t(live.size());
      for (uint32_t i = 0; i < k; ++i) {
        const size_t j = rng() % live.size();
        hs[i] = live[j];
        live[j] = live.back();
        live.pop_back();
      }
      REQUIRE(st.free_units(hs, k, &upd) == 0);
      REQUIRE(st.free_units(hs, 1, &upd) == 2);          // stale now
    } else if (u < 91) {
      uint32_t gain; uint64_t wasted;
      const int rc = st.absorb_gap(pool, &gain, &wasted);
      REQUIRE(rc == 0 || rc == 1);
    } else if (u < 97) {
      uint32_t gain; uint64_t wasted;
      const int rc = st.migrate(pool, 1 + rng() % 6, &moves, &upd, &gain, &wasted);
      REQUIRE(rc == 0 || rc == 1);
      for (const Move& m : moves) REQUIRE(m.dst_slot < st.capacity(pool) && m.src_slot >= st.capacity(pool));
    } else {
      uint32_t bad = rng();
      uint32_t p, s; uint64_t off;
      if (st.resolve(bad, &p, &s, &off)) REQUIRE(s < st.capacity(int(p)));
    }
    // invariants: conservation of bytes, live handles resolve to distinct in-capacity slots
    REQUIRE(uint64_t(st.capacity(0)) * g.unit[0] + uint64_t(st.capacity(1)) * g.unit[1] + st.gap() == g.usable);
    if (step % 64 == 0) {
      std::set<uint64_t> seen;
      uint32_t cnt[2] = {0, 0};
      for (uint32_t h : live) {
        uint32_t p, s; uint64_t off;
        REQUIRE(st.resolve(h, &p, &s, &off));
        REQUIRE(s < st.capacity(int(p)));
        REQUIRE(off + g.unit[p] <= g.usable && off % 16 == 0);
        REQUIRE(seen.insert((uint64_t(p) << 32) | s).second);
        ++cnt[p];
      }
      REQUIRE(cnt[0] == st.live(0) && cnt[1] == st.live(1));
    }
  }
  std::printf("ok seed=%u ops=%llu migrations=%llu rebalances=%llu capacity_errors=%llu\n", seed,
              (unsigned long long)st.counters().ops, (unsigned long long)st.counters().migrations,
              (unsigned long long)rb.rebalance_count, (unsigned long long)st.counters().capacity_errors);
  return 0;
}
