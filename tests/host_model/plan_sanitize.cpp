// Exercises the host-only planning code (csrc/ntp_plan.cpp: shard plans, sub-shard lists for contiguous and
// mapped layouts, the comp / sync rank assignment, row segments) under AddressSanitizer and
// UndefinedBehaviorSanitizer, with invariants checked on every result.  Built with g++ by the test suite; no GPU.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "ntp_internal.h"

#define CHECK(c)                                                   \
  do {                                                             \
    if (!(c)) {                                                    \
      printf("FAIL %s:%d: %s\n", __FILE__, __LINE__, #c);          \
      return 1;                                                    \
    }                                                              \
  } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(uint32_t n) {
  rng_state ^= rng_state << 13;
  rng_state ^= rng_state >> 7;
  rng_state ^= rng_state << 17;
  return uint32_t(rng_state >> 33) % n;
}

int main() {
  int64_t checks = 0;
  // contiguous plans: widths sum to dim, offsets are the prefix sums
  for (int64_t dim : {0, 1, 7, 64, 586, 12000, 53248})
    for (int32_t tp : {1, 2, 7, 8, 30, 32, 71, 72, 100}) {
      int64_t sum = 0;
      for (int32_t r = 0; r < tp; ++r) {
        int64_t off = -1, w = -1;
        CHECK(ntp_shard_plan(dim, tp, r, &off, &w) == NTP_OK);
        CHECK(off == sum && w >= 0);
        sum += w;
        ++checks;
      }
      CHECK(sum == dim);
    }
  // sub-shard lists: every destination unit exactly once, sources in range
  struct Case {
    int64_t units;
    int32_t unit, kind, n_q, n_kv;
  };
  const Case cases[] = {{37, 1, NTP_KIND_PLAIN, 0, 0},   {64, 4, NTP_KIND_PLAIN, 0, 0},      {53248, 1, NTP_KIND_PLAIN, 0, 0},
                        {12, 2, NTP_KIND_QKV_GQA, 8, 2}, {144, 128, NTP_KIND_QKV_GQA, 128, 8}, {80, 64, NTP_KIND_QKV_GQA, 64, 8},
                        {288, 8, NTP_KIND_QKV_GQA, 96, 96}};
  for (const Case& c : cases)
    for (int32_t a : {1, 3, 7, 8, 30, 32, 71, 72})
      for (int32_t b : {1, 4, 7, 8, 30, 32, 71, 72}) {
        ntp_tensor_spec_t spec{c.units * c.unit, 16, 0, c.unit, 4, c.kind, c.n_q, c.n_kv};
        std::vector<ntp_segment_t> segs;
        CHECK(ntp::build_segments(&spec, a, b, &segs) == NTP_OK);
        std::vector<int64_t> su(a), du(b);
        for (int32_t r = 0; r < a; ++r) CHECK(ntp::shard_units(&spec, c.units, a, r, &su[r]) == NTP_OK);
        for (int32_t r = 0; r < b; ++r) CHECK(ntp::shard_units(&spec, c.units, b, r, &du[r]) == NTP_OK);
        std::vector<std::vector<int>> cover(b);
        for (int32_t r = 0; r < b; ++r) cover[r].assign(size_t(du[r]), 0);
        for (const ntp_segment_t& g : segs) {
          CHECK(g.src_rank >= 0 && g.src_rank < a && g.dst_rank >= 0 && g.dst_rank < b && g.units > 0);
          CHECK(g.src_unit >= 0 && g.src_unit + g.units <= su[g.src_rank]);
          CHECK(g.dst_unit >= 0 && g.dst_unit + g.units <= du[g.dst_rank]);
          for (int64_t i = 0; i < g.units; ++i) ++cover[g.dst_rank][size_t(g.dst_unit + i)];
        }
        for (int32_t r = 0; r < b; ++r)
          for (int x : cover[r]) CHECK(x == 1);
        // the C entry point with a short output array writes no more than it was given
        std::vector<ntp_segment_t> few(3);
        int64_t n = -1;
        CHECK(ntp_reshard_segments(&spec, a, b, few.data(), 3, &n) == NTP_OK && n == int64_t(segs.size()));
        // row segments of every source rank with every second destination absent
        std::vector<void*> dst(b);
        std::vector<int64_t> ld(b, 16);
        static float arena[4];
        for (int32_t r = 0; r < b; ++r) dst[r] = (r & 1) ? nullptr : arena;
        for (int32_t r = 0; r < a; ++r) {
          std::vector<ntp_row_segment_t> rows(4);
          int64_t cnt = -1;
          const int rs = ntp_reshard_row_segments(&spec, a, r, b, dst.data(), ld.data(), rows.data(), 4, &cnt);
          if (rs == NTP_ERR_UNSUPPORTED && c.kind == NTP_KIND_QKV_GQA) continue;  // a KV head of this rank has other holders
          CHECK(rs == NTP_OK && cnt >= 0);
          for (int64_t i = 0; i < std::min<int64_t>(cnt, 4); ++i)
            CHECK(rows[size_t(i)].row_begin >= 0 && rows[size_t(i)].row_begin + rows[size_t(i)].rows <= su[r] * c.unit);
        }
        ++checks;
      }
  // comp / sync assignment and mapped sub-shards, also with random maps
  for (int64_t k : {0, 1, 12, 1000, 12000, 53248})
    for (int32_t t : {1, 4, 8, 32, 72})
      for (int32_t tr : {1, 3, 7, 30, 71}) {
        if (tr > t) continue;
        std::vector<int32_t> comp(size_t(k) + 1, -7), sync(size_t(k) + 1, -7);
        CHECK(ntp_comp_sync_plan(k, t, tr, comp.data(), sync.data()) == NTP_OK);
        CHECK(comp[size_t(k)] == -7 && sync[size_t(k)] == -7);  // nothing written past k entries
        for (int64_t u = 0; u < k; ++u) CHECK(comp[size_t(u)] >= 0 && comp[size_t(u)] < t && sync[size_t(u)] >= 0 && sync[size_t(u)] < tr);
        std::vector<ntp_segment_t> segs;
        std::vector<int64_t> su, du;
        CHECK(ntp::build_segments_mapped(k, t, comp.data(), tr, sync.data(), &segs, &su, &du) == NTP_OK);
        int64_t total = 0;
        for (const ntp_segment_t& g : segs) {
          CHECK(g.src_unit + g.units <= su[size_t(g.src_rank)] && g.dst_unit + g.units <= du[size_t(g.dst_rank)]);
          total += g.units;
        }
        CHECK(total == k);
        ++checks;
      }
  for (int rep = 0; rep < 200; ++rep) {
    const int64_t k = 1 + rnd(400);
    const int32_t a = 1 + int32_t(rnd(9)), b = 1 + int32_t(rnd(9));
    std::vector<int32_t> sm, dm;
    sm.resize(size_t(k));
    dm.resize(size_t(k));
    for (int64_t u = 0; u < k; ++u) {
      sm[size_t(u)] = int32_t(rnd(uint32_t(a)));
      dm[size_t(u)] = int32_t(rnd(uint32_t(b)));
    }
    std::vector<ntp_segment_t> segs;
    std::vector<int64_t> su, du;
    CHECK(ntp::build_segments_mapped(k, a, sm.data(), b, dm.data(), &segs, &su, &du) == NTP_OK);
    int64_t total = 0;
    for (const ntp_segment_t& g : segs) total += g.units;
    CHECK(total == k);
    dm[size_t(rnd(uint32_t(k)))] = b;  // a rank out of range is refused, not indexed with
    CHECK(ntp::build_segments_mapped(k, a, sm.data(), b, dm.data(), &segs, &su, &du) == NTP_ERR_INVALID_ARG);
    ++checks;
  }
  printf("OK %lld\n", (long long)checks);
  return 0;
}
