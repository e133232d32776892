// Driver for the host-only part of the library (table rules, tile planning, write-set runs,
// table replication, timing statistics), built by tests/test_host_sanitized.py with
// AddressSanitizer and UndefinedBehaviorSanitizer and run on the CPU.  It checks structural
// invariants of what those routines produce on seeded random inputs; any sanitizer report or
// failed check ends it with a non-zero status.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "r3_internal.h"

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); \
      std::exit(1);                                                        \
    }                                                                      \
  } while (0)

static std::vector<r3_region> random_table(std::mt19937_64& rng, uint32_t n, uint64_t max_bytes,
                                           uint64_t* arena_out) {
  std::vector<r3_region> t(n);
  uint64_t at = 0;
  for (uint32_t i = 0; i < n; ++i) {
    const uint32_t dt = (uint32_t)(rng() % 5);
    const uint32_t es = r3::elem_size(dt);
    uint64_t nb = rng() % 7 == 0 ? 0 : (rng() % max_bytes) / es * es;
    at = (at + es - 1) / es * es + (rng() % 3) * es;
    t[i] = r3_region{at, nb, dt, (uint32_t)(rng() % 2), 1e-3, 1e-6};
    at += nb;
  }
  *arena_out = at + 16;
  return t;
}

static void check_plan(const std::vector<r3_region>& t, uint64_t arena) {
  const uint32_t n = (uint32_t)t.size();
  CHECK(r3_table_validate(t.data(), n, arena) == R3_OK);
  r3::TablePlan plan;
  r3::plan_table(t.data(), n, &plan);
  CHECK(plan.tile_begin.size() == (size_t)n + 1);
  CHECK(plan.tiles.size() == plan.tile_begin[n]);
  CHECK(plan.tiles.size() == r3::count_tiles(t.data(), n));
  CHECK(plan.tiles.size() <= r3::max_tiles(n, arena));
  CHECK(r3_table_workspace_bytes_exact(t.data(), n, arena) <= r3_table_workspace_bytes(n, arena));
  // the tiles of a region cover it exactly, in order, and none is larger than its shift allows
  uint64_t total = 0;
  for (uint32_t i = 0; i < n; ++i) {
    uint64_t covered = 0;
    for (uint64_t k = plan.tile_begin[i]; k < plan.tile_begin[i + 1]; ++k) {
      const r3::Tile& tl = plan.tiles[k];
      const uint32_t shift = tl.packed >> 24, index = tl.packed & 0xFFFFFFu;
      CHECK(tl.region == i);
      CHECK(index == k - plan.tile_begin[i]);
      CHECK(shift >= plan.min_shift && shift <= plan.max_shift);
      const uint64_t rel = (uint64_t)index << shift;
      CHECK(rel == covered && rel < t[i].bytes);
      const uint64_t left = t[i].bytes - rel, full = 1ull << shift;
      covered += left < full ? left : full;
    }
    CHECK(covered == t[i].bytes);
    CHECK(plan.tile_begin[i + 1] - plan.tile_begin[i] <= (1ull << plan.cap_log2));
    total += t[i].bytes;
  }
  CHECK(total == plan.total_bytes);
  // the copy tiles are the same spans, grouped by size class
  uint64_t in_classes = 0, copy_bytes = 0;
  for (uint32_t c = 0; c < r3::kMaxCopyClasses; ++c) in_classes += plan.class_count[c];
  CHECK(in_classes == plan.tiles.size() && plan.copy_tiles.size() == plan.tiles.size());
  uint64_t k = 0;
  for (uint32_t c = 0; c < r3::kMaxCopyClasses; ++c) {
    uint64_t prev_at = 0;
    for (uint32_t j = 0; j < plan.class_count[c]; ++j, ++k) {
      const r3::CopyTile& ct = plan.copy_tiles[k];
      CHECK(ct.len >= 1 && ct.len <= (1ull << (plan.min_shift + c)));
      CHECK(ct.at + ct.len <= arena);
      CHECK(j == 0 || ct.at >= prev_at);  // address order inside a class (table order of offsets here)
      CHECK(ct.es == 1 || ct.es == 2 || ct.es == 4 || ct.es == 8);
      prev_at = ct.at;
      copy_bytes += ct.len;
    }
  }
  CHECK(copy_bytes == plan.total_bytes);
}

int main() {
  std::mt19937_64 rng(20260411);
  // --- tables and plans, under several tile tunings
  const uint32_t tunings[][2] = {{0, 0}, {1024, 64}, {65536, 256}, {1u << 20, 65536}, {4096, 8192}};
  for (const auto& tu : tunings) {
    CHECK(r3_tune_tiles(tu[0], tu[1]) == R3_OK);
    for (int rep = 0; rep < 20; ++rep) {
      uint64_t arena = 0;
      const uint32_t n = 1 + (uint32_t)(rng() % 300);
      const uint64_t max_bytes = rep % 4 == 0 ? (64ull << 20) : (rep % 4 == 1 ? 300000 : 5000);
      std::vector<r3_region> t = random_table(rng, n, max_bytes, &arena);
      check_plan(t, arena);
    }
  }
  CHECK(r3_tune_tiles(3000, 0) == R3_EINVAL && r3_tune_tiles(512, 0) == R3_EINVAL);
  CHECK(r3_tune_tiles(0, 0) == R3_OK);
  {  // one very large region: the tile count stays under the cap and the shift grows
    std::vector<r3_region> t = {r3_region{0, 40ull << 30, R3_U8, R3_CMP_BITWISE, 0, 0}};
    check_plan(t, 40ull << 30);
  }
  // --- rejected tables
  {
    uint64_t arena = 0;
    std::vector<r3_region> t = random_table(rng, 50, 5000, &arena);
    CHECK(r3_table_validate(nullptr, 3, arena) == R3_EINVAL);
    CHECK(r3_table_validate(t.data(), 0, arena) == R3_EINVAL);
    std::vector<r3_region> u = t;
    u[7].dtype = 9;
    CHECK(r3_table_validate(u.data(), 50, arena) == R3_EINVAL);
    u = t;
    u[7].rtol = -1.0;
    CHECK(r3_table_validate(u.data(), 50, arena) == R3_EINVAL);
    u = t;
    u[9].dtype = R3_F64;
    u[9].offset = 8 * (u[9].offset / 8) + 4;
    u[9].bytes = 16;
    CHECK(r3_table_validate(u.data(), 50, arena) == R3_EALIGN);
    u = t;
    u[49].bytes = (arena - u[49].offset) / 8 * 8 + 64;
    u[49].dtype = R3_U8;
    CHECK(r3_table_validate(u.data(), 50, arena) == R3_ERANGE);
    u = t;
    u[3].offset = UINT64_MAX - 7;  // offset + bytes wraps around
    u[3].bytes = 64;
    u[3].dtype = R3_U8;
    CHECK(r3_table_validate(u.data(), 50, arena) == R3_ERANGE);
    u = t;
    u[20] = r3_region{u[30].offset, u[30].bytes ? u[30].bytes : 8, u[30].dtype, 0, 0, 0};
    if (u[30].bytes) CHECK(r3_table_validate(u.data(), 50, arena) == R3_EOVERLAP);
    CHECK(r3_table_workspace_bytes_exact(u.data(), 0, arena) == 0);
  }
  // --- write-set runs: dirty and clean runs partition the pages and alternate
  for (int rep = 0; rep < 50; ++rep) {
    const uint32_t page = 256u << (rng() % 5);
    const uint64_t bytes = rng() % (page * 700ull);
    const uint64_t pages = (bytes + page - 1) / page;
    std::vector<uint64_t> bm((pages + 63) / 64 + 1, 0);
    const int density = (int)(rng() % 4);
    for (uint64_t p = 0; p < pages; ++p) {
      const bool d = density == 0 ? false : density == 1 ? true : density == 2 ? (rng() % 2) : (rng() % 50 == 0);
      if (d) bm[p >> 6] |= 1ull << (p & 63);
    }
    uint32_t nd = 0, nc = 0;
    int rc = r3_writeset_regions(bm.data(), bytes, page, 1, nullptr, 0, &nd);
    CHECK(rc == R3_OK || rc == R3_ENOSPC);
    rc = r3_writeset_regions(bm.data(), bytes, page, 0, nullptr, 0, &nc);
    CHECK(rc == R3_OK || rc == R3_ENOSPC);
    std::vector<r3_region> dirty(nd + 1), clean(nc + 1);
    uint32_t nd2 = 0, nc2 = 0;
    CHECK(r3_writeset_regions(bm.data(), bytes, page, 1, dirty.data(), nd, &nd2) == R3_OK && nd2 == nd);
    CHECK(r3_writeset_regions(bm.data(), bytes, page, 0, clean.data(), nc, &nc2) == R3_OK && nc2 == nc);
    if (nd > 1) {
      uint32_t few = 0;
      CHECK(r3_writeset_regions(bm.data(), bytes, page, 1, dirty.data(), nd - 1, &few) == R3_ENOSPC && few == nd);
    }
    uint64_t sum = 0;
    for (uint32_t i = 0; i < nd; ++i) {
      sum += dirty[i].bytes;
      CHECK(dirty[i].offset % page == 0 && dirty[i].bytes > 0 && dirty[i].offset + dirty[i].bytes <= bytes);
      CHECK(i == 0 || dirty[i].offset > dirty[i - 1].offset + dirty[i - 1].bytes);  // maximal runs
      for (uint64_t p = dirty[i].offset / page; p * page < dirty[i].offset + dirty[i].bytes; ++p)
        CHECK((bm[p >> 6] >> (p & 63)) & 1);
    }
    for (uint32_t i = 0; i < nc; ++i) {
      sum += clean[i].bytes;
      CHECK(clean[i].offset % page == 0 && clean[i].bytes > 0 && clean[i].offset + clean[i].bytes <= bytes);
      for (uint64_t p = clean[i].offset / page; p * page < clean[i].offset + clean[i].bytes; ++p)
        CHECK(!((bm[p >> 6] >> (p & 63)) & 1));
    }
    CHECK(sum == bytes);
    CHECK((nd > nc ? nd - nc : nc - nd) <= 1);
    if (nd + nc) {  // together they are a valid table of the arena
      std::vector<r3_region> both(dirty.begin(), dirty.begin() + nd);
      both.insert(both.end(), clean.begin(), clean.begin() + nc);
      CHECK(r3_table_validate(both.data(), nd + nc, bytes) == R3_OK);
    }
  }
  {
    uint32_t n_out = 0;
    uint64_t word = 1;
    CHECK(r3_writeset_regions(&word, 100, 0, 1, nullptr, 0, &n_out) == R3_EINVAL);
    CHECK(r3_writeset_regions(nullptr, 100, 4096, 1, nullptr, 0, &n_out) == R3_EINVAL);
    CHECK(r3_writeset_regions(&word, 100, 4096, 1, nullptr, 0, nullptr) == R3_EINVAL);
    CHECK(r3_writeset_regions(nullptr, 0, 4096, 1, nullptr, 0, &n_out) == R3_OK && n_out == 0);
  }
  // --- replicated tables
  for (int rep = 0; rep < 20; ++rep) {
    uint64_t arena = 0;
    const uint32_t n = 1 + (uint32_t)(rng() % 40), inst = 1 + (uint32_t)(rng() % 6);
    std::vector<r3_region> t = random_table(rng, n, 20000, &arena);
    const uint64_t stride = (arena + 255) / 256 * 256;
    std::vector<r3_region> out((size_t)n * inst);
    CHECK(r3_table_replicate(t.data(), n, stride, inst, out.data()) == R3_OK);
    for (uint32_t i = 0; i < inst; ++i)
      for (uint32_t r = 0; r < n; ++r) {
        const r3_region& o = out[(size_t)i * n + r];
        CHECK(o.offset == t[r].offset + (uint64_t)i * stride && o.bytes == t[r].bytes);
        CHECK(o.dtype == t[r].dtype && o.mode == t[r].mode && o.rtol == t[r].rtol && o.atol == t[r].atol);
      }
    CHECK(r3_table_validate(out.data(), n * inst, stride * inst) == R3_OK);
  }
  // --- timing statistics against a direct computation
  for (int rep = 0; rep < 50; ++rep) {
    const uint32_t n = 1 + (uint32_t)(rng() % 40);
    std::vector<float> ms(n);
    for (float& v : ms) v = 0.05f + (float)(rng() % 10000) * 1e-4f;
    r3_timing st;
    CHECK(r3_timing_stats(ms.data(), n, 0.05f, &st) == R3_OK);
    std::vector<float> s = ms;
    std::sort(s.begin(), s.end());
    CHECK(st.min == s.front() && st.max == s.back());
    const float med = n % 2 ? s[n / 2] : 0.5f * (s[n / 2 - 1] + s[n / 2]);
    CHECK(st.median == med);
    CHECK(st.mad >= 0 && st.mean >= st.min && st.mean <= st.max);
    CHECK(st.n == n);
  }
  {
    r3_timing st;
    float one = 1.0f;
    CHECK(r3_timing_stats(nullptr, 3, 0.1f, &st) == R3_EINVAL);
    CHECK(r3_timing_stats(&one, 0, 0.1f, &st) == R3_OK && st.n == 0 && st.stable == 0);
    CHECK(r3_timing_stats(&one, 1, 0.1f, nullptr) == R3_EINVAL);
  }
  std::printf("host checks passed\n");
  return 0;
}
