// Host-only part of region tables: the validity rules of r3_table_validate and the split of
// regions into wavefront tiles.  No GPU call in this file.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <numeric>

#include "r3_internal.h"

namespace r3 {

static std::atomic<uint32_t> g_min_shift{12};
static std::atomic<uint32_t> g_cap_log2{13};

Tuning tuning() { return Tuning{g_min_shift.load(), g_cap_log2.load()}; }

uint32_t elem_size(uint32_t dtype) {
  switch (dtype) {
    case R3_U8: return 1;
    case R3_F32: return 4;
    case R3_F64: return 8;
    case R3_I32: return 4;
    case R3_BF16: return 2;
    case R3_F16: return 2;
    default: return 0;
  }
}

// Upper bound on the tiles of any valid table of n regions inside arena_bytes: each
// region has at most 2^cap tiles, and ceil(bytes/T) <= bytes/T_min + 1.
uint64_t max_tiles(uint32_t n, uint64_t arena_bytes) {
  Tuning tu = tuning();
  uint64_t by_cap = (uint64_t)n << tu.cap_log2;
  uint64_t by_bytes = (uint64_t)n + (arena_bytes >> tu.min_shift);
  return by_cap < by_bytes ? by_cap : by_bytes;
}

uint64_t count_tiles(const r3_region* t, uint32_t n) {
  Tuning tu = tuning();
  uint64_t count = 0;
  for (uint32_t i = 0; i < n; ++i) {
    uint32_t s = tile_shift(t[i].bytes, tu.min_shift, tu.cap_log2);
    count += (t[i].bytes + ((1ull << s) - 1)) >> s;
  }
  return count;
}

static size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

WorkspaceLayout workspace_layout(uint32_t n, uint64_t tiles) {
  WorkspaceLayout w;
  size_t at = 0;
  w.regions = at;     at += up256((size_t)n * sizeof(r3_region));
  w.tile_begin = at;  at += up256(((size_t)n + 1) * sizeof(uint64_t));
  w.tiles = at;       at += up256((size_t)tiles * sizeof(Tile));
  w.partials = at;    at += up256((size_t)tiles * sizeof(Partial));
  w.copy_tiles = at;  at += up256((size_t)tiles * sizeof(CopyTile));
  w.total = at;
  return w;
}

int validate_table(const r3_region* t, uint32_t n, uint64_t arena_bytes) {
  if (t == nullptr || n == 0) return R3_EINVAL;
  for (uint32_t i = 0; i < n; ++i) {
    const r3_region& r = t[i];
    uint32_t es = elem_size(r.dtype);
    if (es == 0) return R3_EINVAL;
    if (r.mode != R3_CMP_BITWISE && r.mode != R3_CMP_TOL) return R3_EINVAL;
    if (!std::isfinite(r.rtol) || !std::isfinite(r.atol) || r.rtol < 0 || r.atol < 0)
      return R3_EINVAL;
    if ((r.offset % es) || (r.bytes % es)) return R3_EALIGN;
    if (r.offset > arena_bytes || r.bytes > arena_bytes - r.offset) return R3_ERANGE;
  }
  // Disjointness by one sweep over the non-empty regions in address order.
  std::vector<uint32_t> order;
  order.reserve(n);
  for (uint32_t i = 0; i < n; ++i)
    if (t[i].bytes) order.push_back(i);
  std::sort(order.begin(), order.end(),
            [&](uint32_t a, uint32_t b) { return t[a].offset < t[b].offset; });
  uint64_t end = 0;
  for (uint32_t i : order) {
    if (t[i].offset < end) return R3_EOVERLAP;
    end = t[i].offset + t[i].bytes;
  }
  return R3_OK;
}

void plan_table(const r3_region* t, uint32_t n, TablePlan* plan) {
  Tuning tu = tuning();
  plan->min_shift = tu.min_shift;
  plan->cap_log2 = tu.cap_log2;
  plan->total_bytes = 0;
  plan->max_region_tiles = 0;
  plan->max_shift = tu.min_shift;
  plan->tile_begin.assign((size_t)n + 1, 0);
  uint64_t count = 0;
  for (uint32_t i = 0; i < n; ++i) {
    plan->tile_begin[i] = count;
    uint32_t s = tile_shift(t[i].bytes, tu.min_shift, tu.cap_log2);
    uint64_t k = (t[i].bytes + ((1ull << s) - 1)) >> s;
    if (k > plan->max_region_tiles) plan->max_region_tiles = (uint32_t)k;
    if (k && s > plan->max_shift) plan->max_shift = s;
    count += k;
    plan->total_bytes += t[i].bytes;
  }
  plan->tile_begin[n] = count;
  plan->tiles.resize(count);
  for (uint32_t c = 0; c < kMaxCopyClasses; ++c) plan->class_count[c] = 0;
  for (uint32_t i = 0; i < n; ++i) {
    uint32_t s = tile_shift(t[i].bytes, tu.min_shift, tu.cap_log2);
    uint64_t k = plan->tile_begin[i], e = plan->tile_begin[i + 1];
    for (uint32_t j = 0; k < e; ++k, ++j) plan->tiles[k] = Tile{i, j | (s << 24)};
    const uint32_t c = s - tu.min_shift;
    if (c < kMaxCopyClasses) plan->class_count[c] += (uint32_t)(e - plan->tile_begin[i]);
  }
  // Counting sort of the tile ids by class, address order kept inside a class.
  uint64_t at[kMaxCopyClasses];
  uint64_t run = 0;
  for (uint32_t c = 0; c < kMaxCopyClasses; ++c) {
    at[c] = run;
    run += plan->class_count[c];
  }
  plan->copy_tiles.assign(count, CopyTile{0, 0, 0});
  for (uint64_t k = 0; k < count; ++k) {
    const Tile& tl = plan->tiles[k];
    const uint32_t shift = tl.packed >> 24, index = tl.packed & 0xFFFFFFu;
    const uint32_t c = shift - tu.min_shift;
    if (c >= kMaxCopyClasses) continue;
    const r3_region& rg = t[tl.region];
    const uint64_t rel = (uint64_t)index << shift;
    const uint64_t left = rg.bytes - rel;
    const uint64_t full = 1ull << shift;
    plan->copy_tiles[at[c]++] = CopyTile{rg.offset + rel, (uint32_t)(left < full ? left : full),
                                          elem_size(rg.dtype)};
  }
}

}  // namespace r3

extern "C" {

int r3_table_validate(const r3_region* host_tbl, uint32_t n, uint64_t arena_bytes) {
  return r3::validate_table(host_tbl, n, arena_bytes);
}

size_t r3_table_workspace_bytes(uint32_t n, uint64_t arena_bytes) {
  return r3::workspace_layout(n, r3::max_tiles(n, arena_bytes)).total;
}

size_t r3_table_workspace_bytes_exact(const r3_region* host_tbl, uint32_t n,
                                      uint64_t arena_bytes) {
  if (r3::validate_table(host_tbl, n, arena_bytes) != R3_OK) return 0;
  return r3::workspace_layout(n, r3::count_tiles(host_tbl, n)).total;
}

int r3_writeset_regions(const uint64_t* host_bitmap, uint64_t bytes, uint32_t page_bytes,
                        int want_dirty, r3_region* out, uint32_t cap, uint32_t* n_out) {
  if (n_out == nullptr || page_bytes == 0 || (bytes && host_bitmap == nullptr) || (cap && out == nullptr))
    return R3_EINVAL;
  const uint64_t n_pages = (bytes + page_bytes - 1) / page_bytes;
  uint64_t runs = 0, start = 0;
  bool in_run = false;
  auto close_run = [&](uint64_t end_page) {
    if (runs < cap) {
      r3_region r{};
      r.offset = start * page_bytes;
      const uint64_t end = end_page * page_bytes;
      r.bytes = (end < bytes ? end : bytes) - r.offset;
      r.dtype = R3_U8;
      r.mode = R3_CMP_BITWISE;
      out[runs] = r;
    }
    ++runs;
  };
  for (uint64_t p = 0; p < n_pages; ++p) {
    const bool dirty = (host_bitmap[p >> 6] >> (p & 63)) & 1u;
    const bool want = dirty == (want_dirty != 0);
    if (want && !in_run) {
      in_run = true;
      start = p;
    } else if (!want && in_run) {
      in_run = false;
      close_run(p);
    }
  }
  if (in_run) close_run(n_pages);
  if (runs > 0xFFFFFFFFull) return R3_ERANGE;
  *n_out = (uint32_t)runs;
  return runs > cap ? R3_ENOSPC : R3_OK;
}

int r3_table_replicate(const r3_region* host_tbl, uint32_t n, uint64_t instance_stride,
                       uint32_t instances, r3_region* out) {
  if (host_tbl == nullptr || out == nullptr || n == 0 || instances == 0) return R3_EINVAL;
  if ((uint64_t)n * instances > 0xFFFFFFFFull) return R3_ERANGE;
  for (uint32_t i = 0; i < instances; ++i)
    for (uint32_t r = 0; r < n; ++r) {
      r3_region g = host_tbl[r];
      const uint64_t shift = (uint64_t)i * instance_stride;
      if (g.offset > UINT64_MAX - shift) return R3_ERANGE;
      g.offset += shift;
      out[(size_t)i * n + r] = g;
    }
  return R3_OK;
}

int r3_timing_stats(const float* ms, uint32_t n, float rel_noise, r3_timing* out) {
  if (out == nullptr || (n && ms == nullptr)) return R3_EINVAL;
  *out = r3_timing{};
  if (n == 0) return R3_OK;
  std::vector<float> v(ms, ms + n);
  std::sort(v.begin(), v.end());
  auto median_of = [](const std::vector<float>& s) {
    const size_t m = s.size();
    return m % 2 ? s[m / 2] : 0.5f * (s[m / 2 - 1] + s[m / 2]);
  };
  out->n = n;
  out->min = v.front();
  out->max = v.back();
  out->median = median_of(v);
  double sum = 0;
  for (float x : v) sum += x;
  out->mean = (float)(sum / n);
  std::vector<float> dev(n);
  for (uint32_t i = 0; i < n; ++i) dev[i] = std::fabs(v[i] - out->median);
  std::sort(dev.begin(), dev.end());
  out->mad = median_of(dev);
  out->stable = (out->median > 0 && out->mad <= rel_noise * out->median) ? 1u : 0u;
  return R3_OK;
}

int r3_tune_tiles(uint32_t min_tile_bytes, uint32_t max_tiles_per_region) {
  auto log2_exact = [](uint32_t v) -> int {
    if (v == 0 || (v & (v - 1))) return -1;
    int s = 0;
    while ((1u << s) < v) ++s;
    return s;
  };
  int ms = min_tile_bytes ? log2_exact(min_tile_bytes) : 12;
  int cs = max_tiles_per_region ? log2_exact(max_tiles_per_region) : 13;
  if (ms < 10 || ms > 24 || cs < 6 || cs > 16) return R3_EINVAL;
  r3::g_min_shift.store((uint32_t)ms);
  r3::g_cap_log2.store((uint32_t)cs);
  return R3_OK;
}

}  // extern "C"
