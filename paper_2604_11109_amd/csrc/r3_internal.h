// Internal declarations shared by the host side and the kernels of libr3.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "r3.h"

namespace r3 {

constexpr uint64_t kPhi = 0x9E3779B97F4A7C15ull;  // floor(2^64 * (sqrt(5)-1)/2)
constexpr uint64_t kLen = 0xBB67AE8584CAA73Bull;  // floor(2^64 * frac(sqrt(3)))

constexpr int kWaveSize = 64;
constexpr int kWavesPerBlock = 4;
constexpr int kBlock = kWaveSize * kWavesPerBlock;

// A tile is the unit of work of one wavefront: up to 2^shift consecutive bytes of one
// region, starting at a multiple of 2^shift from the region's first byte.  The shift is
// a function of the region's size (tile_shift below): small regions use the minimum
// tile, large ones grow so that no region has more than 2^cap_log2 tiles, which bounds
// the per-region finalize pass.
struct Tile {
  uint32_t region;
  uint32_t packed;  // bits 0..23: tile number inside the region; bits 24..31: shift
};

__host__ __device__ inline uint32_t tile_shift(uint64_t bytes, uint32_t min_shift,
                                               uint32_t cap_log2) {
  uint64_t q = (bytes + ((1ull << cap_log2) - 1)) >> cap_log2;  // ceil(bytes / cap)
  uint32_t s = 0;
  while (s < 63 && (1ull << s) < q) ++s;  // ceil(log2(q)), at most ~40 steps, scalar
  return s < min_shift ? min_shift : s;
}

// What one wavefront leaves behind for the per-region finalize pass.
struct Partial {
  uint64_t count;
  uint64_t first;  // region-relative element index, R3_NO_INDEX if none
  uint64_t max_abs_bits;
  uint64_t max_rel_bits;
  uint64_t cks;  // sum of word products only; the length term is added at finalize
};
static_assert(sizeof(Partial) == 40, "partial layout");
static_assert(sizeof(r3_region) == 40 && sizeof(r3_region_result) == 40, "ABI layout");
static_assert(sizeof(r3_summary) == 40 && sizeof(r3_eval_result) == 56, "ABI layout");

// Tiles grouped by size class (class c holds the tiles of 2^(min_shift + c) bytes) so that
// the copy kernels can give every tile exactly as many 1 KiB wavefront slots as it has
// bytes for, whatever mix of region sizes a table holds.
constexpr uint32_t kMaxCopyClasses = 32;
struct CopyClasses {
  uint32_t n;                           // classes in use (max_shift - min_shift + 1)
  uint32_t sub_log2[kMaxCopyClasses];   // log2 of the slots per tile of the class
  uint32_t first[kMaxCopyClasses];      // first position of the class in copy_order
  uint64_t slot_base[kMaxCopyClasses + 1];  // first slot of the class; [n] = all slots
};

// What a copy wavefront needs to know about its tile, in one 16-byte load.
struct CopyTile {
  uint64_t at;    // arena offset of the tile's first byte
  uint32_t len;   // bytes in the tile
  uint32_t es;    // element size of the region (unit of unaligned heads and tails)
};

// Device-side view of a table's workspace.
struct TableDev {
  const r3_region* regions;   // n
  const uint64_t* tile_begin; // n + 1, prefix sum of tiles per region
  const Tile* tiles;          // n_tiles
  Partial* partials;          // n_tiles (checksum-only calls use the first 8 bytes * n_tiles)
  const CopyTile* copy_tiles; // n_tiles: the tiles again, sorted by size class
  uint32_t n_regions;
  uint32_t min_shift;         // log2 of the smallest tile
  uint32_t cap_log2;          // log2 of the most tiles a region may have
  uint32_t max_region_tiles;  // largest tile count of any region (sizes the finalize block)
  uint32_t max_shift;         // log2 of the largest tile of any region
  uint64_t n_tiles;
};

// A small table that travels in the launch arguments (r3_compare_static): every region is
// split into tiles of the same size 2^shift; tile_begin is the prefix sum of tiles per region.
struct StaticTable {
  r3_region regions[R3_STATIC_MAX_REGIONS];
  uint32_t tile_begin[R3_STATIC_MAX_REGIONS + 1];
  uint32_t n;
  uint32_t shift;
};

// One slot of the pinned host buffer that the replay loop hands to the finalize pass: the
// table summary and, written after it with a system-scope release, the sequence number of
// the validation that produced it (what the host polls for).
struct HostSlot {
  r3_summary summary;
  uint64_t seq;
  uint64_t pad[2];
};
static_assert(sizeof(HostSlot) == 64, "host slot layout");

// Pinned host slot of one guard check: how many regions changed, the first of them, and
// the sequence number posted after both.
struct GuardSlot {
  uint64_t changed;
  uint64_t first_region;
  uint64_t seq;
  uint64_t pad;
};

// Host-side plan of a table: how the regions split into tiles.
struct TablePlan {
  uint32_t min_shift = 0, cap_log2 = 0, max_region_tiles = 0, max_shift = 0;
  uint64_t total_bytes = 0;
  std::vector<uint64_t> tile_begin;  // n + 1
  std::vector<Tile> tiles;
  std::vector<CopyTile> copy_tiles;          // by size class, address order inside a class
  uint32_t class_count[kMaxCopyClasses] = {};  // tiles per class
};

struct WorkspaceLayout {
  size_t regions, tile_begin, tiles, partials, copy_tiles, total;
};

struct Tuning {
  uint32_t min_shift;  // default 12 (4 KiB)
  uint32_t cap_log2;   // default 13 (8192 tiles per region)
};

uint32_t elem_size(uint32_t dtype);  // 0 for an unknown dtype
Tuning tuning();
uint64_t max_tiles(uint32_t n, uint64_t arena_bytes);
uint64_t count_tiles(const r3_region* t, uint32_t n);
WorkspaceLayout workspace_layout(uint32_t n, uint64_t tiles);
int validate_table(const r3_region* t, uint32_t n, uint64_t arena_bytes);
void plan_table(const r3_region* t, uint32_t n, TablePlan* plan);

// Kernel launchers (r3_kernels.hip).  All enqueue on `s` and return the launch status.
void set_copy_shape(uint32_t shift, uint32_t block);
hipError_t launch_restore(const TableDev& t, const uint32_t* class_count, const void* src, void* dst,
                          hipStream_t s);
hipError_t launch_copy_flat(const void* src, void* dst, uint64_t bytes, hipStream_t s);
hipError_t launch_checksum(const TableDev& t, const void* arena, uint64_t* out, hipStream_t s);
hipError_t launch_compare(const TableDev& t, const void* live, const void* golden,
                          r3_region_result* out, r3_summary* summary, HostSlot* host_slot,
                          uint64_t host_seq, const uint32_t* rep_counter, hipStream_t s);
// The library's own partials buffer on the current device (resolved once per device; the
// device must be current).  launch_compare_static takes that address, never the symbol.
hipError_t static_scratch_address(int device, Partial** out);
hipError_t launch_compare_static(const StaticTable& st, const void* live, const void* golden,
                                 Partial* scratch, r3_region_result* out, r3_summary* summary,
                                 hipStream_t s);
hipError_t launch_stamp(uint32_t* rep_counter, uint64_t* stamps, uint32_t which, hipStream_t s);
hipError_t launch_set_counter(uint32_t* rep_counter, uint32_t value, hipStream_t s);
hipError_t launch_guard_compare(const uint64_t* got, const uint64_t* expected, uint32_t n,
                                GuardSlot* host_slot, uint64_t host_seq, hipStream_t s);
hipError_t launch_dirty_diff(const void* pre, const void* post, uint64_t bytes, uint32_t page_bytes,
                             uint64_t* bitmap, uint64_t* dirty_count, hipStream_t s);

}  // namespace r3

namespace r3 {

// What one evaluation in flight owns: its verdict slots in pinned host memory, its events, and
// what the host has to remember between enqueueing the work and reading the verdict.
struct EvalLane {
  HostSlot* pinned = nullptr;      // R3_MAX_REPLAYS slots, pinned host memory
  HostSlot* pinned_dev = nullptr;  // the same memory as the device addresses it
  GuardSlot* guard_pinned = nullptr;  // R3_MAX_REPLAYS slots, pinned host memory
  GuardSlot* guard_pinned_dev = nullptr;
  std::vector<hipEvent_t> events;  // 4 per replay, grown on demand
  hipEvent_t end_event = nullptr;  // marks the end of a submission whose last work posts no number

  bool busy = false;  // enqueued, verdict not yet collected
  bool prof = false;
  bool has_launch = false;
  bool has_guard = false;
  bool end_recorded = false;
  uint32_t warmup = 0, total = 0, done = 0, n_validated = 0;
  int cand = 0;                        // status of the candidate callback
  hipError_t status = hipSuccess;      // status of the enqueueing
  std::vector<uint8_t> validated, guarded;  // per replay: validation / guard check enqueued
  const uint64_t* last_flag = nullptr;      // where the last work enqueued posts its number, if it does
  uint64_t last_want = 0;
  hipStream_t stream = nullptr;
  r3_guard guard{};
  const void* d_prologue = nullptr;
  void* d_live = nullptr;
};

}  // namespace r3

namespace r3 {

// Two streams of the context's own on which consecutive overlapped evaluations alternate, and
// the events that keep the timed candidate alone on the GPU (r3_eval_submit_overlapped).
struct Pipe {
  hipStream_t s[2] = {nullptr, nullptr};
  hipEvent_t cand_end[2] = {nullptr, nullptr};  // after the last candidate launch of an evaluation
  hipEvent_t val_end[2] = {nullptr, nullptr};   // after its last validation
  hipEvent_t join = nullptr;                    // the caller's stream at submission
  bool cand_valid[2] = {false, false};
  bool val_valid[2] = {false, false};
  uint64_t n = 0;                               // evaluations submitted this way
  bool ready = false;
};

}  // namespace r3

struct r3_ctx {
  int device = 0;
  std::string err;
  r3::EvalLane lanes[1 + R3_MAX_INFLIGHT];  // [0]: the synchronous calls; the rest: tickets
  uint64_t seq = 0;                    // sequence number of the last validation enqueued
  std::vector<float> last_times;       // candidate ms of the timed replays of the last evaluation
  uint32_t profile_period = 0;         // 0 = off, n = stage events on every n-th evaluation
  uint64_t evals = 0;
  r3_profile profile{};
  r3::Pipe pipe;
  r3::Partial* static_scratch = nullptr;  // this device's copy of the library's partials buffer
  hipError_t static_scratch_status = hipSuccess;
};

struct r3_table {
  r3_ctx* ctx = nullptr;
  r3::TableDev dev{};
  uint64_t arena_bytes = 0;
  uint64_t total_bytes = 0;
  uint32_t class_count[r3::kMaxCopyClasses] = {};
};

// One replay (restore, candidate, validation) captured as a HIP graph.
struct r3_replay {
  r3_ctx* ctx = nullptr;
  const r3_table* check_tbl = nullptr;
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  hipStream_t capture_stream = nullptr;
  uint32_t* d_counter = nullptr;            // in the caller's workspace
  r3::HostSlot* slots = nullptr;            // pinned: one verdict per replay
  r3::HostSlot* slots_dev = nullptr;
  uint64_t* stamps = nullptr;               // pinned: start/end wall clock per replay
  uint64_t* stamps_dev = nullptr;
  double ticks_per_ms = 0;
  bool has_candidate = false;
  uint32_t replays = 0;                     // replays recorded in the graph
};
