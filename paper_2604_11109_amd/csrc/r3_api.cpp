// Entry points of libr3.so: argument checks, table upload, and the replay / record loops
// that string the kernels together on the caller's stream.
#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstring>
#include <new>

#include "r3_internal.h"

namespace {

int fail(r3_ctx* ctx, int status, const char* what) {
  if (ctx) ctx->err = what;
  return status;
}

int fail_hip(r3_ctx* ctx, hipError_t e, const char* where) {
  if (ctx) {
    ctx->err = std::string(where) + ": " + hipGetErrorString(e);
  }
  return R3_EHIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

// Bind the calling thread to the context's device for the duration of one entry point.
struct DeviceGuard {
  int prev = -1;
  bool ok = true;
  explicit DeviceGuard(int device) {
    if (hipGetDevice(&prev) != hipSuccess) prev = -1;
    if (prev != device) ok = hipSetDevice(device) == hipSuccess;
  }
  ~DeviceGuard() {
    if (prev >= 0) (void)hipSetDevice(prev);
  }
};

int check_common(r3_ctx* ctx, const r3_table* tbl) {
  if (ctx == nullptr) return R3_EINVAL;
  ctx->err.clear();
  if (tbl == nullptr) return fail(ctx, R3_EINVAL, "table is NULL");
  if (tbl->ctx != ctx) return fail(ctx, R3_EINVAL, "table belongs to another context");
  return R3_OK;
}

// Pinned verdict slots of a lane, allocated the first time the lane is used.
int lane_init(r3_ctx* ctx, r3::EvalLane& lane) {
  if (lane.pinned != nullptr) return R3_OK;
  hipError_t e = hipHostMalloc(reinterpret_cast<void**>(&lane.pinned),
                               R3_MAX_REPLAYS * sizeof(r3::HostSlot), hipHostMallocMapped);
  if (e == hipSuccess) e = hipHostGetDevicePointer(reinterpret_cast<void**>(&lane.pinned_dev), lane.pinned, 0);
  if (e == hipSuccess)
    e = hipHostMalloc(reinterpret_cast<void**>(&lane.guard_pinned), R3_MAX_REPLAYS * sizeof(r3::GuardSlot),
                      hipHostMallocMapped);
  if (e == hipSuccess)
    e = hipHostGetDevicePointer(reinterpret_cast<void**>(&lane.guard_pinned_dev), lane.guard_pinned, 0);
  if (e == hipSuccess) e = hipEventCreate(&lane.end_event);
  if (e != hipSuccess) {
    if (lane.guard_pinned) (void)hipHostFree(lane.guard_pinned);
    if (lane.pinned) (void)hipHostFree(lane.pinned);
    lane.pinned = nullptr;
    lane.guard_pinned = nullptr;
    return fail_hip(ctx, e, "pinned verdict slots");
  }
  return R3_OK;
}

// The context's own pair of streams and ordering events, created at the first overlapped
// submission.  Default priority, like every stream this library touches.
void pipe_release(r3::Pipe& p);

int pipe_init(r3_ctx* ctx) {
  r3::Pipe& p = ctx->pipe;
  if (p.ready) return R3_OK;
  hipError_t e = hipSuccess;
  for (int i = 0; i < 2 && e == hipSuccess; ++i) {
    e = hipStreamCreateWithFlags(&p.s[i], hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&p.cand_end[i], hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&p.val_end[i], hipEventDisableTiming);
  }
  if (e == hipSuccess) e = hipEventCreateWithFlags(&p.join, hipEventDisableTiming);
  if (e != hipSuccess) {
    pipe_release(p);  // nothing half-made is kept: the next submission starts over
    return fail_hip(ctx, e, "streams of the overlapped pipeline");
  }
  p.ready = true;
  return R3_OK;
}

void pipe_release(r3::Pipe& p) {
  for (int i = 0; i < 2; ++i) {
    if (p.s[i]) (void)hipStreamSynchronize(p.s[i]);
    if (p.cand_end[i]) (void)hipEventDestroy(p.cand_end[i]);
    if (p.val_end[i]) (void)hipEventDestroy(p.val_end[i]);
    if (p.s[i]) (void)hipStreamDestroy(p.s[i]);
  }
  if (p.join) (void)hipEventDestroy(p.join);
  p = r3::Pipe{};
}

void lane_release(r3::EvalLane& lane) {
  for (hipEvent_t e : lane.events) (void)hipEventDestroy(e);
  lane.events.clear();
  if (lane.end_event) (void)hipEventDestroy(lane.end_event);
  if (lane.pinned) (void)hipHostFree(lane.pinned);
  if (lane.guard_pinned) (void)hipHostFree(lane.guard_pinned);
  lane.pinned = nullptr;
  lane.guard_pinned = nullptr;
  lane.end_event = nullptr;
}

}  // namespace

extern "C" {

uint32_t r3_version(void) { return 1; }

const char* r3_strerror(int status) {
  switch (status) {
    case R3_OK: return "ok";
    case R3_EINVAL: return "invalid argument";
    case R3_EALIGN: return "misaligned offset, size or pointer";
    case R3_ERANGE: return "region outside the arena";
    case R3_EOVERLAP: return "regions overlap";
    case R3_ENOSPC: return "workspace too small";
    case R3_EHIP: return "HIP runtime error";
    case R3_ECANDIDATE: return "candidate failed to launch";
    case R3_EBUSY: return "not finished yet";
    default: return "unknown status";
  }
}

int r3_ctx_create(r3_ctx** out, int device) {
  if (out == nullptr) return R3_EINVAL;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return R3_EHIP;
  r3_ctx* ctx = new (std::nothrow) r3_ctx();
  if (ctx == nullptr) return R3_ENOSPC;
  ctx->device = device;
  DeviceGuard guard(device);
  if (!guard.ok || lane_init(ctx, ctx->lanes[0]) != R3_OK) {
    delete ctx;
    return R3_EHIP;
  }
  // Where this device keeps the library's own partials buffer (used by r3_compare_static only;
  // a failure here is reported by that call).
  ctx->static_scratch_status = r3::static_scratch_address(device, &ctx->static_scratch);
  *out = ctx;
  return R3_OK;
}

int r3_ctx_destroy(r3_ctx* ctx) {
  if (ctx == nullptr) return R3_EINVAL;
  DeviceGuard guard(ctx->device);
  // Work that still posts into a lane's pinned memory must have run before the memory goes.
  for (r3::EvalLane& lane : ctx->lanes)
    if (lane.busy) (void)hipStreamSynchronize(lane.stream);
  for (r3::EvalLane& lane : ctx->lanes) lane_release(lane);
  pipe_release(ctx->pipe);
  delete ctx;
  return R3_OK;
}

int r3_tune_copy(uint32_t bytes_per_wavefront, uint32_t block_threads) {
  uint32_t shift = 0;
  while ((1u << shift) < bytes_per_wavefront) ++shift;
  if (bytes_per_wavefront == 0) shift = 10;
  if (block_threads == 0) block_threads = 64;
  if ((1u << shift) != (bytes_per_wavefront ? bytes_per_wavefront : 1024u) || shift < 10 || shift > 20)
    return R3_EINVAL;
  if (block_threads != 64 && block_threads != 128 && block_threads != 256) return R3_EINVAL;
  r3::set_copy_shape(shift, block_threads);
  return R3_OK;
}

int r3_ctx_profile(r3_ctx* ctx, int period) {
  if (ctx == nullptr || period < 0) return R3_EINVAL;
  ctx->profile_period = (uint32_t)period;
  ctx->evals = 0;
  return R3_OK;
}

int r3_ctx_profile_read(r3_ctx* ctx, r3_profile* out, int reset) {
  if (ctx == nullptr || out == nullptr) return R3_EINVAL;
  *out = ctx->profile;
  if (reset) ctx->profile = r3_profile{};
  return R3_OK;
}

const char* r3_last_error(const r3_ctx* ctx) { return ctx ? ctx->err.c_str() : "context is NULL"; }

int r3_table_create(r3_ctx* ctx, const r3_region* host_tbl, uint32_t n, uint64_t arena_bytes,
                    void* d_ws, size_t ws_bytes, r3_table** out) {
  if (ctx == nullptr || out == nullptr) return R3_EINVAL;
  ctx->err.clear();
  *out = nullptr;
  int rc = r3::validate_table(host_tbl, n, arena_bytes);
  if (rc != R3_OK) return fail(ctx, rc, "region table rejected");
  if (d_ws == nullptr) return fail(ctx, R3_EINVAL, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(d_ws) & 255u) return fail(ctx, R3_EALIGN, "workspace not 256-byte aligned");
  r3::TablePlan plan;
  r3::plan_table(host_tbl, n, &plan);
  if (plan.max_region_tiles > 0xFFFFFFu || plan.max_shift - plan.min_shift >= r3::kMaxCopyClasses ||
      plan.tiles.size() > 0xFFFFFFFFull)
    return fail(ctx, R3_EINVAL, "region too large");
  const r3::WorkspaceLayout lay = r3::workspace_layout(n, plan.tiles.size());
  if (ws_bytes < lay.total) return fail(ctx, R3_ENOSPC, "workspace smaller than the table needs");

  DeviceGuard guard(ctx->device);
  if (!guard.ok) return fail(ctx, R3_EHIP, "cannot select the device");
  uint8_t* ws = static_cast<uint8_t*>(d_ws);
  hipError_t e = hipMemcpy(ws + lay.regions, host_tbl, (size_t)n * sizeof(r3_region), hipMemcpyHostToDevice);
  if (e == hipSuccess)
    e = hipMemcpy(ws + lay.tile_begin, plan.tile_begin.data(), plan.tile_begin.size() * sizeof(uint64_t),
                  hipMemcpyHostToDevice);
  if (e == hipSuccess && !plan.tiles.empty())
    e = hipMemcpy(ws + lay.tiles, plan.tiles.data(), plan.tiles.size() * sizeof(r3::Tile),
                  hipMemcpyHostToDevice);
  if (e == hipSuccess && !plan.copy_tiles.empty())
    e = hipMemcpy(ws + lay.copy_tiles, plan.copy_tiles.data(), plan.copy_tiles.size() * sizeof(r3::CopyTile),
                  hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) return fail_hip(ctx, e, "table upload");

  r3_table* tbl = new (std::nothrow) r3_table();
  if (tbl == nullptr) return fail(ctx, R3_ENOSPC, "out of host memory");
  tbl->ctx = ctx;
  tbl->arena_bytes = arena_bytes;
  tbl->total_bytes = plan.total_bytes;
  tbl->dev.regions = reinterpret_cast<const r3_region*>(ws + lay.regions);
  tbl->dev.tile_begin = reinterpret_cast<const uint64_t*>(ws + lay.tile_begin);
  tbl->dev.tiles = reinterpret_cast<const r3::Tile*>(ws + lay.tiles);
  tbl->dev.partials = reinterpret_cast<r3::Partial*>(ws + lay.partials);
  tbl->dev.copy_tiles = reinterpret_cast<const r3::CopyTile*>(ws + lay.copy_tiles);
  std::memcpy(tbl->class_count, plan.class_count, sizeof(tbl->class_count));
  tbl->dev.n_regions = n;
  tbl->dev.min_shift = plan.min_shift;
  tbl->dev.cap_log2 = plan.cap_log2;
  tbl->dev.max_region_tiles = plan.max_region_tiles;
  tbl->dev.max_shift = plan.max_shift;
  tbl->dev.n_tiles = plan.tiles.size();
  *out = tbl;
  return R3_OK;
}

int r3_table_destroy(r3_table* tbl) {
  if (tbl == nullptr) return R3_EINVAL;
  delete tbl;
  return R3_OK;
}

int r3_table_info(const r3_table* tbl, uint32_t* n_regions, uint64_t* n_tiles, uint32_t* tile_bytes,
                  uint64_t* total_bytes, uint64_t* arena_bytes) {
  if (tbl == nullptr) return R3_EINVAL;
  if (n_regions) *n_regions = tbl->dev.n_regions;
  if (n_tiles) *n_tiles = tbl->dev.n_tiles;
  if (tile_bytes) *tile_bytes = 1u << tbl->dev.min_shift;
  if (total_bytes) *total_bytes = tbl->total_bytes;
  if (arena_bytes) *arena_bytes = tbl->arena_bytes;
  return R3_OK;
}

int r3_restore(r3_ctx* ctx, const r3_table* tbl, const void* d_snapshot, void* d_live, void* stream) {
  int rc = check_common(ctx, tbl);
  if (rc != R3_OK) return rc;
  if (d_snapshot == nullptr || d_live == nullptr) return fail(ctx, R3_EINVAL, "arena pointer is NULL");
  if (!aligned16(d_snapshot) || !aligned16(d_live)) return fail(ctx, R3_EALIGN, "arena base not 16-byte aligned");
  const uint8_t* s = static_cast<const uint8_t*>(d_snapshot);
  const uint8_t* l = static_cast<const uint8_t*>(d_live);
  if (s < l + tbl->arena_bytes && l < s + tbl->arena_bytes && tbl->arena_bytes)
    return fail(ctx, R3_EINVAL, "snapshot and live arenas overlap");
  DeviceGuard guard(ctx->device);
  hipError_t e = r3::launch_restore(tbl->dev, tbl->class_count, d_snapshot, d_live, as_stream(stream));
  return e == hipSuccess ? R3_OK : fail_hip(ctx, e, "restore launch");
}

int r3_checksum(r3_ctx* ctx, const r3_table* tbl, const void* d_arena, uint64_t* d_out, void* stream) {
  int rc = check_common(ctx, tbl);
  if (rc != R3_OK) return rc;
  if (d_arena == nullptr || d_out == nullptr) return fail(ctx, R3_EINVAL, "pointer is NULL");
  if (!aligned16(d_arena)) return fail(ctx, R3_EALIGN, "arena base not 16-byte aligned");
  DeviceGuard guard(ctx->device);
  hipError_t e = r3::launch_checksum(tbl->dev, d_arena, d_out, as_stream(stream));
  return e == hipSuccess ? R3_OK : fail_hip(ctx, e, "checksum launch");
}

int r3_compare(r3_ctx* ctx, const r3_table* tbl, const void* d_live, const void* d_golden,
               r3_region_result* d_out, r3_summary* d_summary, void* stream) {
  int rc = check_common(ctx, tbl);
  if (rc != R3_OK) return rc;
  if (d_live == nullptr || d_golden == nullptr || d_out == nullptr)
    return fail(ctx, R3_EINVAL, "pointer is NULL");
  if (!aligned16(d_live) || !aligned16(d_golden)) return fail(ctx, R3_EALIGN, "arena base not 16-byte aligned");
  DeviceGuard guard(ctx->device);
  hipError_t e = r3::launch_compare(tbl->dev, d_live, d_golden, d_out, d_summary, nullptr, 0, nullptr,
                                    as_stream(stream));
  return e == hipSuccess ? R3_OK : fail_hip(ctx, e, "compare launch");
}

int r3_compare_static(r3_ctx* ctx, const r3_region* host_tbl, uint32_t n, uint64_t arena_bytes,
                      const void* d_live, const void* d_golden, r3_region_result* d_out,
                      r3_summary* d_summary, void* stream) {
  if (ctx == nullptr) return R3_EINVAL;
  ctx->err.clear();
  if (host_tbl == nullptr || n == 0) return fail(ctx, R3_EINVAL, "region table is empty");
  if (n > R3_STATIC_MAX_REGIONS) return fail(ctx, R3_ENOSPC, "more than R3_STATIC_MAX_REGIONS regions");
  // The rules of r3_table_validate, written without host allocations (n is small).
  for (uint32_t i = 0; i < n; ++i) {
    const r3_region& r = host_tbl[i];
    const uint32_t es = r3::elem_size(r.dtype);
    if (es == 0 || (r.mode != R3_CMP_BITWISE && r.mode != R3_CMP_TOL) || !(r.rtol >= 0) || !(r.atol >= 0) ||
        r.rtol > 1.7976931348623157e308 || r.atol > 1.7976931348623157e308)
      return fail(ctx, R3_EINVAL, "region table rejected");
    if ((r.offset % es) || (r.bytes % es)) return fail(ctx, R3_EALIGN, "region table rejected");
    if (r.offset > arena_bytes || r.bytes > arena_bytes - r.offset)
      return fail(ctx, R3_ERANGE, "region table rejected");
  }
  for (uint32_t i = 0; i < n; ++i)
    for (uint32_t j = i + 1; j < n; ++j) {
      const r3_region &a = host_tbl[i], &b = host_tbl[j];
      if (a.bytes && b.bytes && a.offset < b.offset + b.bytes && b.offset < a.offset + a.bytes)
        return fail(ctx, R3_EOVERLAP, "region table rejected");
    }
  if (d_live == nullptr || d_golden == nullptr || d_out == nullptr)
    return fail(ctx, R3_EINVAL, "pointer is NULL");
  if (!aligned16(d_live) || !aligned16(d_golden)) return fail(ctx, R3_EALIGN, "arena base not 16-byte aligned");
  if (ctx->static_scratch == nullptr)
    return fail_hip(ctx, ctx->static_scratch_status != hipSuccess ? ctx->static_scratch_status : hipErrorInvalidSymbol,
                    "the library's partials buffer could not be resolved on this device");
  // One tile size for all regions: the smallest that keeps the tile count within the buffer.
  r3::StaticTable st{};
  st.n = n;
  uint32_t shift = 12;
  for (;; ++shift) {
    if ((1ull << shift) > R3_STATIC_MAX_TILE_BYTES)
      return fail(ctx, R3_ENOSPC, "regions need more than R3_STATIC_MAX_TILES tiles of R3_STATIC_MAX_TILE_BYTES");
    uint64_t tiles = 0;
    for (uint32_t i = 0; i < n; ++i) tiles += (host_tbl[i].bytes + ((1ull << shift) - 1)) >> shift;
    if (tiles <= R3_STATIC_MAX_TILES) break;
  }
  st.shift = shift;
  uint32_t at = 0;
  for (uint32_t i = 0; i < n; ++i) {
    st.regions[i] = host_tbl[i];
    st.tile_begin[i] = at;
    at += (uint32_t)((host_tbl[i].bytes + ((1ull << shift) - 1)) >> shift);
  }
  for (uint32_t i = n; i <= R3_STATIC_MAX_REGIONS; ++i) st.tile_begin[i] = at;
  DeviceGuard guard(ctx->device);
  hipError_t e = r3::launch_compare_static(st, d_live, d_golden, ctx->static_scratch, d_out, d_summary,
                                           as_stream(stream));
  return e == hipSuccess ? R3_OK : fail_hip(ctx, e, "static compare launch");
}

static bool page_ok(uint32_t page_bytes) {
  return page_bytes >= 256 && page_bytes <= (1u << 20) && (page_bytes & (page_bytes - 1)) == 0;
}

int r3_dirty_diff(r3_ctx* ctx, const void* d_pre, const void* d_post, uint64_t bytes,
                  uint32_t page_bytes, uint64_t* d_bitmap, uint64_t* d_dirty_count, void* stream) {
  if (ctx == nullptr) return R3_EINVAL;
  ctx->err.clear();
  if (!page_ok(page_bytes)) return fail(ctx, R3_EINVAL, "page_bytes must be a power of two in 256..1 MiB");
  if (bytes && (d_pre == nullptr || d_post == nullptr || d_bitmap == nullptr))
    return fail(ctx, R3_EINVAL, "pointer is NULL");
  if (!aligned16(d_pre) || !aligned16(d_post)) return fail(ctx, R3_EALIGN, "state base not 16-byte aligned");
  if (reinterpret_cast<uintptr_t>(d_bitmap) & 7u) return fail(ctx, R3_EALIGN, "bitmap not 8-byte aligned");
  DeviceGuard guard(ctx->device);
  hipError_t e = r3::launch_dirty_diff(d_pre, d_post, bytes, page_bytes, d_bitmap, d_dirty_count,
                                       as_stream(stream));
  return e == hipSuccess ? R3_OK : fail_hip(ctx, e, "dirty-diff launch");
}

int r3_record(r3_ctx* ctx, const r3_table* tbl, void* d_live, r3_launch_fn launch, void* user,
              void* d_prologue, void* d_epilogue, uint32_t page_bytes, uint64_t* d_bitmap,
              uint64_t* d_dirty_count, uint64_t* d_pro_cs, uint64_t* d_epi_cs, void* stream) {
  int rc = check_common(ctx, tbl);
  if (rc != R3_OK) return rc;
  if (d_live == nullptr || d_prologue == nullptr || d_epilogue == nullptr || launch == nullptr)
    return fail(ctx, R3_EINVAL, "pointer is NULL");
  if (!aligned16(d_live) || !aligned16(d_prologue) || !aligned16(d_epilogue))
    return fail(ctx, R3_EALIGN, "arena base not 16-byte aligned");
  if (d_bitmap && !page_ok(page_bytes)) return fail(ctx, R3_EINVAL, "page_bytes must be a power of two in 256..1 MiB");
  if (d_dirty_count && !d_bitmap) return fail(ctx, R3_EINVAL, "dirty count needs the bitmap");
  DeviceGuard guard(ctx->device);
  hipStream_t s = as_stream(stream);
  const uint64_t n = tbl->arena_bytes;
  hipError_t e = r3::launch_copy_flat(d_live, d_prologue, n, s);
  if (e != hipSuccess) return fail_hip(ctx, e, "prologue copy");
  const int cand = launch(user, d_live, stream);
  hipError_t le = hipGetLastError();
  if (cand != 0 || le != hipSuccess) {
    (void)hipStreamSynchronize(s);
    return fail(ctx, R3_ECANDIDATE, "the recorded kernel failed to launch");
  }
  e = r3::launch_copy_flat(d_live, d_epilogue, n, s);
  if (e == hipSuccess && d_bitmap)
    e = r3::launch_dirty_diff(d_prologue, d_epilogue, n, page_bytes, d_bitmap, d_dirty_count, s);
  if (e == hipSuccess && d_pro_cs) e = r3::launch_checksum(tbl->dev, d_prologue, d_pro_cs, s);
  if (e == hipSuccess && d_epi_cs) e = r3::launch_checksum(tbl->dev, d_epilogue, d_epi_cs, s);
  if (e != hipSuccess) return fail_hip(ctx, e, "record launch");
  e = hipStreamSynchronize(s);
  return e == hipSuccess ? R3_OK : fail_hip(ctx, e, "record wait");
}

// First half of an evaluation: check the arguments and enqueue every replay on the stream.
// Returns before any of it has run.  R3_OK means the lane is busy and eval_collect must follow,
// also when the candidate's callback failed (that is part of the verdict).
static int eval_enqueue(r3_ctx* ctx, r3::EvalLane& lane, const r3_table* restore_tbl, const void* d_prologue,
                        const r3_table* check_tbl, const void* d_epilogue, void* d_live,
                        r3_launch_fn launch, void* user, uint32_t warmup, uint32_t reps,
                        uint32_t compare_policy, r3_region_result* d_regions, const r3_guard* guard,
                        uint32_t instances, uint64_t instance_stride, bool mark_end, void* stream,
                        bool overlapped = false) {
  int rc = check_common(ctx, restore_tbl);
  if (rc == R3_OK) rc = check_common(ctx, check_tbl);
  if (rc != R3_OK) return rc;
  if (guard) {
    rc = check_common(ctx, guard->guard_tbl);
    if (rc == R3_OK && guard->heal_tbl) rc = check_common(ctx, guard->heal_tbl);
    if (rc != R3_OK) return rc;
    if (guard->d_expected == nullptr || guard->d_scratch == nullptr)
      return fail(ctx, R3_EINVAL, "guard pointer is NULL");
  }
  if (d_prologue == nullptr || d_epilogue == nullptr || d_live == nullptr || d_regions == nullptr)
    return fail(ctx, R3_EINVAL, "pointer is NULL");
  if (!aligned16(d_prologue) || !aligned16(d_epilogue) || !aligned16(d_live))
    return fail(ctx, R3_EALIGN, "arena base not 16-byte aligned");
  if (compare_policy > R3_POLICY_LAST) return fail(ctx, R3_EINVAL, "unknown compare policy");
  const uint64_t total = (uint64_t)warmup + reps;
  if (reps == 0) return fail(ctx, R3_EINVAL, "reps must be at least 1");
  if (total > R3_MAX_REPLAYS) return fail(ctx, R3_ENOSPC, "warmup + reps exceeds R3_MAX_REPLAYS");
  if (lane.busy) return fail(ctx, R3_EINVAL, "an evaluation is still in flight here");

  DeviceGuard device_guard(ctx->device);
  rc = lane_init(ctx, lane);
  if (rc != R3_OK) return rc;
  hipStream_t s = as_stream(stream);
  // Overlapped: the evaluation runs on one of the context's two streams, after what the
  // caller's stream holds now.  Its first restore waits for the previous evaluation's last
  // candidate (a restore never runs beside a timed candidate) and may overlap that
  // evaluation's last validation; its first candidate waits for that validation.
  r3::Pipe& pipe = ctx->pipe;
  const uint32_t side = overlapped ? (uint32_t)(pipe.n & 1) : 0, other = side ^ 1;
  if (overlapped) {
    rc = pipe_init(ctx);
    if (rc != R3_OK) return rc;
    // nothing to wait for when the caller's stream is idle (the usual state inside a search loop)
    hipError_t je = hipStreamQuery(s);
    if (je == hipErrorNotReady) {
      je = hipEventRecord(pipe.join, s);
      if (je == hipSuccess) je = hipStreamWaitEvent(pipe.s[side], pipe.join, 0);
    }
    s = pipe.s[side];
    if (je == hipSuccess && pipe.cand_valid[other]) je = hipStreamWaitEvent(s, pipe.cand_end[other], 0);
    if (je != hipSuccess) return fail_hip(ctx, je, "overlapped pipeline ordering");
    stream = reinterpret_cast<void*>(s);
    pipe.cand_valid[side] = false;
  }
  // Events of replay r: [4r] before the restore and [4r+3] after the validation (only when
  // profiling), [4r+1] / [4r+2] around the candidate.
  const bool prof = ctx->profile_period != 0 && (ctx->evals++ % ctx->profile_period) == 0;
  while (lane.events.size() < 4 * total) {
    hipEvent_t ev;
    hipError_t e = hipEventCreate(&ev);
    if (e != hipSuccess) return fail_hip(ctx, e, "event create");
    lane.events.push_back(ev);
  }

  lane.prof = prof;
  lane.has_launch = launch != nullptr;
  lane.has_guard = guard != nullptr;
  lane.guard = guard ? *guard : r3_guard{};
  lane.warmup = warmup;
  lane.total = (uint32_t)total;
  lane.done = 0;
  lane.n_validated = 0;
  lane.cand = 0;
  lane.validated.assign(total, 0);
  lane.guarded.assign(total, 0);
  lane.last_flag = nullptr;
  lane.last_want = 0;
  lane.end_recorded = false;
  lane.stream = s;
  lane.d_prologue = d_prologue;
  lane.d_live = d_live;

  int cand = 0;
  hipError_t e = hipSuccess;
  for (uint32_t rep = 0; rep < total; ++rep) {
    lane.last_flag = nullptr;
    if (prof) {
      e = hipEventRecord(lane.events[4 * rep], s);
      if (e != hipSuccess) break;
    }
    e = r3::launch_restore(restore_tbl->dev, restore_tbl->class_count, d_prologue, d_live, s);
    if (e != hipSuccess) break;
    if (overlapped && rep == 0 && launch && pipe.val_valid[other]) {
      // The candidate runs alone: it waits for what the other stream holds now, which ends with the
      // previous evaluation's last validation (recorded only here, where it is needed).
      e = hipEventRecord(pipe.val_end[other], pipe.s[other]);
      if (e == hipSuccess) e = hipStreamWaitEvent(s, pipe.val_end[other], 0);
      if (e != hipSuccess) break;
    }
    if (launch || prof) {
      e = hipEventRecord(lane.events[4 * rep + 1], s);
      if (e != hipSuccess) break;
    }
    if (launch) {
      for (uint32_t inst = 0; inst < instances && cand == 0; ++inst) {
        cand = launch(user, static_cast<uint8_t*>(d_live) + (uint64_t)inst * instance_stride, stream);
        hipError_t le = hipGetLastError();
        if (cand == 0 && le != hipSuccess) cand = -(int)le;
      }
      if (cand != 0) break;
    }
    if (launch || prof) {
      e = hipEventRecord(lane.events[4 * rep + 2], s);
      if (e != hipSuccess) break;
    }
    if (overlapped && launch && rep == total - 1) {  // the next evaluation's restore may start here
      e = hipEventRecord(pipe.cand_end[side], s);
      if (e != hipSuccess) break;
      pipe.cand_valid[side] = true;
    }
    const bool validate = compare_policy == R3_POLICY_EVERY ||
                          (compare_policy == R3_POLICY_FIRST && rep == 0) ||
                          (compare_policy == R3_POLICY_LAST && rep == total - 1);
    if (validate) {
      e = r3::launch_compare(check_tbl->dev, d_live, d_epilogue, d_regions, nullptr,
                             &lane.pinned_dev[lane.n_validated], ++ctx->seq, nullptr, s);
      lane.last_flag = &lane.pinned[lane.n_validated].seq;
      lane.last_want = ctx->seq;
      if (e != hipSuccess) break;
      ++lane.n_validated;
      lane.validated[rep] = 1;
      if (prof) {
        e = hipEventRecord(lane.events[4 * rep + 3], s);
        if (e != hipSuccess) break;
      }
    }
    if (guard && ((guard->every != 0 && (rep + 1) % guard->every == 0) || rep == total - 1)) {
      e = r3::launch_checksum(guard->guard_tbl->dev, d_live, guard->d_scratch, s);
      if (e == hipSuccess)
        e = r3::launch_guard_compare(guard->d_scratch, guard->d_expected, guard->guard_tbl->dev.n_regions,
                                     &lane.guard_pinned_dev[rep], ++ctx->seq, s);
      if (e != hipSuccess) break;
      lane.guarded[rep] = 1;
      lane.last_flag = &lane.guard_pinned[rep].seq;
      lane.last_want = ctx->seq;
    }
    ++lane.done;
  }
  if (overlapped) {
    // what the next overlapped evaluation has to wait for
    pipe.val_valid[side] = true;  // this stream now holds work a later candidate must wait for
    if (e != hipSuccess || cand != 0 || !launch) pipe.cand_valid[side] = false;
    ++pipe.n;
  }
  lane.cand = cand;
  lane.status = e;
  if (e != hipSuccess || cand != 0) lane.last_flag = nullptr;
  // A submission whose end posts no number is marked with an event, so that waiting for it
  // does not have to wait for whatever was enqueued on the stream afterwards.
  if (mark_end && lane.last_flag == nullptr && e == hipSuccess)
    lane.end_recorded = hipEventRecord(lane.end_event, s) == hipSuccess;
  lane.busy = true;
  return R3_OK;
}

// Second half: wait for the verdict of the evaluation enqueued on this lane and report it.
static int eval_collect(r3_ctx* ctx, r3::EvalLane& lane, r3_eval_result* host_out,
                        r3_guard_result* host_guard_out) {
  DeviceGuard device_guard(ctx->device);
  hipStream_t s = lane.stream;
  const uint32_t total = lane.total, done = lane.done;
  hipError_t e = lane.status;
  const int cand = lane.cand;
  lane.busy = false;

  std::memset(host_out, 0, sizeof(*host_out));
  host_out->first_index = R3_NO_INDEX;
  host_out->first_region = R3_NO_REGION;
  if (host_guard_out) {
    std::memset(host_guard_out, 0, sizeof(*host_guard_out));
    host_guard_out->first_region = R3_NO_REGION;
  }

  // When the last thing enqueued is a validation, its sequence number arriving in pinned memory
  // says that everything before it on the stream has run; polling for it (bounded) avoids the
  // wake-up latency of a stream wait.  Anything else, and any doubt, takes the event or the
  // stream wait.
  bool arrived = false;
  if (lane.last_flag != nullptr) {
    for (uint32_t spin = 0; spin < (1u << 22) && !arrived; ++spin)
      arrived = __atomic_load_n(lane.last_flag, __ATOMIC_ACQUIRE) == lane.last_want;
    if (arrived && lane.prof && lane.validated[total - 1])
      arrived = hipEventSynchronize(lane.events[4 * (total - 1) + 3]) == hipSuccess;
  } else if (lane.end_recorded) {
    arrived = hipEventSynchronize(lane.end_event) == hipSuccess;
  }
  if (!arrived) {
    hipError_t we = hipStreamSynchronize(s);
    if (e == hipSuccess) e = we;
  }
  if (e != hipSuccess) return fail_hip(ctx, e, "replay loop");

  host_out->candidate_status = cand;
  for (uint32_t i = 0; i < lane.n_validated; ++i)
    host_out->total_mismatch = std::max(host_out->total_mismatch, lane.pinned[i].summary.total_mismatch);
  if (lane.n_validated) {
    const r3_summary& last = lane.pinned[lane.n_validated - 1].summary;
    host_out->first_index = last.first_index;
    host_out->first_region = last.first_region;
    host_out->max_abs_err = last.max_abs_err;
    host_out->max_rel_err = last.max_rel_err;
  }
  host_out->pass = (cand == 0 && host_out->total_mismatch == 0) ? 1u : 0u;
  if (lane.has_guard) {
    r3_guard_result g{};
    g.first_region = R3_NO_REGION;
    for (uint32_t rep = 0; rep < done; ++rep) {
      if (!lane.guarded[rep]) continue;
      const r3::GuardSlot& gs = lane.guard_pinned[rep];
      ++g.checks;
      if (gs.changed) {
        if (g.failed_checks == 0) g.first_region = (uint32_t)gs.first_region;
        ++g.failed_checks;
        g.changed_regions = std::max(g.changed_regions, (uint32_t)gs.changed);
      }
    }
    if (g.failed_checks) {
      host_out->pass = 0;
      if (lane.guard.heal_tbl) {
        hipError_t he = r3::launch_restore(lane.guard.heal_tbl->dev, lane.guard.heal_tbl->class_count,
                                           lane.d_prologue, lane.d_live, s);
        if (he == hipSuccess) he = hipStreamSynchronize(s);
        if (he != hipSuccess) return fail_hip(ctx, he, "heal restore");
        g.healed = 1;
      }
    }
    if (host_guard_out) *host_guard_out = g;
  }

  // Candidate times of the replays after the warm-up that ran to the end.
  ctx->last_times.clear();
  if (lane.has_launch) {
    // The verdict may have arrived by polling pinned memory, which says nothing about event
    // state: wait for the last candidate's end event (it has passed; this is cheap) before
    // reading times, and refuse to report a runtime that is not there (a search that keeps the
    // fastest correct candidate must never see a zero).
    if (done > 0) (void)hipEventSynchronize(lane.events[4 * (done - 1) + 2]);
    std::vector<float> ms;
    for (uint32_t rep = lane.warmup; rep < done; ++rep) {
      float t = 0.f;
      const hipError_t te = hipEventElapsedTime(&t, lane.events[4 * rep + 1], lane.events[4 * rep + 2]);
      if (te != hipSuccess) return fail_hip(ctx, te, "candidate time of a finished replay");
      ms.push_back(t);
    }
    ctx->last_times = ms;
    if (!ms.empty()) {
      std::sort(ms.begin(), ms.end());
      host_out->ms_min = ms.front();
      host_out->ms_max = ms.back();
      host_out->ms_median = ms.size() % 2 ? ms[ms.size() / 2]
                                          : 0.5f * (ms[ms.size() / 2 - 1] + ms[ms.size() / 2]);
    }
  }
  if (lane.prof) {
    for (uint32_t rep = 0; rep < done; ++rep) {
      float t = 0.f;
      if (hipEventElapsedTime(&t, lane.events[4 * rep], lane.events[4 * rep + 1]) == hipSuccess) {
        ctx->profile.restore_ms += t;
        ctx->profile.restore_launches += 1;
      }
      if (lane.has_launch &&
          hipEventElapsedTime(&t, lane.events[4 * rep + 1], lane.events[4 * rep + 2]) == hipSuccess) {
        ctx->profile.candidate_ms += t;
        ctx->profile.candidate_launches += 1;
      }
      if (lane.validated[rep] &&
          hipEventElapsedTime(&t, lane.events[4 * rep + 2], lane.events[4 * rep + 3]) == hipSuccess) {
        ctx->profile.validate_ms += t;
        ctx->profile.validate_launches += 1;
      }
    }
  }
  if (cand != 0) return fail(ctx, R3_ECANDIDATE, "the candidate failed to launch");
  return R3_OK;
}

static int eval_impl(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologue,
                     const r3_table* check_tbl, const void* d_epilogue, void* d_live,
                     r3_launch_fn launch, void* user, uint32_t warmup, uint32_t reps,
                     uint32_t compare_policy, r3_region_result* d_regions, r3_eval_result* host_out,
                     const r3_guard* guard, r3_guard_result* host_guard_out, uint32_t instances,
                     uint64_t instance_stride, void* stream) {
  if (ctx == nullptr) return R3_EINVAL;
  if (host_out == nullptr) return fail(ctx, R3_EINVAL, "pointer is NULL");
  int rc = eval_enqueue(ctx, ctx->lanes[0], restore_tbl, d_prologue, check_tbl, d_epilogue, d_live, launch,
                        user, warmup, reps, compare_policy, d_regions, guard, instances, instance_stride,
                        false, stream);
  if (rc != R3_OK) return rc;
  return eval_collect(ctx, ctx->lanes[0], host_out, host_guard_out);
}

static int submit_impl(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologue,
                       const r3_table* check_tbl, const void* d_epilogue, void* d_live, r3_launch_fn launch,
                       void* user, uint32_t warmup, uint32_t reps, uint32_t compare_policy,
                       r3_region_result* d_regions, const r3_guard* guard, uint32_t* ticket_out, void* stream,
                       bool overlapped = false) {
  if (ctx == nullptr) return R3_EINVAL;
  if (ticket_out == nullptr) return fail(ctx, R3_EINVAL, "pointer is NULL");
  *ticket_out = 0;
  uint32_t lane = 0;
  for (uint32_t i = 1; i <= R3_MAX_INFLIGHT && lane == 0; ++i)
    if (!ctx->lanes[i].busy) lane = i;
  if (lane == 0) return fail(ctx, R3_ENOSPC, "R3_MAX_INFLIGHT evaluations are in flight already");
  int rc = eval_enqueue(ctx, ctx->lanes[lane], restore_tbl, d_prologue, check_tbl, d_epilogue, d_live, launch,
                        user, warmup, reps, compare_policy, d_regions, guard, 1, 0, true, stream, overlapped);
  if (rc == R3_OK) *ticket_out = lane;
  return rc;
}

int r3_eval_submit(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologue,
                   const r3_table* check_tbl, const void* d_epilogue, void* d_live, r3_launch_fn launch,
                   void* user, uint32_t warmup, uint32_t reps, uint32_t compare_policy,
                   r3_region_result* d_regions, uint32_t* ticket_out, void* stream) {
  return submit_impl(ctx, restore_tbl, d_prologue, check_tbl, d_epilogue, d_live, launch, user, warmup, reps,
                     compare_policy, d_regions, nullptr, ticket_out, stream);
}

int r3_eval_submit_overlapped(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologue,
                              const r3_table* check_tbl, const void* d_epilogue, void* d_live,
                              r3_launch_fn launch, void* user, uint32_t warmup, uint32_t reps,
                              uint32_t compare_policy, r3_region_result* d_regions, uint32_t* ticket_out,
                              void* stream) {
  return submit_impl(ctx, restore_tbl, d_prologue, check_tbl, d_epilogue, d_live, launch, user, warmup, reps,
                     compare_policy, d_regions, nullptr, ticket_out, stream, true);
}

int r3_eval_submit_guarded(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologue,
                           const r3_table* check_tbl, const void* d_epilogue, void* d_live,
                           r3_launch_fn launch, void* user, uint32_t warmup, uint32_t reps,
                           uint32_t compare_policy, r3_region_result* d_regions, const r3_guard* guard,
                           uint32_t* ticket_out, void* stream) {
  return submit_impl(ctx, restore_tbl, d_prologue, check_tbl, d_epilogue, d_live, launch, user, warmup, reps,
                     compare_policy, d_regions, guard, ticket_out, stream);
}

int r3_eval_wait(r3_ctx* ctx, uint32_t ticket, r3_eval_result* host_out, r3_guard_result* host_guard_out) {
  if (ctx == nullptr) return R3_EINVAL;
  ctx->err.clear();
  if (host_out == nullptr) return fail(ctx, R3_EINVAL, "pointer is NULL");
  if (ticket == 0 || ticket > R3_MAX_INFLIGHT || !ctx->lanes[ticket].busy)
    return fail(ctx, R3_EINVAL, "no evaluation in flight under this ticket");
  return eval_collect(ctx, ctx->lanes[ticket], host_out, host_guard_out);
}

int r3_eval_try_wait(r3_ctx* ctx, uint32_t ticket, uint32_t timeout_us, r3_eval_result* host_out,
                     r3_guard_result* host_guard_out) {
  if (ctx == nullptr) return R3_EINVAL;
  ctx->err.clear();
  if (host_out == nullptr) return fail(ctx, R3_EINVAL, "pointer is NULL");
  if (ticket == 0 || ticket > R3_MAX_INFLIGHT || !ctx->lanes[ticket].busy)
    return fail(ctx, R3_EINVAL, "no evaluation in flight under this ticket");
  r3::EvalLane& lane = ctx->lanes[ticket];
  DeviceGuard device_guard(ctx->device);
  const auto deadline = std::chrono::steady_clock::now() + std::chrono::microseconds(timeout_us);
  for (;;) {
    bool done;
    if (lane.last_flag != nullptr)
      done = __atomic_load_n(lane.last_flag, __ATOMIC_ACQUIRE) == lane.last_want;
    else if (lane.end_recorded)
      done = hipEventQuery(lane.end_event) != hipErrorNotReady;
    else
      done = hipStreamQuery(lane.stream) != hipErrorNotReady;
    if (done) return eval_collect(ctx, lane, host_out, host_guard_out);
    if (std::chrono::steady_clock::now() >= deadline) break;
  }
  return fail(ctx, R3_EBUSY, "the evaluation has not finished yet");
}

int r3_eval_candidate(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologue,
                      const r3_table* check_tbl, const void* d_epilogue, void* d_live,
                      r3_launch_fn launch, void* user, uint32_t warmup, uint32_t reps,
                      uint32_t compare_policy, r3_region_result* d_regions,
                      r3_eval_result* host_out, void* stream) {
  return eval_impl(ctx, restore_tbl, d_prologue, check_tbl, d_epilogue, d_live, launch, user, warmup,
                   reps, compare_policy, d_regions, host_out, nullptr, nullptr, 1, 0, stream);
}

int r3_eval_candidate_guarded(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologue,
                              const r3_table* check_tbl, const void* d_epilogue, void* d_live,
                              r3_launch_fn launch, void* user, uint32_t warmup, uint32_t reps,
                              uint32_t compare_policy, r3_region_result* d_regions,
                              r3_eval_result* host_out, const r3_guard* guard,
                              r3_guard_result* host_guard_out, void* stream) {
  return eval_impl(ctx, restore_tbl, d_prologue, check_tbl, d_epilogue, d_live, launch, user, warmup,
                   reps, compare_policy, d_regions, host_out, guard, host_guard_out, 1, 0, stream);
}

int r3_eval_candidate_instances(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologues,
                                const r3_table* check_tbl, const void* d_epilogues, void* d_live,
                                r3_launch_fn launch, void* user, uint32_t instances,
                                uint64_t instance_stride, uint32_t warmup, uint32_t reps,
                                uint32_t compare_policy, r3_region_result* d_regions,
                                r3_eval_result* host_out, uint8_t* host_instance_pass, void* stream) {
  if (ctx == nullptr) return R3_EINVAL;
  if (instances == 0 || check_tbl == nullptr || check_tbl->dev.n_regions % instances != 0)
    return fail(ctx, R3_EINVAL, "check table is not a whole number of instances");
  if (instance_stride & 15u) return fail(ctx, R3_EALIGN, "instance stride not a multiple of 16");
  if (instances > 1 && (check_tbl->arena_bytes < (uint64_t)(instances - 1) * instance_stride ||
                        (restore_tbl && restore_tbl->arena_bytes < (uint64_t)(instances - 1) * instance_stride)))
    return fail(ctx, R3_ERANGE, "instances reach past the super arena");
  int rc = eval_impl(ctx, restore_tbl, d_prologues, check_tbl, d_epilogues, d_live, launch, user, warmup,
                     reps, compare_policy, d_regions, host_out, nullptr, nullptr, instances,
                     instance_stride, stream);
  if ((rc == R3_OK || rc == R3_ECANDIDATE) && host_instance_pass) {
    const uint32_t n = check_tbl->dev.n_regions, per = n / instances;
    std::vector<r3_region_result> res(n);
    DeviceGuard device_guard(ctx->device);
    hipError_t e = hipMemcpyAsync(res.data(), d_regions, (size_t)n * sizeof(r3_region_result),
                                  hipMemcpyDeviceToHost, as_stream(stream));
    if (e == hipSuccess) e = hipStreamSynchronize(as_stream(stream));
    if (e != hipSuccess) return fail_hip(ctx, e, "instance verdicts");
    for (uint32_t i = 0; i < instances; ++i) {
      uint8_t ok = host_out->candidate_status == 0 ? 1 : 0;
      for (uint32_t r = 0; r < per; ++r)
        if (res[(size_t)i * per + r].mismatch_count != 0) ok = 0;
      host_instance_pass[i] = ok;
    }
  }
  return rc;
}

size_t r3_replay_workspace_bytes(void) { return 256; }

int r3_replay_destroy(r3_replay* rp) {
  if (rp == nullptr) return R3_EINVAL;
  DeviceGuard device_guard(rp->ctx->device);
  if (rp->exec) (void)hipGraphExecDestroy(rp->exec);
  if (rp->graph) (void)hipGraphDestroy(rp->graph);
  if (rp->capture_stream) (void)hipStreamDestroy(rp->capture_stream);
  if (rp->slots) (void)hipHostFree(rp->slots);
  if (rp->stamps) (void)hipHostFree(rp->stamps);
  delete rp;
  return R3_OK;
}

int r3_replay_create(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologue,
                     const r3_table* check_tbl, const void* d_epilogue, void* d_live,
                     r3_launch_fn launch, void* user, r3_region_result* d_regions, void* d_ws,
                     uint32_t replays, r3_replay** out) {
  int rc = check_common(ctx, restore_tbl);
  if (rc == R3_OK) rc = check_common(ctx, check_tbl);
  if (rc != R3_OK) return rc;
  if (out == nullptr || d_prologue == nullptr || d_epilogue == nullptr || d_live == nullptr ||
      d_regions == nullptr || d_ws == nullptr)
    return fail(ctx, R3_EINVAL, "pointer is NULL");
  *out = nullptr;
  if (!aligned16(d_prologue) || !aligned16(d_epilogue) || !aligned16(d_live) || !aligned16(d_ws))
    return fail(ctx, R3_EALIGN, "pointer not 16-byte aligned");
  if (replays == 0 || replays > R3_MAX_REPLAYS) return fail(ctx, R3_EINVAL, "replays must be 1..R3_MAX_REPLAYS");
  DeviceGuard device_guard(ctx->device);
  r3_replay* rp = new (std::nothrow) r3_replay();
  if (rp == nullptr) return fail(ctx, R3_ENOSPC, "out of host memory");
  rp->ctx = ctx;
  rp->check_tbl = check_tbl;
  rp->d_counter = static_cast<uint32_t*>(d_ws);
  rp->has_candidate = launch != nullptr;
  int khz = 0;
  hipError_t e = hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, ctx->device);
  if (e == hipSuccess && khz <= 0) e = hipErrorInvalidValue;
  rp->ticks_per_ms = (double)khz;
  if (e == hipSuccess)
    e = hipHostMalloc(reinterpret_cast<void**>(&rp->slots), R3_MAX_REPLAYS * sizeof(r3::HostSlot),
                      hipHostMallocMapped);
  if (e == hipSuccess) e = hipHostGetDevicePointer(reinterpret_cast<void**>(&rp->slots_dev), rp->slots, 0);
  if (e == hipSuccess)
    e = hipHostMalloc(reinterpret_cast<void**>(&rp->stamps), R3_MAX_REPLAYS * 2 * sizeof(uint64_t),
                      hipHostMallocMapped);
  if (e == hipSuccess) e = hipHostGetDevicePointer(reinterpret_cast<void**>(&rp->stamps_dev), rp->stamps, 0);
  if (e == hipSuccess) {
    std::memset(rp->slots, 0, R3_MAX_REPLAYS * sizeof(r3::HostSlot));
    e = hipStreamCreateWithFlags(&rp->capture_stream, hipStreamNonBlocking);
  }
  if (e != hipSuccess) {
    (void)r3_replay_destroy(rp);
    return fail_hip(ctx, e, "replay set-up");
  }
  // Record the replay: nothing below executes now, the launches become graph nodes.
  hipStream_t cs = rp->capture_stream;
  e = hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal);
  int cand = 0;
  if (e == hipSuccess) {
    hipError_t ce = hipSuccess;
    for (uint32_t r = 0; r < replays && ce == hipSuccess && cand == 0; ++r) {
      ce = r3::launch_restore(restore_tbl->dev, restore_tbl->class_count, d_prologue, d_live, cs);
      // stamp 0 also advances the replay counter, so it is always there
      if (ce == hipSuccess) ce = r3::launch_stamp(rp->d_counter, rp->stamps_dev, 0, cs);
      if (ce == hipSuccess && launch) {
        cand = launch(user, d_live, cs);
        hipError_t le = hipGetLastError();
        if (cand == 0 && le != hipSuccess) cand = -(int)le;
        if (cand == 0) ce = r3::launch_stamp(rp->d_counter, rp->stamps_dev, 1, cs);
      }
      if (ce == hipSuccess && cand == 0)
        ce = r3::launch_compare(check_tbl->dev, d_live, d_epilogue, d_regions, nullptr, rp->slots_dev, 1,
                                rp->d_counter, cs);
    }
    hipError_t ee = hipStreamEndCapture(cs, &rp->graph);
    e = ce != hipSuccess ? ce : ee;
  }
  rp->replays = replays;
  if (e == hipSuccess && cand == 0) e = hipGraphInstantiate(&rp->exec, rp->graph, nullptr, nullptr, 0);
  if (cand != 0) {
    (void)r3_replay_destroy(rp);
    return fail(ctx, R3_ECANDIDATE, "the candidate failed to launch during capture");
  }
  if (e != hipSuccess) {
    (void)r3_replay_destroy(rp);
    return fail_hip(ctx, e, "replay capture");
  }
  *out = rp;
  return R3_OK;
}

int r3_replay_run(r3_replay* rp, uint32_t warmup, uint32_t reps, r3_eval_result* host_out, void* stream) {
  if (rp == nullptr || host_out == nullptr) return R3_EINVAL;
  r3_ctx* ctx = rp->ctx;
  ctx->err.clear();
  const uint64_t total = (uint64_t)warmup + reps;
  if (reps == 0) return fail(ctx, R3_EINVAL, "reps must be at least 1");
  if (total != rp->replays) return fail(ctx, R3_EINVAL, "warmup + reps differs from the captured replay count");
  DeviceGuard device_guard(ctx->device);
  hipStream_t s = as_stream(stream);
  std::memset(host_out, 0, sizeof(*host_out));
  host_out->first_index = R3_NO_INDEX;
  host_out->first_region = R3_NO_REGION;
  for (uint64_t i = 0; i < total; ++i) rp->slots[i].seq = 0;
  hipError_t e = r3::launch_set_counter(rp->d_counter, 0, s);
  if (e == hipSuccess) e = hipGraphLaunch(rp->exec, s);
  bool arrived = false;
  if (e == hipSuccess) {
    const uint64_t want = total;  // replay k posts sequence number k + 1
    for (uint32_t spin = 0; spin < (1u << 22) && !arrived; ++spin)
      arrived = __atomic_load_n(&rp->slots[total - 1].seq, __ATOMIC_ACQUIRE) == want;
  }
  if (!arrived) {
    hipError_t we = hipStreamSynchronize(s);
    if (e == hipSuccess) e = we;
  }
  if (e != hipSuccess) return fail_hip(ctx, e, "captured replay");
  for (uint64_t i = 0; i < total; ++i)
    host_out->total_mismatch = std::max(host_out->total_mismatch, rp->slots[i].summary.total_mismatch);
  const r3_summary& last = rp->slots[total - 1].summary;
  host_out->first_index = last.first_index;
  host_out->first_region = last.first_region;
  host_out->max_abs_err = last.max_abs_err;
  host_out->max_rel_err = last.max_rel_err;
  host_out->pass = host_out->total_mismatch == 0 ? 1u : 0u;
  ctx->last_times.clear();
  if (rp->has_candidate) {
    std::vector<float> ms;
    for (uint64_t i = warmup; i < total; ++i)
      ms.push_back((float)((double)(rp->stamps[2 * i + 1] - rp->stamps[2 * i]) / rp->ticks_per_ms));
    ctx->last_times = ms;
    std::sort(ms.begin(), ms.end());
    host_out->ms_min = ms.front();
    host_out->ms_max = ms.back();
    host_out->ms_median = ms.size() % 2 ? ms[ms.size() / 2] : 0.5f * (ms[ms.size() / 2 - 1] + ms[ms.size() / 2]);
  }
  return R3_OK;
}

int r3_ctx_last_times(const r3_ctx* ctx, float* out, uint32_t cap, uint32_t* n_out) {
  if (ctx == nullptr || n_out == nullptr || (cap && out == nullptr)) return R3_EINVAL;
  *n_out = (uint32_t)ctx->last_times.size();
  for (uint32_t i = 0; i < cap && i < ctx->last_times.size(); ++i) out[i] = ctx->last_times[i];
  return R3_OK;
}

}  // extern "C"
