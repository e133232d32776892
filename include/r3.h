/*
 * r3.h -- C ABI of the replay-evaluation library (libr3.so), gfx950 / HIP.
 *
 * The library implements the device-side inner loop of replay-based kernel
 * evaluation as the paper's Section V describes it: a recorded pre-execution
 * device state (prologue snapshot) is restored, a candidate kernel runs on it,
 * and the resulting state is checked against the recorded post-execution state
 * (epilogue snapshot), bitwise by default or under per-variable tolerances
 * (Section V-B "Replay, Transformation, and Auto-Tuning", Section V-C
 * "Correctness Checking").  Snapshots stay resident on the device and all
 * verdicts are reduced on the device, which is the design rule of the
 * persistent replay server (Section V-D).
 *
 * Conventions that hold for every entry point
 *   - Return value: R3_OK (0) or a negative r3_status.  Nothing throws or
 *     aborts across this boundary.  r3_last_error() gives a message for the
 *     last failure on a context.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP
 *     device allocations on the context's GPU.  The library never allocates or
 *     frees device memory: snapshots, live arena, result arrays and the table
 *     workspace are owned by the caller for as long as the objects that refer
 *     to them are in use.
 *   - Device base pointers of arenas must be 16-byte aligned.
 *   - All GPU work is enqueued on the caller's stream (a hipStream_t passed as
 *     void*, NULL = the default stream).  Calls return without waiting unless
 *     stated otherwise.
 *   - One r3_ctx, and one r3_table, may be used by one host thread and one
 *     stream at a time: a table's workspace holds the partial results of the
 *     call in flight.
 *   - Arguments that the host can check (NULL pointers, table contents,
 *     workspace size) are rejected before any GPU work is enqueued.
 *
 * Memory model ("arena"): a recorded device state is a flat byte range
 * [0, arena_bytes).  The prologue snapshot, the epilogue snapshot and the live
 * memory the candidate runs on share this layout, so one offset addresses the
 * same variable in all of them.  A region table names the spans of the arena
 * that an operation touches.
 */
#ifndef R3_H
#define R3_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  R3_OK = 0,
  R3_EINVAL = -1,     /* NULL pointer, n == 0, unknown dtype/mode/policy, bad tolerance   */
  R3_EALIGN = -2,     /* offset/bytes not a multiple of the element size; base not 16 B   */
  R3_ERANGE = -3,     /* region reaches past arena_bytes                                   */
  R3_EOVERLAP = -4,   /* two non-empty regions share a byte                                */
  R3_ENOSPC = -5,     /* workspace too small / too many replays for the workspace          */
  R3_EHIP = -6,       /* a HIP runtime call failed                                         */
  R3_ECANDIDATE = -7, /* the candidate's launch callback or its kernel launch failed       */
  R3_EBUSY = -8       /* r3_eval_try_wait: the evaluation has not finished in the time given */
} r3_status;

/* Element types of a region: 1, 4, 8, 4, 2, 2 bytes (R3_F16 = IEEE binary16). */
typedef enum { R3_U8 = 0, R3_F32 = 1, R3_F64 = 2, R3_I32 = 3, R3_BF16 = 4, R3_F16 = 5 } r3_dtype;

/* Section V-C: bitwise equality is the default criterion; tolerances apply only
 * to regions the user marks (the role of the paper's `annotate`). */
typedef enum { R3_CMP_BITWISE = 0, R3_CMP_TOL = 1 } r3_cmp_mode;

/* When r3_eval_candidate validates: after every replay, only the first, only the last. */
typedef enum { R3_POLICY_EVERY = 0, R3_POLICY_FIRST = 1, R3_POLICY_LAST = 2 } r3_compare_policy;

#define R3_NO_INDEX UINT64_MAX   /* first_mismatch / first_index when nothing mismatched */
#define R3_NO_REGION UINT32_MAX  /* first_region when nothing mismatched                 */
#define R3_MAX_REPLAYS 1024u     /* warmup + reps accepted by r3_eval_candidate          */
#define R3_MAX_INFLIGHT 8u       /* evaluations submitted and not yet waited for         */

/* One span of the arena (40 bytes, host memory, caller-owned).
 * offset and bytes are multiples of the element size; bytes may be 0.
 * rtol and atol are finite and >= 0 (checked in both modes, used in R3_CMP_TOL). */
typedef struct {
  uint64_t offset;
  uint64_t bytes;
  uint32_t dtype; /* r3_dtype    */
  uint32_t mode;  /* r3_cmp_mode */
  double rtol;
  double atol;
} r3_region;

/* Verdict for one region (40 bytes, device memory, written by r3_compare).
 * Element i of the region is "c" in live memory and "g" in the golden snapshot.
 *   - equal bit patterns: match, error 0 (also equal NaNs and infinities);
 *   - different bits and, for F32/F64/BF16, c or g NaN or infinite: mismatch,
 *     both errors +Inf;
 *   - else, in binary64 with one rounding per operation and no fused
 *     multiply-add:  d = |C - G|,  r = (G == 0) ? 0 : d / |G|;
 *     BITWISE: mismatch;   TOL: mismatch iff d > atol + rtol*|G|.
 * max_abs_err / max_rel_err are the maxima of d / r over ALL elements.
 * first_mismatch is the smallest mismatching element index (region-relative),
 * R3_NO_INDEX if none.  checksum is the region checksum of the LIVE bytes. */
typedef struct {
  uint64_t mismatch_count;
  uint64_t first_mismatch;
  double max_abs_err;
  double max_rel_err;
  uint64_t checksum;
} r3_region_result;

/* Verdict over a whole table (40 bytes, device memory, written by r3_compare). */
typedef struct {
  uint64_t total_mismatch; /* sum of mismatch_count                               */
  uint64_t first_index;    /* first_mismatch of region first_region, R3_NO_INDEX  */
  uint32_t first_region;   /* first region in table order with a mismatch         */
  uint32_t pass;           /* total_mismatch == 0                                 */
  double max_abs_err;      /* max over regions                                    */
  double max_rel_err;
} r3_summary;

/* What one candidate evaluation returns to the host (56 bytes, host memory).
 * Section V-B: a replay experiment returns the measured runtime if correct. */
typedef struct {
  uint64_t total_mismatch; /* max over the validated replays                       */
  uint64_t first_index;    /* of the last validated replay                         */
  uint32_t first_region;
  uint32_t pass;           /* every validated replay clean and the candidate ran   */
  double max_abs_err;      /* of the last validated replay                         */
  double max_rel_err;
  float ms_min;            /* candidate time over the timed replays (HIP events)   */
  float ms_median;
  float ms_max;
  int32_t candidate_status; /* value the launch callback returned, 0 = launched     */
} r3_eval_result;

/* Accumulated stage times of r3_eval_candidate while profiling is on (host memory).
 * Each stage is bracketed by HIP events on the caller's stream, so a stage time is the
 * device time of its kernels plus their dispatch gaps. */
typedef struct {
  double restore_ms;   /* batched restore launches                         */
  double candidate_ms; /* the launch callback's kernels                    */
  double validate_ms;  /* fused compare+checksum launches and their finalize */
  uint64_t restore_launches;
  uint64_t candidate_launches;
  uint64_t validate_launches;
} r3_profile;

/* Whole-state guard for replays that restore only a write-set (host memory).  The regions of
 * guard_tbl are the part of the state the recorded kernel does NOT write; their checksums
 * must stay what they were at record time, otherwise the candidate wrote outside its
 * write-set and later replays would start from a wrong state. */
typedef struct {
  const struct r3_table* guard_tbl; /* table over the never-written part of the arena          */
  const uint64_t* d_expected;       /* device: recorded checksums of its regions (n values)    */
  uint64_t* d_scratch;              /* device: n values, overwritten by every check            */
  const struct r3_table* heal_tbl;  /* optional: restored from the prologue if a check fails   */
  uint32_t every;                   /* check after every `every`-th replay and after the last;
                                       0 = only after the last                                 */
  uint32_t reserved;
} r3_guard;

typedef struct {
  uint32_t checks;          /* guard checks that ran                                        */
  uint32_t failed_checks;   /* checks in which at least one region had changed              */
  uint32_t changed_regions; /* most regions changed in any one check                        */
  uint32_t first_region;    /* first changed region of the first failing check, R3_NO_REGION */
  uint32_t healed;          /* 1 if heal_tbl was restored after a failure                   */
  uint32_t reserved;
} r3_guard_result;

/* The candidate: enqueue the kernel(s) under test on `stream`, operating in
 * place on the arena at d_live.  Must not synchronise.  Non-zero = failure. */
typedef int (*r3_launch_fn)(void* user, void* d_live, void* stream);

typedef struct r3_ctx r3_ctx;
typedef struct r3_table r3_table;

/* ---- library / context ------------------------------------------------- */

/* ABI version, bumped when a struct or signature changes. */
uint32_t r3_version(void);

/* Static text for a status code; never NULL. */
const char* r3_strerror(int status);

/* Create a context bound to GPU `device`.  Holds only host-side state (events,
 * a small pinned staging buffer).  R3_EHIP if the device cannot be used. */
int r3_ctx_create(r3_ctx** out, int device);
int r3_ctx_destroy(r3_ctx* ctx);

/* Stage profiling of r3_eval_candidate: period 0 = off (default), n > 0 = bracket the stages
 * of every n-th evaluation with events (two extra events per replay of that evaluation).
 * r3_ctx_profile_read copies the totals since the last reset into *out (host) and clears
 * them when reset != 0. */
int r3_ctx_profile(r3_ctx* ctx, int period);
int r3_ctx_profile_read(r3_ctx* ctx, r3_profile* out, int reset);

/* Message of the last failing call on ctx ("" if none); valid until the next call. */
const char* r3_last_error(const r3_ctx* ctx);

/* ---- region tables ----------------------------------------------------- */

/* Host-only check of a table, usable without a GPU.  Regions are examined in
 * table order and the first violation decides: per region R3_EINVAL (dtype,
 * mode, tolerance), then R3_EALIGN, then R3_ERANGE; once every region passes,
 * R3_EOVERLAP.  host_tbl == NULL or n == 0: R3_EINVAL. */
int r3_table_validate(const r3_region* host_tbl, uint32_t n, uint64_t arena_bytes);

/* Bytes of device workspace r3_table_create needs for n regions in an arena of
 * arena_bytes (an upper bound that depends on nothing else). */
size_t r3_table_workspace_bytes(uint32_t n, uint64_t arena_bytes);

/* The same for one concrete table: exact rather than an upper bound (0 if the table is
 * not valid). */
size_t r3_table_workspace_bytes_exact(const r3_region* host_tbl, uint32_t n, uint64_t arena_bytes);

/* Tuning hook (process-wide, affects tables created afterwards and the two size queries
 * above): smallest tile a wavefront works on, a power of two 1 KiB .. 16 MiB, and the most
 * tiles one region is split into, a power of two 64 .. 65536.  0 = default (4 KiB, 8192). */
int r3_tune_tiles(uint32_t min_tile_bytes, uint32_t max_tiles_per_region);

/* Tuning hook (process-wide): bytes one wavefront moves in the copy kernels (a power of two,
 * 1 KiB .. 1 MiB) and their threads per block (64, 128 or 256).  0 = default. */
int r3_tune_copy(uint32_t bytes_per_wavefront, uint32_t block_threads);

/* Validate host_tbl, split its regions into tiles, and upload regions and tile
 * list into the caller's workspace d_ws (device, 256-byte aligned, at least
 * r3_table_workspace_bytes).  Synchronous (uses blocking copies).  The table
 * refers to d_ws until r3_table_destroy.  host_tbl is not retained. */
int r3_table_create(r3_ctx* ctx, const r3_region* host_tbl, uint32_t n, uint64_t arena_bytes,
                    void* d_ws, size_t ws_bytes, r3_table** out);
int r3_table_destroy(r3_table* tbl);

/* Host-side facts about a table; any out pointer may be NULL. */
int r3_table_info(const r3_table* tbl, uint32_t* n_regions, uint64_t* n_tiles,
                  uint32_t* tile_bytes, uint64_t* total_bytes, uint64_t* arena_bytes);

/* ---- the hot path ------------------------------------------------------ */

/* Batched restore (Section V-B "restores the recorded execution context";
 * Section V-D resident prologue buffers):
 *   for every region r:  d_live[offset_r .. +bytes_r) = d_snapshot[offset_r .. +bytes_r)
 * One launch for the whole table.  Bytes outside the regions are not written.
 * d_snapshot and d_live must not overlap. */
int r3_restore(r3_ctx* ctx, const r3_table* tbl, const void* d_snapshot, void* d_live,
               void* stream);

/* Per-region order-independent 64-bit checksum of d_arena's bytes, the cheap
 * form of the default bitwise criterion of Section V-C (equal checksums of
 * live and recorded state).  With n = bytes of the region, w_j the j-th
 * little-endian 64-bit word of the region (bytes past n read as 0),
 * PHI = 0x9E3779B97F4A7C15, LEN = 0xBB67AE8584CAA73B, all mod 2^64:
 *   k_j = (j+1)*PHI
 *   sum = SUM_j ((lo32(w_j)+lo32(k_j)) mod 2^32) * ((hi32(w_j)+hi32(k_j)) mod 2^32) + n*LEN
 * d_out: device, n_regions values. */
int r3_checksum(r3_ctx* ctx, const r3_table* tbl, const void* d_arena, uint64_t* d_out,
                void* stream);

/* Fused validation (Section V-C): one pass over live and golden memory gives,
 * per region, mismatch count, first mismatching index, max abs / rel error and
 * the checksum of the live bytes (see r3_region_result), plus the table verdict.
 * d_out: device, n_regions results.  d_summary: device, one r3_summary, or NULL. */
int r3_compare(r3_ctx* ctx, const r3_table* tbl, const void* d_live, const void* d_golden,
               r3_region_result* d_out, r3_summary* d_summary, void* stream);

/* Page-level write-set between two states of `bytes` bytes (Section V-A: the
 * recorder stores pre- and post-execution state; the pages that differ are what
 * the kernel wrote).  Bit (p % 64) of d_bitmap[p / 64] is 1 iff page p differs
 * in any of its valid bytes; unused high bits of the last word are 0.
 * page_bytes: a power of two, 256 .. 1 MiB.  d_bitmap: device,
 * ceil(ceil(bytes/page_bytes)/64) words, fully overwritten.  d_dirty_count:
 * device, one value (number of set bits), or NULL.  bytes == 0 is legal. */
int r3_dirty_diff(r3_ctx* ctx, const void* d_pre, const void* d_post, uint64_t bytes,
                  uint32_t page_bytes, uint64_t* d_bitmap, uint64_t* d_dirty_count,
                  void* stream);

/* Record one replay unit's memory state (Section V-A items "pre-execution
 * device state" and "post-execution device state"):
 *   d_prologue[0..arena) = d_live;  launch(user, d_live, stream);
 *   d_epilogue[0..arena) = d_live;  bitmap = dirty_diff(prologue, epilogue);
 *   d_pro_cs / d_epi_cs  = per-region checksums of the two snapshots.
 * The whole arena is copied, not only the table's regions, so the write-set is
 * defined on every page.  Any of d_bitmap, d_dirty_count, d_pro_cs, d_epi_cs
 * may be NULL to skip that product.  Waits for the stream before returning.
 * R3_ECANDIDATE if launch fails. */
int r3_record(r3_ctx* ctx, const r3_table* tbl, void* d_live, r3_launch_fn launch, void* user,
              void* d_prologue, void* d_epilogue, uint32_t page_bytes, uint64_t* d_bitmap,
              uint64_t* d_dirty_count, uint64_t* d_pro_cs, uint64_t* d_epi_cs, void* stream);

/* Evaluate one candidate (Sections V-B, V-C: restore the prologue, execute the
 * candidate, compare with the epilogue, return the runtime if correct):
 *   for each of warmup + reps replays:
 *     r3_restore(restore_tbl, d_prologue -> d_live); time{ launch(user, d_live, stream) };
 *     r3_compare(check_tbl, d_live, d_epilogue) when compare_policy selects this replay
 * d_regions (device, check_tbl's n results) holds the last validated replay.
 * host_out (host) is filled after one wait on the stream at the end.
 * launch == NULL evaluates the restored state itself (a pure restore+validate
 * replay).  warmup + reps must be 1 .. R3_MAX_REPLAYS and reps >= 1.
 * A failing launch stops the loop: R3_ECANDIDATE, host_out->pass = 0. */
int r3_eval_candidate(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologue,
                      const r3_table* check_tbl, const void* d_epilogue, void* d_live,
                      r3_launch_fn launch, void* user, uint32_t warmup, uint32_t reps,
                      uint32_t compare_policy, r3_region_result* d_regions,
                      r3_eval_result* host_out, void* stream);

/* r3_eval_candidate in two halves, for a search that has several candidates ready at once
 * (Section II-C: several controllers run the sample / evaluate / update cycle concurrently;
 * Section V-D: replay workers persist across requests so that nothing is paid per candidate
 * that can be paid once).  r3_eval_submit checks the arguments, enqueues all
 * replays of one evaluation on the stream and returns a ticket without waiting; the host can
 * enqueue the next evaluation while this one runs, which hides the launch latency between
 * evaluations.  r3_eval_wait blocks until that evaluation's verdict is on the host and fills
 * host_out exactly as r3_eval_candidate would have; the ticket is then free again.
 * Evaluations submitted on one stream run in submission order, so they may share d_live, the
 * snapshots and the tables; evaluations that share any of these must use the same stream.
 * d_regions is overwritten by each evaluation that names it: give evaluations in flight
 * different arrays if the per-region results of each are wanted.  At most R3_MAX_INFLIGHT
 * tickets are outstanding (R3_ENOSPC beyond).  Tickets can be waited for in any order;
 * r3_eval_candidate may be called while tickets are outstanding; r3_ctx_destroy waits for
 * what is in flight.  A failing launch callback is reported by r3_eval_wait
 * (R3_ECANDIDATE, pass = 0), not by r3_eval_submit.  Errors: as r3_eval_candidate;
 * r3_eval_wait: R3_EINVAL for a ticket that is not outstanding.
 * host_guard_out (host, may be NULL) is filled for evaluations submitted with
 * r3_eval_submit_guarded (declared with the write-set calls below) and zeroed for others. */
int r3_eval_submit(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologue,
                   const r3_table* check_tbl, const void* d_epilogue, void* d_live,
                   r3_launch_fn launch, void* user, uint32_t warmup, uint32_t reps,
                   uint32_t compare_policy, r3_region_result* d_regions, uint32_t* ticket_out,
                   void* stream);
int r3_eval_wait(r3_ctx* ctx, uint32_t ticket, r3_eval_result* host_out,
                 r3_guard_result* host_guard_out);

/* r3_eval_submit with double-buffered live memory (Section V-D: the replay server keeps state
 * resident and pre-allocated so that nothing of one evaluation's set-up and tear-down has to
 * wait for another's).  The caller keeps TWO live arenas and passes them alternately; the
 * context owns two streams (default priority) and runs consecutive overlapped evaluations on
 * them alternately, after the work that `stream` holds at submission.  Ordering between
 * evaluation k and k+1:
 *   - the first restore of k+1 starts when the last candidate launch of k has finished, so it
 *     overlaps the last validation of k;
 *   - the first candidate launch of k+1 starts when that validation has finished: a timed
 *     candidate never shares the GPU with restore or validation work of this library.
 * Two consecutive submissions must therefore name different d_live (the same one is legal but
 * serialises nothing less: it races), and different d_regions if both results are wanted;
 * tables and snapshots may be shared.  This pays when restore and validation are bound by
 * latency (small states); for large states both are bound by HBM bandwidth and the overlap
 * gains nothing.  Tickets, r3_eval_wait and the error rules are those of r3_eval_submit; the
 * results are complete when r3_eval_wait returns (later work on `stream` is not ordered after
 * them). */
int r3_eval_submit_overlapped(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologue,
                              const r3_table* check_tbl, const void* d_epilogue, void* d_live,
                              r3_launch_fn launch, void* user, uint32_t warmup, uint32_t reps,
                              uint32_t compare_policy, r3_region_result* d_regions,
                              uint32_t* ticket_out, void* stream);

/* r3_eval_wait that gives up: looks for the evaluation's end for at most timeout_us
 * microseconds (0 = look once).  Finished: behaves exactly like r3_eval_wait.  Not finished:
 * R3_EBUSY, nothing is written, the ticket stays outstanding and can be waited for again.
 * This is how a caller notices a candidate that runs far longer than anything it could
 * accept (Section V-C rejects candidates that do not behave); what to do with a kernel that
 * never ends is the caller's decision, the library cannot stop it. */
int r3_eval_try_wait(r3_ctx* ctx, uint32_t ticket, uint32_t timeout_us, r3_eval_result* host_out,
                     r3_guard_result* host_guard_out);

/* ---- write-set driven replay ------------------------------------------- */

/* Turn a page bitmap (host copy of what r3_dirty_diff / r3_record wrote) into regions:
 * maximal runs of dirty pages (want_dirty != 0) or of clean pages (want_dirty == 0), as
 * R3_U8 / R3_CMP_BITWISE regions in address order, the last one clipped to `bytes`.
 * Writes at most cap regions to out (host; may be NULL when cap == 0) and the number of
 * runs to *n_out; R3_ENOSPC if there are more runs than cap (then *n_out says how many). */
int r3_writeset_regions(const uint64_t* host_bitmap, uint64_t bytes, uint32_t page_bytes,
                        int want_dirty, r3_region* out, uint32_t cap, uint32_t* n_out);

/* r3_eval_candidate with a restore table that covers only the recorded write-set, plus the
 * guard above: after the replays selected by guard->every the checksums of guard_tbl's
 * regions in live memory are compared, on the device, with guard->d_expected.  A failed check
 * makes host_out->pass 0; if guard->heal_tbl is given it is then restored from d_prologue so
 * that the next evaluation starts from the recorded state.  guard == NULL behaves exactly
 * like r3_eval_candidate.  host_guard_out (host) may be NULL. */
int r3_eval_candidate_guarded(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologue,
                              const r3_table* check_tbl, const void* d_epilogue, void* d_live,
                              r3_launch_fn launch, void* user, uint32_t warmup, uint32_t reps,
                              uint32_t compare_policy, r3_region_result* d_regions,
                              r3_eval_result* host_out, const r3_guard* guard,
                              r3_guard_result* host_guard_out, void* stream);

/* r3_eval_candidate_guarded in two halves (see r3_eval_submit; the verdict and the guard result
 * come from r3_eval_wait).  The guard structure is copied; what it points to must stay valid
 * until the wait.  d_scratch may be shared by evaluations on one stream.  The heal table, if
 * any, is restored by the r3_eval_wait that finds a failed check: evaluations that were in
 * flight behind the failing one ran on the damaged state, fail their own final check and are
 * to be submitted again. */
int r3_eval_submit_guarded(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologue,
                           const r3_table* check_tbl, const void* d_epilogue, void* d_live,
                           r3_launch_fn launch, void* user, uint32_t warmup, uint32_t reps,
                           uint32_t compare_policy, r3_region_result* d_regions,
                           const r3_guard* guard, uint32_t* ticket_out, void* stream);

/* ---- several recorded instances of one kernel --------------------------- */

/* Section V-C: promising candidates are validated against additional recorded instances of
 * the same kernel.  Instances are laid out back to back in "super arenas": instance i of the
 * prologue, epilogue and live state occupies [i*instance_stride, i*instance_stride + arena).
 * r3_table_replicate writes `instances` copies of an n-region table, copy i shifted by
 * i*instance_stride, to out (host, n*instances regions): tables created from it restore and
 * validate all instances in one launch each. */
int r3_table_replicate(const r3_region* host_tbl, uint32_t n, uint64_t instance_stride,
                       uint32_t instances, r3_region* out);

/* r3_eval_candidate over `instances` recorded instances: per replay one restore launch (all
 * instances), `instances` calls of the launch callback (call i gets d_live + i*instance_stride;
 * their total time is the replay's candidate time) and one validation launch (all instances).
 * restore_tbl and check_tbl are tables over the super arena (see r3_table_replicate);
 * check_tbl's region count must be a multiple of `instances`, copy i holding instance i's
 * regions.  host_instance_pass (host, `instances` bytes, may be NULL): 1 where every region of
 * that instance matched in the last validated replay.  Waits for the stream. */
int r3_eval_candidate_instances(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologues,
                                const r3_table* check_tbl, const void* d_epilogues, void* d_live,
                                r3_launch_fn launch, void* user, uint32_t instances,
                                uint64_t instance_stride, uint32_t warmup, uint32_t reps,
                                uint32_t compare_policy, r3_region_result* d_regions,
                                r3_eval_result* host_out, uint8_t* host_instance_pass, void* stream);

/* ---- a replay captured as a HIP graph ----------------------------------- */

/* For evaluations bound by launch latency (small states, many replays): the whole
 * evaluation -- `replays` times restore, the candidate's launches, validation -- is recorded
 * once as a HIP graph and then launched as a unit.  The candidate is timed by wall-clock
 * stamps taken on the device before and after it (their difference includes the dispatch
 * gap of the candidate).
 *
 * r3_replay_create records the graph; the launch callback is called `replays` times, on an
 * internal capture stream, and must only enqueue kernels on the stream it is given.  d_ws:
 * device, r3_replay_workspace_bytes() bytes, 16-byte aligned, owned by the caller until
 * r3_replay_destroy; all other pointers as in r3_eval_candidate and equally long-lived.
 * r3_replay_run launches the graph once on `stream` (warmup + reps must equal `replays`),
 * waits, and fills host_out like r3_eval_candidate with policy R3_POLICY_EVERY (d_regions
 * holds the last replay).  One run at a time per replay object. */
typedef struct r3_replay r3_replay;
size_t r3_replay_workspace_bytes(void);
int r3_replay_create(r3_ctx* ctx, const r3_table* restore_tbl, const void* d_prologue,
                     const r3_table* check_tbl, const void* d_epilogue, void* d_live,
                     r3_launch_fn launch, void* user, r3_region_result* d_regions, void* d_ws,
                     uint32_t replays, r3_replay** out);
int r3_replay_run(r3_replay* rp, uint32_t warmup, uint32_t reps, r3_eval_result* host_out,
                  void* stream);
int r3_replay_destroy(r3_replay* rp);

/* ---- validation for callers that cannot allocate ------------------------- */

/* r3_compare for callers that may not allocate device memory and hold no table object: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The caller
 * passes the regions themselves (host memory, read during the call, not retained) instead of a
 * table; they travel to the kernels as launch arguments, and the per-tile partial results go to
 * a buffer that is part of the library's device image (R3_STATIC_MAX_TILES x 40 bytes = 640 KiB
 * on every GPU the library has a context on, held until the process ends) instead of a
 * caller-provided workspace.  The call enqueues two or three kernels on `stream` and returns;
 * it calls no allocating routine, performs no copy and does not wait.
 * Results: d_out (device, n results) and d_summary (device, may be NULL) exactly as r3_compare
 * on a table made from the same regions.
 * Limits: n <= R3_STATIC_MAX_REGIONS, and the regions must split into at most
 * R3_STATIC_MAX_TILES tiles of at most R3_STATIC_MAX_TILE_BYTES bytes each (the tile size is the
 * smallest power of two >= 4 KiB for which the tile count fits): R3_ENOSPC beyond, with
 * r3_last_error saying which limit.  Table rules and their status codes as r3_table_validate.
 * Every call on one GPU uses that GPU's one buffer, and the buffer keeps the previous call's
 * partials until they are overwritten: calls on the same GPU must not overlap in time (same
 * stream, or ordered by events); overlapping calls race. */
#define R3_STATIC_MAX_REGIONS 16u
#define R3_STATIC_MAX_TILES 16384u
#define R3_STATIC_MAX_TILE_BYTES (16u << 20)
int r3_compare_static(r3_ctx* ctx, const r3_region* host_tbl, uint32_t n, uint64_t arena_bytes,
                      const void* d_live, const void* d_golden, r3_region_result* d_out,
                      r3_summary* d_summary, void* stream);

/* ---- timing statistics -------------------------------------------------- */

/* Candidate times (ms) of the timed replays of the last evaluation on ctx, in replay order:
 * copies at most cap values to out (host) and the number available to *n_out. */
int r3_ctx_last_times(const r3_ctx* ctx, float* out, uint32_t cap, uint32_t* n_out);

/* What a driver needs to decide whether a runtime is trustworthy (Section IV: each
 * experiment is replayed K times; Section VII-B: warm-up runs are discarded). */
typedef struct {
  uint32_t n;       /* samples used                                              */
  uint32_t stable;  /* 1 if mad / median <= rel_noise                            */
  float min, median, max, mean;
  float mad;        /* median of |x - median|                                    */
  float reserved;
} r3_timing;

/* Host only: statistics of n samples; rel_noise is the stability bound on mad/median.
 * n == 0 gives zeros and stable = 0. */
int r3_timing_stats(const float* ms, uint32_t n, float rel_noise, r3_timing* out);

#ifdef __cplusplus
}
#endif
#endif /* R3_H */
