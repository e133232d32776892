// Device code of libr3.so for gfx950: batched restore, checksum, fused compare+checksum,
// page dirty-diff and their small finalize passes.
//
// Everything here is a byte stream bounded by HBM bandwidth; there is no contraction, so no
// MFMA.  The common shape: one wavefront (64 lanes) owns one tile of one region, walks it
// with 16-byte loads per lane (1 KiB per wavefront instruction, several in flight), keeps
// its running results in registers, combines them across the wavefront with lane
// exchanges, and leaves one small partial per tile.  A second, tiny launch folds the
// partials of every region (integer sums mod 2^64, min, max of non-negative doubles: all
// independent of order, so the results are bit-exact however the tiles were scheduled).
//
// Floating point in the validation follows the rule in r3.h: binary64, one rounding per
// operation.  This file is compiled with -ffp-contract=off; the pragma below repeats that.
#include <algorithm>

#include "r3_internal.h"

#pragma clang fp contract(off)

namespace r3 {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kUnroll = 4;                       // 16-byte loads in flight per lane and stream
constexpr uint64_t kVecKeyStep = 128ull * kPhi;  // 64 lanes * 2 words per 16-byte vector
constexpr double kInf = __builtin_huge_val();

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }

__device__ __forceinline__ uint32_t wave_in_block() {
  return __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
}

__device__ __forceinline__ uint64_t wave_sum(uint64_t v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}
__device__ __forceinline__ uint32_t wave_min(uint32_t v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    uint32_t o = __shfl_xor(v, m, 64);
    v = o < v ? o : v;
  }
  return v;
}
__device__ __forceinline__ uint64_t wave_min(uint64_t v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    uint64_t o = __shfl_xor(v, m, 64);
    v = o < v ? o : v;
  }
  return v;
}
__device__ __forceinline__ uint32_t wave_or(uint32_t v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v |= __shfl_xor(v, m, 64);
  return v;
}
// Maximum of non-negative doubles (never NaN here): the order of their bit patterns.
__device__ __forceinline__ uint64_t wave_max(uint64_t v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    uint64_t o = __shfl_xor(v, m, 64);
    v = o > v ? o : v;
  }
  return v;
}

__device__ __forceinline__ uint64_t dbits(double d) { return (uint64_t)__double_as_longlong(d); }
__device__ __forceinline__ double bits_d(uint64_t u) { return __longlong_as_double((long long)u); }

// Wavefront reductions over the DPP lane network (no LDS traffic): four steps inside each
// row of 16 lanes, then two row broadcasts; the total lands in lane 63 and is read back as
// a wavefront-uniform scalar.  `ident` is the operation's identity; it fills lanes whose DPP
// source does not exist.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp32(uint32_t ident, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)ident, (int)v, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint64_t dpp64(uint64_t ident, uint64_t v) {
  const uint32_t lo = dpp32<CTRL, ROW_MASK>((uint32_t)ident, (uint32_t)v);
  const uint32_t hi = dpp32<CTRL, ROW_MASK>((uint32_t)(ident >> 32), (uint32_t)(v >> 32));
  return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint32_t last_lane(uint32_t v) { return __builtin_amdgcn_readlane(v, 63); }
__device__ __forceinline__ uint64_t last_lane(uint64_t v) {
  return ((uint64_t)last_lane((uint32_t)(v >> 32)) << 32) | last_lane((uint32_t)v);
}
#define R3_DPP_REDUCE(T, DPP, IDENT, OP)                                \
  v = OP(v, DPP<0xb1, 0xf>(IDENT, v));  /* quad_perm [1,0,3,2] */       \
  v = OP(v, DPP<0x4e, 0xf>(IDENT, v));  /* quad_perm [2,3,0,1] */       \
  v = OP(v, DPP<0x114, 0xf>(IDENT, v)); /* row_shr:4 */                 \
  v = OP(v, DPP<0x118, 0xf>(IDENT, v)); /* row_shr:8 */                 \
  v = OP(v, DPP<0x142, 0xa>(IDENT, v)); /* row_bcast:15 into rows 1,3 */\
  v = OP(v, DPP<0x143, 0xc>(IDENT, v)); /* row_bcast:31 into rows 2,3 */\
  return last_lane(v);
__device__ __forceinline__ uint64_t op_add(uint64_t a, uint64_t b) { return a + b; }
__device__ __forceinline__ uint32_t op_add(uint32_t a, uint32_t b) { return a + b; }
__device__ __forceinline__ uint32_t op_min(uint32_t a, uint32_t b) { return b < a ? b : a; }
__device__ __forceinline__ uint64_t op_max(uint64_t a, uint64_t b) { return b > a ? b : a; }
__device__ __forceinline__ uint64_t dpp_sum(uint64_t v) { R3_DPP_REDUCE(uint64_t, dpp64, 0ull, op_add) }
__device__ __forceinline__ uint32_t dpp_sum(uint32_t v) { R3_DPP_REDUCE(uint32_t, dpp32, 0u, op_add) }
__device__ __forceinline__ uint32_t dpp_min(uint32_t v) { R3_DPP_REDUCE(uint32_t, dpp32, 0xFFFFFFFFu, op_min) }
__device__ __forceinline__ uint64_t dpp_max(uint64_t v) { R3_DPP_REDUCE(uint64_t, dpp64, 0ull, op_max) }
__device__ __forceinline__ uint64_t op_min(uint64_t a, uint64_t b) { return b < a ? b : a; }
__device__ __forceinline__ uint64_t dpp_min(uint64_t v) { R3_DPP_REDUCE(uint64_t, dpp64, ~0ull, op_min) }
#undef R3_DPP_REDUCE

// One checksum term: word w under key k.
__device__ __forceinline__ uint64_t cks_term(uint32_t lo, uint32_t hi, uint64_t k) {
  uint32_t a = lo + (uint32_t)k;
  uint32_t b = hi + (uint32_t)(k >> 32);
  return (uint64_t)a * (uint64_t)b;
}

// The tile a wavefront owns, resolved from the table (all values wavefront-uniform).
struct TileView {
  uint64_t rel_start;  // first byte of the tile, relative to the region
  uint32_t len;        // bytes in the tile
  uint32_t region;
  uint64_t offset;     // region offset in the arena
  uint64_t bytes;      // region size
  uint32_t dtype, mode;
  double rtol, atol;
};

__device__ __forceinline__ uint32_t sgpr(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint64_t sgpr(uint64_t v) {
  return ((uint64_t)sgpr((uint32_t)(v >> 32)) << 32) | sgpr((uint32_t)v);
}

__device__ __forceinline__ TileView resolve_tile(const TableDev& t, uint64_t tile_id) {
  TileView v;
  Tile tl = t.tiles[tile_id];
  v.region = sgpr(tl.region);
  const uint32_t packed = sgpr(tl.packed);
  const uint32_t index = packed & 0xFFFFFFu, shift = packed >> 24;
  const r3_region* rg = &t.regions[v.region];
  v.offset = sgpr(rg->offset);
  v.bytes = sgpr(rg->bytes);
  v.dtype = sgpr(rg->dtype);
  v.mode = sgpr(rg->mode);
  v.rtol = bits_d(sgpr(dbits(rg->rtol)));
  v.atol = bits_d(sgpr(dbits(rg->atol)));
  v.rel_start = (uint64_t)index << shift;
  uint64_t left = v.bytes - v.rel_start;
  uint64_t full = 1ull << shift;
  v.len = (uint32_t)(left < full ? left : full);
  return v;
}

// ---------------------------------------------------------------------------------------
// Word loads for the paths that cannot use 16-byte vectors: region tails and regions whose
// offset is not a multiple of 16.  ES = element size; p is ES-aligned; `valid` (1..8, a
// multiple of ES) bytes belong to the region, the rest of the word reads as zero.
// ---------------------------------------------------------------------------------------
template <int ES>
__device__ __forceinline__ uint64_t load_word(const uint8_t* p, uint32_t valid) {
  uint64_t w = 0;
  if (ES == 8) {
    w = *(const uint64_t*)p;
  } else if (ES == 4) {
    w = *(const uint32_t*)p;
    if (valid > 4) w |= (uint64_t)(*(const uint32_t*)(p + 4)) << 32;
  } else if (ES == 2) {
#pragma unroll
    for (uint32_t b = 0; b < 8; b += 2)
      if (b < valid) w |= (uint64_t)(*(const uint16_t*)(p + b)) << (8 * b);
  } else {
#pragma unroll
    for (uint32_t b = 0; b < 8; ++b)
      if (b < valid) w |= (uint64_t)p[b] << (8 * b);
  }
  return w;
}

// =======================================================================================
// Restore / copy
// =======================================================================================
// Copies `len` bytes from src to dst (same misalignment on both sides because the arenas
// are 16-byte aligned and share offsets): a head up to the next 16-byte boundary, 16-byte
// vectors, a tail.  Head and tail move in units of `es` bytes (the element size, which
// divides offset and length).
__device__ __forceinline__ void copy_span(const uint8_t* src, uint8_t* dst, uint32_t len,
                                          uint32_t es, uint32_t lane) {
  uint32_t head = (uint32_t)((16 - ((uintptr_t)src & 15)) & 15);
  if (head > len) head = len;
  if (head) {
    for (uint32_t b = lane * es; b < head; b += 64 * es) {
      if (es == 1) dst[b] = src[b];
      else if (es == 2) *(uint16_t*)(dst + b) = *(const uint16_t*)(src + b);
      else if (es == 4) *(uint32_t*)(dst + b) = *(const uint32_t*)(src + b);
      else *(uint64_t*)(dst + b) = *(const uint64_t*)(src + b);
    }
  }
  const u32x4* s = (const u32x4*)(src + head);
  u32x4* d = (u32x4*)(dst + head);
  const uint32_t nvec = (len - head) >> 4;
  uint32_t v = lane;
  const uint32_t nfull = nvec / (64 * kUnroll);
  for (uint32_t it = 0; it < nfull; ++it) {
    u32x4 r[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) r[u] = __builtin_nontemporal_load(s + v + 64 * u);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) __builtin_nontemporal_store(r[u], d + v + 64 * u);
    v += 64 * kUnroll;
  }
  for (; v < nvec; v += 64) __builtin_nontemporal_store(__builtin_nontemporal_load(s + v), d + v);
  const uint32_t done = head + (nvec << 4);
  for (uint32_t b = done + lane * es; b < len; b += 64 * es) {
    if (es == 1) dst[b] = src[b];
    else if (es == 2) *(uint16_t*)(dst + b) = *(const uint16_t*)(src + b);
    else if (es == 4) *(uint32_t*)(dst + b) = *(const uint32_t*)(src + b);
    else *(uint64_t*)(dst + b) = *(const uint64_t*)(src + b);
  }
}

__device__ __forceinline__ uint32_t elem_size_dev(uint32_t dtype) {
  return dtype == R3_U8 ? 1u : (dtype == R3_BF16 || dtype == R3_F16) ? 2u : dtype == R3_F64 ? 8u : 4u;
}

// Copy kernels run best here as very many short wavefronts that each move 1 KiB (one
// 16-byte load and store per lane, no loop) in address order: measured 6.6 TB/s against
// 5.1-5.4 TB/s for wavefronts that walk 64 KiB or more.  A table tile is therefore spread
// over 2^sub_log2 consecutive wavefront slots; slots past the end of a tile exit at once.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void restore_kernel(TableDev t, const uint8_t* src, uint8_t* dst,
                                                        uint32_t copy_shift, uint32_t n_classes,
                                                        uint32_t sub_log2_0, uint64_t total_slots,
                                                        CopyClasses cls) {
  const uint64_t slot = (uint64_t)blockIdx.x * (BLOCK / 64) + wave_in_block();
  if (slot >= total_slots) return;
  uint64_t rel = slot;
  uint32_t sub_log2 = sub_log2_0, first = 0;
  if (n_classes > 1) {  // size class of this slot: a short scalar scan of the launch arguments
    uint32_t c = 0;
    while (c + 1 < n_classes && slot >= cls.slot_base[c + 1]) ++c;
    rel = slot - cls.slot_base[c];
    sub_log2 = cls.sub_log2[c];
    first = cls.first[c];
  }
  const CopyTile* ct = &t.copy_tiles[first + (rel >> sub_log2)];
  const uint64_t tile_at = sgpr(ct->at);
  const uint32_t tile_len = sgpr(ct->len), es = sgpr(ct->es);
  const uint32_t sub = (uint32_t)(rel & ((1ull << sub_log2) - 1));
  const uint64_t begin = (uint64_t)sub << copy_shift;
  if (begin >= tile_len) return;
  const uint32_t left = tile_len - (uint32_t)begin;
  // a class whose tiles are smaller than the copy unit has one slot per tile
  const uint32_t unit = sub_log2 ? (1u << copy_shift) : 0xFFFFFFFFu;
  const uint32_t len = left < unit ? left : unit;
  const uint64_t at = tile_at + begin;
  copy_span(src + at, dst + at, len, es, lane_id());
}

// Whole-range copy for r3_record: wavefront k moves bytes [k << copy_shift, (k+1) << copy_shift).
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void copy_flat_kernel(const uint8_t* src, uint8_t* dst,
                                                          uint64_t bytes, uint64_t n_slots,
                                                          uint32_t copy_shift) {
  const uint64_t slot = (uint64_t)blockIdx.x * (BLOCK / 64) + wave_in_block();
  if (slot >= n_slots) return;
  const uint64_t at = slot << copy_shift;
  const uint64_t left = bytes - at;
  const uint32_t len = (uint32_t)(left < (1ull << copy_shift) ? left : (1ull << copy_shift));
  copy_span(src + at, dst + at, len, 1, lane_id());
}

// =======================================================================================
// Checksum
// =======================================================================================
// Sum of the word terms of one tile.  word0 = region word index of the tile's first word.
template <int ES>
__device__ __forceinline__ uint64_t checksum_tile(const uint8_t* base, uint32_t len,
                                                  uint64_t word0, uint32_t lane) {
  uint64_t acc = 0;
  if (((uintptr_t)base & 15) == 0) {
    const u32x4* p = (const u32x4*)base;
    const uint32_t nvec = len >> 4;
    uint64_t k = (word0 + 2ull * lane + 1) * kPhi;
    uint32_t v = lane;
    const uint32_t nfull = nvec / (64 * kUnroll);
    for (uint32_t it = 0; it < nfull; ++it) {
      u32x4 r[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) r[u] = __builtin_nontemporal_load(p + v + 64 * u);
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const uint64_t ku = k + (uint64_t)u * kVecKeyStep;
        acc += cks_term(r[u].x, r[u].y, ku);
        acc += cks_term(r[u].z, r[u].w, ku + kPhi);
      }
      v += 64 * kUnroll;
      k += (uint64_t)kUnroll * kVecKeyStep;
    }
    for (; v < nvec; v += 64) {
      u32x4 r = __builtin_nontemporal_load(p + v);
      acc += cks_term(r.x, r.y, k);
      acc += cks_term(r.z, r.w, k + kPhi);
      k += kVecKeyStep;
    }
    // Fewer than 16 bytes left: at most two words, the last one possibly partial.
    const uint32_t tail = len & 15;
    const uint32_t tail_words = (tail + 7) >> 3;
    if (lane < tail_words) {
      const uint32_t at = (nvec << 4) + 8 * lane;
      const uint32_t valid = (len - at) < 8 ? (len - at) : 8;
      uint64_t w = load_word<ES>(base + at, valid);
      acc += cks_term((uint32_t)w, (uint32_t)(w >> 32), (word0 + 2ull * nvec + lane + 1) * kPhi);
    }
  } else {
    const uint32_t nwords = (len + 7) >> 3;
    for (uint32_t j = lane; j < nwords; j += 64) {
      const uint32_t at = 8 * j;
      const uint32_t valid = (len - at) < 8 ? (len - at) : 8;
      uint64_t w = load_word<ES>(base + at, valid);
      acc += cks_term((uint32_t)w, (uint32_t)(w >> 32), (word0 + j + 1) * kPhi);
    }
  }
  return acc;
}

__global__ __launch_bounds__(kBlock) void checksum_kernel(TableDev t, const uint8_t* arena) {
  const uint64_t tile_id = (uint64_t)blockIdx.x * kWavesPerBlock + wave_in_block();
  if (tile_id >= t.n_tiles) return;
  const TileView tv = resolve_tile(t, tile_id);
  const uint8_t* base = arena + tv.offset + tv.rel_start;
  const uint64_t word0 = tv.rel_start >> 3;  // tiles start at multiples of 16 bytes
  const uint32_t lane = lane_id();
  uint64_t acc;
  switch (elem_size_dev(tv.dtype)) {
    case 1: acc = checksum_tile<1>(base, tv.len, word0, lane); break;
    case 2: acc = checksum_tile<2>(base, tv.len, word0, lane); break;
    case 4: acc = checksum_tile<4>(base, tv.len, word0, lane); break;
    default: acc = checksum_tile<8>(base, tv.len, word0, lane); break;
  }
  acc = dpp_sum(acc);
  if (lane == 0) ((uint64_t*)t.partials)[tile_id] = acc;
}

// One block per region: add up the tile sums, add the length term.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void checksum_finalize_kernel(TableDev t, uint64_t* out) {
  __shared__ uint64_t sh[BLOCK / 64];
  const uint32_t r = blockIdx.x;
  const uint64_t b = t.tile_begin[r], e = t.tile_begin[r + 1];
  const uint64_t* part = (const uint64_t*)t.partials;
  uint64_t acc = 0;
  for (uint64_t i = b + threadIdx.x; i < e; i += (uint64_t)BLOCK * 4) {
    uint64_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint64_t idx = i + (uint64_t)u * BLOCK;
      v[u] = idx < e ? part[idx] : 0;
    }
    acc += (v[0] + v[1]) + (v[2] + v[3]);
  }
  acc = wave_sum(acc);
  if (BLOCK > 64) {
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
      acc = 0;
      for (int w = 0; w < BLOCK / 64; ++w) acc += sh[w];
    }
  }
  if (threadIdx.x == 0) out[r] = acc + t.regions[r].bytes * kLen;
}

// =======================================================================================
// Fused compare + checksum
// =======================================================================================
// What a wavefront knows about its tile.  Everything but max_abs and the checksum is kept
// for the wavefront as a whole (uniform values, scalar registers): the common path updates
// them from lane masks, the rare paths work on a LaneAcc of their own and fold it in when
// they are done.
struct Acc {
  uint32_t wcount;    // mismatches so far
  uint32_t wfirst;    // smallest mismatching element index inside the tile, ~0u if none
  uint64_t top_bits;  // bit pattern of top = the largest relative error so far (the tile's max_rel)
  uint64_t tq_bits;   // bit pattern of tq = top cut down so that tq * |G| is exact (raise_top)
  uint32_t tq_fix;    // floor(top * 2^16), saturated: the same bound in fixed point, for 1-byte elements
  double rtol_cut;    // a little under rtol (tolerance mode), -1 in bitwise mode; see within
  uint32_t within;    // 1 while top <= rtol_cut: an element that cannot raise top is then no mismatch
  uint32_t lut_ready; // 1 once this wavefront has built its table of the 1-byte path
  uint32_t lut_fix;   // the tq_fix that table was built for
  uint32_t imax;      // per lane: largest integer error seen by the 1-byte path
  double max_abs;     // per lane
  uint64_t cks;       // per lane
};

// What one lane gathers inside a rare path.
struct LaneAcc {
  uint32_t count;
  uint32_t first;  // ~0u if none
  double max_rel;
};

// How the elements of the region at hand are read (wavefront-uniform).
struct ElemKind {
  uint32_t dtype;
  uint32_t es;        // element size in bytes
  bool is_float;
  bool tol;
  double rtol, atol;
  uint32_t* lut;      // this wavefront's 1 KiB of LDS (table of the 1-byte path)
};

// binary16 -> binary64 (exact): through the hardware conversion to binary32.
__device__ __forceinline__ double f16_to_f64(uint32_t bits) {
  return (double)(float)__builtin_bit_cast(_Float16, (uint16_t)bits);
}

__device__ __forceinline__ double to_f64(uint64_t bits, uint32_t dtype) {
  switch (dtype) {  // uniform across the wavefront: a scalar branch
    case R3_U8: return (double)(uint32_t)bits;
    case R3_I32: return (double)(int32_t)(uint32_t)bits;
    case R3_F32: return (double)__uint_as_float((uint32_t)bits);
    case R3_BF16: return (double)__uint_as_float((uint32_t)bits << 16);
    case R3_F16: return f16_to_f64((uint32_t)bits);
    default: return bits_d(bits);
  }
}

// Can the quotient d/|G| exceed `top`?  The quotient is needed only when it can raise the
// running maximum of the relative error.  With ph = fl(top*|G|) and pl = fma(top, |G|, -ph)
// the product top*|G| equals ph + pl exactly (pl cannot underflow while ph >= 2^-900), and
// u = fl(fl(d - ph) - pl) has the sign of d - top*|G|: if d and ph are within a factor of two
// the first difference is exact and the second keeps the sign; otherwise |d - ph| >= ph/2
// dwarfs pl.  So
//   ph >= 2^-900 and u <= 0   =>   d <= top*|G|   =>   fl(d/|G|) <= top,
// and the divide can be skipped; equal quotients (ties, frequent with 8- and 16-bit types)
// are skipped as well.  d == 0 never raises anything.  Everything else (ph tiny, zero or NaN,
// d NaN or infinite, overflow of ph) answers "maybe": an answer "no" therefore also says that
// d is finite, hence that both inputs are.  Written with bitwise operators on purpose: the
// compiler must not turn the tests into branches.
constexpr double kTopFloor = 0x1p-900;
__device__ __forceinline__ bool may_raise_max_rel(double d, double aG, double top) {
  const double ph = top * aG;
  const double pl = __builtin_fma(top, aG, -ph);
  const double u = (d - ph) - pl;
  const bool below = (ph >= kTopFloor) & (u <= 0.0);
  return !(below | (d == 0.0));
}

// The quick form for element types of at most 32 significant bits, t = C - G: tq keeps the
// leading 21 significant bits of top, so ph = tq * |G| is exact while it is a normal number
// or zero, and |t| <= ph proves |t|/|G| <= tq <= top (and t == 0 when ph == 0).
__device__ __forceinline__ bool may_raise_quick(double t, double aG, double tq) {
  const double ph = tq * aG;
  const bool exact = __builtin_isnormal(ph) | (ph == 0.0);
  return !((__builtin_fabs(t) <= ph) & exact);
}

// A larger top for the wavefront (m is uniform).  An infinite top (a NaN or infinity
// mismatch was seen, nothing can raise max_rel any more) gets a large finite tq, which lets
// finite errors pass the quick test.
__device__ __forceinline__ void raise_top(Acc& a, double m) {
  if (m > bits_d(a.top_bits)) {
    const uint64_t mb = dbits(m);
    a.top_bits = sgpr(mb);
    const uint64_t cut = m < kInf ? (mb & ~0xFFFFFFFFull) : dbits(0x1p500);
    a.tq_bits = sgpr(cut);
    const uint32_t fix = m < 0x1p15 ? (uint32_t)(m * 0x1p16) : 0x7FFFFFFFu;  // the scaling is exact
    a.tq_fix = sgpr(fix);
    a.within = sgpr((uint32_t)(m <= a.rtol_cut));
  }
}

// Fold what the lanes gathered in a rare path into the wavefront's state.  Called by all
// lanes (uniform control flow).
__device__ __forceinline__ void fold_lanes(Acc& a, const LaneAcc& l) {
  if (__builtin_amdgcn_ballot_w64(l.count != 0) != 0) {
    a.wcount += dpp_sum(l.count);
    const uint32_t f = dpp_min(l.first);
    a.wfirst = f < a.wfirst ? f : a.wfirst;
  }
  if (__builtin_amdgcn_ballot_w64(l.max_rel > bits_d(a.top_bits)) != 0)
    raise_top(a, bits_d(dpp_max(dbits(l.max_rel))));
}

// The relative error of one element whose quotient may raise the maximum (aG == 0 means
// G == 0: no relative error by rule).
__device__ __forceinline__ void raise_max_rel(double d, double aG, LaneAcc& l) {
  const double r = (aG == 0.0) ? 0.0 : d / aG;
  l.max_rel = r > l.max_rel ? r : l.max_rel;
}

// The larger of the wavefront's top and what this lane has found since.
__device__ __forceinline__ double lane_top(const Acc& a, const LaneAcc& l) {
  const double top = bits_d(a.top_bits);
  return l.max_rel > top ? l.max_rel : top;
}

// One element whose bit patterns differ, under the full rules (tails, regions that are not
// 16-byte aligned, and the careful path of the vector code, which also passes equal ones).
__device__ __forceinline__ void full_rules(bool differ, double C, double G, bool is_float, uint32_t idx,
                                           const ElemKind& k, Acc& a, LaneAcc& l) {
  const double aG = __builtin_fabs(G);
  double d = __builtin_fabs(C - G);
  bool forced = false, rel_done = false;
  if (!(d < kInf)) {  // NaN or +Inf: equal non-finite patterns, a non-finite input, fp64 overflow
    if (!differ) {
      d = 0.0;
    } else if (is_float && !(__builtin_fabs(C) < kInf && aG < kInf)) {
      d = kInf;
      forced = true;
      rel_done = true;
      l.max_rel = kInf;
    }
  }
  bool mis;
  if (k.tol) {
    const double t = k.rtol * aG;
    const double thr = k.atol + t;
    mis = forced || d > thr;
  } else {
    mis = differ;
  }
  if (!rel_done && may_raise_max_rel(d, aG, lane_top(a, l))) raise_max_rel(d, aG, l);
  a.max_abs = d > a.max_abs ? d : a.max_abs;
  l.count += mis ? 1u : 0u;
  const uint32_t cand = mis ? idx : 0xFFFFFFFFu;
  l.first = cand < l.first ? cand : l.first;
}

// One 64-bit word of live (wc) and golden (wg) data holding `nvalid` elements; idx = tile
// index of its first element.  The element loop is deliberately not unrolled: this path only
// serves tails and unaligned regions.
__device__ __forceinline__ void differing_word(uint64_t wc, uint64_t wg, uint32_t nvalid, uint32_t idx,
                                               const ElemKind& k, Acc& a, LaneAcc& l) {
  if (wc == wg) return;
  const uint32_t bits = 8 * k.es;
  const uint64_t mask = k.es == 8 ? ~0ull : (1ull << bits) - 1;
#pragma unroll 1
  for (uint32_t e = 0; e < nvalid; ++e) {
    const uint64_t cb = wc & mask, gb = wg & mask;
    if (cb != gb) full_rules(true, to_f64(cb, k.dtype), to_f64(gb, k.dtype), k.is_float, idx + e, k, a, l);
    wc = k.es == 8 ? 0 : wc >> bits;
    wg = k.es == 8 ? 0 : wg >> bits;
  }
}

// ---- whole 16-byte vectors, specialised per element type ------------------------------
// Candidates that are numerically equivalent but not bit-identical differ almost
// everywhere, so this path matters as much as the bit-equal one.  A vector is handled in
// chunks of N elements.  The common case of a chunk needs no branch and no divide: every
// element's error is finite and provably cannot raise max_rel; then the mismatch masks of
// the lanes are counted on the scalar unit and max_abs is one instruction per element (and
// while the largest relative error so far is under rtol, such a chunk cannot hold a mismatch
// either: threshold, masks and counting are skipped).  Only the elements that may raise
// max_rel are divided, one per lane and round; a chunk in which any lane sees NaN or infinity
// is redone element by element under the full rules.
template <int DT> struct Elem;
template <> struct Elem<R3_U8>   { static constexpr int size = 1; [[maybe_unused]] static constexpr bool is_float = false; };
template <> struct Elem<R3_F32>  { static constexpr int size = 4; static constexpr bool is_float = true; };
template <> struct Elem<R3_F64>  { static constexpr int size = 8; static constexpr bool is_float = true; };
template <> struct Elem<R3_I32>  { static constexpr int size = 4; static constexpr bool is_float = false; };
template <> struct Elem<R3_BF16> { static constexpr int size = 2; static constexpr bool is_float = true; };
template <> struct Elem<R3_F16>  { static constexpr int size = 2; static constexpr bool is_float = true; };

template <int DT>
__device__ __forceinline__ double to_f64_t(uint64_t bits) {
  if (DT == R3_U8) return (double)(uint32_t)bits;
  if (DT == R3_I32) return (double)(int32_t)(uint32_t)bits;
  if (DT == R3_F32) return (double)__uint_as_float((uint32_t)bits);
  if (DT == R3_BF16) return (double)__uint_as_float((uint32_t)bits << 16);
  if (DT == R3_F16) return f16_to_f64((uint32_t)bits);
  return bits_d(bits);
}

// Bit pattern of element e of a 16-byte vector.
template <int DT>
__device__ __forceinline__ uint64_t elem_bits(const u32x4& v, int e) {
  constexpr int ES = Elem<DT>::size;
  if constexpr (ES == 8) {
    return ((uint64_t)v[2 * e + 1] << 32) | v[2 * e];
  } else if constexpr (ES == 4) {
    return v[e];
  } else if constexpr (ES == 2) {
    return (v[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
  } else {
    return (v[e >> 2] >> (8 * (e & 3))) & 0xFFu;
  }
}

// A vector is consumed from its low end: drop its first BYTES bytes (a multiple of 4).
template <int BYTES>
__device__ __forceinline__ void drop_front(u32x4& v) {
  if constexpr (BYTES == 4) {
    v = u32x4{v.y, v.z, v.w, 0};
  } else if constexpr (BYTES == 8) {
    v = u32x4{v.z, v.w, 0, 0};
  } else {
    v = u32x4{0, 0, 0, 0};
  }
}

// First element of a vector, and the vector without it.
template <int DT>
__device__ __forceinline__ uint64_t pop_elem(u32x4& v) {
  constexpr int ES = Elem<DT>::size;
  uint64_t bits;
  if constexpr (ES == 8) {
    bits = ((uint64_t)v.y << 32) | v.x;
    drop_front<8>(v);
  } else if constexpr (ES == 4) {
    bits = v.x;
    drop_front<4>(v);
  } else {
    constexpr uint32_t S = 8 * ES;
    bits = v.x & ((1u << S) - 1);
    v.x = (v.x >> S) | (v.y << (32 - S));
    v.y = (v.y >> S) | (v.z << (32 - S));
    v.z = (v.z >> S) | (v.w << (32 - S));
    v.w >>= S;
  }
  return bits;
}

// max(m, |t|) for a finite t in one instruction (a plain fmax costs a second one that
// quiets signalling NaNs, which cannot occur where this is used).
__device__ __forceinline__ double max_with_abs(double m, double t) {
  double r;
  asm("v_max_f64 %0, %1, |%2|" : "=v"(r) : "v"(m), "v"(t));
  return r;
}

// The first N elements of the vectors c and g.  idx0 = tile index of the first of them in
// lane 0; lane L holds the elements EPV * L further on.  All lanes take part (uniform
// control flow).
template <int DT, int N>
__device__ __forceinline__ void compare_chunk(const u32x4& c, const u32x4& g, uint32_t idx0,
                                              const ElemKind& k, Acc& a) {
  constexpr bool kQuick = Elem<DT>::size < 8;
  constexpr uint32_t EPV = 16 / Elem<DT>::size;
  const double top = bits_d(a.top_bits), tq = bits_d(a.tq_bits);
  double aG[N], t[N];  // |G| and the signed difference C - G
  bool any_flag = false;
  bool flag[N];
#pragma unroll
  for (int e = 0; e < N; ++e) {
    const double C = to_f64_t<DT>(elem_bits<DT>(c, e)), G = to_f64_t<DT>(elem_bits<DT>(g, e));
    aG[e] = __builtin_fabs(G);
    t[e] = C - G;
    flag[e] = kQuick ? may_raise_quick(t[e], aG[e], tq) : may_raise_max_rel(__builtin_fabs(t[e]), aG[e], top);
    any_flag |= flag[e];
  }
  // Per lane, which of its elements may raise max_rel (or are NaN / infinite).  Usually none.
  uint32_t pend = 0;
  const bool flagged = __builtin_amdgcn_ballot_w64(any_flag) != 0;
  if (!flagged && a.within) {
    // No element of the chunk can raise top, and top <= rtol_cut: every error is finite and
    //   d <= top * |G| <= rtol * (1 - 2^-51) * |G| <= fl(rtol * |G|) <= fl(atol + fl(rtol * |G|))
    // (the product is a normal number or the element has d == 0; adding atol >= 0 and rounding
    // cannot go below the addend), so no element is a mismatch and the threshold is not needed.
#pragma unroll
    for (int e = 0; e < N; ++e) a.max_abs = max_with_abs(a.max_abs, t[e]);
    return;
  }
  if (flagged) {
    bool odd = false;  // an error that is NaN or infinite: the plain predicate does not apply
#pragma unroll
    for (int e = 0; e < N; ++e) {
      const double d = __builtin_fabs(t[e]);
      if (kQuick) flag[e] = flag[e] & may_raise_max_rel(d, aG[e], top);
      odd |= flag[e] & !(d < kInf);
      pend |= flag[e] ? (1u << e) : 0u;
    }
    if (__builtin_amdgcn_ballot_w64(odd) != 0) {
      // The careful path: element by element under the full rules, one copy of the code.
      u32x4 cw = c, gw = g;
      const uint32_t idx = idx0 + lane_id() * EPV;
      LaneAcc l{0, 0xFFFFFFFFu, 0.0};
#pragma unroll 1
      for (uint32_t e = 0; e < (uint32_t)N; ++e) {
        const uint64_t ce = pop_elem<DT>(cw), ge = pop_elem<DT>(gw);
        full_rules(ce != ge, to_f64_t<DT>(ce), to_f64_t<DT>(ge), Elem<DT>::is_float, idx + e, k, a, l);
      }
      fold_lanes(a, l);
      return;
    }
  }
  // Every error here is finite, so both inputs are finite and the plain predicate applies.
  // Mismatches are counted for the whole wavefront at once from the lane masks.
  uint64_t m[N];
  if (k.tol) {
#pragma unroll
    for (int e = 0; e < N; ++e) {
      const double rt = k.rtol * aG[e];
      const double thr = k.atol + rt;
      m[e] = __builtin_amdgcn_ballot_w64(__builtin_fabs(t[e]) > thr);
    }
  } else {
#pragma unroll
    for (int e = 0; e < N; ++e) m[e] = __builtin_amdgcn_ballot_w64(elem_bits<DT>(c, e) != elem_bits<DT>(g, e));
  }
  uint64_t any = 0;
#pragma unroll
  for (int e = 0; e < N; ++e) {
    any |= m[e];
    a.wcount += (uint32_t)__builtin_popcountll(m[e]);
    a.max_abs = max_with_abs(a.max_abs, t[e]);
  }
  // The smallest index among them: the lowest lane with a mismatch, its lowest element.  Only
  // looked for while this chunk can still hold a smaller index than the one known.
  if (any != 0 && idx0 < a.wfirst) {
    const uint32_t lane = (uint32_t)__builtin_ctzll(any);
    uint32_t e0 = N - 1;
#pragma unroll
    for (int e = N - 2; e >= 0; --e) e0 = ((m[e] >> lane) & 1) ? (uint32_t)e : e0;
    const uint32_t cand = idx0 + lane * EPV + e0;
    a.wfirst = cand < a.wfirst ? cand : a.wfirst;
  }
  // The quotients that may raise max_rel, one per lane and round (usually one round).
  if (__builtin_amdgcn_ballot_w64(pend != 0) != 0) {
    LaneAcc l{0, 0xFFFFFFFFu, 0.0};
    do {
      if (pend != 0) {
        const uint32_t e = (uint32_t)__builtin_ctz(pend);
        pend &= pend - 1;
        double tt = t[0], gg = aG[0];
#pragma unroll
        for (int j = 1; j < N; ++j) {
          tt = e == (uint32_t)j ? t[j] : tt;
          gg = e == (uint32_t)j ? aG[j] : gg;
        }
        const double dd = __builtin_fabs(tt);
        if (may_raise_max_rel(dd, gg, lane_top(a, l))) raise_max_rel(dd, gg, l);
      }
    } while (__builtin_amdgcn_ballot_w64(pend != 0) != 0);
    fold_lanes(a, l);
  }
}

// ---- 1-byte elements: the same chunk in integer arithmetic -----------------------------
// With C, G in 0..255 everything is exact in small integers: d = |C - G|, and both tests of
// an element are comparisons of d with a function of G alone, read from a 256-entry table
// that the wavefront keeps in LDS (one 32-bit word per entry, T in the low half and Q in the
// high half, so that each comparison reads its half of the word in place):
//   T[G] = min(255, floor(atol + fl(rtol*G)))      mismatch under tolerance  <=>  d > T[G]
//          (binary64, the two roundings of the rule; d is an integer, so d > thr <=> d > floor(thr);
//          T[G] = 0 in bitwise mode, where any difference is a mismatch)
//   Q[G] = min(255, floor(F * max(G, 1) / 2^16)),  F = floor(top * 2^16)
//          d <= Q[G]  =>  d * 2^16 <= F * G  =>  d/G <= top: the quotient cannot raise max_rel.
//          G == 0 (no relative error by rule) is entered as G = 1, which flags it only when d
//          itself exceeds top.
// Elements with d > Q[G] take the exact test and the divide like those of every other type.
// The table is rebuilt when top has changed (a few times per tile).
__device__ __forceinline__ void build_byte_table(const ElemKind& k, Acc& a) {
  if (a.lut_ready && a.lut_fix == a.tq_fix) return;
  const uint32_t lane = lane_id();
  uint32_t entry[4];
#pragma unroll
  for (uint32_t j = 0; j < 4; ++j) {
    const uint32_t gi = 4 * lane + j;
    const double G = (double)gi;
    const double rt = k.rtol * G;
    const double thr = k.atol + rt;
    // thr >= 0: truncation is floor.  Bitwise mode: T = 0, any difference is a mismatch.
    const uint32_t T = !k.tol ? 0u : thr >= 255.0 ? 255u : (uint32_t)thr;
    const uint64_t q = ((uint64_t)a.tq_fix * (gi > 1u ? gi : 1u)) >> 16;
    const uint32_t Q = q > 255u ? 255u : (uint32_t)q;
    entry[j] = T | (Q << 16);
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // earlier reads of the table are done
  *(u32x4*)(k.lut + 4 * lane) = u32x4{entry[0], entry[1], entry[2], entry[3]};
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  a.lut_ready = 1;
  a.lut_fix = a.tq_fix;
}

template <int N>  // the first N (<= 8) bytes of c and g
__device__ __forceinline__ void compare_chunk_u8(const u32x4& c, const u32x4& g, uint32_t idx0,
                                                 const ElemKind& k, Acc& a) {
  constexpr uint32_t EPV = 16;
  uint32_t ge[N], d[N], tv[N];
  uint64_t m[N];
  const uint32_t* lut = k.lut;
  build_byte_table(k, a);
#pragma unroll
  for (int e = 0; e < N; ++e) {
    const uint32_t ce = (c[e >> 2] >> (8 * (e & 3))) & 0xFFu;
    ge[e] = (g[e >> 2] >> (8 * (e & 3))) & 0xFFu;
    d[e] = __builtin_amdgcn_sad_u8(ce, ge[e], 0u);  // |ce - ge|: the upper bytes of both are zero
    a.imax = d[e] > a.imax ? d[e] : a.imax;
  }
#pragma unroll
  for (int e = 0; e < N; ++e) tv[e] = lut[ge[e]];  // all table reads first: one wait for the N of them
  uint64_t any = 0, any_rel = 0;
#pragma unroll
  for (int e = 0; e < N; ++e) {
    m[e] = __builtin_amdgcn_ballot_w64(d[e] > (tv[e] & 0xFFFFu));
    any_rel |= __builtin_amdgcn_ballot_w64(d[e] > (tv[e] >> 16));
    any |= m[e];
    a.wcount += (uint32_t)__builtin_popcountll(m[e]);
  }
  if (any != 0 && idx0 < a.wfirst) {
    const uint32_t lane = (uint32_t)__builtin_ctzll(any);
    uint32_t e0 = N - 1;
#pragma unroll
    for (int e = N - 2; e >= 0; --e) e0 = ((m[e] >> lane) & 1) ? (uint32_t)e : e0;
    const uint32_t cand = idx0 + lane * EPV + e0;
    a.wfirst = cand < a.wfirst ? cand : a.wfirst;
  }
  if (any_rel != 0) {
    uint32_t pend = 0;
#pragma unroll
    for (int e = 0; e < N; ++e) pend |= d[e] > (tv[e] >> 16) ? (1u << e) : 0u;
    LaneAcc l{0, 0xFFFFFFFFu, 0.0};
    do {
      if (pend != 0) {
        const uint32_t e = (uint32_t)__builtin_ctz(pend);
        pend &= pend - 1;
        uint32_t di = d[0], gi = ge[0];
#pragma unroll
        for (int j = 1; j < N; ++j) {
          di = e == (uint32_t)j ? d[j] : di;
          gi = e == (uint32_t)j ? ge[j] : gi;
        }
        const double dd = (double)di, gg = (double)gi;
        if (may_raise_max_rel(dd, gg, lane_top(a, l))) raise_max_rel(dd, gg, l);
      }
    } while (__builtin_amdgcn_ballot_w64(pend != 0) != 0);
    fold_lanes(a, l);
  }
}

// One whole vector per lane; idx0 = tile index of the first element of lane 0's vector.  The
// chunks of a vector go through one copy of the code.
template <int DT>
__device__ __forceinline__ void compare_vector(u32x4 c, u32x4 g, uint32_t idx0, const ElemKind& k, Acc& a) {
  constexpr int ES = Elem<DT>::size;
  constexpr int N = ES == 8 ? 2 : ES == 4 ? 4 : 8;  // elements per chunk
  constexpr int CHUNKS = 16 / (ES * N);             // 2 for 1-byte elements, else 1
  if constexpr (CHUNKS == 1) {
    compare_chunk<DT, N>(c, g, idx0, k, a);
  } else {
#pragma unroll 1
    for (uint32_t j = 0; j < (uint32_t)CHUNKS; ++j) {
      compare_chunk_u8<N>(c, g, idx0 + j * N, k, a);
      drop_front<ES * N>(c);
      drop_front<ES * N>(g);
    }
  }
}

__device__ __forceinline__ uint64_t load_word_any(const uint8_t* p, uint32_t valid, uint32_t es) {
  switch (es) {
    case 1: return load_word<1>(p, valid);
    case 2: return load_word<2>(p, valid);
    case 4: return load_word<4>(p, valid);
    default: return load_word<8>(p, valid);
  }
}

__device__ __forceinline__ uint32_t vec_diff(u32x4 c, u32x4 g) {
  return (c.x ^ g.x) | (c.y ^ g.y) | (c.z ^ g.z) | (c.w ^ g.w);
}

// The whole 16-byte vectors of an aligned tile: nvec vectors at C / G, vector v belongs to
// lane v % 64.  key = checksum key of this lane's first word.  The last round may be short:
// its missing vectors read as zeros on both sides and take no part in the checksum.
template <int DT>
__device__ __forceinline__ void compare_vectors(const u32x4* C, const u32x4* G, uint32_t nvec,
                                                uint64_t key, const ElemKind& k, uint32_t lane, Acc& a) {
  constexpr uint32_t EPV = 16 / Elem<DT>::size;  // elements per vector
  constexpr uint32_t kRound = 64 * kUnroll;      // vectors per round of the wavefront
  uint32_t v = lane;
  uint32_t v0 = 0;  // the vector lane 0 starts this round with (uniform)
  const uint32_t nfull = nvec / kRound;
  const uint32_t rounds = (nvec + kRound - 1) / kRound;
  for (uint32_t it = 0; it < rounds; ++it) {
    u32x4 c[kUnroll], g[kUnroll];
    uint32_t diff = 0;
    if (it < nfull) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        c[u] = __builtin_nontemporal_load(C + v + 64 * u);
        g[u] = __builtin_nontemporal_load(G + v + 64 * u);
      }
      // Fast path: checksum every vector, gather one "something differs" flag.
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const uint64_t ku = key + (uint64_t)u * kVecKeyStep;
        a.cks += cks_term(c[u].x, c[u].y, ku);
        a.cks += cks_term(c[u].z, c[u].w, ku + kPhi);
        diff |= vec_diff(c[u], g[u]);
      }
    } else {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        c[u] = u32x4{0, 0, 0, 0};
        g[u] = u32x4{0, 0, 0, 0};
        if (v + 64 * u < nvec) {
          c[u] = __builtin_nontemporal_load(C + v + 64 * u);
          g[u] = __builtin_nontemporal_load(G + v + 64 * u);
          const uint64_t ku = key + (uint64_t)u * kVecKeyStep;
          a.cks += cks_term(c[u].x, c[u].y, ku);
          a.cks += cks_term(c[u].z, c[u].w, ku + kPhi);
        }
        diff |= vec_diff(c[u], g[u]);
      }
    }
    if (__builtin_amdgcn_ballot_w64(diff != 0) != 0) {
      // Each vector has its own copy of the chunk code (no register-indexed copies of the
      // loaded vectors); the element-by-element careful path inside stays a rolled loop, so
      // one element type's path is about 14 KB of the instruction cache.
#pragma unroll
      for (uint32_t u = 0; u < (uint32_t)kUnroll; ++u) {
        const u32x4 cc = c[u], gg = g[u];
        if (__builtin_amdgcn_ballot_w64(vec_diff(cc, gg) != 0) != 0)
          compare_vector<DT>(cc, gg, (v0 + 64 * u) * EPV, k, a);
      }
    }
    v += kRound;
    v0 += kRound;
    key += (uint64_t)kUnroll * kVecKeyStep;
  }
}

__device__ __forceinline__ void compare_tile(const uint8_t* cbase, const uint8_t* gbase, uint32_t len,
                                             uint64_t word0, const ElemKind& k, uint32_t lane, Acc& a) {
  const uint32_t epw = 8 / k.es;
  uint32_t first_word = 0;  // where the word-by-word loop below starts
  if (((uintptr_t)cbase & 15) == 0) {
    const u32x4* C = (const u32x4*)cbase;
    const u32x4* G = (const u32x4*)gbase;
    const uint32_t nvec = len >> 4;
    const uint64_t key = (word0 + 2ull * lane + 1) * kPhi;
    switch (k.dtype) {  // uniform across the wavefront
      case R3_U8: compare_vectors<R3_U8>(C, G, nvec, key, k, lane, a); break;
      case R3_F32: compare_vectors<R3_F32>(C, G, nvec, key, k, lane, a); break;
      case R3_F64: compare_vectors<R3_F64>(C, G, nvec, key, k, lane, a); break;
      case R3_I32: compare_vectors<R3_I32>(C, G, nvec, key, k, lane, a); break;
      case R3_BF16: compare_vectors<R3_BF16>(C, G, nvec, key, k, lane, a); break;
      default: compare_vectors<R3_F16>(C, G, nvec, key, k, lane, a); break;
    }
    first_word = 2 * nvec;  // what is left: fewer than 16 bytes at the end of a region
  }
  // Word by word: the whole tile when the region does not start on a 16-byte boundary,
  // otherwise only the last one or two words of a region whose size is not a multiple of 16.
  const uint32_t nwords = (len + 7) >> 3;
  const uint32_t trips = (nwords - first_word + 63) >> 6;
  uint32_t j = first_word + lane;
  LaneAcc l{0, 0xFFFFFFFFu, 0.0};
  for (uint32_t it = 0; it < trips; ++it, j += 64) {
    if (j < nwords) {
      const uint32_t at = 8 * j;
      const uint32_t valid = (len - at) < 8 ? (len - at) : 8;
      const uint64_t wc = load_word_any(cbase + at, valid, k.es);
      const uint64_t wg = load_word_any(gbase + at, valid, k.es);
      a.cks += cks_term((uint32_t)wc, (uint32_t)(wc >> 32), (word0 + j + 1) * kPhi);
      differing_word(wc, wg, valid / k.es, j * epw, k, a, l);
    }
    // share the relative error found so far: it spares the later words their divides
    if (__builtin_amdgcn_ballot_w64(l.max_rel > bits_d(a.top_bits)) != 0)
      raise_top(a, bits_d(dpp_max(dbits(l.max_rel))));
  }
  if (trips) fold_lanes(a, l);
}

// Validate one tile and leave its partial at *dst (all 64 lanes of the wavefront take part).
__device__ __forceinline__ void compare_tile_to_partial(const TileView& tv, const uint8_t* live,
                                                        const uint8_t* golden, Partial* dst) {
  const uint64_t at = tv.offset + tv.rel_start;
  const uint64_t word0 = tv.rel_start >> 3;
  const uint32_t lane = lane_id();
  ElemKind k;
  k.dtype = tv.dtype;
  k.es = elem_size_dev(tv.dtype);
  k.is_float = tv.dtype == R3_F32 || tv.dtype == R3_F64 || tv.dtype == R3_BF16 || tv.dtype == R3_F16;
  k.tol = tv.mode == R3_CMP_TOL;
  k.rtol = tv.rtol;
  k.atol = tv.atol;
  __shared__ uint32_t lut[kWavesPerBlock][256];
  k.lut = lut[wave_in_block()];
  Acc a;
  a.tq_fix = 0;
  // rtol * (1 - 2^-50), rounded: at most rtol * (1 - 2^-51).  Tiny rtol: only top == 0 counts.
  a.rtol_cut = !k.tol ? -1.0 : k.rtol >= kTopFloor ? k.rtol - k.rtol * 0x1p-50 : 0.0;
  a.within = k.tol ? 1u : 0u;  // top starts at 0
  a.lut_ready = 0;
  a.lut_fix = 0;
  a.imax = 0;
  a.wcount = 0;
  a.wfirst = 0xFFFFFFFFu;
  a.top_bits = 0;
  a.tq_bits = 0;
  a.max_abs = 0.0;
  a.cks = 0;
  compare_tile(live + at, golden + at, tv.len, word0, k, lane, a);
  // Fold the two per-lane values.  A tile in which nothing differed (the usual case) only
  // has a checksum to add up.
  const uint64_t cks = dpp_sum(a.cks);
  uint64_t max_abs = 0;
  const double lane_abs = (double)a.imax > a.max_abs ? (double)a.imax : a.max_abs;
  if (__builtin_amdgcn_ballot_w64(dbits(lane_abs) != 0) != 0) max_abs = dpp_max(dbits(lane_abs));
  const uint64_t count = a.wcount;
  const uint64_t first_elem = a.wfirst != 0xFFFFFFFFu ? tv.rel_start / k.es + a.wfirst : R3_NO_INDEX;
  const uint64_t max_rel = a.top_bits;
  uint64_t* out = (uint64_t*)dst;
  if (lane < 5) {
    const uint64_t val = lane == 0 ? count : lane == 1 ? first_elem : lane == 2 ? max_abs
                       : lane == 3 ? max_rel : cks;
    out[lane] = val;
  }
}

__global__ __launch_bounds__(kBlock) void compare_kernel(TableDev t, const uint8_t* live,
                                                         const uint8_t* golden) {
  const uint64_t tile_id = (uint64_t)blockIdx.x * kWavesPerBlock + wave_in_block();
  if (tile_id >= t.n_tiles) return;
  const TileView tv = resolve_tile(t, tile_id);
  compare_tile_to_partial(tv, live, golden, &t.partials[tile_id]);
}

// One block per region folds that region's partials into its r3_region_result.  The table
// summary goes to `summary` (device) and, when given, to `host_slot` (pinned host memory
// mapped into the device's address space) followed by its sequence number, which saves the
// caller a copy and lets it poll for the verdict instead of waiting for the stream.
struct Folded {
  uint64_t count, first, max_abs, max_rel, cks;
};

__device__ __forceinline__ void publish_seq(HostSlot* slot, uint64_t seq) {
  __threadfence_system();  // the summary is in host memory before its sequence number
  __hip_atomic_store(&slot->seq, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__device__ __forceinline__ void write_summary(r3_summary* dst, uint64_t total, uint32_t first_region,
                                              uint64_t first_index, uint64_t max_abs,
                                              uint64_t max_rel) {
  dst->total_mismatch = total;
  dst->first_index = first_index;
  dst->first_region = first_region;
  dst->pass = total == 0 ? 1u : 0u;
  dst->max_abs_err = bits_d(max_abs);
  dst->max_rel_err = bits_d(max_rel);
}

// Fold partials [b, e) with one block; the result is complete in thread 0.
template <int BLOCK>
__device__ __forceinline__ Folded fold_partials(const Partial* partials, uint64_t b, uint64_t e,
                                                uint64_t (*sh)[BLOCK / 64]) {
  constexpr int NW = BLOCK / 64;
  constexpr int kAhead = 8;  // partials fetched per thread before any is folded
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  Folded f{0, R3_NO_INDEX, 0, 0, 0};
  for (uint64_t i = b + tid; i < e; i += (uint64_t)BLOCK * kAhead) {
    uint64_t v[kAhead][5];
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      const uint64_t idx = i + (uint64_t)u * BLOCK;
      if (idx < e) {
        const uint64_t* p = (const uint64_t*)&partials[idx];
#pragma unroll
        for (int k = 0; k < 5; ++k) v[u][k] = p[k];
      } else {
        v[u][0] = 0; v[u][1] = R3_NO_INDEX; v[u][2] = 0; v[u][3] = 0; v[u][4] = 0;
      }
    }
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      f.count += v[u][0];
      f.first = v[u][1] < f.first ? v[u][1] : f.first;
      f.max_abs = v[u][2] > f.max_abs ? v[u][2] : f.max_abs;
      f.max_rel = v[u][3] > f.max_rel ? v[u][3] : f.max_rel;
      f.cks += v[u][4];
    }
  }
  f.count = dpp_sum(f.count);
  f.first = dpp_min(f.first);
  f.max_abs = dpp_max(f.max_abs);
  f.max_rel = dpp_max(f.max_rel);
  f.cks = dpp_sum(f.cks);
  if (NW > 1) {
    if (lane == 0) {
      sh[0][wave] = f.count; sh[1][wave] = f.first; sh[2][wave] = f.max_abs;
      sh[3][wave] = f.max_rel; sh[4][wave] = f.cks;
    }
    __syncthreads();
    if (wave == 0) {  // the first wavefront folds the per-wavefront values, again over DPP
      const bool on = lane < (uint32_t)NW;
      const uint64_t zero = 0, none = R3_NO_INDEX;
      f.count = dpp_sum((uint64_t)(on ? sh[0][lane] : zero));
      f.first = dpp_min((uint64_t)(on ? sh[1][lane] : none));
      f.max_abs = dpp_max((uint64_t)(on ? sh[2][lane] : zero));
      f.max_rel = dpp_max((uint64_t)(on ? sh[3][lane] : zero));
      f.cks = dpp_sum((uint64_t)(on ? sh[4][lane] : zero));
    }
  }
  return f;
}

__device__ __forceinline__ void write_region_result(r3_region_result* dst, const Folded& f,
                                                    uint64_t region_bytes) {
  uint64_t* o = (uint64_t*)dst;
  o[0] = f.count;
  o[1] = f.first;
  o[2] = f.max_abs;
  o[3] = f.max_rel;
  o[4] = f.cks + region_bytes * kLen;
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void compare_finalize_kernel(TableDev t, r3_region_result* out,
                                                                 r3_summary* summary,
                                                                 HostSlot* host_slot, uint64_t host_seq,
                                                                 const uint32_t* rep_counter) {
  __shared__ uint64_t sh[5][BLOCK / 64];
  const uint32_t r = blockIdx.x;
  const uint32_t tid = threadIdx.x;
  const Folded f = fold_partials<BLOCK>(t.partials, t.tile_begin[r], t.tile_begin[r + 1], sh);
  if (tid == 0) write_region_result(&out[r], f, t.regions[r].bytes);
  // A table of one region: its result is the summary.  Larger tables get their summary from
  // summary_kernel, a separate launch: folding it in here through a "last block" ticket
  // needs a device-wide release fence per block, which cost 37 ns per region (150 us for
  // 4096 regions) when measured.
  if (gridDim.x == 1 && tid == 0 && (summary != nullptr || host_slot != nullptr)) {
    const uint32_t fr = f.count ? 0u : R3_NO_REGION;
    const uint64_t fi = f.count ? f.first : R3_NO_INDEX;
    if (summary) write_summary(summary, f.count, fr, fi, f.max_abs, f.max_rel);
    if (host_slot) {
      // inside a captured replay the slot and sequence number advance with the replay count
      const uint32_t k = rep_counter ? *rep_counter - 1 : 0;
      write_summary(&host_slot[k].summary, f.count, fr, fi, f.max_abs, f.max_rel);
      publish_seq(host_slot + k, host_seq + k);
    }
  }
}

// ---- validation without a table object or a caller workspace (r3_compare_static) -------
// The partials of these launches live in the library's device image.  In host code the
// array's name is only a handle for hipGetSymbolAddress; kernels get the resolved address.
static __device__ __align__(256) unsigned char scratch[(size_t)R3_STATIC_MAX_TILES * sizeof(Partial)];

__global__ __launch_bounds__(kBlock) void compare_static_kernel(StaticTable st, const uint8_t* live,
                                                                const uint8_t* golden, Partial* partials) {
  const uint32_t tile_id = blockIdx.x * kWavesPerBlock + wave_in_block();
  if (tile_id >= st.tile_begin[st.n]) return;
  uint32_t r = 0;  // the region whose tile range holds tile_id (empty regions are skipped)
  while (r + 1 < st.n && tile_id >= st.tile_begin[r + 1]) ++r;
  r = sgpr(r);
  const r3_region& rg = st.regions[r];
  TileView tv;
  tv.region = r;
  tv.offset = rg.offset;
  tv.bytes = rg.bytes;
  tv.dtype = rg.dtype;
  tv.mode = rg.mode;
  tv.rtol = rg.rtol;
  tv.atol = rg.atol;
  tv.rel_start = (uint64_t)(tile_id - st.tile_begin[r]) << st.shift;
  const uint64_t left = tv.bytes - tv.rel_start, full = 1ull << st.shift;
  tv.len = (uint32_t)(left < full ? left : full);
  compare_tile_to_partial(tv, live, golden, &partials[tile_id]);
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void compare_static_finalize_kernel(StaticTable st,
                                                                        const Partial* partials,
                                                                        r3_region_result* out,
                                                                        r3_summary* summary) {
  __shared__ uint64_t sh[5][BLOCK / 64];
  const uint32_t r = blockIdx.x;
  const Folded f = fold_partials<BLOCK>(partials, st.tile_begin[r], st.tile_begin[r + 1], sh);
  if (threadIdx.x == 0) {
    write_region_result(&out[r], f, st.regions[r].bytes);
    if (gridDim.x == 1 && summary != nullptr)
      write_summary(summary, f.count, f.count ? 0u : R3_NO_REGION, f.count ? f.first : R3_NO_INDEX,
                    f.max_abs, f.max_rel);
  }
}

// Table verdict from the per-region results (one block; runs after the finalize launch).
__global__ __launch_bounds__(kBlock) void summary_kernel(const r3_region_result* out, uint32_t n,
                                                         r3_summary* summary, HostSlot* host_slot,
                                                         uint64_t host_seq, const uint32_t* rep_counter) {
  __shared__ uint64_t sh[3][kWavesPerBlock];
  __shared__ uint32_t sh_first_region[kWavesPerBlock];
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint64_t total = 0, max_abs = 0, max_rel = 0;
  uint32_t first_region = R3_NO_REGION;
  for (uint32_t i = tid; i < n; i += kBlock) {
    const uint64_t* o = (const uint64_t*)&out[i];
    const uint64_t cnt = o[0], ma = o[2], mr = o[3];
    total += cnt;
    if (cnt != 0 && i < first_region) first_region = i;
    max_abs = ma > max_abs ? ma : max_abs;
    max_rel = mr > max_rel ? mr : max_rel;
  }
  total = wave_sum(total);
  first_region = wave_min(first_region);
  max_abs = wave_max(max_abs);
  max_rel = wave_max(max_rel);
  if (lane == 0) {
    sh[0][wave] = total; sh[1][wave] = max_abs; sh[2][wave] = max_rel;
    sh_first_region[wave] = first_region;
  }
  __syncthreads();
  if (tid == 0) {
    total = 0; max_abs = 0; max_rel = 0; first_region = R3_NO_REGION;
    for (int w = 0; w < kWavesPerBlock; ++w) {
      total += sh[0][w];
      max_abs = sh[1][w] > max_abs ? sh[1][w] : max_abs;
      max_rel = sh[2][w] > max_rel ? sh[2][w] : max_rel;
      first_region = sh_first_region[w] < first_region ? sh_first_region[w] : first_region;
    }
    const uint64_t first_index = first_region == R3_NO_REGION ? R3_NO_INDEX : out[first_region].first_mismatch;
    if (summary) write_summary(summary, total, first_region, first_index, max_abs, max_rel);
    if (host_slot) {
      const uint32_t k = rep_counter ? *rep_counter - 1 : 0;
      write_summary(&host_slot[k].summary, total, first_region, first_index, max_abs, max_rel);
      publish_seq(host_slot + k, host_seq + k);
    }
  }
}

// =======================================================================================
// Page dirty-diff
// =======================================================================================
// One wavefront owns 16 consecutive pages (one 16-bit slice of a bitmap word) and ORs the
// per-page "differs" flags of its lanes.  vec_shift = log2(page_bytes / 16).
__global__ __launch_bounds__(kBlock) void dirty_diff_kernel(const uint8_t* pre, const uint8_t* post,
                                                            uint64_t bytes, uint32_t page_shift,
                                                            uint16_t* bitmap16, uint64_t n_slices) {
  const uint64_t slice = (uint64_t)blockIdx.x * kWavesPerBlock + wave_in_block();
  if (slice >= n_slices) return;
  const uint32_t lane = lane_id();
  const uint64_t span_start = (slice * 16) << page_shift;
  uint32_t bits = 0;
  if (span_start < bytes) {
    const uint64_t span_full = 16ull << page_shift;
    const uint64_t left = bytes - span_start;
    const uint64_t span = left < span_full ? left : span_full;
    const u32x4* A = (const u32x4*)(pre + span_start);
    const u32x4* B = (const u32x4*)(post + span_start);
    const uint32_t vec_shift = page_shift - 4;
    const uint32_t nvec = (uint32_t)(span >> 4);
    uint32_t v = lane;
    const uint32_t nfull = nvec / (64 * kUnroll);
    for (uint32_t it = 0; it < nfull; ++it) {
      u32x4 a[kUnroll], b[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        a[u] = __builtin_nontemporal_load(A + v + 64 * u);
        b[u] = __builtin_nontemporal_load(B + v + 64 * u);
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const uint32_t d = (a[u].x ^ b[u].x) | (a[u].y ^ b[u].y) | (a[u].z ^ b[u].z) | (a[u].w ^ b[u].w);
        bits |= (d != 0 ? 1u : 0u) << ((v + 64 * u) >> vec_shift);
      }
      v += 64 * kUnroll;
    }
    for (; v < nvec; v += 64) {
      const u32x4 a = __builtin_nontemporal_load(A + v), b = __builtin_nontemporal_load(B + v);
      const uint32_t d = (a.x ^ b.x) | (a.y ^ b.y) | (a.z ^ b.z) | (a.w ^ b.w);
      bits |= (d != 0 ? 1u : 0u) << (v >> vec_shift);
    }
    // Bytes after the last whole vector (only at the very end of the state).
    const uint32_t done = nvec << 4;
    const uint32_t tail = (uint32_t)(span - done);
    if (lane < tail) {
      const uint32_t at = done + lane;
      bits |= (pre[span_start + at] != post[span_start + at] ? 1u : 0u) << (at >> page_shift);
    }
  }
  bits = wave_or(bits);
  if (lane == 0) bitmap16[slice] = (uint16_t)bits;
}

__global__ __launch_bounds__(1024) void popcount_kernel(const uint64_t* bitmap, uint64_t n_words,
                                                        uint64_t* count) {
  __shared__ uint64_t sh[16];
  uint64_t acc = 0;
  for (uint64_t i = threadIdx.x; i < n_words; i += 1024 * 4) {  // four loads in flight
    uint64_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint64_t idx = i + (uint64_t)u * 1024;
      v[u] = idx < n_words ? bitmap[idx] : 0;
    }
    acc += __popcll(v[0]) + __popcll(v[1]) + __popcll(v[2]) + __popcll(v[3]);
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    acc = 0;
    for (int w = 0; w < 16; ++w) acc += sh[w];
    *count = acc;
  }
}

// Guard check: how many of n checksums differ from the recorded ones, and the first such
// region; one block, result straight into pinned host memory.
__global__ __launch_bounds__(kBlock) void guard_compare_kernel(const uint64_t* got,
                                                               const uint64_t* expected, uint32_t n,
                                                               GuardSlot* host_slot, uint64_t host_seq) {
  __shared__ uint32_t sh_count[kWavesPerBlock], sh_first[kWavesPerBlock];
  uint32_t count = 0, first = R3_NO_REGION;
  for (uint32_t i = threadIdx.x; i < n; i += kBlock) {
    if (got[i] != expected[i]) {
      ++count;
      first = i < first ? i : first;
    }
  }
  count = wave_sum(count);
  first = wave_min(first);
  if ((threadIdx.x & 63) == 0) {
    sh_count[threadIdx.x >> 6] = count;
    sh_first[threadIdx.x >> 6] = first;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    count = 0;
    first = R3_NO_REGION;
    for (int w = 0; w < kWavesPerBlock; ++w) {
      count += sh_count[w];
      first = sh_first[w] < first ? sh_first[w] : first;
    }
    host_slot->changed = count;
    host_slot->first_region = first;
    __threadfence_system();
    __hip_atomic_store(&host_slot->seq, host_seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}

// Time stamps around the candidate inside a captured replay.  `which` 0: take the next replay
// number (the counter advances) and stamp its start; 1: stamp its end.  The stamps go to
// pinned host memory, the counter lives in device memory.
__global__ void stamp_kernel(uint32_t* rep_counter, uint64_t* stamps, uint32_t which) {
  if (threadIdx.x == 0) {
    uint32_t k;
    if (which == 0) {
      k = *rep_counter;
      *rep_counter = k + 1;
    } else {
      k = *rep_counter - 1;
    }
    stamps[2 * k + which] = wall_clock64();
  }
}

__global__ void set_counter_kernel(uint32_t* rep_counter, uint32_t value) {
  if (threadIdx.x == 0) *rep_counter = value;
}

uint32_t grid_for(uint64_t tiles) { return (uint32_t)((tiles + kWavesPerBlock - 1) / kWavesPerBlock); }

}  // namespace

// Bytes one wavefront copies (log2) and threads per block of the copy kernels.  Measured on
// MI355X (restore of 2 x 128 MiB / 4 x 2 GiB): 1 KiB per wavefront in 64-thread blocks 6.6
// TB/s, 4 KiB in 256-thread blocks 6.2 / 5.8 TB/s, 8 KiB 6.1 / 5.3 TB/s.
static uint32_t g_copy_shift = 10;
static uint32_t g_copy_block = 64;

void set_copy_shape(uint32_t shift, uint32_t block) {
  g_copy_shift = shift;
  g_copy_block = block;
}

hipError_t launch_restore(const TableDev& t, const uint32_t* class_count, const void* src, void* dst,
                          hipStream_t s) {
  if (t.n_tiles == 0) return hipSuccess;
  const uint32_t cs = g_copy_shift, wpb = g_copy_block / 64;
  CopyClasses cls{};
  cls.n = t.max_shift - t.min_shift + 1;
  uint64_t slots = 0;
  uint32_t first = 0;
  for (uint32_t c = 0; c < cls.n; ++c) {
    const uint32_t shift = t.min_shift + c;
    cls.sub_log2[c] = shift > cs ? shift - cs : 0;
    cls.first[c] = first;
    cls.slot_base[c] = slots;
    slots += (uint64_t)class_count[c] << cls.sub_log2[c];
    first += class_count[c];
  }
  cls.slot_base[cls.n] = slots;
  const uint64_t blocks = (slots + wpb - 1) / wpb;
  if (blocks > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
  const uint8_t* a = (const uint8_t*)src;
  uint8_t* b = (uint8_t*)dst;
  // a table with a single size class (the common case) is resolved from the plain arguments
  uint32_t used = 0, only = 0;
  for (uint32_t c = 0; c < cls.n; ++c)
    if (class_count[c]) {
      ++used;
      only = c;
    }
  const uint32_t n_classes = used <= 1 ? 1 : cls.n;
  const uint32_t sub0 = used <= 1 ? cls.sub_log2[only] : 0;
  switch (g_copy_block) {
    case 64: restore_kernel<64><<<(uint32_t)blocks, 64, 0, s>>>(t, a, b, cs, n_classes, sub0, slots, cls); break;
    case 128: restore_kernel<128><<<(uint32_t)blocks, 128, 0, s>>>(t, a, b, cs, n_classes, sub0, slots, cls); break;
    default: restore_kernel<256><<<(uint32_t)blocks, 256, 0, s>>>(t, a, b, cs, n_classes, sub0, slots, cls); break;
  }
  return hipGetLastError();
}

hipError_t launch_copy_flat(const void* src, void* dst, uint64_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  const uint32_t cs = g_copy_shift, wpb = g_copy_block / 64;
  const uint64_t n_slots = (bytes + ((1ull << cs) - 1)) >> cs;
  const uint64_t blocks = (n_slots + wpb - 1) / wpb;
  if (blocks > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
  const uint8_t* a = (const uint8_t*)src;
  uint8_t* b = (uint8_t*)dst;
  switch (g_copy_block) {
    case 64: copy_flat_kernel<64><<<(uint32_t)blocks, 64, 0, s>>>(a, b, bytes, n_slots, cs); break;
    case 128: copy_flat_kernel<128><<<(uint32_t)blocks, 128, 0, s>>>(a, b, bytes, n_slots, cs); break;
    default: copy_flat_kernel<256><<<(uint32_t)blocks, 256, 0, s>>>(a, b, bytes, n_slots, cs); break;
  }
  return hipGetLastError();
}

static int finalize_block(uint32_t max_region_tiles) {
  return max_region_tiles <= 64 * 4 ? 64 : max_region_tiles <= 256 * 8 ? 256 : 1024;
}

hipError_t launch_checksum(const TableDev& t, const void* arena, uint64_t* out, hipStream_t s) {
  if (t.n_tiles) {
    checksum_kernel<<<grid_for(t.n_tiles), kBlock, 0, s>>>(t, (const uint8_t*)arena);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  switch (finalize_block(t.max_region_tiles)) {
    case 64: checksum_finalize_kernel<64><<<t.n_regions, 64, 0, s>>>(t, out); break;
    case 256: checksum_finalize_kernel<256><<<t.n_regions, 256, 0, s>>>(t, out); break;
    default: checksum_finalize_kernel<1024><<<t.n_regions, 1024, 0, s>>>(t, out); break;
  }
  return hipGetLastError();
}

hipError_t launch_compare(const TableDev& t, const void* live, const void* golden,
                          r3_region_result* out, r3_summary* summary, HostSlot* host_slot,
                          uint64_t host_seq, const uint32_t* rep_counter, hipStream_t s) {
  if (t.n_tiles) {
    compare_kernel<<<grid_for(t.n_tiles), kBlock, 0, s>>>(t, (const uint8_t*)live,
                                                          (const uint8_t*)golden);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  switch (finalize_block(t.max_region_tiles)) {
    case 64:
      compare_finalize_kernel<64><<<t.n_regions, 64, 0, s>>>(t, out, summary, host_slot, host_seq, rep_counter);
      break;
    case 256:
      compare_finalize_kernel<256><<<t.n_regions, 256, 0, s>>>(t, out, summary, host_slot, host_seq, rep_counter);
      break;
    default:
      compare_finalize_kernel<1024><<<t.n_regions, 1024, 0, s>>>(t, out, summary, host_slot, host_seq, rep_counter);
      break;
  }
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && t.n_regions > 1 && (summary != nullptr || host_slot != nullptr)) {
    summary_kernel<<<1, kBlock, 0, s>>>(out, t.n_regions, summary, host_slot, host_seq, rep_counter);
    e = hipGetLastError();
  }
  return e;
}

hipError_t static_scratch_address(int device, Partial** out) {
  constexpr int kMaxDevices = 64;
  static Partial* resolved[kMaxDevices] = {};  // each GPU holds its own copy at its own address
  *out = nullptr;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  Partial* p = __atomic_load_n(&resolved[device], __ATOMIC_ACQUIRE);
  if (p == nullptr) {
    void* addr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (addr == nullptr) return hipErrorInvalidSymbol;
    p = static_cast<Partial*>(addr);
    __atomic_store_n(&resolved[device], p, __ATOMIC_RELEASE);
  }
  *out = p;
  return hipSuccess;
}

hipError_t launch_compare_static(const StaticTable& st, const void* live, const void* golden,
                                 Partial* scratch_ptr, r3_region_result* out, r3_summary* summary,
                                 hipStream_t s) {
  const uint32_t n_tiles = st.tile_begin[st.n];
  uint32_t max_region_tiles = 0;
  for (uint32_t r = 0; r < st.n; ++r)
    max_region_tiles = std::max(max_region_tiles, st.tile_begin[r + 1] - st.tile_begin[r]);
  if (n_tiles) {
    compare_static_kernel<<<grid_for(n_tiles), kBlock, 0, s>>>(st, (const uint8_t*)live,
                                                               (const uint8_t*)golden, scratch_ptr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  switch (finalize_block(max_region_tiles)) {
    case 64: compare_static_finalize_kernel<64><<<st.n, 64, 0, s>>>(st, scratch_ptr, out, summary); break;
    case 256: compare_static_finalize_kernel<256><<<st.n, 256, 0, s>>>(st, scratch_ptr, out, summary); break;
    default: compare_static_finalize_kernel<1024><<<st.n, 1024, 0, s>>>(st, scratch_ptr, out, summary); break;
  }
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && st.n > 1 && summary != nullptr) {
    summary_kernel<<<1, kBlock, 0, s>>>(out, st.n, summary, nullptr, 0, nullptr);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_stamp(uint32_t* rep_counter, uint64_t* stamps, uint32_t which, hipStream_t s) {
  stamp_kernel<<<1, 64, 0, s>>>(rep_counter, stamps, which);
  return hipGetLastError();
}

hipError_t launch_set_counter(uint32_t* rep_counter, uint32_t value, hipStream_t s) {
  set_counter_kernel<<<1, 64, 0, s>>>(rep_counter, value);
  return hipGetLastError();
}

hipError_t launch_guard_compare(const uint64_t* got, const uint64_t* expected, uint32_t n,
                                GuardSlot* host_slot, uint64_t host_seq, hipStream_t s) {
  guard_compare_kernel<<<1, kBlock, 0, s>>>(got, expected, n, host_slot, host_seq);
  return hipGetLastError();
}

hipError_t launch_dirty_diff(const void* pre, const void* post, uint64_t bytes, uint32_t page_bytes,
                             uint64_t* bitmap, uint64_t* dirty_count, hipStream_t s) {
  uint32_t page_shift = 0;
  while ((1u << page_shift) < page_bytes) ++page_shift;
  const uint64_t n_pages = (bytes + page_bytes - 1) >> page_shift;
  const uint64_t n_words = (n_pages + 63) / 64;
  const uint64_t n_slices = n_words * 4;
  if (n_slices) {
    dirty_diff_kernel<<<grid_for(n_slices), kBlock, 0, s>>>(
        (const uint8_t*)pre, (const uint8_t*)post, bytes, page_shift, (uint16_t*)bitmap, n_slices);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (dirty_count) {
    popcount_kernel<<<1, 1024, 0, s>>>(bitmap, n_words, dirty_count);
    return hipGetLastError();
  }
  return hipSuccess;
}

}  // namespace r3
