/*
 * r3_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, single-threaded CPU statement of what the replay-evaluation path
 * computes: restore a recorded state, validate live memory against the recorded
 * epilogue (Section V-C "Correctness Checking": bitwise by default, optional
 * absolute/relative tolerances on marked variables), checksum a state, and find
 * the pages a kernel wrote (Section V-A: pre- and post-execution state).
 * One element, one word, one page at a time, in the order the definitions are
 * written.  Only tests, the smoke check and the benchmark's CPU-baseline leg may
 * call this; the GPU library shares no code, header or table with it.
 *
 * Floating point: IEEE-754 binary64, round to nearest even, one rounding per
 * written operation.  Build with -ffp-contract=off and without fast-math.
 *
 * Pins (tests/test_oracle_*.py): brute-force big-integer checksum, per-element
 * Python-float compare, numpy.isclose for the tolerance decision, closed forms
 * (self-compare, single planted perturbation, swapped words), byte-flip
 * dirty-diff cases.  The timing fields of an evaluation are measurements:
 * parity unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

enum { O_OK = 0, O_EINVAL = -1, O_EALIGN = -2, O_ERANGE = -3, O_EOVERLAP = -4 };
enum { O_U8 = 0, O_F32 = 1, O_F64 = 2, O_I32 = 3, O_BF16 = 4, O_F16 = 5 };
enum { O_BITWISE = 0, O_TOL = 1 };

typedef struct {
  uint64_t offset, bytes;
  uint32_t dtype, mode;
  double rtol, atol;
} r3o_region;

typedef struct {
  uint64_t mismatch_count, first_mismatch;
  double max_abs_err, max_rel_err;
  uint64_t checksum;
} r3o_region_result;

typedef struct {
  uint64_t total_mismatch, first_index;
  uint32_t first_region, pass;
  double max_abs_err, max_rel_err;
} r3o_summary;

static uint64_t elem_size(uint32_t dtype) {
  switch (dtype) {
    case O_U8: return 1;
    case O_F32: return 4;
    case O_F64: return 8;
    case O_I32: return 4;
    case O_BF16: return 2;
    case O_F16: return 2;
    default: return 0;
  }
}

/* Table rules.  Regions are examined in table order; the first violation
 * decides.  Overlap is examined only after every region passed on its own. */
int r3o_validate_table(const r3o_region* t, uint32_t n, uint64_t arena_bytes) {
  if (t == 0 || n == 0) return O_EINVAL;
  for (uint32_t i = 0; i < n; ++i) {
    uint64_t es = elem_size(t[i].dtype);
    if (es == 0) return O_EINVAL;
    if (t[i].mode != O_BITWISE && t[i].mode != O_TOL) return O_EINVAL;
    if (!(t[i].rtol >= 0.0) || !(t[i].atol >= 0.0)) return O_EINVAL; /* also NaN */
    if (isinf(t[i].rtol) || isinf(t[i].atol)) return O_EINVAL;
    if (t[i].offset % es != 0 || t[i].bytes % es != 0) return O_EALIGN;
    if (t[i].offset > arena_bytes || t[i].bytes > arena_bytes - t[i].offset) return O_ERANGE;
  }
  for (uint32_t i = 0; i < n; ++i)
    for (uint32_t j = i + 1; j < n; ++j) {
      if (t[i].bytes == 0 || t[j].bytes == 0) continue;
      if (t[i].offset < t[j].offset + t[j].bytes && t[j].offset < t[i].offset + t[i].bytes)
        return O_EOVERLAP;
    }
  return O_OK;
}

/* Restore: copy each region of the snapshot over the same span of live memory. */
void r3o_restore(const r3o_region* t, uint32_t n, const uint8_t* snapshot, uint8_t* live) {
  for (uint32_t i = 0; i < n; ++i)
    memcpy(live + t[i].offset, snapshot + t[i].offset, t[i].bytes);
}

/* Order-independent 64-bit checksum of n bytes.
 * Word j is bytes [8j, 8j+8) little-endian, bytes beyond n count as zero. */
uint64_t r3o_checksum_bytes(const uint8_t* p, uint64_t n) {
  const uint64_t PHI = 0x9E3779B97F4A7C15ull;
  const uint64_t LEN = 0xBB67AE8584CAA73Bull;
  uint64_t words = n / 8 + (n % 8 != 0);
  uint64_t sum = 0;
  for (uint64_t j = 0; j < words; ++j) {
    uint64_t w = 0;
    for (unsigned b = 0; b < 8; ++b) {
      uint64_t pos = 8 * j + b;
      if (pos < n) w |= (uint64_t)p[pos] << (8 * b);
    }
    uint64_t k = (j + 1) * PHI;
    uint32_t a = (uint32_t)w + (uint32_t)k;
    uint32_t bb = (uint32_t)(w >> 32) + (uint32_t)(k >> 32);
    sum += (uint64_t)a * (uint64_t)bb;
  }
  return sum + n * LEN;
}

void r3o_checksum_table(const r3o_region* t, uint32_t n, const uint8_t* arena, uint64_t* out) {
  for (uint32_t i = 0; i < n; ++i) out[i] = r3o_checksum_bytes(arena + t[i].offset, t[i].bytes);
}

static double f32_from_bits(uint32_t u) {
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* Element i of a region as (bit pattern, binary64 value, non-finite flag). */
static void load_elem(const uint8_t* base, uint32_t dtype, uint64_t i, uint64_t* bits, double* val,
                      int* nonfinite) {
  *nonfinite = 0;
  switch (dtype) {
    case O_U8: {
      uint8_t v = base[i];
      *bits = v;
      *val = (double)v;
      break;
    }
    case O_I32: {
      int32_t v;
      memcpy(&v, base + 4 * i, 4);
      *bits = (uint32_t)v;
      *val = (double)v;
      break;
    }
    case O_F32: {
      uint32_t u;
      memcpy(&u, base + 4 * i, 4);
      *bits = u;
      *val = f32_from_bits(u);
      *nonfinite = isnan(*val) || isinf(*val);
      break;
    }
    case O_BF16: {
      uint16_t h;
      memcpy(&h, base + 2 * i, 2);
      *bits = h;
      *val = f32_from_bits((uint32_t)h << 16); /* bf16 is the top half of a binary32 */
      *nonfinite = isnan(*val) || isinf(*val);
      break;
    }
    case O_F16: {
      /* IEEE binary16: 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits.  Every
       * value is exactly representable in binary64. */
      uint16_t h;
      memcpy(&h, base + 2 * i, 2);
      *bits = h;
      int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;
      if (e == 31) {
        *val = m ? NAN : INFINITY;
        *nonfinite = 1;
      } else if (e == 0) {
        *val = ldexp((double)m, -24); /* zero and subnormals: m * 2^-10 * 2^-14 */
      } else {
        *val = ldexp((double)(1024 + m), e - 25); /* (1 + m/1024) * 2^(e-15) */
      }
      if (sign) *val = -*val;
      break;
    }
    default: { /* O_F64 */
      uint64_t u;
      memcpy(&u, base + 8 * i, 8);
      *bits = u;
      memcpy(val, &u, 8);
      *nonfinite = isnan(*val) || isinf(*val);
      break;
    }
  }
}

/* Validation of one region: c = live element, g = recorded (golden) element. */
void r3o_compare_region(const r3o_region* rg, const uint8_t* live_arena,
                        const uint8_t* golden_arena, r3o_region_result* out) {
  const uint8_t* c_base = live_arena + rg->offset;
  const uint8_t* g_base = golden_arena + rg->offset;
  uint64_t n_elem = rg->bytes / elem_size(rg->dtype);
  uint64_t count = 0, first = UINT64_MAX;
  double max_abs = 0.0, max_rel = 0.0;
  for (uint64_t i = 0; i < n_elem; ++i) {
    uint64_t cb, gb;
    double C, G;
    int cnf, gnf;
    load_elem(c_base, rg->dtype, i, &cb, &C, &cnf);
    load_elem(g_base, rg->dtype, i, &gb, &G, &gnf);
    double d, r;
    int mismatch;
    if (cb == gb) {
      d = 0.0;
      r = 0.0;
      mismatch = 0;
    } else if (cnf || gnf) {
      d = INFINITY;
      r = INFINITY;
      mismatch = 1;
    } else {
      d = fabs(C - G);
      r = (G == 0.0) ? 0.0 : d / fabs(G);
      if (rg->mode == O_BITWISE) {
        mismatch = 1;
      } else {
        double t = rg->rtol * fabs(G);
        double thr = rg->atol + t;
        mismatch = d > thr;
      }
    }
    if (mismatch) {
      ++count;
      if (i < first) first = i;
    }
    if (d > max_abs) max_abs = d;
    if (r > max_rel) max_rel = r;
  }
  out->mismatch_count = count;
  out->first_mismatch = first;
  out->max_abs_err = max_abs;
  out->max_rel_err = max_rel;
  out->checksum = r3o_checksum_bytes(c_base, rg->bytes);
}

void r3o_compare_table(const r3o_region* t, uint32_t n, const uint8_t* live_arena,
                       const uint8_t* golden_arena, r3o_region_result* out) {
  for (uint32_t i = 0; i < n; ++i) r3o_compare_region(&t[i], live_arena, golden_arena, &out[i]);
}

/* Table verdict: totals, the first mismatching region in table order, maxima. */
void r3o_summarize(const r3o_region_result* res, uint32_t n, r3o_summary* s) {
  s->total_mismatch = 0;
  s->first_index = UINT64_MAX;
  s->first_region = UINT32_MAX;
  s->max_abs_err = 0.0;
  s->max_rel_err = 0.0;
  for (uint32_t i = 0; i < n; ++i) {
    s->total_mismatch += res[i].mismatch_count;
    if (res[i].mismatch_count != 0 && s->first_region == UINT32_MAX) {
      s->first_region = i;
      s->first_index = res[i].first_mismatch;
    }
    if (res[i].max_abs_err > s->max_abs_err) s->max_abs_err = res[i].max_abs_err;
    if (res[i].max_rel_err > s->max_rel_err) s->max_rel_err = res[i].max_rel_err;
  }
  s->pass = s->total_mismatch == 0;
}

/* Page write-set: bit p is set iff page p of the two states differs in any
 * valid byte.  bitmap has ceil(ceil(n/page)/64) words and is fully written. */
void r3o_dirty_diff(const uint8_t* pre, const uint8_t* post, uint64_t n, uint64_t page,
                    uint64_t* bitmap, uint64_t* dirty_count) {
  uint64_t npages = n / page + (n % page != 0);
  uint64_t nwords = npages / 64 + (npages % 64 != 0);
  for (uint64_t w = 0; w < nwords; ++w) bitmap[w] = 0;
  uint64_t count = 0;
  for (uint64_t p = 0; p < npages; ++p) {
    uint64_t lo = p * page;
    uint64_t len = (n - lo < page) ? n - lo : page;
    if (memcmp(pre + lo, post + lo, len) != 0) {
      bitmap[p / 64] |= 1ull << (p % 64);
      ++count;
    }
  }
  *dirty_count = count;
}
