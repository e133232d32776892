"""CPU-only: every planted mistake in a copy of the oracle must trip at least one pin.

Each case edits one line of a temporary copy of oracle/r3_oracle.c (a dropped
term, a wrong sign or index, a swapped operand), builds it with the oracle's own
flags and runs the pin suite against it.  The real oracle is never modified.
"""
import importlib.util
import os

import pytest

import pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "r3_oracle.c")
PY = os.path.join(ROOT, "oracle", "r3_oracle.py")

MUTANTS = [
    ("key_index_off_by_one", "uint64_t k = (j + 1) * PHI;", "uint64_t k = j * PHI;"),
    ("key_high_half_dropped", "(uint32_t)(w >> 32) + (uint32_t)(k >> 32)", "(uint32_t)(w >> 32) + (uint32_t)k"),
    ("length_term_in_words", "return sum + n * LEN;", "return sum + words * LEN;"),
    ("length_term_dropped", "return sum + n * LEN;", "return sum;"),
    ("product_truncated", "sum += (uint64_t)a * (uint64_t)bb;", "sum += (uint64_t)(a * bb);"),
    ("big_endian_word", "w |= (uint64_t)p[pos] << (8 * b);", "w |= (uint64_t)p[pos] << (8 * (7 - b));"),
    ("abs_err_sign", "d = fabs(C - G);", "d = fabs(C + G);"),
    ("rel_err_wrong_reference", "d / fabs(G);", "d / fabs(C);"),
    ("threshold_on_candidate", "double t = rg->rtol * fabs(G);", "double t = rg->rtol * fabs(C);"),
    ("threshold_inclusive", "mismatch = d > thr;", "mismatch = d >= thr;"),
    ("threshold_fused", "double thr = rg->atol + t;", "double thr = fma(rg->rtol, fabs(G), rg->atol);"),
    ("atol_dropped", "double thr = rg->atol + t;", "double thr = t;"),
    ("zero_reference_divides", "r = (G == 0.0) ? 0.0 : d / fabs(G);", "r = d / fabs(G);"),
    ("last_instead_of_first", "if (i < first) first = i;", "first = i;"),
    ("nonfinite_needs_both", "} else if (cnf || gnf) {", "} else if (cnf && gnf) {"),
    ("value_equality", "if (cb == gb) {", "if (C == G) {"),
    ("max_only_over_mismatches", "if (d > max_abs) max_abs = d;", "if (mismatch && d > max_abs) max_abs = d;"),
    ("rel_max_only_over_mismatches", "if (r > max_rel) max_rel = r;", "if (mismatch && r > max_rel) max_rel = r;"),
    ("bf16_low_half", "f32_from_bits((uint32_t)h << 16)", "f32_from_bits((uint32_t)h)"),
    ("f16_exponent_bias", "ldexp((double)(1024 + m), e - 25)", "ldexp((double)(1024 + m), e - 24)"),
    ("f16_subnormal_scale", "ldexp((double)m, -24)", "ldexp((double)m, -25)"),
    ("f16_hidden_bit_dropped", "ldexp((double)(1024 + m), e - 25)", "ldexp((double)m, e - 25)"),
    ("f16_nonfinite_not_flagged", "*val = m ? NAN : INFINITY;\n        *nonfinite = 1;", "*val = m ? NAN : INFINITY;"),
    ("checksum_of_golden", "out->checksum = r3o_checksum_bytes(c_base, rg->bytes);",
     "out->checksum = r3o_checksum_bytes(g_base, rg->bytes);"),
    ("dirty_bit_order", "bitmap[p / 64] |= 1ull << (p % 64);", "bitmap[p / 64] |= 1ull << (63 - p % 64);"),
    ("dirty_word_index", "bitmap[p / 64] |= 1ull << (p % 64);", "bitmap[p / 63] |= 1ull << (p % 64);"),
    ("dirty_skips_partial_page", "uint64_t npages = n / page + (n % page != 0);\n  uint64_t nwords",
     "uint64_t npages = n / page + (n % page != 0);\n  if (n % page != 0 && n > page) n -= n % page;\n  uint64_t nwords"),
    ("restore_ignores_offset", "memcpy(live + t[i].offset, snapshot + t[i].offset, t[i].bytes);",
     "memcpy(live + t[i].offset, snapshot, t[i].bytes);"),
    ("summary_last_region", "if (res[i].mismatch_count != 0 && s->first_region == UINT32_MAX) {",
     "if (res[i].mismatch_count != 0) {"),
    ("range_check_overflows", "t[i].bytes > arena_bytes - t[i].offset", "t[i].offset + t[i].bytes > arena_bytes"),
    ("empty_regions_overlap", "if (t[i].bytes == 0 || t[j].bytes == 0) continue;", ""),
    ("overlap_touching_counts", "t[i].offset < t[j].offset + t[j].bytes &&", "t[i].offset <= t[j].offset + t[j].bytes &&"),
    ("inf_tolerance_allowed", "if (isinf(t[i].rtol) || isinf(t[i].atol)) return O_EINVAL;", ""),
    ("align_before_dtype", "if (t[i].offset % es != 0 || t[i].bytes % es != 0) return O_EALIGN;",
     "if (t[i].offset % es != 0) return O_EALIGN;"),
]


def _mutant_api(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation site not unique: %r" % old
    src = tmp_path / ("mut_%s.c" % name)
    src.write_text(text.replace(old, new))
    spec = importlib.util.spec_from_file_location("r3_oracle_mut_%s" % name, PY)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod._SRC = str(src)
    mod._LIB = str(tmp_path / ("libmut_%s.so" % name))
    mod.lib()
    return mod


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, name, old, new):
    api = _mutant_api(tmp_path, name, old, new)
    caught = None
    for check in pins.ALL_CHECKS:
        try:
            check(api)
        except AssertionError:
            caught = check.__name__
            break
    assert caught is not None, "no pin notices mutant %s" % name


def test_unmutated_copy_passes(tmp_path):
    api = _mutant_api(tmp_path, "identity", "uint64_t sum = 0;", "uint64_t sum = 0u;")
    for check in pins.ALL_CHECKS:
        check(api)
