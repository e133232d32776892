"""Writes the text fixtures in this folder.  Calls only the CPU oracle (oracle/).

    python tests/golden/make_golden.py

The paper prints no numeric example for its correctness check, so these are
worked examples of the definitions in include/r3.h: each input was chosen by
hand, the expected values are what the oracle returns, and tests/pins.py checks
the same rows against a brute-force restatement in Python integers / rationals.
"""
import os
import struct
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import numpy as np  # noqa: E402

from oracle import r3_oracle as o  # noqa: E402

CHECKSUM_INPUTS = [
    ("empty", "-"),
    ("eight_zero_bytes", "00x8"),
    ("bytes_00_to_0f", bytes(range(16)).hex()),
    ("bf16_1_-2_0.5_tail_padded", "803f00c0003f"),
    ("f32_1_2_3_4", struct.pack("<4f", 1, 2, 3, 4).hex()),
    ("f32_2_1_3_4_swap_in_word", struct.pack("<4f", 2, 1, 3, 4).hex()),
    ("f32_3_4_1_2_swap_words", struct.pack("<4f", 3, 4, 1, 2).hex()),
    ("f64_0.5_-0.25_1e-3", struct.pack("<3d", 0.5, -0.25, 1e-3).hex()),
    ("i32_-1_0_1_max_min_tail_padded", struct.pack("<5i", -1, 0, 1, 2**31 - 1, -2**31).hex()),
    ("ff_times_4096", "ffx4096"),
]

# (golden bits, candidate bits) of fp32 elements; rtol 1e-5, atol 1e-7
COMPARE_ROWS = [
    (0x3F800000, 0x3F800000),  # equal
    (0x40000000, 0x40000001),  # one step above 2.0
    (0x00000000, 0x322BCC77),  # 1e-8 against 0: under atol
    (0xC0400000, 0xC04004EA),  # -3 against -3.0003
    (0x3A83126F, 0x3A83126F),  # equal
    (0x00000000, 0x3456BF95),  # 2e-7 against 0: over atol
    (0x80000000, 0x00000000),  # -0 against +0
    (0x7FC00000, 0x7FC00000),  # the same NaN
    (0x40A00000, 0x7FC00000),  # NaN against 5
    (0x40E00000, 0x7F800000),  # +Inf against 7
]


def parse_hex(spec):
    if spec == "-":
        return b""
    base, _, rep = spec.partition("x")
    return bytes.fromhex(base) * int(rep or 1)


def main():
    with open(os.path.join(HERE, "checksum_vectors.txt"), "w") as f:
        f.write("# Worked examples of the region checksum defined in include/r3.h (r3_checksum).\n")
        f.write("# name  input bytes (hex, 'AAxN' = AA repeated N times, '-' = empty)  checksum\n")
        f.write("# Second row by hand: one zero word gives lo32(PHI)*hi32(PHI) + 8*LEN\n")
        f.write("#   = 0x7F4A7C15*0x9E3779B9 + 8*0xBB67AE8584CAA73B mod 2^64.\n")
        for name, spec in CHECKSUM_INPUTS:
            f.write("%s %s %016X\n" % (name, spec, o.checksum_bytes(parse_hex(spec))))
    with open(os.path.join(HERE, "compare_worked_f32.txt"), "w") as f:
        f.write("# Worked example of the validation rule in include/r3.h (r3_region_result), fp32,\n")
        f.write("# rtol 1e-5, atol 1e-7: the paper's relaxed check with absolute and relative\n")
        f.write("# tolerances next to its default bitwise check (Section V-C).\n")
        f.write("# i  golden_bits  candidate_bits  abs_err_f64_bits  rel_err_f64_bits  TOL  BITWISE\n")
        f.write("# verdict: M = mismatch, ok = match\n")
        for i, (g, c) in enumerate(COMPARE_ROWS):
            gold = np.frombuffer(struct.pack("<I", g), dtype=np.uint8).copy()
            live = np.frombuffer(struct.pack("<I", c), dtype=np.uint8).copy()
            verdicts = []
            for mode in (o.TOL, o.BITWISE):
                res, _ = o.compare(o.make_table([(0, 4, o.F32, mode, 1e-5, 1e-7)]), live, gold)
                verdicts.append("M" if int(res[0]["mismatch_count"]) else "ok")
            d = struct.unpack("<Q", struct.pack("<d", float(res[0]["max_abs_err"])))[0]
            r = struct.unpack("<Q", struct.pack("<d", float(res[0]["max_rel_err"])))[0]
            f.write("%d %08X %08X %016X %016X %s %s\n" % (i, g, c, d, r, verdicts[0], verdicts[1]))


if __name__ == "__main__":
    main()
