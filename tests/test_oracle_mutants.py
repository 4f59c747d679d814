"""Planted mistakes in the oracle (CPU only): every one must be caught by at least one pin.

Each mutant is the oracle's C file with one plausible slip (a dropped term, an off-by-one, a wrong
index) compiled to a temporary library.  This shows the pins are strong enough to notice such
slips; it does not touch the GPU path.
"""
import os
import subprocess
import sys

import pytest

import oracle
from oracle_pins import ALL_PINS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(os.path.dirname(oracle.__file__), "reft_oracle.c")

MUTANTS = {
    # encode forgets the last shard
    "encode_drops_last": ("for (uint32_t s = 0; s < k; ++s) p ^= shards[s][i];",
                          "for (uint32_t s = 0; s + 1 < k; ++s) p ^= shards[s][i];"),
    # encode starts from the wrong identity
    "encode_bad_identity": ("uint8_t p = 0;\n        for (uint32_t s = 0; s < k; ++s) p ^= shards",
                            "uint8_t p = 1;\n        for (uint32_t s = 0; s < k; ++s) p ^= shards"),
    # encode uses OR instead of XOR
    "encode_or": ("p ^= shards[s][i];", "p |= shards[s][i];"),
    # reconstruct forgets the parity
    "reconstruct_no_parity": ("uint8_t v = parity[i];", "uint8_t v = 0;"),
    # reconstruct skips the first survivor
    "reconstruct_skips_first": ("for (uint32_t s = 0; s < n_survivors; ++s) v ^=",
                                "for (uint32_t s = 1; s < n_survivors; ++s) v ^="),
    # bucketed pack reads the neighbouring byte in every odd bucket
    "bucketed_wrong_byte": ("host[o] = spans[t][o - span_start];",
                            "host[o] = spans[t][(o - span_start) ^ (b & 1)];"),
    # bucketed pack steps over at most one span boundary per byte (breaks on empty spans)
    "bucketed_single_step": ("while (o >= span_start + span_nbytes[t]) {",
                             "if (o >= span_start + span_nbytes[t]) {"),
    # pack leaves a gap of one byte after each span
    "pack_gap": ("        o += n;\n    }\n    return 0;\n}\n\n/*\n * The bucketed",
                 "        o += n + (n > 200);\n    }\n    return 0;\n}\n\n/*\n * The bucketed"),
    # unpack slices from the wrong offset
    "unpack_offset": ("dst[i] = stream[o + i];", "dst[i] = stream[o + i + (t > 2)];"),
    # rotated placement: every member takes segment 0 (Eq. 1 applied to all members alike)
    "rotated_all_segment0": ("static uint32_t oracle_rot_index(uint32_t i, uint32_t j) { return i < j ? i : i - 1; }",
                             "static uint32_t oracle_rot_index(uint32_t i, uint32_t j) { (void)i; (void)j; return 0; }"),
    # rotated placement: the other rotation (index by the protected shard, not by the member)
    "rotated_transposed": ("static uint32_t oracle_rot_index(uint32_t i, uint32_t j) { return i < j ? i : i - 1; }",
                           "static uint32_t oracle_rot_index(uint32_t i, uint32_t j) { return j < i ? j : j - 1; }"),
    # rotated decode: the protecting member's own shard is XORed in as well
    "rotated_decode_skips_member": ("if (j == i || j == lost) continue;", "if (j == lost) continue;"),
    # rotated placement: the zero extension of the last segment forgotten (the bytes beyond the
    # stream read as a repeat of its last byte instead of zero)
    "rotated_no_zero_extension": ("            if (y < L) p ^= shards[j][y];",
                                  "            if (L) p ^= shards[j][y < L ? y : L - 1];"),
    # collaborative recovery: the copy of S_x looked for on the wrong side (x + d instead of x - d)
    "collab_wrong_holder": ("const uint32_t holder = (x + k - arc_offsets[a]) % k;",
                            "const uint32_t holder = (x + arc_offsets[a]) % k;"),
    # collaborative recovery: a segment decoded although the unit covers another unknown segment
    "collab_decodes_too_early": ("!seg_known[j * nseg + oracle_rot_index(i, j)]) ready = 0;",
                                 "!seg_known[j * nseg + oracle_rot_index(i, j)]) ready = 1;"),
    # collaborative recovery: the member that covers segment r taken to be member r
    "collab_wrong_protector": ("const uint32_t i = r < x ? r : r + 1;               /* r(i, x) == r */",
                               "const uint32_t i = r;"),
    # collaborative recovery: a lost member's recovered bytes not used when decoding another
    "collab_ignores_recovered": ("if (y < L) v ^= lost[j] ? out[j][y] : shards[j][y];",
                                 "if (y < L) v ^= shards[j][y];"),
    # padded encode ignores the lengths
    "padded_ignores_len": ("p ^= (i < lens[s]) ? shards[s][i] : 0;",
                           "p ^= (i < lens[0]) ? shards[s][i < lens[s] ? i : 0] : 0;"),
}

@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name, tmp_path):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found"
    mutated = text.replace(old, new, 1)
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"lib{name}.so"
    c.write_text(mutated)
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", str(so),
                           str(c)])
    # The pins run in a child process: a mutant that indexes out of bounds may corrupt the heap
    # or crash, which also counts as noticed.
    code = (
        "import sys; sys.path[:0] = [%r, %r]\n"
        "import oracle\n"
        "from oracle_pins import ALL_PINS\n"
        "orc = oracle.Oracle(%r)\n"
        "bad = 0\n"
        "for pin in ALL_PINS:\n"
        "    try:\n"
        "        pin(orc)\n"
        "    except (AssertionError, ValueError):\n"
        "        bad += 1\n"
        "sys.exit(3 if bad else 0)\n"
    ) % (ROOT, os.path.join(ROOT, "tests"), str(so))
    rc = subprocess.run([sys.executable, "-c", code]).returncode
    assert rc != 0, f"no pin noticed the planted mistake '{name}'"
