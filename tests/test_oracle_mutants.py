"""Do the pins notice a plausible mistake in the oracle?  (CPU only.)

Each case patches one line of a copy of oracle/tc_oracle.c - a transposed index, a dropped stride,
a missing pad, an off-by-one table write - builds it with gcc, swaps it in as the oracle under test
and runs the pin suite: at least one pin must fail for every planted mistake.  The mistakes are
planted in copies of the oracle, on the CPU, and every one of them stays inside the buffers it is
given; nothing here touches the product.
"""
import os

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "tc_oracle.c")

MUTANTS = {
    "offload reads pool[block][plane] instead of pool[plane][block]":
        ("memcpy(record + p * pb, pool + (p * NB + blk) * pb, pb);",
         "memcpy(record + p * pb, pool + (blk * P + p) * pb, pb);"),
    "offload packs records without the pad":
        ("uint8_t *record = host + j * rec;", "uint8_t *record = host + j * (P * pb + 4u * S);"),
    "offload leaves the pad unwritten":
        ("while (at < rec) record[at++] = 0;", "(void)at;"),
    "offload takes scales as [block][s]":
        ("uint32_t w = scales[(uint64_t)s * NB + blk];", "uint32_t w = scales[blk * S + s];"),
    "offload skips the last plane":
        ("for (uint64_t p = 0; p < P; ++p)\n            memcpy(record + p * pb, pool",
         "for (uint64_t p = 0; p + 1 < P; ++p)\n            memcpy(record + p * pb, pool"),
    "upload writes the pages of plane p into plane P-1-p":
        ("memcpy(pool + (p * NB + blk) * pb, record + p * pb, pb);",
         "memcpy(pool + ((P - 1 - p) * NB + blk) * pb, record + p * pb, pb);"),
    "upload reads scale words one word late":
        ("memcpy(&w, record + P * pb + (uint64_t)4 * s, 4);", "memcpy(&w, record + P * pb + (uint64_t)4 * s + 4, 4);"),
    "upload writes the table one entry late":
        ("for (uint64_t i = 0; i < n; ++i) table_row[i] = new_ids[i];",
         "for (uint64_t i = 0; i + 1 < n; ++i) table_row[i + 1] = new_ids[i];"),
    "upload leaves the table alone":
        ("for (uint64_t i = 0; i < n; ++i) table_row[i] = new_ids[i];", "{ (void)new_ids; }"),
    "upload returns success, having done nothing, on a bad id":
        ("if (new_ids[i] < 0 || (uint64_t)new_ids[i] >= NB) return TCO_BAD_ID;",
         "if (new_ids[i] < 0 || (uint64_t)new_ids[i] >= NB) return TCO_OK;"),
    "record size counts the scale words twice":
        ("uint64_t raw = (uint64_t)2 * L * pb + (uint64_t)4 * S;", "uint64_t raw = (uint64_t)2 * L * pb + (uint64_t)8 * S;"),
    "record size rounds to 128":
        ("return (raw + 255u) / 256u * 256u;", "return (raw + 127u) / 128u * 128u;"),
    "blocks for tokens rounds down":
        ("return (tokens + block_size - 1) / block_size;", "return tokens / block_size;"),
    "read_token ignores the slot inside the block":
        ("+ (t % block_size) * tok, tok);", ", tok);"),
    "read_token swaps K and V":
        ("const uint64_t p = (uint64_t)2 * layer + kv;", "const uint64_t p = (uint64_t)2 * layer + (1 - kv);"),
}

PIN_CALLS = [
    (pins.test_block_bytes_matches_paper, [()]),
    (pins.test_tokens_to_blocks_matches_paper, [()]),
    (pins.test_benchmark_config_record_sizes, [()]),
    (pins.test_offload_is_numpy_take, [(2, 64, 48, 0, 9), (3, 37, 80, 6, 11), (1, 19, 16, 1, 5)]),
    (pins.test_upload_is_numpy_put, [(2, 64, 48, 0, 9), (3, 37, 80, 6, 11), (1, 19, 16, 1, 5)]),
    (pins.test_round_trip_byte_identical_and_foreign_blocks_untouched, [(False,), (True,)]),
    (pins.test_round_trip_with_scales_and_ragged_page, [()]),
    (pins.test_remapped_table_addresses_same_logical_tokens, [()]),
    (pins.test_empty_and_bad_ids, [()]),
    (pins.test_opaque_bytes_survive, [()]),
]


def _failing_pins(lib):
    failed = []
    saved = pins.O
    pins.O = lib
    try:
        for fn, argsets in PIN_CALLS:
            for args in argsets:
                try:
                    fn(*args)
                except (AssertionError, oracle.OracleError, ValueError, IndexError, pytest.fail.Exception):
                    failed.append(fn.__name__)
                    break
    finally:
        pins.O = saved
    return failed


def test_the_unmodified_oracle_passes_the_same_calls(tmp_path):
    lib = oracle.OracleLibrary(oracle.compile_c(SRC, str(tmp_path / "liboracle_copy.so")))
    assert _failing_pins(lib) == []


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name, tmp_path):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, "the line to break is not in the oracle any more"
    mutated = tmp_path / "tc_oracle_mutant.c"
    mutated.write_text(text.replace(old, new, 1))
    lib = oracle.OracleLibrary(oracle.compile_c(str(mutated), str(tmp_path / "libmutant.so")))
    failed = _failing_pins(lib)
    assert failed, f"no pin noticed: {name}"
