"""The pins must be able to fail: plant one plausible mistake at a time in a COPY of the oracle's
source (a dropped term, a wrong index, swapped sides, an off-by-one), build it, and check that at
least one pin of tests/test_oracle_pins.py rejects it.  Everything here runs on the CPU."""
import os
import subprocess
import sys

import pytest

import test_oracle_pins as pins
from oracle import kvd_oracle as orc

SRC = os.path.join(os.path.dirname(orc.__file__), "kvd_oracle.c")

# (name, text in the oracle source, what a mistaken author might have typed instead)
MUTANTS = [
    ("stride-dropped", "dot += index[a] * t->stride[a];", "dot += index[a];"),
    ("shape-for-stride", "dot += index[a] * t->stride[a];", "dot += index[a] * t->shape[a];"),
    ("elem-size-dropped", "return dot * t->elem_bytes;", "return dot;"),
    ("last-axis-skipped", "for (int a = 0; a < 5; ++a)\n        dot +=", "for (int a = 0; a < 4; ++a)\n        dot +="),
    ("src-slot-from-dst-block-size", "offset_by_role(s, sa, src_table[t / Ls], kv, t % Ls, h, x);\n                        int64_t dofs",
     "offset_by_role(s, sa, src_table[t / Ls], kv, t % Ld, h, x);\n                        int64_t dofs"),
    ("dst-block-from-src-block-size", "offset_by_role(d, da, dst_table[t / Ld], kv, t % Ld, h, x);\n                        memcpy",
     "offset_by_role(d, da, dst_table[t / Ls], kv, t % Ld, h, x);\n                        memcpy"),
    ("copy-direction", "memcpy(d->address + dofs, s->address + so, (size_t)e);", "memcpy(s->address + so, d->address + dofs, (size_t)e);"),
    ("v-never-copied", "for (int64_t kv = 0; kv < 2; ++kv)\n            for (int64_t t = 0; t < seq_len; ++t)",
     "for (int64_t kv = 0; kv < 1; ++kv)\n            for (int64_t t = 0; t < seq_len; ++t)"),
    ("whole-last-block", "for (int64_t t = 0; t < seq_len; ++t)\n                for (int64_t h = 0; h < H; ++h)\n                    for (int64_t x = 0; x < D; ++x) {\n                        int64_t so",
     "for (int64_t t = 0; t < (seq_len + Ls - 1) / Ls * Ls; ++t)\n                for (int64_t h = 0; h < H; ++h)\n                    for (int64_t x = 0; x < D; ++x) {\n                        int64_t so"),
    ("layer-range-off-by-one", "for (int64_t layer = layer_begin; layer < layer_end; ++layer) {", "for (int64_t layer = layer_begin; layer <= layer_end - 2; ++layer) {"),
    ("head-and-token-swapped", "index[role_axis[KVDO_L]] = l;\n    index[role_axis[KVDO_H]] = h;", "index[role_axis[KVDO_L]] = h;\n    index[role_axis[KVDO_H]] = l;"),
    ("span-uses-smallest-stride", "if (t->stride[a] > t->stride[best])", "if (t->stride[a] < t->stride[best])"),
    ("span-forgets-extent", "return t->shape[best] * t->stride[best] * t->elem_bytes;", "return t->stride[best] * t->elem_bytes;"),
    ("merge-on-remote-only", "if (m > 0 && out[m - 1].remote + out[m - 1].size == cur.remote &&\n            out[m - 1].local + out[m - 1].size == cur.local)",
     "if (m > 0 && out[m - 1].remote + out[m - 1].size == cur.remote)"),
    ("merge-on-local-only", "if (m > 0 && out[m - 1].remote + out[m - 1].size == cur.remote &&\n            out[m - 1].local + out[m - 1].size == cur.local)",
     "if (m > 0 && out[m - 1].local + out[m - 1].size == cur.local)"),
    ("merge-keeps-old-size", "out[m - 1].size += cur.size;\n        else\n            out[m++] = cur;", "out[m - 1].size = cur.size;\n        else\n            out[m++] = cur;"),
    ("merge-never", "            out[m - 1].size += cur.size;\n        else\n            out[m++] = cur;", "            out[m++] = cur;\n        else\n            out[m++] = cur;"),
    ("transfer-bytes-forgets-v", "return tokens * layers * 2 * kv_heads * head_dim * elem_bytes;", "return tokens * layers * kv_heads * head_dim * elem_bytes;"),
    ("transactions-ignore-seq-len", "while (t1 < seq_len && t1 / Ls == t0 / Ls && t1 / Ld == t0 / Ld)", "while (t1 / Ls == t0 / Ls && t1 / Ld == t0 / Ld)"),
]


def pin_checks():
    """The pins, as callables that raise AssertionError when the oracle is wrong."""
    checks = [pins.test_block8_offsets_match_paper, pins.test_offset_uses_every_axis,
              pins.test_span_size_matches_paper, pins.test_span_size_follows_largest_stride_axis,
              pins.test_block8_is_two_transactions_and_blocks01_merge,
              pins.test_partial_last_block_moves_only_the_request_tokens,
              pins.test_adjacent_k_and_v_are_queued_k_first_and_merge,
              pins.test_queue_example_merges_across_requests, pins.test_merge_needs_both_sides_contiguous,
              lambda: pins.test_run_count_closed_form(0), pins.test_sizes_quoted_in_paper,
              pins.test_round_trip_is_identity_on_valid_tokens, pins.test_identity_tables_reduce_to_memcpy]
    for w in pins.tiny_workloads():
        checks.append(lambda w=w: pins.test_oracle_equals_brute_force_and_writes_each_element_once(w))
    checks.append(lambda: pins.test_unique_ids_arrive_where_reshape_says("BHTD", "BTHD", 16, 32, (False, False)))
    checks.append(lambda: pins.test_unique_ids_arrive_where_reshape_says("BHTD", "BHTD", 8, 16, (True, True)))
    checks.append(pins.test_block_major_pools_coalesce_a_block_over_all_its_layers)
    checks.append(pins.test_runs_of_fixed_length_coalesce_to_one_transaction_per_run)
    return checks


def test_the_unmutated_oracle_passes_every_pin():
    for c in pin_checks():
        c()


RUNNER = r"""
import ctypes, sys
sys.path.insert(0, sys.argv[2]); sys.path.insert(0, sys.argv[3])
from oracle import kvd_oracle as orc
import test_oracle_mutants as tm
good = orc.lib()
mutant = ctypes.CDLL(sys.argv[1])
for fn in ("kvdo_offset_bytes", "kvdo_block_span_bytes", "kvdo_transfer_bytes", "kvdo_pull",
           "kvdo_request_transactions", "kvdo_coalesce"):
    getattr(mutant, fn).restype = getattr(good, fn).restype
    getattr(mutant, fn).argtypes = getattr(good, fn).argtypes
orc._lib = mutant
caught = 0
for c in tm.pin_checks():
    try:
        c()
    except (AssertionError, RuntimeError, ValueError):
        caught += 1
sys.exit(1 if caught else 0)
"""


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_is_caught(name, old, new, tmp_path):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for {name} not found exactly once"
    c_file, so_file = tmp_path / "mutant.c", tmp_path / "libmutant.so"
    c_file.write_text(text.replace(old, new))
    subprocess.check_call(["gcc", "-O1", "-std=c99", "-shared", "-fPIC", "-o", str(so_file), str(c_file)])
    # in a child process: a mutant that runs off the end of a table may crash, which also counts
    here = os.path.dirname(os.path.abspath(__file__))
    rc = subprocess.run([sys.executable, "-c", RUNNER, str(so_file), os.path.dirname(here), here],
                        stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL, timeout=300).returncode
    assert rc != 0, f"no pin noticed the planted mistake '{name}'"
