"""The pins must bite: plant one plausible mistake at a time in a copy of the
oracle's source (on the CPU, in a temporary directory), rebuild it, and check
that at least one pin fails for every planted mistake."""
import ctypes
import os
import subprocess
import sys

import pytest

from oracle import kvxo
from tests import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(kvxo.__file__), "kvxo.c")

MUTANTS = {
    "kv_swapped_in_buffer": ("(((uint64_t)(l - l0) * 2 + c) * n + t) * row",
                             "(((uint64_t)(l - l0) * 2 + (1 - c)) * n + t) * row"),
    "layer_not_relative_to_range": ("(((uint64_t)(l - l0) * 2 + c) * n + t) * row",
                                    "(((uint64_t)(l) * 2 + c) * n + t) * row"),
    "token_major_buffer": ("(((uint64_t)(l - l0) * 2 + c) * n + t) * row",
                           "(((uint64_t)t * (l1 - l0) + (l - l0)) * 2 + c) * row"),
    "request_offset_dropped": ("return T_r * bytes_per_token +", "return 0 * T_r +"),
    "page_major_strides_wrong": ("*sp = (uint64_t)p->num_layers * *sl;", "*sp = *sl;"),
    "layer_major_kv_stride_wrong": ("*sk = (uint64_t)p->num_pages * *sp;", "*sk = *sp;"),
    "slot_uses_division": ("uint64_t slot = t % p->page_tokens;", "uint64_t slot = t / p->page_tokens;"),
    "logical_page_off_by_one": ("uint64_t logical = t / p->page_tokens;",
                                "uint64_t logical = (t + 1) / p->page_tokens;"),
    "block_table_not_indirected": ("uint32_t page = b->block_ids[b->block_offsets[r] + logical];",
                                   "uint32_t page = (uint32_t)logical;"),
    "csr_offset_ignored": ("uint32_t page = b->block_ids[b->block_offsets[r] + logical];",
                           "uint32_t page = b->block_ids[logical];"),
    "convert_uses_sender_table_twice": ("if (pool_place(pd, bd, (uint32_t)r, l, c, t, &to))",
                                        "if (pool_place(pd, bs, (uint32_t)r, l, c, t, &to))"),
    "head_major_forgets_slot": ("return w->base + (h * P + w->slot) * D * e + d * e;",
                                "return w->base + (h * P) * D * e + d * e;"),
    "head_major_is_token_major": ("return w->base + (h * P + w->slot) * D * e + d * e;",
                                  "return w->base + (w->slot * g->num_kv_heads + h) * D * e + d * e;"),
    "split_groups_not_16_bytes": ("uint64_t x = 16 / e;", "uint64_t x = 8 / e ? 8 / e : 1;"),
    "split_token_outside_group": ("return w->base + ((h * (D / x) + d / x) * P + w->slot) * 16 + (d % x) * e;",
                                  "return w->base + ((h * P + w->slot) * (D / x) + d / x) * 16 + (d % x) * e;"),
    "split_lane_order_reversed": ("+ (d % x) * e;", "+ (x - 1 - d % x) * e;"),
    "tinner_forgets_slot": ("return w->base + ((h * D + d) * P + w->slot) * e;",
                            "return w->base + ((h * D + d) * P) * e;"),
    "tinner_column_pitch_is_head_dim": ("return w->base + ((h * D + d) * P + w->slot) * e;",
                                        "return w->base + ((h * D + d) * D + w->slot) * e;"),
    "tinner_heads_innermost": ("return w->base + ((h * D + d) * P + w->slot) * e;",
                               "return w->base + ((d * g->num_kv_heads + h) * P + w->slot) * e;"),
    "tinner_slot_not_scaled_by_element": ("return w->base + ((h * D + d) * P + w->slot) * e;",
                                          "return w->base + ((h * D + d) * P) * e + w->slot;"),
    "segment_length_half": ("*len = 2 * (uint64_t)b->seq_lens[r] * row_bytes(p);",
                            "*len = (uint64_t)b->seq_lens[r] * row_bytes(p);"),
    "total_forgets_kv_factor": ("* 2\n                 * tokens_before(b, b->num_requests);",
                                "\n                 * tokens_before(b, b->num_requests);"),
    "row_ignores_elem_bytes": ("return (uint64_t)p->num_kv_heads * p->head_dim * p->elem_bytes;",
                               "return (uint64_t)p->num_kv_heads * p->head_dim;"),
}
MUTANTS["unpack_writes_one_row_past_length"] = (
    "                    copy_token(p, pool, &to, buf, &from);",
    "                    copy_token(p, pool, &to, buf, &from);\n"
    "                    if (t + 1 == b->seq_lens[r] && (t + 1) % p->page_tokens) {\n"
    "                        to.slot += 1; copy_token(p, pool, &to, buf, &from); }")


def _run_pins():
    """A cross-section of the pins; returns the names of those that fail."""
    failed = []
    cases = [
        ("bruteforce", lambda: [pins.test_bruteforce_tiny(*c) for c in pins.TINY[::5]]),
        ("paper_sizes", lambda: [pins.test_paper_kv_sizes(*g) for g in pins._golden_rows()]),
        ("closed_form", lambda: [pins.test_closed_form_and_segments_tile_buffer(s) for s in range(3)]),
        ("stamps", lambda: [pins.test_roundtrip_stamps_and_canaries(pins.LM, pins.PM, 128, 16),
                            pins.test_roundtrip_stamps_and_canaries(pins.PM, pins.LM, 16, 128),
                            pins.test_roundtrip_stamps_and_canaries(pins.LM, pins.LM, 5, 7)]),
        ("take", lambda: pins.test_pack_reduces_to_numpy_take(0)),
        ("inner_bruteforce", lambda: [pins.test_bruteforce_tiny(*c) for c in pins.INNER[::7]]),
        ("inner_transposes", lambda: pins.test_inner_arrangements_reduce_to_transposes(2, 16)),
        ("transpose", pins.test_convert_reduces_to_transpose),
        ("algebra", pins.test_convert_equals_unpack_of_pack),
        ("ranges", pins.test_whole_range_is_per_layer_ranges_at_segment_offsets),
    ]
    for name, fn in cases:
        try:
            fn()
        except (AssertionError, ValueError, IndexError, KeyError):
            failed.append(name)
    return failed


def test_unmutated_oracle_passes_the_cross_section():
    assert _run_pins() == []


_CHILD = """
import ctypes, sys
sys.path.insert(0, {root!r})
from oracle import kvxo
from tests import test_oracle_mutants as m
mut = ctypes.CDLL({so!r})
for fn in ("kvxo_total_bytes", "kvxo_segment", "kvxo_pack", "kvxo_unpack", "kvxo_convert"):
    getattr(mut, fn).restype = ctypes.c_int
kvxo._lib = mut
print("FAILED_PINS=" + ",".join(m._run_pins()), flush=True)
"""


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistake(name, tmp_path):
    """Runs in a child process: a planted indexing mistake may write out of
    bounds and take the interpreter down, which also counts as noticed."""
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found in the oracle source"
    c = tmp_path / "kvxo_mut.c"
    so = tmp_path / "libkvxo_mut.so"
    c.write_text(text.replace(old, new))
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", str(so), str(c)],
                   check=True)
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, "-c", _CHILD.format(root=root, so=str(so))],
                         capture_output=True, text=True, timeout=300)
    if res.returncode < 0:
        return                                    # crashed on a wild access: noticed
    assert res.returncode == 0, res.stderr[-2000:]
    line = [x for x in res.stdout.splitlines() if x.startswith("FAILED_PINS=")][-1]
    assert line != "FAILED_PINS=", f"no pin noticed the planted mistake '{name}'"
