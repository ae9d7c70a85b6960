"""CPU-only checks of libkvx: the library loads and exports the whole boundary,
and the host side of kvx_plan (validation, sizes, segments) behaves as
include/kvx.h states.  No kernel is launched: plans are host-only."""
import os
import re
import subprocess

import numpy as np
import pytest

from oracle import kvxo
from paper_2408_08147_amd import kvx
from paper_2408_08147_amd import workloads as W
from tests import gpu_util as G

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    import ctypes
    hdr = open(os.path.join(ROOT, "include", "kvx.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(kvx_[a-z_]+)\s*\(", hdr))
    assert declared == set(kvx.EXPORTS), declared ^ set(kvx.EXPORTS)
    lib = ctypes.CDLL(kvx.lib_path())
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings():
    seen = {kvx.status_string(i) for i in range(9)}
    assert len(seen) == 9 and "ok" in seen and kvx.status_string(8) == "out of host memory"
    assert kvx.status_string(9) == "unknown status"


def _simple(n=(100, 33), P=16, NP=64):
    need = [(x + P - 1) // P for x in n]
    ids = np.arange(sum(need), dtype=np.uint32)
    offs = np.concatenate([[0], np.cumsum(need)]).astype(np.uint64)
    return kvx.pool_desc(2, 8, 128, 2, P, NP), kvx.BatchDesc(n, ids, offs)


def expect(status, fn, *a, **k):
    with pytest.raises(kvx.KvxError) as e:
        fn(*a, **k)
    assert e.value.status == status, e.value


def test_argument_errors():
    s, b = _simple()
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, None, None, None, None, 0, 1)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, s, None, None, None, 0, 1)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, s, b, None, None, 1, 0)          # range reversed
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, s, b, None, None, 0, 3)          # beyond num_layers
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, s, b, None, None, 0, 2, 0, 4096) # size without pointer
    expect(kvx.ERR_ALIGNMENT, kvx.kvx_plan, s, b, None, None, 0, 2, 128, 1 << 20)
    zero = kvx.pool_desc(2, 8, 128, 2, 0, 64)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, zero, b, None, None, 0, 2)
    odd = kvx.pool_desc(2, 1, 4, 2, 16, 64)                                    # row = 8 bytes
    expect(kvx.ERR_ALIGNMENT, kvx.kvx_plan, odd, b, None, None, 0, 2)
    badlayout = kvx.pool_desc(2, 8, 128, 2, 16, 64, layout=7)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, badlayout, b, None, None, 0, 2)
    part = kvx.pool_desc(2, 8, 128, 2, 16, 64, strides=(1 << 20, 0, 0, 0))
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, part, b, None, None, 0, 2)
    mis = kvx.pool_desc(2, 8, 128, 2, 16, 64, strides=(1 << 20, 1 << 19, 32776, 2048))
    expect(kvx.ERR_ALIGNMENT, kvx.kvx_plan, mis, b, None, None, 0, 2)
    short = kvx.pool_desc(2, 8, 128, 2, 16, 64, strides=(1 << 22, 1 << 21, 1 << 15, 1024))
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, short, b, None, None, 0, 2)      # stride_token < row
    huge = kvx.pool_desc(1, 64, 256, 4, 1 << 16, 2)                            # page_tokens*row = 2^32
    expect(kvx.ERR_UNSUPPORTED, kvx.kvx_plan, huge, kvx.BatchDesc([1], [0], [0, 1]), None, None, 0, 1)


def test_inner_arrangement_errors():
    _, b = _simple()
    ok = kvx.pool_desc(2, 8, 128, 2, 16, 64, inner=kvx.INNER_DIM_SPLIT_TOKEN)
    kvx.kvx_plan(ok, b, ok, b, 0, 2).destroy()
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, kvx.pool_desc(2, 8, 128, 2, 16, 64, inner=4), b, None, None, 0, 2)
    # token axis innermost: elements of 1, 2, 4 or 8 bytes, no condition on the head dimension but the row's
    tin = kvx.pool_desc(2, 8, 128, 2, 16, 64, inner=kvx.INNER_TOKEN_INNERMOST)
    kvx.kvx_plan(tin, b, ok, b, 0, 2).destroy()
    kvx.kvx_plan(kvx.pool_desc(2, 4, 4, 1, 16, 64, inner=3), b, None, None, 0, 2).destroy()   # 4-byte heads, 16-byte row
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, kvx.pool_desc(2, 1, 16, 3, 16, 64, inner=3), b, None, None, 0, 2)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, kvx.pool_desc(2, 1, 16, 16, 16, 64, inner=3), b, None, None, 0, 2)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan,
           kvx.pool_desc(2, 8, 128, 2, 16, 64, strides=(1 << 22, 1 << 21, 1 << 15, 2048), inner=3), b, None, None, 0, 2)
    strided = kvx.pool_desc(2, 8, 128, 2, 16, 64, strides=(1 << 22, 1 << 21, 1 << 15, 2048), inner=1)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, strided, b, None, None, 0, 2)
    # head_dim*elem_bytes must be a multiple of 16 even when the whole row is
    expect(kvx.ERR_ALIGNMENT, kvx.kvx_plan, kvx.pool_desc(2, 4, 4, 2, 16, 64, inner=1), b, None, None, 0, 2)
    # 16-byte groups need an element size that divides 16
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, kvx.pool_desc(2, 1, 16, 3, 16, 64, inner=2), b, None, None, 0, 2)
    # the two sides may differ in arrangement, not in shape
    other = kvx.pool_desc(2, 8, 128, 2, 8, 128, layout=1, inner=kvx.INNER_HEAD_MAJOR)
    b8 = kvx.BatchDesc([100, 33], np.arange(18), [0, 13, 18])
    p = kvx.kvx_plan(ok, b, other, b8, 0, 2)
    assert kvx.kvx_plan_total_bytes(p) == 133 * 2 * 2 * 2048


def test_receiver_strides_must_not_alias():
    """A pool that is written must not let two rows share bytes: its four axes have to nest.  A sender is
    only read and may overlap itself."""
    _, b = _simple()                              # pages of 16 tokens, rows of 2048 bytes, 64 pages, 2 layers
    row, P, NP = 2048, 16, 64
    good = (2 * NP * P * row, NP * P * row, P * row, row)                    # (layer, kv, page, token)
    padded = (2 * NP * (P * 2304 + 512) + 4096, NP * (P * 2304 + 512), P * 2304 + 512, 2304)
    page_major = (2 * P * row, P * row, 2 * 2 * P * row, row)                # pages outermost
    for st in (good, padded, page_major):
        kvx.kvx_plan(None, None, kvx.pool_desc(2, 8, 128, 2, P, NP, strides=st), b, 0, 2).destroy()
    bad = {
        "pages overlap": (good[0], good[1], (P - 1) * row, row),
        "K and V overlap": (good[0], good[1] - 16, good[2], good[3]),
        "layers overlap": (good[1], good[1], good[2], good[3]),
        "layers inside a page": (16 * 1024, good[1], good[2], good[3]),
        "page stride below one row": (good[0], good[1], 1024, row),
    }
    for what, st in bad.items():
        recv = kvx.pool_desc(2, 8, 128, 2, P, NP, strides=st)
        with pytest.raises(kvx.KvxError) as e:
            kvx.kvx_plan(None, None, recv, b, 0, 2)
        assert e.value.status == kvx.ERR_INVALID_ARG, what
        with pytest.raises(kvx.KvxError) as e:
            kvx.kvx_plan_workspace_bytes(None, None, recv, b)
        assert e.value.status == kvx.ERR_INVALID_ARG, what
        kvx.kvx_plan(recv, b, None, None, 0, 2).destroy()                    # as a sender: allowed
    # an axis of extent 1 has no say: one layer, any layer stride
    one_layer = kvx.pool_desc(1, 8, 128, 2, P, NP, strides=(16, good[1], good[2], good[3]))
    kvx.kvx_plan(None, None, one_layer, b, 0, 1).destroy()


def test_unpack_noalloc_refuses_on_the_host():
    """Everything kvx_unpack_noalloc can refuse, it refuses before any HIP call."""
    d = kvx.pool_desc(2, 8, 128, 2, 16, 4096)
    ok = kvx.BatchDesc([100, 33], np.arange(10), [0, 7, 10])
    f = kvx.kvx_unpack_noalloc
    expect(kvx.ERR_INVALID_ARG, f, None, ok, 0, 2, 4096, 1 << 30, 8192)
    expect(kvx.ERR_INVALID_ARG, f, d, None, 0, 2, 4096, 1 << 30, 8192)
    expect(kvx.ERR_INVALID_ARG, f, d, ok, 1, 0, 4096, 1 << 30, 8192)
    expect(kvx.ERR_INVALID_ARG, f, d, ok, 0, 3, 4096, 1 << 30, 8192)
    expect(kvx.ERR_CAPACITY, f, d, ok, 0, 2, 4096, 133 * 2 * 2 * 2048 - 1, 8192)       # buffer too small
    expect(kvx.ERR_INVALID_ARG, f, d, ok, 0, 2, 0, 1 << 30, 8192)
    expect(kvx.ERR_ALIGNMENT, f, d, ok, 0, 2, 4096 + 8, 1 << 30, 8192)
    dup = kvx.BatchDesc([100, 33], [0, 1, 2, 3, 4, 5, 6, 0, 1, 9], [0, 7, 10])
    expect(kvx.ERR_BLOCK_TABLE, f, d, dup, 0, 2, 4096, 1 << 30, 8192)
    expect(kvx.ERR_BLOCK_TABLE, f, d, kvx.BatchDesc([100, 33], np.arange(9), [0, 6, 9]), 0, 2, 4096, 1 << 30, 8192)
    expect(kvx.ERR_BLOCK_TABLE, f, d, kvx.BatchDesc([16], [4096], [0, 1]), 0, 2, 4096, 1 << 30, 8192)
    # the limit: requests + used pages <= 896 words
    n_ok, n_over = [16] * 448, [16] * 449
    at_limit = kvx.BatchDesc(n_ok, np.arange(448), np.arange(449))
    over = kvx.BatchDesc(n_over, np.arange(449), np.arange(450))
    assert 2 * 448 == kvx.NOALLOC_MAX_TABLE_WORDS
    expect(kvx.ERR_CAPACITY, f, d, over, 0, 2, 4096, 1 << 40, 8192)
    expect(kvx.ERR_CAPACITY, f, d, kvx.BatchDesc([1] * 897, np.arange(897), np.arange(898)), 0, 2, 4096, 1 << 40, 8192)
    # at the limit the tables fit the scratch array: the call gets past every host check (and, with no GPU
    # here, stops at the first HIP call)
    ws = kvx.kvx_plan_workspace_bytes(None, None, d, at_limit)
    assert ws <= kvx.NOALLOC_SCRATCH_BYTES
    # an empty transfer is a no-op that touches no device
    f(d, kvx.BatchDesc([0, 0], [], [0, 0, 0]), 0, 2, 0, 0, 0)
    f(d, ok, 1, 1, 0, 0, 0)


def test_release_cached_with_nothing_cached():
    assert kvx.kvx_release_cached() == 0


def test_sides_must_agree():
    s, b = _simple()
    d_heads = kvx.pool_desc(2, 4, 128, 2, 16, 64)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, s, b, d_heads, b, 0, 2)
    d_elem = kvx.pool_desc(2, 8, 128, 1, 16, 64)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, s, b, d_elem, b, 0, 2)
    _, b_other = _simple(n=(100, 34))
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, s, b, s, b_other, 0, 2)
    _, b_three = _simple(n=(100, 33, 1))
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, s, b, s, b_three, 0, 2)
    d_fewer_layers = kvx.pool_desc(1, 8, 128, 2, 16, 64)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan, s, b, d_fewer_layers, b, 0, 2)
    kvx.kvx_plan(s, b, d_fewer_layers, b, 0, 1).destroy()


def test_block_table_errors():
    s = kvx.pool_desc(2, 8, 128, 2, 16, 64)
    ok = kvx.BatchDesc([100, 33], np.arange(10), [0, 7, 10])
    kvx.kvx_plan(s, ok, s, ok, 0, 2).destroy()
    too_short = kvx.BatchDesc([100, 33], np.arange(9), [0, 6, 9])
    expect(kvx.ERR_BLOCK_TABLE, kvx.kvx_plan, s, too_short, None, None, 0, 2)
    out_of_pool = kvx.BatchDesc([100, 33], [0, 1, 2, 3, 4, 5, 64, 7, 8, 9], [0, 7, 10])
    expect(kvx.ERR_BLOCK_TABLE, kvx.kvx_plan, s, out_of_pool, None, None, 0, 2)
    descending = kvx.BatchDesc([100, 33], np.arange(10), [0, 7, 5])
    expect(kvx.ERR_BLOCK_TABLE, kvx.kvx_plan, s, descending, None, None, 0, 2)
    nonzero_start = kvx.BatchDesc([100, 33], np.arange(12), [1, 8, 11])
    expect(kvx.ERR_BLOCK_TABLE, kvx.kvx_plan, s, nonzero_start, None, None, 0, 2)
    # a page twice: fine for a sender (shared prefix), an error for a receiver
    dup = kvx.BatchDesc([100, 33], [0, 1, 2, 3, 4, 5, 6, 0, 1, 9], [0, 7, 10])
    kvx.kvx_plan(s, dup, None, None, 0, 2).destroy()
    kvx.kvx_plan(s, dup, s, ok, 0, 2).destroy()
    expect(kvx.ERR_BLOCK_TABLE, kvx.kvx_plan, None, None, s, dup, 0, 2)
    expect(kvx.ERR_BLOCK_TABLE, kvx.kvx_plan, s, ok, s, dup, 0, 2)
    # ids beyond ceil(n/P) are ignored: they may repeat or leave the pool
    extra = kvx.BatchDesc([100, 33], [0, 1, 2, 3, 4, 5, 6, 6, 999, 7, 8, 9, 7], [0, 9, 13])
    kvx.kvx_plan(None, None, s, extra, 0, 2).destroy()
    # zero-length requests need no pages
    empty = kvx.BatchDesc([0, 16, 0], [3], [0, 0, 1, 1])
    p = kvx.kvx_plan(s, empty, s, empty, 0, 2)
    assert kvx.kvx_plan_total_bytes(p) == 16 * 2 * 2 * 2048
    assert kvx.kvx_plan_request_segment(p, 0) == (0, 0)
    assert kvx.kvx_plan_request_segment(p, 2) == (16 * 8192, 0)
    none = kvx.BatchDesc([], [], [0])
    p0 = kvx.kvx_plan(s, none, None, None, 0, 2)
    assert kvx.kvx_plan_total_bytes(p0) == 0


def test_host_only_plan_cannot_launch():
    s, b = _simple()
    p = kvx.kvx_plan(s, b, s, b, 0, 2)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_pack, p, 4096, 8192, 1 << 40)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_unpack, p, 4096, 1 << 40, 8192)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_convert, p, 4096, 8192)
    expect(kvx.ERR_CAPACITY, kvx.kvx_pack, p, 4096, 8192, 10)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan_get_tables, p)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan_segment, p, 2, 0)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan_segment, p, 0, 2)


def test_small_one_sided_plans_without_a_workspace_can_launch():
    """One side, token-row pages, at most KVX_INLINE_RUNS used pages: the host builds the run records, and
    the plan says so."""
    hdr = open(os.path.join(ROOT, "include", "kvx.h")).read()
    assert int(re.search(r"#define KVX_INLINE_RUNS (\d+)u", hdr).group(1)) == kvx.INLINE_RUNS == 96
    s, b = _simple()
    for p in (kvx.kvx_plan(s, b, None, None, 0, 2), kvx.kvx_plan(None, None, s, b, 1, 2)):
        assert kvx.kvx_plan_can_launch(p)
        expect(kvx.ERR_INVALID_ARG, kvx.kvx_convert, p, 4096, 8192)
        expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan_get_tables, p)
    p = kvx.kvx_plan(s, b, None, None, 0, 2)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_unpack, p, 4096, 1 << 40, 8192)     # the side it does not have
    expect(kvx.ERR_CAPACITY, kvx.kvx_pack, p, 4096, 8192, 10)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_pack, p, 0, 8192, 1 << 40)
    expect(kvx.ERR_ALIGNMENT, kvx.kvx_pack, p, 4096 + 8, 8192, 1 << 40)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_pack_layers, p, 1, 3, 4096, 8192, 1 << 40)
    s96, b96 = _simple(n=(16 * 90, 16 * 6 - 1), NP=200)
    assert kvx.kvx_plan_can_launch(kvx.kvx_plan(s96, b96, None, None, 0, 2))


@pytest.mark.parametrize("what", ["ninety_seven_pages", "two_sided", "head_major_pages", "padded_rows", "empty"])
def test_plans_without_a_workspace_that_cannot_run(what):
    """Everything else without a workspace answers the size queries and refuses to launch, before any device
    call: the pointers handed over here are never touched."""
    rng = np.random.default_rng(11)
    lens = {"ninety_seven_pages": [16 * 96 + 1], "empty": [0, 0]}.get(what, [100, 40])
    inner = 1 if what == "head_major_pages" else 0
    case = G.make_case(rng, 2, 2, 16, 2, lens, 16, 16, 0, 0, inner_s=inner, inner_d=inner)
    sp, sb = case.kvx_pool(case.s), kvx.BatchDesc(case.seq_lens, case.ids_s, case.offs_s)
    dp, db = case.kvx_pool(case.d), kvx.BatchDesc(case.seq_lens, case.ids_d, case.offs_d)
    if what == "padded_rows":
        st = case.row + 16                 # layer, K|V, page, token
        strides = (2 * st * 16 * case.s.num_pages, st * 16 * case.s.num_pages, st * 16, st)
        sp = kvx.pool_desc(2, 2, 16, 2, 16, case.s.num_pages, 0, strides, 0)
    if what == "two_sided":
        plans = [kvx.kvx_plan(sp, sb, dp, db, 0, 2)]
    else:
        plans = [kvx.kvx_plan(sp, sb, None, None, 0, 2)]
        if what != "padded_rows":
            plans.append(kvx.kvx_plan(None, None, dp, db, 0, 2))
    for p in plans:
        assert not kvx.kvx_plan_can_launch(p)
        if what != "empty":
            with pytest.raises(kvx.KvxError) as e:
                kvx.kvx_pack(p, 4096, 8192, 1 << 40)
            assert e.value.status == kvx.ERR_INVALID_ARG
            with pytest.raises(kvx.KvxError) as e:
                kvx.kvx_unpack(p, 4096, 1 << 40, 8192)
            assert e.value.status == kvx.ERR_INVALID_ARG
        p.destroy()


def test_launch_config_round_trip():
    s, b = _simple()
    p = kvx.kvx_plan(s, b, None, None, 0, 2)
    d = kvx.kvx_plan_get_launch(p)
    assert d.unroll in (0, 1, 2, 4, 8) and d.nontemporal in (0, 1, 2, 3) and d.order in (0, 1, 2, 3)
    kvx.kvx_plan_set_launch(p, unroll=8, nontemporal=1, order=2, xcd_swizzle=2, max_workgroups=4096, threads=512)
    g = kvx.kvx_plan_get_launch(p)
    assert (g.unroll, g.nontemporal, g.order, g.xcd_swizzle, g.max_workgroups, g.threads) == (8, 1, 2, 2, 4096, 512)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan_set_launch, p, unroll=3)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan_set_launch, p, threads=96)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan_set_launch, p, order=5)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan_set_launch, p, nontemporal=4)
    expect(kvx.ERR_INVALID_ARG, kvx.kvx_plan_set_launch, p, workgroups_per_cu=9)


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_totals_and_segments_match_oracle_on_the_five_workloads(idx):
    """Host arithmetic of the library against the oracle's, at the full sizes
    of the five synthetic workloads (64-bit offsets included)."""
    w = W.CONFIGS[idx]
    bt = W.draw_batch(w)
    s = kvx.pool_desc(w.num_layers, w.num_kv_heads, w.head_dim, w.elem_bytes, w.page_s, bt.num_pages_s, w.layout_s)
    d = kvx.pool_desc(w.num_layers, w.num_kv_heads, w.head_dim, w.elem_bytes, w.page_d, bt.num_pages_d, w.layout_d)
    sb = kvx.BatchDesc(bt.seq_lens, bt.ids_s, bt.offs_s)
    db = kvx.BatchDesc(bt.seq_lens, bt.ids_d, bt.offs_d)
    op = kvxo.Pool(w.num_layers, w.num_kv_heads, w.head_dim, w.elem_bytes, w.page_s, bt.num_pages_s, w.layout_s)
    ob = kvxo.Batch(bt.seq_lens, bt.ids_s, bt.offs_s)
    rng = np.random.default_rng(idx)
    for l0, l1 in [(0, w.num_layers), (1, 2), (w.num_layers - 1, w.num_layers)]:
        p = kvx.kvx_plan(s, sb, d, db, l0, l1)
        assert kvx.kvx_plan_total_bytes(p) == kvxo.total_bytes(op, ob, l0, l1)
        for r in rng.integers(0, w.num_requests, size=8):
            r = int(r)
            for l in {l0, l1 - 1, int(rng.integers(l0, l1))}:
                assert kvx.kvx_plan_segment(p, r, l) == kvxo.segment(op, ob, l0, l1, r, l)
            off0, _ = kvxo.segment(op, ob, l0, l1, r, l0)
            offn, lenn = kvxo.segment(op, ob, l0, l1, r, l1 - 1)
            assert kvx.kvx_plan_request_segment(p, r) == (off0, offn + lenn - off0)
        p.destroy()
    assert kvx.kvx_plan_workspace_bytes(s, sb, d, db) % 256 == 0


def test_header_is_plain_c(tmp_path):
    """include/kvx.h must be usable from C99 and from C++ without any other header of this library."""
    import subprocess
    src = tmp_path / "use_kvx.c"
    src.write_text('#include "kvx.h"\nint main(void) { kvx_pool_desc d; kvx_launch_cfg c; (void)d; (void)c; '
                   'return (int)sizeof(kvx_run) - 32; }\n')
    inc = os.path.join(ROOT, "include")
    for cmd in (["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc, str(src)],
                ["g++", "-std=c++17", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++",
                 "-I", inc, str(src)]):
        res = subprocess.run(cmd, capture_output=True, text=True)
        assert res.returncode == 0, res.stderr


def test_retriever_sizing_errors():
    assert kvx.kvx_retriever_arena_bytes(3, 1000, 100) == 3 * (1024 + 256)
    for args, code in (((0, 1, 1), kvx.ERR_INVALID_ARG), ((1, 0, 1), kvx.ERR_INVALID_ARG),
                       ((1, 1, 0), kvx.ERR_INVALID_ARG), ((1025, 1, 1), kvx.ERR_UNSUPPORTED),
                       ((1, (1 << 48) + 1, 1), kvx.ERR_UNSUPPORTED), ((1, 1, (1 << 48) + 1), kvx.ERR_UNSUPPORTED)):
        with pytest.raises(kvx.KvxError) as ei:
            kvx.kvx_retriever_arena_bytes(*args)
        assert ei.value.status == code, args


def test_public_header_is_plain_c99_and_cxx17(tmp_path):
    """include/kvx.h on its own, pedantic and warning-free, as C99 and as C++17."""
    inc = os.path.join(ROOT, "include")
    for compiler, std, ext in (("gcc", "-std=c99", "c"), ("g++", "-std=c++17", "cpp")):
        src = tmp_path / f"only_header.{ext}"
        src.write_text('#include "kvx.h"\nint main(void) { return (int)sizeof(kvx_run) - 32; }\n')
        res = subprocess.run([compiler, std, "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", inc, "-c", str(src),
                              "-o", str(tmp_path / f"only_header_{ext}.o")], capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-2000:]


def test_no_library_no_result(monkeypatch, tmp_path):
    """Without the HIP library every entry point of the binding raises: there is no other path to fall back to."""
    from paper_2408_08147_amd import build as B

    def no_compiler():
        raise RuntimeError("hipcc is not here")
    monkeypatch.setattr(kvx, "_lib", None)
    monkeypatch.setattr(B, "LIB", str(tmp_path / "libkvx_absent.so"))
    monkeypatch.setattr(B, "build", no_compiler)
    sp, sb = _simple()
    with pytest.raises(RuntimeError, match="hipcc is not here"):
        kvx.kvx_plan_workspace_bytes(sp, sb, None, None)
    with pytest.raises(RuntimeError, match="hipcc is not here"):
        kvx.kvx_plan(sp, sb, None, None, 0, 2)
    # a file that was not built from the sources beside it (no id, or another id) is not loaded either:
    # the binding asks for a rebuild, and fails as loudly when there is no compiler
    for blob in (b"not an ELF file", B.ID_TAG.encode() + b"0" * 32):
        bad = tmp_path / "libkvx_stale.so"
        bad.write_bytes(blob)
        monkeypatch.setattr(B, "LIB", str(bad))
        assert B.is_stale()
        with pytest.raises(RuntimeError, match="hipcc is not here"):
            kvx.kvx_plan_workspace_bytes(sp, sb, None, None)


def test_built_library_names_its_sources():
    from paper_2408_08147_amd import build as B
    assert not B.is_stale()
    assert kvx.kvx_build_id() == B.ID_TAG + B.source_id()
