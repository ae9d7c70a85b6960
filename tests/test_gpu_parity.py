"""GPU parity: kvx_pack / kvx_unpack / kvx_convert through the C ABI against the
CPU oracle, byte for byte (buffer incl. slack, destination pools incl. every
byte that must stay untouched), at sizes the oracle finishes in seconds."""
import numpy as np
import pytest

from paper_2408_08147_amd import kvx
from paper_2408_08147_amd import workloads as W
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

LM, PM = 0, 1


def check(case, seed, ranges=None, launch=None, kind="bytes"):
    rng = np.random.default_rng(seed)
    if kind == "bytes":
        src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    else:
        src = W.values_numpy(kind, case.pool_bytes(case.s), rng)
    for l0, l1 in ranges or [(0, case.num_layers)]:
        want = G.run_oracle(case, src, l0, l1)
        got = G.run_gpu(case, src, l0, l1, launch=launch)
        G.assert_same(got, want, f"layers [{l0},{l1})")


# ------------------------------------------------------------------ edge cases
EDGE_LENS = {
    "empty_batch": [],
    "all_zero": [0, 0, 0],
    "single_token": [1],
    "around_page": [15, 16, 17, 0, 31, 32, 33, 1],
    "ragged_multi_tile": [1000, 3, 517, 128, 129, 2047],
}


@pytest.mark.parametrize("name", sorted(EDGE_LENS))
@pytest.mark.parametrize("Ps,Pd,ls,ld", [(16, 16, LM, LM), (128, 16, LM, PM), (16, 128, PM, LM)])
def test_edge_lengths(name, Ps, Pd, ls, ld):
    rng = np.random.default_rng(sum(map(ord, name)) + Ps)
    case = G.make_case(rng, 3, 2, 64, 2, EDGE_LENS[name], Ps, Pd, ls, ld)
    check(case, 1, ranges=[(0, 3), (1, 2), (2, 2)])


@pytest.mark.parametrize("Ps,Pd", [(5, 7), (7, 5), (24, 16), (1, 1), (1, 64), (64, 1), (3, 128)])
@pytest.mark.parametrize("ls,ld", [(LM, LM), (PM, PM), (LM, PM)])
def test_page_sizes_that_do_not_divide(Ps, Pd, ls, ld):
    rng = np.random.default_rng(Ps * 1000 + Pd)
    lens = [0, 1, 34, 35, 36, 211, 500, Ps, Pd, Ps * Pd + 1]
    case = G.make_case(rng, 2, 1, 16, 1, lens, Ps, Pd, ls, ld)      # 16-byte rows: the smallest allowed
    check(case, 2)


def test_shared_source_pages_and_extra_ids():
    rng = np.random.default_rng(5)
    case = G.make_case(rng, 2, 2, 32, 2, [100, 7, 260, 33], 16, 8, LM, PM, shared_src=True, extra=2)
    check(case, 3)


def test_explicit_strides_padded_rows_and_pages():
    """Caller-given strides: rows padded (no two tokens adjacent) on the sender,
    pages padded on the receiver."""
    rng = np.random.default_rng(6)
    L, H, D, e, Ps, Pd = 2, 2, 32, 2, 8, 4
    row = H * D * e
    lens = np.array([9, 0, 40, 8, 17], dtype=np.uint32)
    nps, npd = 24, 48
    st_tok_s = row + 32
    st_page_s = Ps * st_tok_s + 64
    st_kv_s = nps * st_page_s
    st_layer_s = 2 * st_kv_s + 256
    s = G.Side(Ps, nps, 0, (st_layer_s, st_kv_s, st_page_s, st_tok_s), L * st_layer_s)
    st_page_d = Pd * row + 48
    st_kv_d = npd * st_page_d
    st_layer_d = 2 * st_kv_d
    d = G.Side(Pd, npd, 0, (st_layer_d, st_kv_d, st_page_d, row), L * st_layer_d)
    ids_s, offs_s = G.tables(rng, lens, Ps, nps)
    ids_d, offs_d = G.tables(rng, lens, Pd, npd)
    case = G.Case(L, H, D, e, lens, s, d, ids_s, offs_s, ids_d, offs_d)
    check(case, 4, ranges=[(0, 2), (1, 2)])


# ------------------------------------------------------------------ launch geometry does not matter
@pytest.mark.parametrize("launch", [
    dict(unroll=1), dict(unroll=2, nontemporal=1), dict(unroll=8, order=2),
    dict(unroll=4, xcd_swizzle=2), dict(unroll=8, xcd_swizzle=2, order=2, max_workgroups=24),
    dict(unroll=2, max_workgroups=7), dict(unroll=4, nontemporal=1, max_workgroups=1),
    dict(threads=64), dict(threads=128, unroll=2, xcd_swizzle=1), dict(threads=512, unroll=4, order=2),
    dict(threads=1024, unroll=8), dict(threads=1024, unroll=1, max_workgroups=16),
    dict(order=1), dict(order=2, xcd_swizzle=1), dict(order=2, threads=512, unroll=4),
    dict(order=3), dict(order=3, xcd_swizzle=1, max_workgroups=37), dict(order=3, threads=512, unroll=2, nontemporal=3),
    dict(order=3, xcd_block_tiles=64, max_workgroups=24),
    dict(threads=256, unroll=4, workgroups_per_cu=2), dict(threads=512, unroll=4, workgroups_per_cu=1),
    dict(nontemporal=3), dict(nontemporal=3, threads=512, unroll=4, order=2), dict(nontemporal=3, unroll=8),
    dict(nontemporal=2), dict(workgroups_per_cu=6), dict(xcd_block_tiles=8), dict(xcd_block_tiles=64, threads=64),
    dict(xcd_block_tiles=4096, order=2), dict(xcd_block_tiles=2, max_workgroups=40),
])
def test_results_do_not_depend_on_launch_config(launch):
    rng = np.random.default_rng(7)
    case = G.make_case(rng, 3, 4, 64, 2, [700, 1, 129, 64, 300, 0, 33], 32, 16, LM, PM)
    check(case, 5, launch=launch)


# ------------------------------------------------------------------ the five workloads, oracle-sized
def workload_case(idx, **scaled):
    w = W.CONFIGS[idx].scaled(**scaled) if scaled else W.CONFIGS[idx]
    b = W.draw_batch(w)
    return w, G.Case(w.num_layers, w.num_kv_heads, w.head_dim, w.elem_bytes, b.seq_lens,
                     G.Side(w.page_s, b.num_pages_s, w.layout_s), G.Side(w.page_d, b.num_pages_d, w.layout_d),
                     b.ids_s, b.offs_s, b.ids_d, b.offs_d)


def test_workload_1_tiny_full():
    w, case = workload_case(1)
    check(case, w.seed, kind=w.value_kind, ranges=[(0, 2), (1, 2)])


def test_workload_2_scaled():
    w, case = workload_case(2, num_layers=2, num_requests=4)
    check(case, w.seed, kind=w.value_kind)


def test_workload_3_scaled():
    w, case = workload_case(3, num_layers=4, num_requests=24)
    check(case, w.seed, kind=w.value_kind, ranges=[(0, 4), (3, 4)])


def test_workload_4_scaled():
    w, case = workload_case(4, num_layers=2, num_requests=8, len_hi=6000)
    check(case, w.seed, kind=w.value_kind)


def test_workload_5_scaled():
    w, case = workload_case(5, num_layers=2, num_requests=256)
    check(case, w.seed, kind=w.value_kind)


# ------------------------------------------------------------------ the device-built plan itself
def plan_table_lens(rng, batch, Ps, Pd):
    if batch == "staged":                  # more requests than one scan pass holds; tables copied from pinned memory
        lens = rng.integers(0, 900, size=1500).astype(np.uint32)
        lens[::97] = 0
        return lens
    # batches whose tables ride in the launch arguments (lengths + both sides' page ids <= 896 words): one
    # launch plans them, with 1, 4 or 16 waves
    count = {"one": 1, "four": 4, "five": 5, "sixty_four": 64, "sixty_five": 65, "three_hundred": 300}[batch]
    pages_each = (896 - count) // count    # pages a request may use on both sides together
    if pages_each >= 4:
        hi = int((pages_each - 2) / (1.0 / Ps + 1.0 / Pd))     # ceil() on either side costs at most one page
    else:
        hi = min(Ps, Pd)                   # one page per side; the empty requests below make the room
    lens = rng.integers(1, hi + 1, size=count).astype(np.uint32)
    if count > 4:
        lens[1::7] = 0
    return lens


@pytest.mark.parametrize("batch", ["staged", "one", "four", "five", "sixty_four", "sixty_five", "three_hundred"])
@pytest.mark.parametrize("Ps,Pd", [(16, 16), (128, 16), (5, 7)])
def test_device_plan_tables(Ps, Pd, batch):
    """The prefix scans and run records the kernels wrote: T_r is the exclusive
    sum of lengths, and per operation the runs of a request tile its tokens
    exactly once, in order, each run inside one page on both sides."""
    rng = np.random.default_rng(Ps + Pd + len(batch))
    lens = plan_table_lens(rng, batch, Ps, Pd)
    if batch != "staged":
        pages = lambda q: int(np.sum((lens.astype(np.int64) + q - 1) // q))
        assert len(lens) + pages(Ps) + pages(Pd) <= kvx.NOALLOC_MAX_TABLE_WORDS, "meant to fit the launch arguments"
    case = G.make_case(rng, 2, 1, 16, 1, lens, Ps, Pd, LM, PM)
    src = np.zeros(case.pool_bytes(case.s), dtype=np.uint8)
    res = G.run_gpu(case, src, 0, 2, want_tables=True)
    T = np.concatenate([[0], np.cumsum(lens.astype(np.uint64))])
    assert np.array_equal(res.extra["token_prefix"], T)
    row, bpt = case.row, 2 * 2 * case.row
    for op, (qa, qb) in enumerate([(Ps, None), (None, Pd), (Ps, Pd)]):
        runs, pre = res.extra[f"runs{op}"], res.extra[f"run_prefix{op}"]
        assert pre[0] == 0 and pre[-1] == len(runs)
        assert np.all(np.diff(pre.astype(np.int64)) >= 0)
        owner = np.repeat(np.arange(len(lens)), np.diff(pre.astype(np.int64)))
        if op == 2:
            # convert keeps a fixed number of slots per page of the coarser side; unclaimed slots are empty
            coarse, fine = max(Ps, Pd), min(Ps, Pd)
            slots = coarse // fine if coarse % fine == 0 else coarse // fine + 2
            pages = (lens.astype(np.int64) + coarse - 1) // coarse
            assert np.array_equal(np.diff(pre.astype(np.int64)), pages * slots)
            live = runs["bytes"] > 0
            assert np.all(runs["token"][live] // coarse == (np.arange(len(runs))[live] - pre[owner[live]]) // slots)
            runs, owner = runs[live], owner[live]
        req = runs["request"].astype(np.int64)
        assert np.array_equal(req, owner)
        assert np.array_equal(runs["seq_len"], lens[req])
        tok, ntok = runs["token"].astype(np.int64), runs["bytes"].astype(np.int64) // row
        assert np.all(runs["bytes"] % row == 0) and np.all(ntok > 0)
        nxt = tok + ntok
        same_req = req[1:] == req[:-1]
        first = np.ones(len(runs), dtype=bool)
        first[1:] = ~same_req
        assert np.all(tok[first] == 0)
        assert np.all(tok[1:][same_req] == nxt[:-1][same_req])                 # contiguous inside a request
        last = np.ones(len(runs), dtype=bool)
        last[:-1] = ~same_req
        assert np.array_equal(nxt[last], lens[req[last]].astype(np.int64))     # and they end at n_r
        assert np.array_equal(np.unique(req), np.flatnonzero(lens))           # every non-empty request is there
        for q in (qa, qb):
            if q:
                assert np.all(tok // q == (nxt - 1) // q)                      # never crosses a page
        buf_off = T[req].astype(np.int64) * bpt + tok * row
        if qa is None:
            assert np.array_equal(runs["src_off"].astype(np.int64), buf_off)
        if qb is None:
            assert np.array_equal(runs["dst_off"].astype(np.int64), buf_off)


@pytest.mark.parametrize("pages_second", [45, 46, 47, 48, 49])
def test_tables_on_either_side_of_the_launch_argument_limit(pages_second):
    """Small batches hand their tables to the device inside a kernel's launch arguments (896 words: lengths
    plus both sides' used page ids), larger ones through a staged copy.  2 requests with 400 + k pages per
    side give 2 + 2*(400 + k) words: k = 47 is the last that fits."""
    rng = np.random.default_rng(500 + pages_second)
    lens = [16 * 400 - 3, 16 * pages_second - 5]
    case = G.make_case(rng, 2, 1, 16, 1, lens, 16, 16, LM, PM)
    words = 2 + 2 * (400 + pages_second)
    assert (words <= 896) == (pages_second <= 47)
    check(case, 600 + pages_second)


ONE_SIDED = {
    # tables in the plan kernel's launch arguments
    "one_request": [16 * 20 - 7],
    "four_requests": [100, 0, 33, 16],
    "six_requests": [50, 7, 0, 160, 16, 1],
    "forty_requests": [3 * k % 41 for k in range(40)],
    "sixty_five_requests": [9] * 65,
    "one_request_895_pages": [16 * 895 - 1],        # 1 + 895 words: the most the launch arguments take
    # tables staged in pinned memory and copied
    "one_request_896_pages": [16 * 896],
    "one_request_2000_pages": [16 * 2000 - 7],
}


@pytest.mark.parametrize("name", sorted(ONE_SIDED))
def test_sender_only_and_receiver_only_plans(name):
    """One-sided plans (what a real sender or receiver builds) through both ways the tables reach the device."""
    import torch
    dev = torch.device("cuda:0")
    lens = ONE_SIDED[name]
    rng = np.random.default_rng(len(lens) + sum(lens))
    case = G.make_case(rng, 2, 2, 16, 2, lens, 16, 16, LM, LM)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    want = G.run_oracle(case, src, 0, 2)
    sb = kvx.BatchDesc(case.seq_lens, case.ids_s, case.offs_s)
    db = kvx.BatchDesc(case.seq_lens, case.ids_d, case.offs_d)
    sp, dp = case.kvx_pool(case.s), case.kvx_pool(case.d)
    stream = torch.cuda.Stream(device=dev)
    with torch.cuda.stream(stream):
        src_t = torch.from_numpy(src).to(dev)
        ws_s = torch.zeros(kvx.kvx_plan_workspace_bytes(sp, sb, None, None), dtype=torch.uint8, device=dev)
        ws_d = torch.zeros(kvx.kvx_plan_workspace_bytes(None, None, dp, db), dtype=torch.uint8, device=dev)
        buf = torch.full((want.total + G.BUF_SLACK,), G.CANARY_BUF, dtype=torch.uint8, device=dev)
        dst = torch.full((case.pool_bytes(case.d),), G.CANARY_POOL, dtype=torch.uint8, device=dev)
        ps = kvx.kvx_plan(sp, sb, None, None, 0, 2, ws_s.data_ptr(), ws_s.numel(), stream.cuda_stream)
        pd = kvx.kvx_plan(None, None, dp, db, 0, 2, ws_d.data_ptr(), ws_d.numel(), stream.cuda_stream)
        kvx.kvx_pack(ps, src_t.data_ptr(), buf.data_ptr(), want.total, stream.cuda_stream)
        kvx.kvx_unpack(pd, buf.data_ptr(), want.total, dst.data_ptr(), stream.cuda_stream)
        ps.destroy()
        pd.destroy()
    stream.synchronize()
    assert np.array_equal(buf.cpu().numpy(), want.buf)
    assert np.array_equal(dst.cpu().numpy(), want.dst_unpack)


@pytest.mark.parametrize("lens,Ps,Pd", [([77], 16, 16), ([1], 16, 4), ([4000], 128, 16), ([1700], 5, 7),
                                        ([16 * 447], 16, 16), ([16 * 447 + 1], 16, 16)])
def test_single_request_two_sided_plans(lens, Ps, Pd):
    """One request with both sides given, around the point where its tables stop fitting the launch
    arguments (1 + 2 x 447 words do, 1 + 2 x 448 do not)."""
    rng = np.random.default_rng(lens[0] + Ps)
    case = G.make_case(rng, 2, 1, 16, 1, lens, Ps, Pd, LM, PM)
    check(case, lens[0] + Pd)


def test_many_requests_whose_tables_still_fit_the_launch_arguments():
    """600 requests, 140 of them non-empty with one page each: 600 + 140 + 140 words ride in the launch
    arguments, and the scan runs with ten waves."""
    rng = np.random.default_rng(880)
    lens = np.zeros(600, dtype=np.uint32)
    lens[rng.choice(600, size=140, replace=False)] = rng.integers(1, 17, size=140)
    case = G.make_case(rng, 2, 2, 16, 2, lens, 16, 16, LM, PM)
    assert len(lens) + len(case.ids_s) + len(case.ids_d) == 880
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    want = G.run_oracle(case, src, 0, 2)
    got = G.run_gpu(case, src, 0, 2, want_tables=True)
    G.assert_same(got, want, "600 requests inline")
    assert np.array_equal(got.extra["token_prefix"], np.concatenate([[0], np.cumsum(lens.astype(np.uint64))]))


def test_plan_reuse_and_immediate_destroy():
    """A plan can be used many times, and destroyed right after enqueueing."""
    import torch
    rng = np.random.default_rng(9)
    case = G.make_case(rng, 2, 2, 64, 2, [300, 45, 1000], 16, 16)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    want = G.run_oracle(case, src, 0, 2)
    dev = torch.device("cuda:0")
    st = torch.cuda.Stream(device=dev)
    sp, dp = case.kvx_pool(case.s), case.kvx_pool(case.d)
    sb = kvx.BatchDesc(case.seq_lens, case.ids_s, case.offs_s)
    db = kvx.BatchDesc(case.seq_lens, case.ids_d, case.offs_d)
    nws = kvx.kvx_plan_workspace_bytes(sp, sb, dp, db)
    with torch.cuda.stream(st):
        src_t = torch.from_numpy(src).to(dev)
        outs = []
        for it in range(6):
            ws = torch.empty(nws, dtype=torch.uint8, device=dev)
            plan = kvx.kvx_plan(sp, sb, dp, db, 0, 2, ws.data_ptr(), nws, st.cuda_stream)
            buf = torch.full((want.total + G.BUF_SLACK,), G.CANARY_BUF, dtype=torch.uint8, device=dev)
            dst = torch.full((case.pool_bytes(case.d),), G.CANARY_POOL, dtype=torch.uint8, device=dev)
            for _ in range(2):
                kvx.kvx_pack(plan, src_t.data_ptr(), buf.data_ptr(), want.total, st.cuda_stream)
                kvx.kvx_unpack(plan, buf.data_ptr(), want.total, dst.data_ptr(), st.cuda_stream)
            plan.destroy()
            outs.append((ws, buf, dst))
    st.synchronize()
    for ws, buf, dst in outs:
        assert np.array_equal(buf.cpu().numpy(), want.buf)
        assert np.array_equal(dst.cpu().numpy(), want.dst_unpack)


def test_pinned_staging_blocks_are_reused_and_released_on_request():
    """Tables too large for a launch's arguments are staged in pinned blocks the library keeps between plans:
    plans made back to back (nothing completes in between) each get their own, idle ones are handed out
    again, kvx_release_cached gives them all back, and a plan made afterwards still comes out right."""
    import torch
    rng = np.random.default_rng(12)
    lens = rng.integers(1, 40, size=700).astype(np.uint32)          # 700 + 2 x ~1100 words: beyond 896
    case = G.make_case(rng, 1, 1, 16, 1, lens, 16, 16)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    want = G.run_oracle(case, src, 0, 1)
    dev = torch.device("cuda:0")
    st = torch.cuda.Stream(device=dev)
    sp, dp = case.kvx_pool(case.s), case.kvx_pool(case.d)
    sb = kvx.BatchDesc(case.seq_lens, case.ids_s, case.offs_s)
    db = kvx.BatchDesc(case.seq_lens, case.ids_d, case.offs_d)
    nws = kvx.kvx_plan_workspace_bytes(sp, sb, dp, db)
    torch.cuda.synchronize()
    kvx.kvx_release_cached()                                          # whatever earlier tests left behind
    assert kvx.kvx_release_cached() == 0
    with torch.cuda.stream(st):
        src_t = torch.from_numpy(src).to(dev)
        wss = [torch.empty(nws, dtype=torch.uint8, device=dev) for _ in range(5)]
        for ws in wss:
            kvx.kvx_plan(sp, sb, dp, db, 0, 1, ws.data_ptr(), nws, st.cuda_stream).destroy()
    st.synchronize()
    freed = kvx.kvx_release_cached()
    assert 0 < freed <= 5 * 64 * 1024 and freed % 4096 == 0, freed
    assert kvx.kvx_release_cached() == 0
    got = G.run_gpu(case, src, 0, 1)
    G.assert_same(got, want, "after the release")
    torch.cuda.synchronize()
    assert kvx.kvx_release_cached() > 0


def test_runtime_argument_errors():
    import torch
    rng = np.random.default_rng(10)
    case = G.make_case(rng, 1, 1, 64, 2, [40], 16, 16)
    dev = torch.device("cuda:0")
    sp = case.kvx_pool(case.s)
    sb = kvx.BatchDesc(case.seq_lens, case.ids_s, case.offs_s)
    nws = kvx.kvx_plan_workspace_bytes(sp, sb, None, None)
    ws = torch.empty(nws, dtype=torch.uint8, device=dev)
    with pytest.raises(kvx.KvxError) as e:
        kvx.kvx_plan(sp, sb, None, None, 0, 1, ws.data_ptr(), nws - 256)
    assert e.value.status == kvx.ERR_CAPACITY
    plan = kvx.kvx_plan(sp, sb, None, None, 0, 1, ws.data_ptr(), nws)
    total = kvx.kvx_plan_total_bytes(plan)
    pool = torch.zeros(case.pool_bytes(case.s), dtype=torch.uint8, device=dev)
    buf = torch.zeros(total + 64, dtype=torch.uint8, device=dev)
    for fn, args, status in [
        (kvx.kvx_pack, (plan, pool.data_ptr(), buf.data_ptr(), total - 1), kvx.ERR_CAPACITY),
        (kvx.kvx_pack, (plan, pool.data_ptr(), buf.data_ptr() + 8, total), kvx.ERR_ALIGNMENT),
        (kvx.kvx_pack, (plan, 0, buf.data_ptr(), total), kvx.ERR_INVALID_ARG),
        (kvx.kvx_unpack, (plan, buf.data_ptr(), total, pool.data_ptr()), kvx.ERR_INVALID_ARG),   # no receiver side
        (kvx.kvx_convert, (plan, pool.data_ptr(), pool.data_ptr()), kvx.ERR_INVALID_ARG),
    ]:
        with pytest.raises(kvx.KvxError) as e:
            fn(*args)
        assert e.value.status == status
    torch.cuda.synchronize()
    plan.destroy()


def test_convert_between_overlapping_dense_pools_is_refused():
    """Two pools with derived strides have known extents: a convert whose pools share bytes is turned down
    before anything is launched, in either order, and one whose pools only touch end to end is not."""
    import torch
    rng = np.random.default_rng(11)
    case = G.make_case(rng, 2, 2, 64, 2, [40, 9], 16, 8, LM, PM)
    dev = torch.device("cuda:0")
    sp, dp = case.kvx_pool(case.s), case.kvx_pool(case.d)
    sb = kvx.BatchDesc(case.seq_lens, case.ids_s, case.offs_s)
    db = kvx.BatchDesc(case.seq_lens, case.ids_d, case.offs_d)
    nws = kvx.kvx_plan_workspace_bytes(sp, sb, dp, db)
    ns, nd = case.pool_bytes(case.s), case.pool_bytes(case.d)
    ws = torch.empty(nws, dtype=torch.uint8, device=dev)
    arena = torch.full((ns + nd,), G.CANARY_POOL, dtype=torch.uint8, device=dev)
    plan = kvx.kvx_plan(sp, sb, dp, db, 0, 2, ws.data_ptr(), nws)
    a = arena.data_ptr()
    for src, dst in ((a, a), (a, a + ns - 16), (a + nd - 16, a), (a + 16, a)):
        with pytest.raises(kvx.KvxError) as e:
            kvx.kvx_convert(plan, src, dst)
        assert e.value.status == kvx.ERR_INVALID_ARG, (src - a, dst - a)
    torch.cuda.synchronize()
    assert bool((arena == G.CANARY_POOL).all())
    kvx.kvx_convert(plan, a, a + ns)          # back to back: allowed
    kvx.kvx_convert(plan, a + nd, a)          # receiver first
    torch.cuda.synchronize()
    plan.destroy()


# ------------------------------------------------------------------ extreme shapes
def test_many_tiny_requests_and_single_token_pages():
    """40 000 requests (40 passes of the scan kernel), pages of one token, 16-byte rows."""
    rng = np.random.default_rng(101)
    lens = rng.integers(0, 4, size=40000).astype(np.uint32)
    case = G.make_case(rng, 2, 1, 16, 1, lens, 1, 2, LM, PM)
    check(case, 102)


def test_one_very_long_request():
    """A single request of 300 000 tokens: offsets beyond 32 bits inside one request's segment."""
    rng = np.random.default_rng(103)
    case = G.make_case(rng, 1, 8, 128, 2, [300000], 128, 16, LM, LM, slack_pages=0)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    assert case.pool_bytes(case.s) > 2 ** 31
    want = G.run_oracle(case, src, 0, 1)
    got = G.run_gpu(case, src, 0, 1)
    G.assert_same(got, want, "long request")


def test_page_sizes_whose_lcm_exceeds_32_bits():
    """Pages of 65 537 and 65 539 tokens (coprime: the two grids never meet again below 2^32 tokens), 16-byte
    rows; the planner's run counts and ranks must not depend on the common multiple fitting a word."""
    rng = np.random.default_rng(107)
    case = G.make_case(rng, 1, 1, 8, 2, [150000, 70000, 65537, 65539, 5, 0], 65537, 65539, LM, LM, slack_pages=1)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    want = G.run_oracle(case, src, 0, 1)
    got = G.run_gpu(case, src, 0, 1, want_tables=True)
    G.assert_same(got, want, "huge lcm")
    # runs of convert: one per cut of either grid -> ceil(n/Ps) + ceil(n/Pd) - 1 per non-empty request,
    # stored in groups of (65539 // 65537 + 2) slots per receiver page
    runs = got.extra["runs2"]
    live = runs[runs["bytes"] > 0]
    expect = sum(-(-n // 65537) + -(-n // 65539) - 1 for n in (150000, 70000, 65537, 65539, 5))
    assert len(live) == expect
    assert int(live["bytes"].astype(np.int64).sum()) == (150000 + 70000 + 65537 + 65539 + 5) * 16


def test_wide_rows_and_large_pages():
    """64 KiB rows (64 heads x 256 x 4 bytes) in pages of 512 tokens: a 32 MiB page chunk."""
    rng = np.random.default_rng(104)
    case = G.make_case(rng, 1, 64, 256, 4, [513, 40], 512, 256, LM, PM, slack_pages=0)
    check(case, 105)


def test_head_slice_through_explicit_strides():
    """A slice of the heads of a wider pool (unequal tensor-parallel degrees between the sides): the
    pool is described with the slice's head count, the full pool's strides, and a base pointer moved to
    the first head of the slice."""
    rng = np.random.default_rng(106)
    L, H_full, D, e, Ps, Pd = 2, 8, 64, 2, 16, 8
    h0, h1 = 2, 5
    row_full = H_full * D * e
    lens = np.array([100, 7, 0, 260, 33], dtype=np.uint32)
    nps = 2 * int(sum((int(n) + Ps - 1) // Ps for n in lens)) + 1
    st_page = Ps * row_full
    st_kv = nps * st_page
    st_layer = 2 * st_kv
    full_bytes = L * st_layer
    off = h0 * D * e
    s = G.Side(Ps, nps, 0, (st_layer, st_kv, st_page, row_full), full_bytes - off)
    npd = 2 * int(sum((int(n) + Pd - 1) // Pd for n in lens)) + 1
    d = G.Side(Pd, npd, 1)                                            # the receiver holds just the slice, densely
    ids_s, offs_s = G.tables(rng, lens, Ps, nps)
    ids_d, offs_d = G.tables(rng, lens, Pd, npd)
    case = G.Case(L, h1 - h0, D, e, lens, s, d, ids_s, offs_s, ids_d, offs_d)
    full = rng.integers(0, 256, size=full_bytes, dtype=np.uint8)
    src = np.ascontiguousarray(full[off:])
    want = G.run_oracle(case, src, 0, L)
    got = G.run_gpu(case, src, 0, L)
    G.assert_same(got, want, "head slice")
    # and the slice really is heads [h0,h1) of every token: check one row against the full pool by hand
    r, t = 3, 41
    page = int(ids_s[int(offs_s[r]) + t // Ps])
    row = full[0 * st_layer + 1 * st_kv + page * st_page + (t % Ps) * row_full:][:row_full]
    T_r = int(lens[:r].sum())
    slice_row = (h1 - h0) * D * e
    o = T_r * L * 2 * slice_row + ((0 * 2 + 1) * int(lens[r]) + t) * slice_row
    assert np.array_equal(got.buf[o:o + slice_row], row[off:off + slice_row])
