"""Per-layer triggers: kvx_pack_layers / kvx_unpack_layers / kvx_convert_layers
touch exactly the chosen layers' segments of the whole-range buffer (and the
chosen layers of the receiver's pool) and nothing else.  Expected bytes come
from the oracle run on one-layer ranges, placed at the whole-range `segment`
offsets (section 3.6: per-layer or whole-model transfer into the same buffer)."""
import numpy as np
import pytest

from oracle import kvxo
from paper_2408_08147_amd import kvx
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def setup_case(ls, ld, Ps, Pd):
    rng = np.random.default_rng(31 + Ps + Pd)
    case = G.make_case(rng, 5, 2, 64, 2, [300, 0, 17, 129, 1000, 64], Ps, Pd, ls, ld)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    return case, src


@pytest.mark.parametrize("ls,ld,Ps,Pd", [(0, 0, 16, 16), (0, 1, 128, 16), (1, 0, 8, 24)])
def test_layer_subranges_touch_only_their_segments(ls, ld, Ps, Pd):
    import torch
    case, src = setup_case(ls, ld, Ps, Pd)
    L0, L1 = 1, 5                                  # the plan's range does not start at layer 0
    picks = [(2, 3), (4, 5)]
    ps, pd = case.oracle_pool(case.s), case.oracle_pool(case.d)
    bs = kvxo.Batch(case.seq_lens, case.ids_s, case.offs_s)
    bd = kvxo.Batch(case.seq_lens, case.ids_d, case.offs_d)
    total = kvxo.total_bytes(ps, bs, L0, L1)
    R = len(case.seq_lens)

    # expected: canaries, plus one-layer oracle results at whole-range segment offsets
    want_buf = np.full(total + G.BUF_SLACK, G.CANARY_BUF, dtype=np.uint8)
    full_buf = np.zeros(total, dtype=np.uint8)
    kvxo.pack(ps, bs, L0, L1, src, full_buf)
    want_unpack = np.full(case.pool_bytes(case.d), G.CANARY_POOL, dtype=np.uint8)
    want_convert = want_unpack.copy()
    for lb, le in picks:
        for l in range(lb, le):
            part = np.zeros(kvxo.total_bytes(ps, bs, l, l + 1), dtype=np.uint8)
            kvxo.pack(ps, bs, l, l + 1, src, part)
            for r in range(R):
                ow, nw = kvxo.segment(ps, bs, L0, L1, r, l)
                op, n1 = kvxo.segment(ps, bs, l, l + 1, r, l)
                want_buf[ow:ow + nw] = part[op:op + n1]
            kvxo.unpack(pd, bd, l, l + 1, part, want_unpack)
            kvxo.convert(ps, bs, pd, bd, l, l + 1, src, want_convert)

    dev = torch.device("cuda:0")
    st = torch.cuda.Stream(device=dev)
    sp, dp = case.kvx_pool(case.s), case.kvx_pool(case.d)
    sb = kvx.BatchDesc(case.seq_lens, case.ids_s, case.offs_s)
    db = kvx.BatchDesc(case.seq_lens, case.ids_d, case.offs_d)
    nws = kvx.kvx_plan_workspace_bytes(sp, sb, dp, db)
    with torch.cuda.stream(st):
        ws = torch.empty(nws, dtype=torch.uint8, device=dev)
        src_t = torch.from_numpy(src).to(dev)
        full_t = torch.from_numpy(full_buf).to(dev)
        plan = kvx.kvx_plan(sp, sb, dp, db, L0, L1, ws.data_ptr(), nws, st.cuda_stream)
        assert kvx.kvx_plan_total_bytes(plan) == total
        buf = torch.full((total + G.BUF_SLACK,), G.CANARY_BUF, dtype=torch.uint8, device=dev)
        du = torch.full((case.pool_bytes(case.d),), G.CANARY_POOL, dtype=torch.uint8, device=dev)
        dc = torch.full((case.pool_bytes(case.d),), G.CANARY_POOL, dtype=torch.uint8, device=dev)
        for lb, le in picks:
            kvx.kvx_pack_layers(plan, lb, le, src_t.data_ptr(), buf.data_ptr(), total, st.cuda_stream)
            kvx.kvx_unpack_layers(plan, lb, le, full_t.data_ptr(), total, du.data_ptr(), st.cuda_stream)
            kvx.kvx_convert_layers(plan, lb, le, src_t.data_ptr(), dc.data_ptr(), st.cuda_stream)
        kvx.kvx_pack_layers(plan, 3, 3, src_t.data_ptr(), buf.data_ptr(), total, st.cuda_stream)   # empty: no-op
    st.synchronize()
    assert np.array_equal(buf.cpu().numpy(), want_buf)
    assert np.array_equal(du.cpu().numpy(), want_unpack)
    assert np.array_equal(dc.cpu().numpy(), want_convert)

    for bad in [(0, 2), (4, 6), (3, 2)]:
        with pytest.raises(kvx.KvxError) as e:
            kvx.kvx_pack_layers(plan, bad[0], bad[1], src_t.data_ptr(), buf.data_ptr(), total, st.cuda_stream)
        assert e.value.status == kvx.ERR_INVALID_ARG
    plan.destroy()


def test_all_layers_one_by_one_equal_the_whole():
    import torch
    case, src = setup_case(0, 1, 32, 16)
    want = G.run_oracle(case, src, 0, case.num_layers)
    dev = torch.device("cuda:0")
    st = torch.cuda.Stream(device=dev)
    sp, dp = case.kvx_pool(case.s), case.kvx_pool(case.d)
    sb = kvx.BatchDesc(case.seq_lens, case.ids_s, case.offs_s)
    db = kvx.BatchDesc(case.seq_lens, case.ids_d, case.offs_d)
    nws = kvx.kvx_plan_workspace_bytes(sp, sb, dp, db)
    with torch.cuda.stream(st):
        ws = torch.empty(nws, dtype=torch.uint8, device=dev)
        src_t = torch.from_numpy(src).to(dev)
        plan = kvx.kvx_plan(sp, sb, dp, db, 0, case.num_layers, ws.data_ptr(), nws, st.cuda_stream)
        buf = torch.full((want.total + G.BUF_SLACK,), G.CANARY_BUF, dtype=torch.uint8, device=dev)
        du = torch.full((case.pool_bytes(case.d),), G.CANARY_POOL, dtype=torch.uint8, device=dev)
        dc = torch.full((case.pool_bytes(case.d),), G.CANARY_POOL, dtype=torch.uint8, device=dev)
        for l in reversed(range(case.num_layers)):          # order of the triggers does not matter
            kvx.kvx_pack_layers(plan, l, l + 1, src_t.data_ptr(), buf.data_ptr(), want.total, st.cuda_stream)
        for l in range(case.num_layers):
            kvx.kvx_unpack_layers(plan, l, l + 1, buf.data_ptr(), want.total, du.data_ptr(), st.cuda_stream)
            kvx.kvx_convert_layers(plan, l, l + 1, src_t.data_ptr(), dc.data_ptr(), st.cuda_stream)
    st.synchronize()
    got = G.Result(want.total, buf.cpu().numpy(), du.cpu().numpy(), dc.cpu().numpy())
    G.assert_same(got, want, "layer by layer")
    plan.destroy()


@pytest.mark.parametrize("confirm_every", [0, 1, 7])
def test_blockwise_baseline_gives_the_same_buffer(confirm_every):
    """The block-by-block reference point must produce kvx_pack's bytes."""
    import torch
    case, src = setup_case(0, 0, 16, 16)
    want = G.run_oracle(case, src, 1, 4)
    dev = torch.device("cuda:0")
    st = torch.cuda.Stream(device=dev)
    sp = case.kvx_pool(case.s)
    sb = kvx.BatchDesc(case.seq_lens, case.ids_s, case.offs_s)
    plan = kvx.kvx_plan(sp, sb, None, None, 1, 4)            # host-only plan: no workspace needed
    with torch.cuda.stream(st):
        src_t = torch.from_numpy(src).to(dev)
        buf = torch.full((want.total + G.BUF_SLACK,), G.CANARY_BUF, dtype=torch.uint8, device=dev)
    st.synchronize()
    kvx.kvx_pack_blockwise(plan, src_t.data_ptr(), buf.data_ptr(), want.total, confirm_every, st.cuda_stream)
    st.synchronize()
    assert np.array_equal(buf.cpu().numpy(), want.buf)
    plan.destroy()


def test_blockwise_baseline_with_padded_rows():
    import torch
    rng = np.random.default_rng(77)
    L, H, D, e, Ps = 2, 2, 32, 2, 8
    row = H * D * e
    lens = np.array([9, 0, 40, 8], dtype=np.uint32)
    nps = 24
    st_tok = row + 32
    st_page = Ps * st_tok + 64
    st_kv = nps * st_page
    st_layer = 2 * st_kv + 256
    s = G.Side(Ps, nps, 0, (st_layer, st_kv, st_page, st_tok), L * st_layer)
    ids, offs = G.tables(rng, lens, Ps, nps)
    case = G.Case(L, H, D, e, lens, s, s, ids, offs, ids, offs)
    src = rng.integers(0, 256, size=case.pool_bytes(s), dtype=np.uint8)
    po, bo = case.oracle_pool(s), kvxo.Batch(lens, ids, offs)
    total = kvxo.total_bytes(po, bo, 0, L)
    want = np.full(total + 64, 0x5A, dtype=np.uint8)
    kvxo.pack(po, bo, 0, L, src, want)
    dev = torch.device("cuda:0")
    plan = kvx.kvx_plan(case.kvx_pool(s), kvx.BatchDesc(lens, ids, offs), None, None, 0, L)
    src_t = torch.from_numpy(src).to(dev)
    buf = torch.full((total + 64,), 0x5A, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    kvx.kvx_pack_blockwise(plan, src_t.data_ptr(), buf.data_ptr(), total, 0, 0)
    torch.cuda.synchronize()
    assert np.array_equal(buf.cpu().numpy(), want)
    plan.destroy()


def test_layer_triggers_captured_in_a_hip_graph():
    """The per-layer launches carry plain kernel arguments and no memset, so a whole layer-by-layer
    transfer can be captured once and replayed; every replay, with eager work in between, must give
    what the eager calls give on the data of that moment."""
    import torch
    case, src = setup_case(0, 1, 32, 16)
    L = case.num_layers
    dev = torch.device("cuda:0")
    st = torch.cuda.Stream(device=dev)
    sp, dp = case.kvx_pool(case.s), case.kvx_pool(case.d)
    sb = kvx.BatchDesc(case.seq_lens, case.ids_s, case.offs_s)
    db = kvx.BatchDesc(case.seq_lens, case.ids_d, case.offs_d)
    nws = kvx.kvx_plan_workspace_bytes(sp, sb, dp, db)
    with torch.cuda.stream(st):
        ws = torch.empty(nws, dtype=torch.uint8, device=dev)
        src_t = torch.from_numpy(src).to(dev)
        plan = kvx.kvx_plan(sp, sb, dp, db, 0, L, ws.data_ptr(), nws, st.cuda_stream)   # built eagerly, outside the graph
        total = kvx.kvx_plan_total_bytes(plan)
        buf = torch.full((total + G.BUF_SLACK,), G.CANARY_BUF, dtype=torch.uint8, device=dev)
        dst = torch.full((case.pool_bytes(case.d),), G.CANARY_POOL, dtype=torch.uint8, device=dev)
    st.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=st):
        for l in range(L):
            kvx.kvx_pack_layers(plan, l, l + 1, src_t.data_ptr(), buf.data_ptr(), total, st.cuda_stream)
        for l in range(L):
            kvx.kvx_unpack_layers(plan, l, l + 1, buf.data_ptr(), total, dst.data_ptr(), st.cuda_stream)
    torch.cuda.synchronize()
    rng = np.random.default_rng(55)
    for rep in range(4):
        # eager work between the replays: new source bytes, destination and buffer back to canaries
        new_src = rng.integers(0, 256, size=src.size, dtype=np.uint8)
        src_t.copy_(torch.from_numpy(new_src))
        buf.fill_(G.CANARY_BUF)
        dst.fill_(G.CANARY_POOL)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = G.run_oracle(case, new_src, 0, L)
        assert np.array_equal(buf.cpu().numpy(), want.buf), f"replay {rep}: buffer"
        assert np.array_equal(dst.cpu().numpy(), want.dst_unpack), f"replay {rep}: receiver pool"
    plan.destroy()
