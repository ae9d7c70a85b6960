"""Plans without a device workspace that can still run: one side, token-row pages, at most KVX_INLINE_RUNS used
pages.  The host works the run records out and kvx_pack / kvx_unpack carry them in their launch arguments, so
nothing is planned on the device (section 3.6: the sender's gather and the receiver's RecvScatter, one launch
each).  Every result is compared byte for byte with the oracle, canaries included."""
import numpy as np
import pytest

from oracle import kvxo
from paper_2408_08147_amd import kvx
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

LM, PM = 0, 1

# name -> (lens, sender page, receiver page, sender layout, receiver layout)
CASES = {
    "one_token": ([1], 16, 16, LM, LM),
    "one_request": ([16 * 20 - 7], 16, 16, LM, LM),
    "one_request_page_major": ([16 * 20 - 7], 16, 16, PM, PM),
    "ninety_six_pages": ([16 * 96], 16, 16, LM, PM),
    "ninety_six_pages_ragged": ([16 * 50 - 1, 0, 16 * 45 + 1], 16, 16, LM, LM),     # 50 + 46 pages
    "several_requests": ([100, 0, 33, 16, 1, 250], 16, 16, LM, PM),
    "odd_pages": ([77, 5, 0, 130], 5, 7, PM, LM),
    "coarse_pages": ([4000, 129], 128, 128, LM, LM),
    "ninety_six_requests": ([3] * 96, 16, 16, LM, LM),
}


def sides(case):
    return (case.kvx_pool(case.s), kvx.BatchDesc(case.seq_lens, case.ids_s, case.offs_s),
            case.kvx_pool(case.d), kvx.BatchDesc(case.seq_lens, case.ids_d, case.offs_d))


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("launch", [None, dict(threads=64, unroll=8), dict(threads=1024, unroll=2, order=1),
                                    dict(max_workgroups=8, nontemporal=1), dict(workgroups_per_cu=1)])
def test_pack_and_unpack_without_a_workspace(name, launch):
    import torch
    dev = torch.device("cuda:0")
    lens, Ps, Pd, ls, ld = CASES[name]
    rng = np.random.default_rng(len(lens) + sum(lens) + Ps)
    case = G.make_case(rng, 3, 2, 16, 2, lens, Ps, Pd, ls, ld)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    want = G.run_oracle(case, src, 0, 3)
    sp, sb, dp, db = sides(case)
    stream = torch.cuda.Stream(device=dev)
    with torch.cuda.stream(stream):
        src_t = torch.from_numpy(src).to(dev)
        buf = torch.full((want.total + G.BUF_SLACK,), G.CANARY_BUF, dtype=torch.uint8, device=dev)
        dst = torch.full((case.pool_bytes(case.d),), G.CANARY_POOL, dtype=torch.uint8, device=dev)
        ps = kvx.kvx_plan(sp, sb, None, None, 0, 3)
        pd = kvx.kvx_plan(None, None, dp, db, 0, 3)
        assert kvx.kvx_plan_can_launch(ps) and kvx.kvx_plan_can_launch(pd)
        assert kvx.kvx_plan_total_bytes(ps) == want.total == kvx.kvx_plan_total_bytes(pd)
        if launch:
            kvx.kvx_plan_set_launch(ps, **launch)
            kvx.kvx_plan_set_launch(pd, **launch)
        kvx.kvx_pack(ps, src_t.data_ptr(), buf.data_ptr(), want.total, stream.cuda_stream)
        kvx.kvx_unpack(pd, buf.data_ptr(), want.total, dst.data_ptr(), stream.cuda_stream)
        ps.destroy()        # the launches carry all they need
        pd.destroy()
    stream.synchronize()
    assert np.array_equal(buf.cpu().numpy(), want.buf)
    assert np.array_equal(dst.cpu().numpy(), want.dst_unpack)
    assert np.array_equal(src_t.cpu().numpy(), src)


def test_layer_subranges_without_a_workspace():
    """kvx_pack_layers / kvx_unpack_layers on such a plan touch their layers' segments only; all sub-ranges
    together give the whole-range result."""
    import torch
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(96)
    case = G.make_case(rng, 5, 2, 32, 2, [300, 0, 17, 129], 16, 16, LM, PM)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    L0, L1 = 1, 5
    want = G.run_oracle(case, src, L0, L1)
    ops, obs = case.oracle_pool(case.s), kvxo.Batch(case.seq_lens, case.ids_s, case.offs_s)
    sp, sb, dp, db = sides(case)
    stream = torch.cuda.Stream(device=dev)
    with torch.cuda.stream(stream):
        src_t = torch.from_numpy(src).to(dev)
        buf = torch.full((want.total + G.BUF_SLACK,), G.CANARY_BUF, dtype=torch.uint8, device=dev)
        dst = torch.full((case.pool_bytes(case.d),), G.CANARY_POOL, dtype=torch.uint8, device=dev)
        ps = kvx.kvx_plan(sp, sb, None, None, L0, L1)
        pd = kvx.kvx_plan(None, None, dp, db, L0, L1)
        kvx.kvx_pack_layers(ps, 2, 3, src_t.data_ptr(), buf.data_ptr(), want.total, stream.cuda_stream)
        stream.synchronize()
        part = buf.cpu().numpy()
        expect = np.full_like(part, G.CANARY_BUF)
        for r in range(len(case.seq_lens)):
            off, n = kvxo.segment(ops, obs, L0, L1, r, 2)
            expect[off:off + n] = want.buf[off:off + n]
        assert np.array_equal(part, expect), "one layer's segments and nothing else"
        for lb, le in [(1, 2), (3, 5)]:
            kvx.kvx_pack_layers(ps, lb, le, src_t.data_ptr(), buf.data_ptr(), want.total, stream.cuda_stream)
        for lb, le in [(4, 5), (1, 4)]:
            kvx.kvx_unpack_layers(pd, lb, le, buf.data_ptr(), want.total, dst.data_ptr(), stream.cuda_stream)
    stream.synchronize()
    assert np.array_equal(buf.cpu().numpy(), want.buf)
    assert np.array_equal(dst.cpu().numpy(), want.dst_unpack)


def test_same_bytes_as_the_plan_with_a_workspace_under_graph_replay():
    """The launch of such a plan recorded into a HIP graph: its arguments hold the run records, so replays
    after the plan is gone, with eager work in between, keep giving the oracle's bytes."""
    import torch
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(7)
    case = G.make_case(rng, 2, 2, 32, 2, [200, 31, 0, 64], 16, 16, LM, LM)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    want = G.run_oracle(case, src, 0, 2)
    sp, sb, dp, db = sides(case)
    src_t = torch.from_numpy(src).to(dev)
    buf = torch.zeros(want.total + G.BUF_SLACK, dtype=torch.uint8, device=dev)
    dst = torch.zeros(case.pool_bytes(case.d), dtype=torch.uint8, device=dev)
    ps = kvx.kvx_plan(sp, sb, None, None, 0, 2)
    pd = kvx.kvx_plan(None, None, dp, db, 0, 2)
    side = torch.cuda.Stream(device=dev)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # one eager pass first: nothing is set up lazily under capture
        kvx.kvx_pack(ps, src_t.data_ptr(), buf.data_ptr(), want.total, side.cuda_stream)
        kvx.kvx_unpack(pd, buf.data_ptr(), want.total, dst.data_ptr(), side.cuda_stream)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        kvx.kvx_pack(ps, src_t.data_ptr(), buf.data_ptr(), want.total, side.cuda_stream)
        kvx.kvx_unpack(pd, buf.data_ptr(), want.total, dst.data_ptr(), side.cuda_stream)
    ps.destroy()
    pd.destroy()
    for replay in range(3):
        buf.fill_(G.CANARY_BUF)         # eager work between the replays
        dst.fill_(G.CANARY_POOL)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(buf.cpu().numpy(), want.buf), replay
        assert np.array_equal(dst.cpu().numpy(), want.dst_unpack), replay
