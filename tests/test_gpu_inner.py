"""GPU parity for pools whose pages are not [token][head][dim] inside: head-major
pages, pages with the token axis inside 16-byte groups of the head dimension, and
pages with the token axis innermost element by element, on either side, against
the oracle, byte for byte (canaries included)."""
import numpy as np
import pytest

from paper_2408_08147_amd import kvx
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

ROWS, HEADS, SPLIT, TINNER = 0, 1, 2, 3
LM, PM = 0, 1


def check(case, seed, ranges=None, launch=None):
    rng = np.random.default_rng(seed)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    for l0, l1 in ranges or [(0, case.num_layers)]:
        want = G.run_oracle(case, src, l0, l1)
        got = G.run_gpu(case, src, l0, l1, launch=launch)
        G.assert_same(got, want, f"layers [{l0},{l1})")


COMBOS = [(HEADS, ROWS), (ROWS, HEADS), (ROWS, SPLIT), (SPLIT, ROWS), (SPLIT, HEADS), (HEADS, SPLIT),
          (SPLIT, SPLIT), (HEADS, HEADS)]
# the token axis innermost on at least one side: elements change place below the 16-byte grain
COMBOS_TINNER = [(ROWS, TINNER), (TINNER, ROWS), (TINNER, TINNER), (HEADS, TINNER), (TINNER, HEADS),
                 (SPLIT, TINNER), (TINNER, SPLIT)]


@pytest.mark.parametrize("ins,ind", COMBOS)
@pytest.mark.parametrize("H,D,e,Ps,Pd,ls,ld", [
    (8, 128, 2, 128, 16, LM, PM),      # 2 KiB rows, 128 -> 16 tokens per page, into page-major
    (1, 128, 2, 16, 16, LM, LM),       # one head: 256-byte rows
    (3, 48, 1, 5, 7, PM, LM),          # odd everything: 3 units per head, pages that do not divide
    (2, 64, 4, 64, 128, LM, LM),       # 4-byte elements, more tokens per page than a tile holds
])
def test_inner_arrangements(ins, ind, H, D, e, Ps, Pd, ls, ld):
    rng = np.random.default_rng(ins * 10 + ind + Ps)
    lens = [0, 1, 15, 16, 17, 200, 129, Ps, Pd, 2 * Pd + 1]
    case = G.make_case(rng, 3, H, D, e, lens, Ps, Pd, ls, ld, inner_s=ins, inner_d=ind)
    check(case, 11, ranges=[(0, 3), (1, 2)])


@pytest.mark.parametrize("ins,ind", COMBOS_TINNER)
@pytest.mark.parametrize("H,D,e,Ps,Pd,ls,ld", [
    (8, 128, 2, 128, 16, LM, PM),      # 2 KiB rows, 128 -> 16 tokens per page: columns of 256 and 32 bytes
    (1, 128, 2, 16, 16, LM, LM),       # one head: 256-byte rows
    (3, 48, 1, 5, 7, PM, LM),          # 1-byte elements, pages of 5 and 7 tokens: no column starts aligned
    (2, 64, 4, 64, 128, LM, LM),       # 4-byte elements
    (1, 16, 8, 512, 40, LM, PM),       # 8-byte elements, more tokens per page than a tile holds, 40*8 = 320-byte columns
    (2, 64, 1, 16, 48, PM, PM),        # 1-byte elements, 16 tokens = exactly one 16-byte piece per column
    (2, 32, 1, 256, 2, LM, LM),        # 128 runs per coarse page: more than a tile spanning the page can take
    (2, 32, 1, 64, 8, LM, PM),         # fine pages of 8 one-byte tokens: half a 16-byte piece per column
    (1, 64, 2, 24, 8, PM, LM),         # three fine pages per coarse one
])
def test_token_innermost_arrangements(ins, ind, H, D, e, Ps, Pd, ls, ld):
    rng = np.random.default_rng(100 + ins * 10 + ind + Ps)
    lens = [0, 1, 15, 16, 17, 200, 129, Ps, Pd, 2 * Pd + 1, 3 * Ps + 7]
    case = G.make_case(rng, 3, H, D, e, lens, Ps, Pd, ls, ld, inner_s=ins, inner_d=ind)
    check(case, 17, ranges=[(0, 3), (1, 2)])


@pytest.mark.parametrize("launch", [dict(order=1), dict(order=2), dict(xcd_swizzle=1), dict(nontemporal=1),
                                    dict(nontemporal=2), dict(nontemporal=3), dict(max_workgroups=5),
                                    dict(order=2, max_workgroups=16), dict(order=3)])
def test_token_innermost_results_do_not_depend_on_launch_config(launch):
    rng = np.random.default_rng(18)
    case = G.make_case(rng, 2, 4, 64, 2, [300, 1, 77, 0, 64, 33], 32, 16, LM, PM, inner_s=TINNER, inner_d=TINNER)
    check(case, 19, launch=launch)
    case = G.make_case(rng, 2, 4, 64, 2, [300, 1, 77, 0, 64, 33], 32, 16, PM, LM, inner_s=SPLIT, inner_d=TINNER)
    check(case, 20, launch=launch)


def test_token_innermost_shared_pages_and_layer_triggers():
    rng = np.random.default_rng(21)
    case = G.make_case(rng, 4, 2, 64, 2, [100, 7, 260, 33], 16, 8, LM, PM, shared_src=True, extra=1,
                       inner_s=TINNER, inner_d=ROWS)
    check(case, 22, ranges=[(0, 4), (3, 4), (1, 3)])
    case = G.make_case(rng, 4, 2, 64, 2, [100, 7, 260, 33], 24, 8, PM, LM, shared_src=True, extra=1,
                       inner_s=ROWS, inner_d=TINNER)
    check(case, 23, ranges=[(0, 4), (2, 3)])


@pytest.mark.parametrize("launch", [dict(order=1), dict(order=2), dict(xcd_swizzle=1), dict(nontemporal=1),
                                    dict(nontemporal=2), dict(nontemporal=3), dict(nontemporal=3, order=2),
                                    dict(max_workgroups=5), dict(order=2, max_workgroups=16), dict(order=3)])
def test_inner_results_do_not_depend_on_launch_config(launch):
    rng = np.random.default_rng(12)
    case = G.make_case(rng, 2, 4, 64, 2, [300, 1, 77, 0, 64, 33], 32, 16, LM, PM, inner_s=ROWS, inner_d=SPLIT)
    check(case, 13, launch=launch)


def test_inner_layer_triggers_and_shared_pages():
    import torch
    rng = np.random.default_rng(14)
    case = G.make_case(rng, 4, 2, 64, 2, [100, 7, 260, 33], 16, 8, LM, PM, shared_src=True, extra=1,
                       inner_s=HEADS, inner_d=SPLIT)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    want = G.run_oracle(case, src, 0, 4)
    dev = torch.device("cuda:0")
    st = torch.cuda.Stream(device=dev)
    sp, dp = case.kvx_pool(case.s), case.kvx_pool(case.d)
    sb = kvx.BatchDesc(case.seq_lens, case.ids_s, case.offs_s)
    db = kvx.BatchDesc(case.seq_lens, case.ids_d, case.offs_d)
    nws = kvx.kvx_plan_workspace_bytes(sp, sb, dp, db)
    with torch.cuda.stream(st):
        ws = torch.empty(nws, dtype=torch.uint8, device=dev)
        src_t = torch.from_numpy(src).to(dev)
        plan = kvx.kvx_plan(sp, sb, dp, db, 0, 4, ws.data_ptr(), nws, st.cuda_stream)
        buf = torch.full((want.total + G.BUF_SLACK,), G.CANARY_BUF, dtype=torch.uint8, device=dev)
        du = torch.full((case.pool_bytes(case.d),), G.CANARY_POOL, dtype=torch.uint8, device=dev)
        dc = torch.full((case.pool_bytes(case.d),), G.CANARY_POOL, dtype=torch.uint8, device=dev)
        for l in (3, 0, 2, 1):
            kvx.kvx_pack_layers(plan, l, l + 1, src_t.data_ptr(), buf.data_ptr(), want.total, st.cuda_stream)
        for l in range(4):
            kvx.kvx_unpack_layers(plan, l, l + 1, buf.data_ptr(), want.total, du.data_ptr(), st.cuda_stream)
            kvx.kvx_convert_layers(plan, l, l + 1, src_t.data_ptr(), dc.data_ptr(), st.cuda_stream)
    st.synchronize()
    G.assert_same(G.Result(want.total, buf.cpu().numpy(), du.cpu().numpy(), dc.cpu().numpy()), want, "layers")
    with pytest.raises(kvx.KvxError) as e:
        kvx.kvx_pack_blockwise(plan, src_t.data_ptr(), buf.data_ptr(), want.total, 0, st.cuda_stream)
    assert e.value.status == kvx.ERR_UNSUPPORTED
    plan.destroy()
