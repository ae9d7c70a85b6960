"""Asynchronous retrieval through a few receive slots (section 3.6): requests
arrive one by one into whichever slot is free, are scattered into the
receiver's pool on the slot's stream while a mock decoding loop keeps running,
and become valid when a poll reports their ticket.  At the end the receiver's
pool must equal the oracle's unpack of every request, byte for byte."""
import numpy as np
import pytest

from oracle import kvxo
from paper_2408_08147_amd import kvx
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def one_request_batches(case, r):
    """Sender- and receiver-side batch of request r alone."""
    a, b = int(case.offs_s[r]), int(case.offs_s[r + 1])
    c, d = int(case.offs_d[r]), int(case.offs_d[r + 1])
    n = [int(case.seq_lens[r])]
    return (n, case.ids_s[a:b], [0, b - a]), (n, case.ids_d[c:d], [0, d - c])


@pytest.mark.parametrize("num_slots", [1, 3])
def test_retrieval_through_slots(num_slots):
    import torch
    rng = np.random.default_rng(41 + num_slots)
    lens = [300, 17, 0, 129, 1000, 64, 5, 777, 256, 31, 400, 90]
    case = G.make_case(rng, 3, 2, 64, 2, lens, 16, 8, 0, 1)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    L, R, row = case.num_layers, len(lens), case.row

    # expected: the oracle scatters request after request into one canary pool
    pd = case.oracle_pool(case.d)
    ps = case.oracle_pool(case.s)
    want = np.full(case.pool_bytes(case.d), G.CANARY_POOL, dtype=np.uint8)
    for r in range(R):
        (n, ids_s, offs_s), (_, ids_d, offs_d) = one_request_batches(case, r)
        bs, bd = kvxo.Batch(n, ids_s, offs_s), kvxo.Batch(n, ids_d, offs_d)
        buf = np.zeros(kvxo.total_bytes(ps, bs, 0, L), dtype=np.uint8)
        kvxo.pack(ps, bs, 0, L, src, buf)
        kvxo.unpack(pd, bd, 0, L, buf, want)

    dev = torch.device("cuda:0")
    sp, dp = case.kvx_pool(case.s), case.kvx_pool(case.d)
    slot_buf = max(lens) * L * 2 * row
    slot_ws = 1 << 16
    arena_bytes = kvx.kvx_retriever_arena_bytes(num_slots, slot_buf, slot_ws)
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device=dev)
    src_t = torch.from_numpy(src).to(dev)
    dst = torch.full((case.pool_bytes(case.d),), G.CANARY_POOL, dtype=torch.uint8, device=dev)
    send_ws = torch.empty(num_slots, 1 << 16, dtype=torch.uint8, device=dev)   # the sender's own plan workspaces
    decode_state = torch.zeros(1 << 20, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    ret = kvx.kvx_retriever_create(num_slots, slot_buf, slot_ws, arena.data_ptr(), arena_bytes)

    with pytest.raises(kvx.KvxError) as e:
        kvx.kvx_retriever_acquire(ret, 99, slot_buf + 4096)
    assert e.value.status == kvx.ERR_CAPACITY

    pending = list(range(R))
    valid, iterations, saw_busy = [], 0, False
    while len(valid) < R:
        iterations += 1
        assert iterations < 100000
        decode_state.add_(1.0)                       # the running batch's step, on the main stream
        done = kvx.kvx_retriever_poll(ret)           # requests that became valid for this iteration
        assert not set(done) & set(valid), "a ticket was reported twice"
        valid += done
        while pending:                               # a completed request triggers the next retrieval
            r = pending[0]
            (n, ids_s, offs_s), (_, ids_d, offs_d) = one_request_batches(case, r)
            need = n[0] * L * 2 * row
            try:
                slot, buf_ptr, stream = kvx.kvx_retriever_acquire(ret, r, need)
            except kvx.KvxError as err:
                assert err.status == kvx.ERR_BUSY
                saw_busy = True
                break
            pending.pop(0)
            # the bytes "arrive": the sender packs this request straight into the slot's buffer
            sb = kvx.BatchDesc(n, ids_s, offs_s)
            plan = kvx.kvx_plan(sp, sb, None, None, 0, L, send_ws[slot].data_ptr(), send_ws.shape[1], stream)
            kvx.kvx_pack(plan, src_t.data_ptr(), buf_ptr, slot_buf, stream)
            plan.destroy()
            launch = kvx.LaunchCfg(0, 0, 0, 0, 256)   # a capped grid leaves the device to the running batch
            kvx.kvx_retriever_scatter(ret, slot, dp, kvx.BatchDesc(n, ids_d, offs_d), 0, L, dst.data_ptr(), launch)
    kvx.kvx_retriever_drain(ret)
    assert kvx.kvx_retriever_poll(ret) == []
    torch.cuda.synchronize()
    assert sorted(valid) == list(range(R))
    assert saw_busy, "the slots never filled up: the test did not exercise the queue"
    assert np.array_equal(dst.cpu().numpy(), want)
    assert float(decode_state[0]) == iterations

    # bookkeeping errors
    slot, _, _ = kvx.kvx_retriever_acquire(ret, 1234, 0)
    with pytest.raises(kvx.KvxError) as e:       # a receiver table with a page listed twice is refused, slot stays ours
        kvx.kvx_retriever_scatter(ret, slot, dp, kvx.BatchDesc([16], [3, 3], [0, 2]), 0, L, dst.data_ptr())
    assert e.value.status == kvx.ERR_BLOCK_TABLE
    kvx.kvx_retriever_abandon(ret, slot)
    with pytest.raises(kvx.KvxError) as e:
        kvx.kvx_retriever_abandon(ret, slot)
    assert e.value.status == kvx.ERR_INVALID_ARG
    ret.destroy()
