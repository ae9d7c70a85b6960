"""GPU parity at the full sizes of the synthetic workloads, in the default launch
configuration (the one bench.py times).

The pools do not fit the oracle in one piece, so the check is streamed by
layer: the GPU runs ONE full-range plan (one launch per operation); for each
layer the sender's slab of that layer is copied to the host, the
oracle runs on it as a one-layer pool, and its buffer segments and receiver
slab (untouched bytes included) are compared byte for byte with what the GPU
produced for that layer.  Segment positions inside the GPU's full-range buffer
come from the oracle's own full-range `segment`, so the layer-range
addressing is cross-checked as well.
"""
import numpy as np
import pytest

from oracle import kvxo
from paper_2408_08147_amd import kvx
from paper_2408_08147_amd import workloads as W
from tests import gpu_util as G

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(400)]

CANARY = 0xC3


def layer_slab(t, w, num_pages, page, layout, layer):
    """One layer of a dense pool tensor as a contiguous host array, laid out as
    a one-layer pool of the same layout."""
    row = w.row_bytes
    if layout == W.LAYER_MAJOR:
        n = 2 * num_pages * page * row
        return t[layer * n:(layer + 1) * n].cpu().numpy()
    v = t.view(num_pages, w.num_layers, 2 * page * row)
    return v[:, layer].contiguous().cpu().numpy().reshape(-1)


def run_fullsize(idx, layers_to_check, ops):
    import gc
    import torch
    w = W.CONFIGS[idx]
    b = W.draw_batch(w)
    dev = torch.device("cuda:0")
    gc.collect()
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    sp = kvx.pool_desc(w.num_layers, w.num_kv_heads, w.head_dim, w.elem_bytes, w.page_s, b.num_pages_s, w.layout_s)
    dp = kvx.pool_desc(w.num_layers, w.num_kv_heads, w.head_dim, w.elem_bytes, w.page_d, b.num_pages_d, w.layout_d)
    payload = w.num_layers * 2 * w.row_bytes * b.total_tokens
    need = sp.dense_bytes + dp.dense_bytes + (payload if "pack" in ops else 0)
    # no skip: on an MI355X (288 GB) every workload fits, and a skipped run would leave the workload unchecked
    assert need <= 0.95 * free, f"needs {need / 2**30:.0f} GiB of device memory, {free / 2**30:.0f} GiB free"
    st = torch.cuda.Stream(device=dev)
    sb = kvx.BatchDesc(b.seq_lens, b.ids_s, b.offs_s)
    db = kvx.BatchDesc(b.seq_lens, b.ids_d, b.offs_d)
    nws = kvx.kvx_plan_workspace_bytes(sp, sb, dp, db)
    print(f"workload {idx}: {b.total_tokens} tokens, payload {payload / 1e9:.2f} GB", flush=True)
    with torch.cuda.stream(st):
        ws = torch.empty(nws, dtype=torch.uint8, device=dev)
        src = torch.empty(sp.dense_bytes, dtype=torch.uint8, device=dev)
        W.fill_values_torch(w.value_kind, src, w.seed)
        dst = torch.full((dp.dense_bytes,), CANARY, dtype=torch.uint8, device=dev)
        plan = kvx.kvx_plan(sp, sb, dp, db, 0, w.num_layers, ws.data_ptr(), nws, st.cuda_stream)
        assert kvx.kvx_plan_total_bytes(plan) == payload
        if "pack" in ops:
            buf = torch.full((payload + G.BUF_SLACK,), G.CANARY_BUF, dtype=torch.uint8, device=dev)
            kvx.kvx_pack(plan, src.data_ptr(), buf.data_ptr(), payload, st.cuda_stream)
            kvx.kvx_unpack(plan, buf.data_ptr(), payload, dst.data_ptr(), st.cuda_stream)
        else:
            kvx.kvx_convert(plan, src.data_ptr(), dst.data_ptr(), st.cuda_stream)
    st.synchronize()

    o_full = kvxo.Pool(w.num_layers, w.num_kv_heads, w.head_dim, w.elem_bytes, w.page_s, b.num_pages_s, w.layout_s)
    o_s = kvxo.Pool(1, w.num_kv_heads, w.head_dim, w.elem_bytes, w.page_s, b.num_pages_s, w.layout_s)
    o_d = kvxo.Pool(1, w.num_kv_heads, w.head_dim, w.elem_bytes, w.page_d, b.num_pages_d, w.layout_d)
    obs, obd = kvxo.Batch(b.seq_lens, b.ids_s, b.offs_s), kvxo.Batch(b.seq_lens, b.ids_d, b.offs_d)
    per_layer = kvxo.total_bytes(o_s, obs, 0, 1)
    R = w.num_requests
    if "pack" in ops:
        assert bool((buf[payload:] == G.CANARY_BUF).all()), "bytes after the payload were written"
        seg_full = np.array([[kvxo.segment(o_full, obs, 0, w.num_layers, r, l) for r in range(R)]
                             for l in layers_to_check], dtype=np.int64)
    for k, layer in enumerate(layers_to_check):
        s_slab = layer_slab(src, w, b.num_pages_s, w.page_s, w.layout_s, layer)
        want_dst = np.full(o_d.nbytes, CANARY, dtype=np.uint8)
        if "pack" in ops:
            want_buf = np.empty(per_layer, dtype=np.uint8)
            kvxo.pack(o_s, obs, 0, 1, s_slab, want_buf, threads=G.ORACLE_THREADS)
            kvxo.unpack(o_d, obd, 0, 1, want_buf, want_dst, threads=G.ORACLE_THREADS)
            # the GPU buffer's bytes for this layer: one segment per request
            idx_lo, idx_len = seg_full[k, :, 0], seg_full[k, :, 1]
            got_parts = [buf[int(o):int(o + n)] for o, n in zip(idx_lo, idx_len) if n]
            got_buf = torch.cat(got_parts).cpu().numpy() if got_parts else np.empty(0, np.uint8)
            assert got_buf.size == want_buf.size
            assert np.array_equal(got_buf, want_buf), f"buffer differs in layer {layer}"
        else:
            kvxo.convert(o_s, obs, o_d, obd, 0, 1, s_slab, want_dst, threads=G.ORACLE_THREADS)
        got_dst = layer_slab(dst, w, b.num_pages_d, w.page_d, w.layout_d, layer)
        if not np.array_equal(got_dst, want_dst):
            bad = np.flatnonzero(got_dst != want_dst)
            raise AssertionError(f"receiver pool differs in layer {layer}: {bad.size} bytes, first {bad[0]}")
        print(f"  layer {layer} ok", flush=True)
    print(f"workload {idx}: {len(layers_to_check)} of {w.num_layers} layers compared", flush=True)
    plan.destroy()


def test_workload_2_full_every_layer():
    run_fullsize(2, list(range(32)), ("pack", "unpack"))


def test_workload_3_full_every_layer():
    run_fullsize(3, list(range(80)), ("pack", "unpack"))


def test_workload_5_full_every_layer():
    run_fullsize(5, list(range(40)), ("pack", "unpack"))


@pytest.mark.timeout(900)
def test_workload_4_full_convert_every_layer():
    run_fullsize(4, list(range(40)), ("convert",))


def test_workload_2_full_convert():
    run_fullsize(2, [0, 15, 31], ("convert",))
