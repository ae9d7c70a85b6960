#!/usr/bin/env python3
"""Side measurements around the hot path (each prints JSON lines; bench.py stays the headline):

  blocks   the block-fixed transfer of section 2.2.3 in one-GPU form: one device copy per
           (request, layer, K|V, page) issued from the host, with and without a host wait per block,
           against ONE planned kernel launch, over a sweep of page sizes at fixed tokens
  layers   per-layer triggers (section 3.6): the whole model in one launch, one launch per layer on the
           same plan and buffer, and the same with the grid capped to a share of the compute units
  retrieval asynchronous retrieval (section 3.6): requests arriving one by one through k receive slots
  overlap  RecvScatter beside a stand-in for the running model (GEMMs on another stream), grid capped or not
  slice    a head slice of a wider sender pool through explicit strides (unequal tensor-parallel degrees)
  ops      every operation of a workload by itself, a few launches in a row each (pack, unpack, convert, then
           the plain contiguous copy of as many bytes): under a hardware-counter run the dispatches come in
           exactly that order, so each counter reading can be given to its operation; `--sorted` first sorts
           the page ids of the named side(s), which keeps the sizes and makes that side's chunks near-sequential
  layouts  pools whose pages are head-major or keep the token axis inside 16-byte groups of the head
           dimension, against plain [token][head][dim] pages of the same shape
"""
import argparse
import json
import sys
import time

import bench


def study_blocks(args):
    from paper_2408_08147_amd import workloads as W
    base = W.CONFIGS[2]
    for P in (16, 32, 64, 128, 256, 512):
        w = base.scaled(page_s=P, page_d=P, num_layers=args.layers)
        s = bench.Setup(w, with_dst=False)
        kvx, torch = s.kvx, s.torch
        p = s.plan()
        t_kernel = s.time_op(lambda: s.pack(p), iters=10, warmup=2)
        blocks = len(s.batch.ids_s) * w.num_layers * 2

        def blockwise(confirm):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            kvx.kvx_pack_blockwise(p, s.src.data_ptr(), s.buf.data_ptr(), s.payload, confirm, s.stream.cuda_stream)
            s.stream.synchronize()
            return (time.perf_counter() - t0) * 1e3
        blockwise(0)
        t_async = min(blockwise(0) for _ in range(2))
        t_confirm = blockwise(1)
        p.destroy()
        print(json.dumps({
            "study": "blocks", "page_tokens": P, "block_bytes": P * w.row_bytes, "blocks": blocks,
            "payload_bytes": s.payload, "layers": w.num_layers,
            "planned_kernel_ms": round(t_kernel, 4), "blockwise_async_ms": round(t_async, 3),
            "blockwise_confirm_each_ms": round(t_confirm, 3),
            "planned_kernel_GBps_moved": round(s.payload / t_kernel / 1e6, 1),
            "blockwise_async_GBps_moved": round(s.payload / t_async / 1e6, 1),
            "blockwise_confirm_each_GBps_moved": round(s.payload / t_confirm / 1e6, 1),
            "time_saved_vs_async": round(1 - t_kernel / t_async, 4),
            "time_saved_vs_confirm_each": round(1 - t_kernel / t_confirm, 4)}), flush=True)
        del s
        torch.cuda.empty_cache()


def study_layers(args):
    s = bench.Setup(args.workload)
    kvx, w = s.kvx, s.w
    L = w.num_layers
    p = s.plan()
    whole = s.time_op(lambda: (s.pack(p), s.unpack(p)), iters=10, warmup=2)

    def per_layer():
        for l in range(L):
            kvx.kvx_pack_layers(p, l, l + 1, s.src.data_ptr(), s.buf.data_ptr(), s.payload, s.stream.cuda_stream)
        for l in range(L):
            kvx.kvx_unpack_layers(p, l, l + 1, s.buf.data_ptr(), s.payload, s.dst.data_ptr(), s.stream.cuda_stream)
    layered = s.time_op(per_layer, iters=10, warmup=2)
    one = s.time_op(lambda: kvx.kvx_pack_layers(p, 0, 1, s.src.data_ptr(), s.buf.data_ptr(), s.payload,
                                                s.stream.cuda_stream), iters=50, warmup=5)
    # the same 2*L launches captured once in a HIP graph and replayed
    import torch
    s.stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s.stream):
        per_layer()
    torch.cuda.synchronize()
    with torch.cuda.stream(s.stream):
        graphed = s.time_op(graph.replay, iters=10, warmup=2)
    print(json.dumps({"study": "layers", "workload": w.name, "layers": L, "payload_bytes": s.payload,
                      "whole_model_pack_unpack_ms": round(whole, 4),
                      "layer_by_layer_pack_unpack_ms": round(layered, 4),
                      "layer_by_layer_hip_graph_replay_ms": round(graphed, 4),
                      "one_layer_pack_us": round(one * 1e3, 2),
                      "one_layer_payload_bytes": s.payload // L,
                      "one_layer_hbm_GBps": round(2 * s.payload / L / one / 1e6, 1)}), flush=True)
    # a transfer that leaves most of the device to the model: cap the grid (256-lane workgroups,
    # up to 8 resident per compute unit, so 8*k workgroups keep about k of the 256 units busy)
    for cus in (8, 16, 32, 64, 128, 256):
        kvx.kvx_plan_set_launch(p, max_workgroups=8 * cus)
        t = s.time_op(lambda: kvx.kvx_pack_layers(p, 0, 1, s.src.data_ptr(), s.buf.data_ptr(), s.payload,
                                                  s.stream.cuda_stream), iters=20, warmup=3)
        print(json.dumps({"study": "layers_cu_capped", "compute_units": cus, "max_workgroups": 8 * cus,
                          "one_layer_pack_us": round(t * 1e3, 2),
                          "hbm_GBps": round(2 * s.payload / L / t / 1e6, 1)}), flush=True)
    p.destroy()


def study_layouts(args):
    from paper_2408_08147_amd import workloads as W
    names = {0: "rows", 1: "head_major", 2: "dim_split_token", 3: "token_innermost"}
    shapes = [("workload2 shape, 128-token pages", W.CONFIGS[2], {}),
              ("workload2 shape, 16-token pages", W.CONFIGS[2], dict(page_s=16, page_d=16)),
              ("workload2 shape, 128 -> 16 tokens, page-major receiver", W.CONFIGS[2],
               dict(page_d=16, layout_d=W.PAGE_MAJOR)),
              ("workload3 shape (one head, 256-byte rows)", W.CONFIGS[3], {})]
    for label, base, kw in shapes:
        for ins, ind in [(0, 0), (0, 1), (1, 0), (0, 2), (2, 0), (2, 2), (1, 2), (0, 3), (3, 0), (3, 3), (2, 3)]:
            w = base.scaled(inner_s=ins, inner_d=ind, **kw)
            s = bench.Setup(w, fill=False)
            p = s.plan()
            tp = s.time_op(lambda: s.pack(p), iters=8, warmup=2)
            tu = s.time_op(lambda: s.unpack(p), iters=8, warmup=2)
            tc = s.time_op(lambda: s.convert(p), iters=8, warmup=2)
            p.destroy()
            g = lambda ms: round(2 * s.payload / ms / 1e6, 1)
            print(json.dumps({"study": "layouts", "shape": label, "sender_pages": names[ins],
                              "receiver_pages": names[ind], "payload_bytes": s.payload,
                              "pack_hbm_GBps": g(tp), "unpack_hbm_GBps": g(tu), "convert_hbm_GBps": g(tc)}),
                  flush=True)
            del s
            import torch
            torch.cuda.empty_cache()


def study_retrieval(args):
    """Requests of the workload-5 shape arrive one by one and are scattered through k receive slots;
    k = 1 is one transfer after another."""
    import numpy as np
    import torch
    from paper_2408_08147_amd import kvx, workloads as W
    w = W.CONFIGS[5].scaled(num_requests=args.requests)
    b = W.draw_batch(w)
    dev = torch.device("cuda:0")
    L, row = w.num_layers, w.row_bytes
    sp = kvx.pool_desc(L, w.num_kv_heads, w.head_dim, w.elem_bytes, w.page_s, b.num_pages_s, w.layout_s)
    dp = kvx.pool_desc(L, w.num_kv_heads, w.head_dim, w.elem_bytes, w.page_d, b.num_pages_d, w.layout_d)
    src = torch.empty(sp.dense_bytes, dtype=torch.uint8, device=dev)
    dst = torch.empty(dp.dense_bytes, dtype=torch.uint8, device=dev)
    reqs = []
    for r in range(w.num_requests):
        n = [int(b.seq_lens[r])]
        a, z = int(b.offs_s[r]), int(b.offs_s[r + 1])
        c, y = int(b.offs_d[r]), int(b.offs_d[r + 1])
        reqs.append((n[0] * L * 2 * row, kvx.BatchDesc(n, b.ids_s[a:z], [0, z - a]),
                     kvx.BatchDesc(n, b.ids_d[c:y], [0, y - c])))
    payload = sum(x[0] for x in reqs)
    slot_buf = max(x[0] for x in reqs)
    for k in (1, 2, 4, 8, 16):
        arena_bytes = kvx.kvx_retriever_arena_bytes(k, slot_buf, 1 << 16)
        arena = torch.empty(arena_bytes, dtype=torch.uint8, device=dev)
        send_ws = torch.empty(k, 1 << 16, dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()
        ret = kvx.kvx_retriever_create(k, slot_buf, 1 << 16, arena.data_ptr(), arena_bytes)
        for timed in (False, True):
            pending, done, polls = list(range(len(reqs))), 0, 0
            submitted_at, latency = {}, []
            t0 = time.perf_counter()
            while done < len(reqs):
                polls += 1
                for t in kvx.kvx_retriever_poll(ret):
                    latency.append(time.perf_counter() - submitted_at[t])
                    done += 1
                while pending:
                    need, sb, db = reqs[pending[0]]
                    try:
                        slot, buf_ptr, stream = kvx.kvx_retriever_acquire(ret, pending[0], need)
                    except kvx.KvxError:
                        break
                    submitted_at[pending.pop(0)] = time.perf_counter()
                    plan = kvx.kvx_plan(sp, sb, None, None, 0, L)      # planned on the host when small enough
                    if not kvx.kvx_plan_can_launch(plan):
                        plan.destroy()
                        plan = kvx.kvx_plan(sp, sb, None, None, 0, L, send_ws[slot].data_ptr(), 1 << 16, stream)
                    kvx.kvx_pack(plan, src.data_ptr(), buf_ptr, slot_buf, stream)
                    plan.destroy()
                    kvx.kvx_retriever_scatter(ret, slot, dp, db, 0, L, dst.data_ptr())
            kvx.kvx_retriever_drain(ret)
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
        ret.destroy()
        print(json.dumps({"study": "retrieval", "slots": k, "requests": len(reqs), "payload_bytes": payload,
                          "total_ms": round(wall * 1e3, 3), "us_per_request": round(wall * 1e6 / len(reqs), 2),
                          "mean_completion_us": round(1e6 * sum(latency) / len(latency), 1),
                          "GBps_moved_pack_plus_unpack": round(2 * payload / wall / 1e9, 1)}), flush=True)


def study_overlap(args):
    """RecvScatter beside a running model (section 3.6: the operator form must not interrupt the other
    operators; retrieval does no harm to the running requests): a stand-in for decoding (bf16 GEMMs from
    torch on one stream) runs alone, then with unpacks of workload 2 in a loop on another stream, with the
    transfer's grid uncapped and capped."""
    import torch
    s = bench.Setup(args.workload)
    kvx = s.kvx
    p = s.plan()
    s.pack(p)
    s.stream.synchronize()
    a = torch.randn(8192, 8192, device=s.dev, dtype=torch.bfloat16)
    b = torch.randn(8192, 8192, device=s.dev, dtype=torch.bfloat16)
    model_stream = torch.cuda.Stream(device=s.dev)
    flops = 2 * 8192 ** 3
    reps = 40

    def gemms():
        with torch.cuda.stream(model_stream):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(model_stream)
            for _ in range(reps):
                torch.matmul(a, b)
            e1.record(model_stream)
        return e0, e1

    e0, e1 = gemms()
    e1.synchronize()
    e0, e1 = gemms()
    e1.synchronize()
    alone_ms = e0.elapsed_time(e1) / reps
    t_alone = s.time_op(lambda: s.unpack(p), iters=10, warmup=2)
    print(json.dumps({"study": "overlap", "case": "each alone", "gemm_ms": round(alone_ms, 4),
                      "gemm_TFLOPs": round(flops / alone_ms / 1e9, 1), "unpack_ms": round(t_alone, 4),
                      "unpack_hbm_GBps": round(2 * s.payload / t_alone / 1e6, 1)}), flush=True)
    for cap in (0, 2048, 512, 256, 128):
        kvx.kvx_plan_set_launch(p, max_workgroups=cap)
        n_unpacks = 30
        t0 = torch.cuda.Event(enable_timing=True)
        t1 = torch.cuda.Event(enable_timing=True)
        t0.record(s.stream)
        for _ in range(n_unpacks):
            s.unpack(p)
        t1.record(s.stream)
        e0, e1 = gemms()
        e1.synchronize()
        t1.synchronize()
        both_gemm = e0.elapsed_time(e1) / reps
        both_unpack = t0.elapsed_time(t1) / n_unpacks
        print(json.dumps({"study": "overlap", "case": "together", "transfer_max_workgroups": cap or "uncapped",
                          "gemm_ms": round(both_gemm, 4), "gemm_slowdown": round(both_gemm / alone_ms, 3),
                          "unpack_ms": round(both_unpack, 4),
                          "unpack_hbm_GBps": round(2 * s.payload / both_unpack / 1e6, 1)}), flush=True)
    p.destroy()


def study_slice(args):
    """A head slice of a wider sender pool (sender with all 8 KV heads, receiver holding heads [2,6)):
    the sender is described by explicit strides and a moved base pointer; rows are 1 KiB pieces at a
    2 KiB pitch, so the tile kernel moves them."""
    import torch
    from paper_2408_08147_amd import kvx, workloads as W
    w = W.CONFIGS[2]
    b = W.draw_batch(w)
    dev = torch.device("cuda:0")
    st = torch.cuda.Stream(device=dev)
    L, D, e, P = w.num_layers, w.head_dim, w.elem_bytes, w.page_s
    h0, h1, H_full = 2, 6, w.num_kv_heads
    row_full = H_full * D * e
    st_page = P * row_full
    st_kv = b.num_pages_s * st_page
    st_layer = 2 * st_kv
    sp = kvx.pool_desc(L, h1 - h0, D, e, P, b.num_pages_s, 0, (st_layer, st_kv, st_page, row_full))
    dp = kvx.pool_desc(L, h1 - h0, D, e, w.page_d, b.num_pages_d, w.layout_d)
    sb = kvx.BatchDesc(b.seq_lens, b.ids_s, b.offs_s)
    db = kvx.BatchDesc(b.seq_lens, b.ids_d, b.offs_d)
    nws = kvx.kvx_plan_workspace_bytes(sp, sb, dp, db)
    src = torch.empty(L * st_layer, dtype=torch.uint8, device=dev)
    dst = torch.empty(dp.dense_bytes, dtype=torch.uint8, device=dev)
    ws = torch.empty(nws, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    plan = kvx.kvx_plan(sp, sb, dp, db, 0, L, ws.data_ptr(), nws, st.cuda_stream)
    total = kvx.kvx_plan_total_bytes(plan)
    buf = torch.empty(total, dtype=torch.uint8, device=dev)
    base = src.data_ptr() + h0 * D * e
    timer = bench.Setup.time_op

    holder = type("H", (), {"torch": torch, "stream": st})()
    tp = timer(holder, lambda: kvx.kvx_pack(plan, base, buf.data_ptr(), total, st.cuda_stream), iters=8, warmup=2)
    tu = timer(holder, lambda: kvx.kvx_unpack(plan, buf.data_ptr(), total, dst.data_ptr(), st.cuda_stream), iters=8,
               warmup=2)
    tc = timer(holder, lambda: kvx.kvx_convert(plan, base, dst.data_ptr(), st.cuda_stream), iters=8, warmup=2)
    plan.destroy()
    g = lambda ms: round(2 * total / ms / 1e6, 1)
    print(json.dumps({"study": "head_slice", "shape": "workload 2, heads [2,6) of 8", "payload_bytes": total,
                      "piece_bytes": (h1 - h0) * D * e, "pitch_bytes": row_full,
                      "pack_hbm_GBps": g(tp), "unpack_hbm_GBps": g(tu), "convert_hbm_GBps": g(tc)}), flush=True)


def study_ops(args):
    import numpy as np
    s = bench.Setup(args.workload, fill=False)
    kvx, b = s.kvx, s.batch
    if "s" in args.sorted:
        b.ids_s = np.sort(b.ids_s)
        s.sb = kvx.BatchDesc(b.seq_lens, b.ids_s, b.offs_s)
    if "d" in args.sorted:
        b.ids_d = np.sort(b.ids_d)
        s.db = kvx.BatchDesc(b.seq_lens, b.ids_d, b.offs_d)
    p = s.plan()
    n = args.reps
    half = min(s.payload, 4 << 30) // 4096 * 4096
    assert s.src.numel() >= half and s.dst.numel() >= half
    order = [("pack", lambda: s.pack(p)), ("unpack", lambda: s.unpack(p)), ("convert", lambda: s.convert(p)),
             ("plain_copy", lambda: kvx.kvx_copy_yardstick(s.dst.data_ptr(), s.src.data_ptr(), half,
                                                            s.stream.cuda_stream))]
    out = {"study": "ops", "workload": f"{s.w.index}:{s.w.name}", "sorted_sides": args.sorted, "launches_each": n + 1,
           "order": [name for name, _ in order], "payload_bytes": s.payload, "plain_copy_bytes": half}
    for name, fn in order:
        ms = s.time_op(fn, iters=n, warmup=1)
        nbytes = half if name == "plain_copy" else s.payload
        out[name + "_ms"] = round(ms, 4)
        out[name + "_hbm_GBps"] = round(2 * nbytes / ms / 1e6, 1)
    p.destroy()
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("study", choices=["blocks", "layers", "layouts", "retrieval", "slice", "overlap", "ops"])
    ap.add_argument("--requests", type=int, default=512, help="retrieval: requests of the workload-5 shape")
    ap.add_argument("--workload", type=int, default=2, choices=[2, 3, 5])
    ap.add_argument("--layers", type=int, default=8, help="blocks: layers of the workload-2 shape to move")
    ap.add_argument("--reps", type=int, default=4, help="ops: timed launches per operation (after one warm-up)")
    ap.add_argument("--sorted", default="", choices=["", "s", "d", "sd"],
                    help="ops: sort the page ids of the sender (s) and/or receiver (d) side first")
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench_studies.py: no GPU visible")
    {"blocks": study_blocks, "layers": study_layers, "layouts": study_layouts,
     "retrieval": study_retrieval, "slice": study_slice, "overlap": study_overlap,
     "ops": study_ops}[args.study](args)


if __name__ == "__main__":
    main()
