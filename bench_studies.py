#!/usr/bin/env python3
"""Side measurements around the hot path (each prints JSON lines; bench.py stays the headline):

  blocks   the block-fixed transfer of section 2.2.3 in one-GPU form: one device copy per
           (request, layer, K|V, page) issued from the host, with and without a host wait per block,
           against ONE planned kernel launch, over a sweep of page sizes at fixed tokens
  layers   per-layer triggers (section 3.6): the whole model in one launch, one launch per layer on the
           same plan and buffer, and the same with the grid capped to a share of the compute units
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
    print(json.dumps({"study": "layers", "workload": w.name, "layers": L, "payload_bytes": s.payload,
                      "whole_model_pack_unpack_ms": round(whole, 4),
                      "layer_by_layer_pack_unpack_ms": round(layered, 4),
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
    names = {0: "rows", 1: "head_major", 2: "dim_split_token"}
    shapes = [("workload2 shape, 128-token pages", W.CONFIGS[2], {}),
              ("workload2 shape, 16-token pages", W.CONFIGS[2], dict(page_s=16, page_d=16)),
              ("workload2 shape, 128 -> 16 tokens, page-major receiver", W.CONFIGS[2],
               dict(page_d=16, layout_d=W.PAGE_MAJOR)),
              ("workload3 shape (one head, 256-byte rows)", W.CONFIGS[3], {})]
    for label, base, kw in shapes:
        for ins, ind in [(0, 0), (0, 1), (1, 0), (0, 2), (2, 0), (2, 2), (1, 2)]:
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("study", choices=["blocks", "layers", "layouts"])
    ap.add_argument("--workload", type=int, default=2, choices=[2, 3, 5])
    ap.add_argument("--layers", type=int, default=8, help="blocks: layers of the workload-2 shape to move")
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench_studies.py: no GPU visible")
    {"blocks": study_blocks, "layers": study_layers, "layouts": study_layouts}[args.study](args)


if __name__ == "__main__":
    main()
