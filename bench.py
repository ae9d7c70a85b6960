#!/usr/bin/env python3
"""Benchmark of the block-free KV transfer hot path on one MI355X.

One step = build the copy plan (kvx_plan: host validation, then the scan and
fill kernels, the lengths and block tables riding in the first one's launch
arguments or, for batches too large for that, in one H2D copy before it),
gather the batch's KV out of the sender's paged pool into the contiguous buffer
(kvx_pack), scatter it into the receiver's paged pool (kvx_unpack).  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.  The headline
is synthetic workload 2 (Llama-3-8B-shaped KV, 16 requests of 1024..4096
tokens, 128-token pages, scattered block tables) unless --workload says
otherwise; the other full-size workloads (3, 5, and 4 whose step is kvx_plan +
kvx_convert) follow under "other_workloads", each measured the same way, each
with its own roofline and CPU-oracle figures.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published peak

# HBM bytes per copy_kernel launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised under
# profiles/ (scaled by the plain-copy calibration).  They are figures of an earlier run, not of this one, and
# are reported only while the library that runs is built from the very sources they were taken on.
COUNTER_RUNS = {
    "build_id": "kvx-sources:941b7b59d54e3d8ae5b00e9ee1880ee4",
    "summary": "profiles/copy_kernel_workloads_2_3_5_4.txt",
    "traffic_bytes_per_launch": {2: 12103914358, 3: 13228422392, 5: 47001687500, 4: 152991552595},
}


def measured_traffic(workload: int):
    """(bytes per launch, where the figure comes from), or (None, None)."""
    from paper_2408_08147_amd import kvx
    if workload not in COUNTER_RUNS["traffic_bytes_per_launch"]:
        return None, None
    if kvx.kvx_build_id() != COUNTER_RUNS["build_id"]:
        return None, None  # the library changed since the counters were taken
    return COUNTER_RUNS["traffic_bytes_per_launch"][workload], COUNTER_RUNS["summary"]


class Setup:
    """Device-resident inputs and outputs of one workload."""

    def __init__(self, idx, with_dst: bool = True, with_buf: bool = True, fill: bool = True):
        import torch
        from paper_2408_08147_amd import kvx, workloads as W
        self.torch, self.kvx, self.W = torch, kvx, W
        kvx.load()
        self.w = w = W.CONFIGS[idx] if isinstance(idx, int) else idx
        self.batch = b = W.draw_batch(w)
        self.dev = torch.device("cuda:0")
        self.stream = torch.cuda.Stream(device=self.dev)
        self.sp = kvx.pool_desc(w.num_layers, w.num_kv_heads, w.head_dim, w.elem_bytes, w.page_s,
                                b.num_pages_s, w.layout_s, inner=w.inner_s)
        self.dp = kvx.pool_desc(w.num_layers, w.num_kv_heads, w.head_dim, w.elem_bytes, w.page_d,
                                b.num_pages_d, w.layout_d, inner=w.inner_d)
        self.sb = kvx.BatchDesc(b.seq_lens, b.ids_s, b.offs_s)
        self.db = kvx.BatchDesc(b.seq_lens, b.ids_d, b.offs_d)
        self.ws_bytes = kvx.kvx_plan_workspace_bytes(self.sp, self.sb, self.dp, self.db)
        self.bpt = w.num_layers * 2 * w.row_bytes
        self.payload = self.bpt * b.total_tokens
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.dev)
        self.src = torch.empty(self.sp.dense_bytes, dtype=torch.uint8, device=self.dev)
        if fill:
            W.fill_values_torch(w.value_kind, self.src, w.seed)
        self.dst = torch.full((self.dp.dense_bytes,), 0xC3, dtype=torch.uint8, device=self.dev) if with_dst else None
        self.buf = torch.empty(self.payload, dtype=torch.uint8, device=self.dev) if with_buf else None
        torch.cuda.synchronize()

    def plan(self, l0=0, l1=None, launch=None):
        l1 = self.w.num_layers if l1 is None else l1
        p = self.kvx.kvx_plan(self.sp, self.sb, self.dp, self.db, l0, l1, self.ws.data_ptr(), self.ws_bytes,
                              self.stream.cuda_stream)
        if launch:
            self.kvx.kvx_plan_set_launch(p, **launch)
        return p

    def pack(self, p):
        self.kvx.kvx_pack(p, self.src.data_ptr(), self.buf.data_ptr(), self.payload, self.stream.cuda_stream)

    def unpack(self, p):
        self.kvx.kvx_unpack(p, self.buf.data_ptr(), self.payload, self.dst.data_ptr(), self.stream.cuda_stream)

    def convert(self, p):
        self.kvx.kvx_convert(p, self.src.data_ptr(), self.dst.data_ptr(), self.stream.cuda_stream)

    def time_op(self, fn, iters=10, warmup=2):
        """Mean milliseconds per call of fn() by events on the library's stream."""
        torch = self.torch
        for _ in range(warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(self.stream)
        for _ in range(iters):
            fn()
        e1.record(self.stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / iters


def first_layers(t, w, num_pages, page, layout, layers):
    """The first `layers` layers of a dense pool tensor, laid out as a pool of that many layers."""
    row = w.row_bytes
    if layout == 0:  # layer-major: a leading slice
        return t[: layers * 2 * num_pages * page * row]
    return t.view(num_pages, w.num_layers, 2 * page * row)[:, :layers].contiguous().view(-1)


def cpu_baseline(setup: Setup, convert_only: bool, target_bytes: float = 1.5e9):
    """Times the CPU oracle on the first few layers of the same workload, copied off the device (pack +
    unpack, or convert for the conversion workload), and checks the GPU result for those layers against it."""
    import numpy as np
    from oracle import kvxo
    w, b = setup.w, setup.batch
    per_layer = 2 * w.row_bytes * b.total_tokens
    layers = int(max(1, min(w.num_layers, target_bytes // per_layer)))
    src = first_layers(setup.src, w, b.num_pages_s, w.page_s, w.layout_s, layers).cpu().numpy()
    ps = kvxo.Pool(layers, w.num_kv_heads, w.head_dim, w.elem_bytes, w.page_s, b.num_pages_s, w.layout_s)
    pd = kvxo.Pool(layers, w.num_kv_heads, w.head_dim, w.elem_bytes, w.page_d, b.num_pages_d, w.layout_d)
    bs, bd = kvxo.Batch(b.seq_lens, b.ids_s, b.offs_s), kvxo.Batch(b.seq_lens, b.ids_d, b.offs_d)
    total = kvxo.total_bytes(ps, bs, 0, layers)
    cores = len(os.sched_getaffinity(0))
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    out = {}
    buf = None if convert_only else np.empty(total, dtype=np.uint8)
    dst = np.full(pd.nbytes, 0xC3, dtype=np.uint8)
    for label, th in (("threads_1", 1), ("all", cores)):
        t0 = time.perf_counter()
        if convert_only:
            kvxo.convert(ps, bs, pd, bd, 0, layers, src, dst, threads=th)
            t1 = t2 = time.perf_counter()
            moved = total
        else:
            kvxo.pack(ps, bs, 0, layers, src, buf, threads=th)
            t1 = time.perf_counter()
            kvxo.unpack(pd, bd, 0, layers, buf, dst, threads=th)
            t2 = time.perf_counter()
            moved = 2 * total
        out[label] = dict(first_s=t1 - t0, second_s=t2 - t1, gbps=moved / (t2 - t0) / 1e9)
    # parity at full shape on the sample: the GPU's result for these layers, through its own full-range plan
    plan = setup.plan()
    with setup.torch.cuda.stream(setup.stream):
        setup.dst.fill_(0xC3)
    if convert_only:
        setup.convert(plan)
    else:
        setup.pack(plan)
        setup.unpack(plan)
    setup.stream.synchronize()
    got_dst = first_layers(setup.dst, w, b.num_pages_d, w.page_d, w.layout_d, layers).cpu().numpy()
    ok = bool(np.array_equal(got_dst, dst))
    if not convert_only:
        gbuf = setup.buf.cpu().numpy()
        for r in range(w.num_requests):
            for l in (0, layers - 1):
                o, n = setup.kvx.kvx_plan_segment(plan, r, l)
                oo, nn = kvxo.segment(ps, bs, 0, layers, r, l)
                ok = ok and n == nn and bool(np.array_equal(gbuf[o:o + n], buf[oo:oo + nn]))
    plan.destroy()
    both = out["all"]["first_s"] + out["all"]["second_s"]
    what = "convert" if convert_only else "pack+unpack"
    return {
        "value": round(out["all"]["gbps"], 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
        "sample": f"{what} of layers [0,{layers}) of the same batch ({total / 1e9:.2f} GB payload), "
                  f"moved bytes = {'payload' if convert_only else '2*payload'}; value is measured on the sample, "
                  f"us_per_request is the sample's time scaled to all {w.num_layers} layers",
        "extrapolated_from_layers": layers, "of_layers": w.num_layers,
        "value_1_thread": round(out["threads_1"]["gbps"], 3),
        "us_per_request": round(both * 1e6 / w.num_requests * (w.num_layers / layers), 1),
        "gpu_matches_oracle_on_sample": ok,
    }


def measure(workload: int, K: int, Wm: int, with_cpu: bool):
    """Times K steps of one workload after Wm warm-up steps; returns the fields of its report."""
    import torch
    convert_only = workload == 4
    s = Setup(workload, with_buf=not convert_only)
    kvx, w = s.kvx, s.w

    def step(events=None):
        p = s.plan()
        if events is not None:
            events[0].record(s.stream)
        if convert_only:
            s.convert(p)
        else:
            s.pack(p)
        if events is not None:
            events[1].record(s.stream)
        if not convert_only:
            s.unpack(p)
        if events is not None:
            events[2].record(s.stream)
        p.destroy()

    for _ in range(Wm):
        step()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        step(evs[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / K
    pack_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / K
    unpack_ms = sum(e[1].elapsed_time(e[2]) for e in evs) / K
    per_step = sorted(e[0].elapsed_time(e[2]) for e in evs)   # the launches of one step, plan kernels excluded

    # outside the step: plan alone (host + device part), convert pool to pool, plain D2D copy ceiling
    t2 = time.perf_counter()
    for _ in range(20):
        s.plan().destroy()
    s.stream.synchronize()
    plan_ms = (time.perf_counter() - t2) * 1e3 / 20
    p = s.plan()
    convert_ms = s.time_op(lambda: s.convert(p), iters=5, warmup=1)
    p.destroy()
    # plain contiguous copy of a known size with the same access shape: the measured ceiling
    scratch = s.dst if convert_only else s.buf
    half = min(scratch.numel() // 2, 4 << 30) // 4096 * 4096
    yard_ms = s.time_op(lambda: kvx.kvx_copy_yardstick(scratch.data_ptr(), scratch.data_ptr() + half, half,
                                                       s.stream.cuda_stream), iters=10, warmup=2)
    with torch.cuda.stream(s.stream):
        memcpy_ms = s.time_op(lambda: scratch[:half].copy_(scratch[half:2 * half]), iters=5, warmup=1)

    if convert_only:
        dom_name, dom_ms = "kvx_convert", pack_ms
        moved = s.payload / (ms_step * 1e-3) / 1e9
        traffic_per_step = 2 * s.payload
    else:
        dom_name, dom_ms = ("kvx_pack", pack_ms) if pack_ms >= unpack_ms else ("kvx_unpack", unpack_ms)
        moved = 2 * s.payload / (ms_step * 1e-3) / 1e9
        traffic_per_step = 4 * s.payload
    achieved = 2 * s.payload / (dom_ms * 1e-3) / 1e9
    R = w.num_requests
    traffic, traffic_from = measured_traffic(workload)
    out = {
        "value": round(moved, 1), "unit": "GB/s", "steps": K, "warmup": Wm, "ms_per_step": round(ms_step, 4),
        "config": {"workload": f"{s.w.index}:{w.name}", "layers": w.num_layers, "kv_heads": w.num_kv_heads,
                   "head_dim": w.head_dim, "elem_bytes": w.elem_bytes, "page_tokens": w.page_s,
                   "requests": R, "total_tokens": s.batch.total_tokens, "payload_bytes": s.payload,
                   "step": "kvx_plan + kvx_convert" if convert_only else "kvx_plan + kvx_pack + kvx_unpack"},
        "hbm_frac_step": round(traffic_per_step / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "us_per_request": round(ms_step * 1e3 / R, 2), "requests_per_s": round(R / (ms_step * 1e-3), 1),
        "ops": {"plan_ms": round(plan_ms, 4),
                "step_kernels_ms_median": round(per_step[len(per_step) // 2], 4),
                "step_kernels_ms_min": round(per_step[0], 4),
                "pack_ms": None if convert_only else round(pack_ms, 4),
                "unpack_ms": None if convert_only else round(unpack_ms, 4),
                "convert_ms": round(convert_ms, 4),
                "pack_hbm_GBps": None if convert_only else round(2 * s.payload / pack_ms / 1e6, 1),
                "unpack_hbm_GBps": None if convert_only else round(2 * s.payload / unpack_ms / 1e6, 1),
                "convert_hbm_GBps": round(2 * s.payload / convert_ms / 1e6, 1),
                "yardstick_copy_hbm_GBps": round(2 * half / yard_ms / 1e6, 1), "yardstick_bytes": half,
                "torch_d2d_copy_hbm_GBps": round(2 * half / memcpy_ms / 1e6, 1)},
        "roofline": {"bound": "hbm", "kernel": dom_name, "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "algorithmic_bytes_per_launch": 2 * s.payload,
                     "traffic": traffic, "traffic_from": traffic_from,
                     # beside the published peak: what a plain contiguous copy of the same access shape
                     # reached in this very process (kvx_copy_yardstick)
                     "frac_of_plain_copy": round(achieved / (2 * half / yard_ms / 1e6), 4)},
    }
    if with_cpu:
        out["cpu_baseline"] = cpu_baseline(s, convert_only)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=2, choices=[1, 2, 3, 4, 5],
                    help="4 = page-size/layout conversion: the step is kvx_plan + kvx_convert")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="only the headline workload (profiling runs use this)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this path runs on one GPU (no collectives, no sharding); use --gpus 1")

    import gc
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    head = measure(args.workload, args.steps, args.warmup, not args.no_cpu_baseline)
    out = {"metric": "kv_pack_unpack_moved", "value": head.pop("value"), "unit": head.pop("unit"),
           "n_gpus": 1, "steps": head.pop("steps"), "warmup": head.pop("warmup"),
           "ms_per_step": head.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "u8", "data": "synthetic"}
    out.update(head)
    if not args.no_other_workloads:
        # the other full-size workloads, each a short run of the same kind: same fields, one entry each
        out["other_workloads"] = []
        for idx in (3, 5, 4):
            if idx == args.workload:
                continue
            gc.collect()
            torch.cuda.empty_cache()
            try:
                out["other_workloads"].append(measure(idx, max(args.steps, 20) if idx != 4 else args.steps,
                                                      args.warmup, not args.no_cpu_baseline))
            except (RuntimeError, MemoryError) as e:
                # the headline must still be printed, e.g. when the device lacks the 163 GB workload 4 takes
                out["other_workloads"].append({"config": {"workload": str(idx)}, "error": str(e)[:300]})
    print(json.dumps(out))


if __name__ == "__main__":
    main()
