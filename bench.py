"""Benchmark of the structured-binary hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Headline workload: the LLaMA-70B-shaped decoder layer (q/o 8192x8192 and k/v 1024x8192 at 6:8, gate/up 28672x8192 at
4:8, down 8192x28672 at 2:4; the largest of the five workloads, 355 MB of packed weights) as decode at batch 1.  A step
is one pass over all seven matrices: four calls of stb_gemv_batched in the order a decoder layer needs them (q, k and v
share their input; o; gate and up share theirs; down).  Each step reads another copy of the packed weights (tiled
device order) out of a pool of more than 1 GiB, so the weights come from HBM and not from the 256 MB last-level cache.
Inputs are resident in HBM before the timed region.  After W warm-up steps (default 200: the step time of a GPU that
has been idle falls for about 180 steps) the K steps are captured once in a HIP graph; the graph is replayed W / K
times untimed, then several times timed, and `ms_per_step` is the median timed replay divided by K (the fastest
replay is reported beside it).
`value` is packed-weight GB/s (bytes of the packed format) over the whole timed region, launch gaps included.

`roofline` describes the dominant kernel, the decode GEMV: algorithmic bytes per launch (packed planes + x + y) divided
by the average duration of a launch, measured with events on the launch stream over the same timed region.

After the timed steps the same JSON line gets: one row per (workload, layer, batch) for the decode shapes of all five
workloads and one per (workload, layer, tokens) for the prefill shapes (stb_gemm, with its own roofline against the
fp16 matrix peak), the streaming-read rate of a plain 128-bit-load kernel on buffers of 18 MB and 93 MB
("stream_read_roof"), the issue rate of the matrix instructions, and the CPU oracle timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure
MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16/bf16 matrix peak, vendor figure
POOL_BYTES = 1 << 30
ROW_POOL_BYTES = 600 << 20     # per-layer rotation of the breakdown rows: more than twice the last-level cache

# HBM bytes per decode step / per prefill launch from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE on this command (offline
# runs, scaled by what the same counters read for a copy of known size); the summaries under profiles/ give the runs.
# None = not measured for the build that is checked in.
# Decode: 94.50 MB read + 0.26 MB written per launch, average of the step's four launches
# (profiles/gemv24_group_kernel_workload5_decode_b1.md).  Prefill: bytes read + written per launch of the cases that were
# measured, keyed by (T, n, k) (profiles/gemm_kernels_workloads4_5_prefill.md).
MEASURED_DECODE_TRAFFIC_BYTES_PER_LAUNCH = 94_760_000
MEASURED_GEMM_TRAFFIC_BYTES_PER_LAUNCH = {
    (2048, 4096, 4096): 89_200_000, (8192, 4096, 4096): 421_500_000, (2048, 11008, 4096): 245_900_000,
    (8192, 11008, 4096): 1_151_000_000, (2048, 8192, 8192): 387_000_000, (2048, 1024, 8192): 75_100_000,
    (2048, 28672, 8192): 1_164_600_000, (2048, 8192, 28672): 1_092_100_000,
}

# The calls of one decode step over workload 5, by layer name: layers of a group share their input vector.
DECODE_GROUPS = (("q", "k", "v"), ("o",), ("gate", "up"), ("down",))


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_pool(S, torch, pm, pool_bytes, tiled=True, min_copies=2):
    """Copies of one packed image (tiled device order) in HBM, each with its own bound layout."""
    lay, img = pm.host_pair(tiled)
    copies = max(min_copies, int(np.ceil(pool_bytes / lay.image_bytes)))
    stride = (lay.image_bytes + S.STB_PLANE_ALIGN - 1) // S.STB_PLANE_ALIGN * S.STB_PLANE_ALIGN
    buf = torch.empty(copies * stride + S.STB_PLANE_ALIGN, dtype=torch.uint8, device="cuda")
    off = (-buf.data_ptr()) % S.STB_PLANE_ALIGN
    src = torch.from_numpy(img).cuda()
    layouts = []
    for c in range(copies):
        view = buf[off + c * stride: off + c * stride + lay.image_bytes]
        view.copy_(src)
        layouts.append(pm.clone_layout_for(view.data_ptr(), tiled))
    return buf, layouts


USE_GRAPHS = True       # --no-graph: every timed launch comes from the host (what a counter run wants to see)


WARM_SECONDS = 0.03       # untimed work before a row is timed: an idle GPU takes about 25 ms of work to reach its steady rate


def timed(torch, fn, reps, warm=3, rounds=3, graph=False):
    """Median and fastest average time of fn() in microseconds over `rounds` runs of `reps` calls, events on the
    stream the calls are launched on.  graph=True: the `reps` calls are captured once in a HIP graph and each run is
    one replay (a launch through the Python binding costs the host more time than a short kernel runs).  Before the
    timed runs the GPU is kept busy with the same calls for WARM_SECONDS (the rows follow host work -- packing the
    next layer -- during which the GPU idles and clocks down)."""
    for _ in range(warm):
        fn(0)
    torch.cuda.synchronize()
    out = []

    def keep_busy(run):
        t_end = time.perf_counter() + WARM_SECONDS
        while time.perf_counter() < t_end:
            run()
    if graph and USE_GRAPHS:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for r in range(reps):
                    fn(r)
            g.replay()
            side.synchronize()
            keep_busy(lambda: (g.replay(), side.synchronize()))
            for _ in range(rounds):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(side)
                g.replay()
                e1.record(side)
                side.synchronize()
                out.append(e0.elapsed_time(e1) * 1e3 / reps)
        torch.cuda.current_stream().wait_stream(side)
        return statistics.median(out), min(out)
    r = 0
    keep_busy(lambda: (fn(0), torch.cuda.synchronize()))
    for _ in range(rounds):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn(r)
            r += 1
        e1.record()
        torch.cuda.synchronize()
        out.append(e0.elapsed_time(e1) * 1e3 / reps)
    return statistics.median(out), min(out)


def tiled_ok(spec):
    return (8 * spec.N) % spec.M == 0 and (8 * spec.N // spec.M) in (3, 4, 5, 6)


PACK_ROWS = []          # (workload layer, host seconds, device seconds) of layers packed both ways


def pack_on_device(S, torch, L, spec, pm):
    """stb_pack_device on the same inputs; returns the median time of three runs and checks the bytes against the
    host packer's."""
    img = S.new_device_scratch(pm.host_layout.image_bytes)
    lay = pm.clone_layout_for(img.data_ptr(), False)
    ws = S.new_device_scratch(S.stb_pack_device_workspace_bytes(pm.cfg))
    Wd = torch.from_numpy(L["W"]).cuda()
    xd = torch.from_numpy(L["xnorm"]).cuda()
    sd = torch.from_numpy(np.ascontiguousarray(L["sal_bitmap"], dtype="<u4").view(np.int32)).cuda()
    times = []
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        S.stb_pack_device(Wd, xd, sd, lay, False, ws)          # waits for its stream
        times.append(time.perf_counter() - t0)
    got = img.cpu().numpy()
    same = all(bool((got[getattr(pm.host_layout, off):getattr(pm.host_layout, off) + getattr(pm.host_layout, size)]
                     == pm.plane(name)).all()) for name, off, size in S.PLANE_FIELDS)
    del img, ws, Wd, xd, sd
    torch.cuda.empty_cache()
    return statistics.median(times), same


def pack_spec(S, make_layer, spec, torch=None):
    L = make_layer(spec.n, spec.k, spec.seed, spec.salient_kind)
    t0 = time.time()
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], spec.N, spec.M, spec.region_mode)
    host_s = time.time() - t0
    if torch is not None:
        dev_s, same = pack_on_device(S, torch, L, spec, pm)
        PACK_ROWS.append(dict(layer=spec.name, n=spec.n, k=spec.k, nm=f"{spec.N}:{spec.M}",
                              host_seconds=round(host_s, 3), host_threads=os.cpu_count(),
                              device_seconds=round(dev_s, 4), weights_gbs_device=round(4.0 * spec.n * spec.k / dev_s / 1e9, 1),
                              same_bytes_as_host=same))
        log("pack row:", PACK_ROWS[-1])
    log(f"packed {spec.name} {spec.n}x{spec.k} {spec.N}:{spec.M}: {pm.packed_bytes / 1e6:.2f} MB in {host_s:.1f} s")
    return pm


def gemm_kernel_name(spec):
    if (spec.N, spec.M) == (2, 4):
        return "gemm24_wide_kernel (v_smfmac_f32_32x32x32_f16)"
    return "gemm_tiled_kernel (v_mfma_f32_16x16x32_f16)"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=200,
                    help="untimed steps before the timed ones (the step time falls for about 180 steps, 25 ms, after the "
                         "GPU has been idle: fewer warm-up steps time the ramp, not the kernel)")
    ap.add_argument("--replays", type=int, default=7, help="timed replays of the graph of K steps (median is reported)")
    ap.add_argument("--no-gemm", action="store_true", help="skip the prefill rows")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-graph", action="store_true", help="time host-side launches instead of a HIP graph replay")
    ap.add_argument("--no-extra", action="store_true", help="skip the per-layer rows, the read probe and the issue probe")
    ap.add_argument("--only-headline", action="store_true", help="the timed steps only (for profiling runs)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")
    if a.only_headline:
        a.no_gemm = a.no_cpu = a.no_extra = True

    import torch
    import paper_2408_01803_amd as S
    from workloads import WORKLOADS, make_layer, make_x

    global USE_GRAPHS
    USE_GRAPHS = not a.no_graph
    if not os.path.exists(S.LIB_PATH):
        sys.exit("bench.py: libstb.so is missing; run __graft_entry__.build() first")
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    prop = torch.cuda.get_device_properties(0)
    log(f"device: {prop.name} {prop.gcnArchName} CUs={prop.multi_processor_count} "
        f"mem={prop.total_memory >> 20} MiB  host cores={os.cpu_count()}")

    # ---------------- headline: decode step over workload 5 at batch 1 ----------------
    wl = WORKLOADS[5]
    B = 1
    packed5 = {spec.name: pack_spec(S, make_layer, spec, None if a.no_extra else torch) for spec in wl["layers"]}
    specs5 = {spec.name: spec for spec in wl["layers"]}
    step_bytes = sum(pm.packed_bytes for pm in packed5.values())
    copies = max(2, int(np.ceil(POOL_BYTES / step_bytes)))
    pools = {}
    for name, pm in packed5.items():
        lay, _ = pm.host_pair(True)
        pools[name] = build_pool(S, torch, pm, copies * lay.image_bytes, min_copies=copies)
    groups = []
    ws_bytes = 0
    for names in DECODE_GROUPS:
        k = specs5[names[0]].k
        x = torch.from_numpy(make_x(B, k, specs5[names[0]].seed)).cuda()
        ys = [torch.empty((B, specs5[nm].n), dtype=torch.float16, device="cuda") for nm in names]
        groups.append(dict(names=names, x=x, ys=ys))
        ws_bytes = max(ws_bytes, S.stb_gemv_batched_workspace_bytes([packed5[nm].cfg for nm in names], B))
    ws = S.new_device_scratch(ws_bytes, zero=True)
    cursor = [0]

    def decode_step():
        c = cursor[0]
        cursor[0] = (c + 1) % copies
        for g in groups:
            S.stb_gemv_batched([pools[nm][1][c] for nm in g["names"]], [g["x"]] * len(g["names"]), B, g["ys"], False, ws)

    launches_per_step = len(groups)
    algo_per_step = sum(packed5[nm].packed_bytes + 2 * B * specs5[nm].k + 2 * B * specs5[nm].n for nm in packed5)
    for _ in range(a.warmup):
        decode_step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(a.steps):
        decode_step()
    ev1.record()
    torch.cuda.synchronize()
    eager_ms_per_step = ev0.elapsed_time(ev1) / a.steps
    ms_per_step = best_ms_per_step = eager_ms_per_step
    launch_mode = "stream launches from the host"
    replays_ms = []
    if not a.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for _ in range(a.steps):
                    decode_step()
            for _ in range(max(1, -(-a.warmup // max(1, a.steps)))):     # untimed replays: the W warm-up steps once more
                graph.replay()
            side.synchronize()
            for _ in range(max(1, a.replays)):   # each timed region is one replay = exactly K steps
                g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                g0.record(side)
                graph.replay()
                g1.record(side)
                side.synchronize()
                replays_ms.append(g0.elapsed_time(g1) / a.steps)
        ms_per_step = statistics.median(replays_ms)
        best_ms_per_step = min(replays_ms)
        launch_mode = f"one HIP graph of the K steps, replayed {len(replays_ms)} times (median)"
        torch.cuda.current_stream().wait_stream(side)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    launch_us = ms_per_step * 1e3 / launches_per_step
    achieved = algo_per_step / (ms_per_step * 1e-3) / 1e9
    log(f"decode: {ms_per_step:.4f} ms/step median, {best_ms_per_step:.4f} best ({launch_mode}; "
        f"{eager_ms_per_step:.4f} ms/step launched one by one), {value:.1f} GB/s packed")

    result = {
        "metric": "packed-weight GB/s (GEMV) & TFLOP/s (GEMM), % of MI355X HBM/MFMA roofline",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "configs[4]: one LLaMA-70B-shaped decoder layer (q/o 8192x8192 and k/v 1024x8192 at 6:8, "
                               "gate/up 28672x8192 at 4:8, down 8192x28672 at 2:4), decode GEMV at batch 1: all seven "
                               "matrices per step in four grouped launches (q+k+v, o, gate+up, down)",
                   "packed_bytes_per_step": step_bytes,
                   "pool_bytes": int(sum(buf.numel() for buf, _ in pools.values())),
                   "launch": launch_mode,
                   "ms_per_step_best_replay": round(best_ms_per_step, 4),
                   "ms_per_step_replays": [round(v, 4) for v in replays_ms],
                   "ms_per_step_host_launches": round(eager_ms_per_step, 4)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": MEASURED_DECODE_TRAFFIC_BYTES_PER_LAUNCH,
                     "kernel": "gemv24_group_kernel (stb_gemv_batched on tiled layouts)", "us_per_launch": round(launch_us, 2),
                     "algorithmic_bytes_per_launch": int(algo_per_step / launches_per_step),
                     "launches_per_step": launches_per_step},
    }
    del pools
    torch.cuda.empty_cache()

    def decode_rows(cfg, spec, pm, batches):
        """One row per batch: a single stb_gemv call per launch, rotating over copies of the layer (30 launches in a
        HIP graph, replayed)."""
        rows = []
        tiled = tiled_ok(spec)
        buf, layouts = build_pool(S, torch, pm, ROW_POOL_BYTES, tiled=tiled)
        wsl = pm.new_workspace()
        for Bq in batches:
            x = torch.from_numpy(make_x(Bq, spec.k, spec.seed)).cuda()
            y = torch.empty((Bq, spec.n), dtype=torch.float16, device="cuda")
            med, best = timed(torch, lambda r: S.stb_gemv(layouts[r % len(layouts)], x, Bq, y, False, wsl), 30, graph=True)
            rows.append(dict(workload=cfg, layer=spec.name, n=spec.n, k=spec.k, nm=f"{spec.N}:{spec.M}", B=Bq,
                             us=round(med, 2), us_best=round(best, 2), packed_mb=round(pm.packed_bytes / 1e6, 2),
                             packed_gbs=round(pm.packed_bytes / med / 1e3, 1),
                             frac_of_hbm_peak=round(pm.packed_bytes / med / 1e3 / HBM_PEAK_GBS, 4)))
            log("decode row:", rows[-1])
        del buf, layouts
        torch.cuda.empty_cache()
        return rows

    def gemm_rows(cfg, spec, pm, tokens, graph=False):
        rows = []
        pm.to_device(tiled=tiled_ok(spec))
        for T in tokens:
            X = torch.from_numpy(make_x(T, spec.k, spec.seed)).cuda()
            Y = torch.empty((T, spec.n), dtype=torch.float16, device="cuda")
            wsg = pm.new_gemm_workspace(T)
            flops = 2.0 * T * spec.n * spec.k
            reps = max(2, min(10, int(2e12 / flops)))
            med, best = timed(torch, lambda r: S.stb_gemm(pm.dev_layout, X, T, Y, False, wsg), reps, warm=2, graph=graph)
            tf = flops / med / 1e6
            row = dict(workload=cfg, layer=spec.name, T=T, n=spec.n, k=spec.k, nm=f"{spec.N}:{spec.M}",
                       us=round(med, 1), us_best=round(best, 1), tflops=round(tf, 2),
                       frac_of_f16_mfma_peak=round(tf / MFMA_F16_PEAK_TFLOPS, 4), kernel=gemm_kernel_name(spec))
            if (spec.N, spec.M) == (2, 4):
                # the sparse instruction multiplies the kept weights only: 2*T*n*k*N/M flops are executed, and
                # `tflops` (2*T*n*k) is the dense-equivalent rate
                row["tflops_kept_weights"] = round(tf * spec.N / spec.M, 2)
                row["frac_of_f16_mfma_peak_kept_weights"] = round(tf * spec.N / spec.M / MFMA_F16_PEAK_TFLOPS, 4)
            rows.append(row)
            log("gemm row:", row)
            del X, Y, wsg
        pm.dev_image = pm.dev_layout = None
        torch.cuda.empty_cache()
        return rows

    decode_all, gemm_all, gemm_small = [], [], []
    if not a.no_extra:
        for spec in wl["layers"]:
            decode_all += decode_rows(5, spec, packed5[spec.name], wl["decode_batches"])
    if not a.no_gemm:
        for spec in wl["layers"]:
            gemm_all += gemm_rows(5, spec, packed5[spec.name], wl["prefill_tokens"])
    cpu_layers = {nm: packed5[nm] for nm in ("q", "k", "v")}      # kept for the CPU leg
    del packed5
    if not (a.no_extra and a.no_gemm):
        for cfg in (1, 2, 3, 4):
            w = WORKLOADS[cfg]
            for spec in w["layers"]:
                if (a.no_extra or not w["decode_batches"]) and (a.no_gemm or not w["prefill_tokens"]):
                    continue
                pm = pack_spec(S, make_layer, spec)
                if not a.no_extra and w["decode_batches"]:
                    decode_all += decode_rows(cfg, spec, pm, w["decode_batches"])
                if not a.no_gemm and w["prefill_tokens"]:
                    gemm_all += gemm_rows(cfg, spec, pm, w["prefill_tokens"])
                if not a.no_gemm and not a.no_extra and cfg == 3:
                    # launches of up to 64 tokens run their own instantiation of the prefill kernels (it is also what
                    # stb_gemv takes for B = 17 .. 32 on these layers: compare the B = 32 decode rows)
                    gemm_small += gemm_rows("3 (small launches)", spec, pm, [32, 64], graph=True)
                del pm
        # the paper's other ratios (Sec. 3.3, Table 1) on the shape of workload 1: 3:8 and 5:8 run on the same kernels as
        # 4:8 and 6:8 (their tiled image carries one unused slot per group of 8 columns)
        from workloads.synth import LayerSpec
        for Nk in (3, 5):
            spec = LayerSpec(f"linear_{Nk}of8", 4096, 4096, Nk, 8, 0, "x8", 10 + Nk)
            pm = pack_spec(S, make_layer, spec)
            if not a.no_extra:
                decode_all += decode_rows("1 (ratio varied)", spec, pm, [1])
            if not a.no_gemm:
                gemm_all += gemm_rows("1 (ratio varied)", spec, pm, [2048])
            del pm
    if PACK_ROWS:
        result["pack_rows"] = {"rows": PACK_ROWS, "note": "stb_pack (host threads) and stb_pack_device (fp32 weights already "
                               "in HBM, the call waits for its kernels) on the layers of workload 5; same bytes"}
    if decode_all:
        result["decode_rows"] = decode_all
    if gemm_all:
        dense = [g for g in gemm_all if g["nm"] != "2:4"]
        best = max(dense, key=lambda g: g["tflops"])
        result["gemm"] = {"rows": gemm_all,
                          "roofline": {"bound": "mfma", "achieved": best["tflops"], "peak": MFMA_F16_PEAK_TFLOPS,
                                       "unit": "TFLOP/s", "frac": best["frac_of_f16_mfma_peak"],
                                       "traffic": MEASURED_GEMM_TRAFFIC_BYTES_PER_LAUNCH.get((best["T"], best["n"], best["k"])),
                                       "kernel": best["kernel"] + " (stb_gemm), flops = 2*T*n*k executed on the "
                                                 f"dequantised tile; best dense-instruction row: workload {best['workload']} "
                                                 f"{best['layer']} T={best['T']}"}}

    if gemm_small:
        result["gemm_small_rows"] = {"rows": gemm_small, "note": "stb_gemm at 32 and 64 tokens (launches in a HIP graph, as "
                                     "the decode rows are timed); not part of the roofline row above"}
    if not a.no_extra:
        # streaming-read rate of a plain kernel on buffers of two sizes (an 18 MB layer and a 93 MB one), rotating over
        # a pool larger than the last-level cache, same launch-to-launch timing as the rows above
        base = torch.empty(ROW_POOL_BYTES + 256, dtype=torch.uint8, device="cuda")
        base.fill_(1)
        off0 = (-base.data_ptr()) % 256
        sink = torch.zeros(1024, dtype=torch.int32, device="cuda")
        roofs = []
        for nbytes in (17_968_384, 93_585_408):
            stride = (nbytes + 255) // 256 * 256
            ncopy = (base.numel() - off0) // stride
            med, best = timed(torch, lambda r: S.stb_probe_read(base[off0 + (r % ncopy) * stride:], nbytes, sink), 30, graph=True)
            roofs.append({"bytes": nbytes, "us": round(med, 2), "us_best": round(best, 2), "gbs": round(nbytes / med / 1e3, 1)})
        result["stream_read_roof"] = {"sizes": roofs, "note": "plain 128-bit-load read kernel, one launch per buffer, "
                                                              "same launch-to-launch timing as decode_rows"}
        log("stream read roof:", roofs)
        del base
        torch.cuda.empty_cache()
        # what the matrix instructions themselves sustain on this GPU: one wavefront per SIMD on every compute unit,
        # independent accumulators, alone and with vector instructions after each
        n_cu = prop.multi_processor_count
        sink = torch.empty(n_cu * 4096, dtype=torch.uint8, device="cuda")
        steps = 2000
        roof = {}
        for kind, name, flop in ((0, "v_mfma_f32_16x16x32_f16", 16384.0), (1, "v_smfmac_f32_16x16x64_f16", 32768.0),
                                 (2, "v_mfma_f32_32x32x16_f16", 32768.0), (3, "v_smfmac_f32_32x32x32_f16", 65536.0)):
            for rnd in (0, 1):           # operands next to 1.0 / operands with every bit random (what a GEMM is fed)
                for valu in ((0, 3, 5, 8) if not rnd else (0, 5)):
                    med, _ = timed(torch, lambda r: S.stb_probe_mfma(kind + 4 * rnd, valu, steps, n_cu, sink), 3, warm=1, rounds=1)
                    ns = med * 1e3 / (steps * 32)
                    roof[f"{name}{'(random operands)' if rnd else ''}+{valu}valu"] = {
                        "ns_per_instruction_per_simd": round(ns, 2), "tflops_all_simds": round(flop * 4 * n_cu / ns / 1e3, 1)}
        result["instruction_issue_roof"] = roof

    # ---------------- CPU baseline: the oracle as it stands, on this machine's host cores ----------------
    if not a.no_cpu:
        from oracle import stb_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        t_total, bytes_total, parts = 0.0, 0, []
        for nm, pm in cpu_layers.items():
            spec = specs5[nm]
            lay = pm.host_layout
            planes = dict(
                mask=pm.plane("mask").reshape(spec.n, lay.mask_stride),
                sign=pm.plane("sign").reshape(spec.n, lay.sign_stride),
                region=pm.plane("region").reshape(spec.n, lay.region_stride),
                res_sign=pm.plane("res_sign").reshape(spec.n, lay.res_stride),
                scales=pm.plane("scales").view(np.float16).reshape(spec.n, lay.n_blocks, 4),
                res_scale=pm.plane("res_scale").view(np.float16).reshape(spec.n, lay.n_blocks),
                sal_bitmap=pm.plane("sal_bitmap").view("<u4"),
                sal_block_prefix=pm.plane("sal_block_prefix").view("<u4"))
            x = make_x(B, spec.k, spec.seed)
            t0 = time.time()
            What = O.unpack(planes, spec.n, spec.k, spec.N, spec.M)
            O.matmul(x, What)
            dt = time.time() - t0
            del What
            t_total += dt
            bytes_total += pm.packed_bytes
            parts.append(f"{nm} {dt:.1f} s")
        result["cpu_baseline"] = {
            "value": round(bytes_total / t_total / 1e9, 5), "unit": "GB/s", "cores": int(cores), "kind": "oracle",
            "sample": "the q, k and v matrices of the step (3 of 7, 41 of 355 MB) at batch 1: numpy dequantisation from "
                      "the packed bytes + float64 product, " + ", ".join(parts)}
        log("cpu baseline:", result["cpu_baseline"])

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
