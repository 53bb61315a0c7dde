"""Benchmark of the structured-binary hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one decode pass over workload 2 (the LLaMA-7B MLP linears 11008x4096 and 4096x11008 at 2:4 with
the residual salient plane): stb_gemv at batch 1, 4 and 16 on both layers, i.e. six launches.  Each launch
reads a different copy of the packed weights (tiled device order) out of a pool of more than 1 GiB, so the
weights come from HBM and not from the 256 MB last-level cache.  Inputs are resident in HBM before the timed
region.  `value` is packed-weight GB/s (STB1 bytes) over the whole timed region, launch gaps included.

`roofline` describes the dominant kernel, the decode GEMV: algorithmic bytes per launch (packed planes + x + y)
divided by the average time of one launch, measured with events on the launch stream over the same timed
region.  After the timed steps the same JSON line gets: a per-(layer, batch) breakdown, the streaming-read
rate of a plain 128-bit-load kernel on a buffer of the same size ("stream_read_roof"), the largest decode
layers of workload 5 ("decode_large"), the prefill leg (stb_gemm on workload 4 shapes, tiled order, with its
own roofline against the fp16 matrix peak) and the CPU oracle timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure
MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16/bf16 matrix peak, vendor figure
POOL_BYTES = 1 << 30

# HBM bytes per decode launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this command, scaled by what
# the same counters read for a copy of known size; see profiles/gemv24_workload2_decode.md.
# Average over the six launches of a step (read + written).
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = 19.5e6


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_pool(S, torch, pm, pool_bytes, tiled=True):
    """Copies of one packed image (tiled device order) in HBM, each with its own bound layout."""
    lay, img = pm.host_pair(tiled)
    copies = max(2, int(np.ceil(pool_bytes / lay.image_bytes)))
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


def timed(torch, fn, reps, warm=3):
    """Average time of fn() in microseconds, events on the current stream."""
    for _ in range(warm):
        fn(0)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for r in range(reps):
        fn(r)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-gemm", action="store_true", help="skip the prefill leg")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-graph", action="store_true", help="time host-side launches instead of a HIP graph replay")
    ap.add_argument("--no-extra", action="store_true", help="skip the breakdown, roof probe and large decode layers")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import torch
    import paper_2408_01803_amd as S
    from workloads import WORKLOADS, make_layer, make_x

    if not os.path.exists(S.LIB_PATH):
        sys.exit("bench.py: libstb.so is missing; run __graft_entry__.build() first")
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    prop = torch.cuda.get_device_properties(0)
    log(f"device: {prop.name} {prop.gcnArchName} CUs={prop.multi_processor_count} "
        f"mem={prop.total_memory >> 20} MiB  host cores={os.cpu_count()}")

    # ---------------- decode leg: workload 2 ----------------
    wl = WORKLOADS[2]
    batches = wl["decode_batches"]
    layers = []
    for spec in wl["layers"]:
        t0 = time.time()
        L = make_layer(spec.n, spec.k, spec.seed, spec.salient_kind)
        pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], spec.N, spec.M, spec.region_mode)
        buf, layouts = build_pool(S, torch, pm, POOL_BYTES // len(wl["layers"]))
        xs = {B: torch.from_numpy(make_x(B, spec.k, spec.seed)).cuda() for B in batches}
        ys = {B: torch.empty((B, spec.n), dtype=torch.float16, device="cuda") for B in batches}
        layers.append(dict(spec=spec, pm=pm, buf=buf, layouts=layouts, xs=xs, ys=ys, cursor=0,
                           ws=pm.new_workspace()))
        log(f"packed {spec.name} {spec.n}x{spec.k} {spec.N}:{spec.M}: {pm.packed_bytes / 1e6:.2f} MB, "
            f"{len(layouts)} copies, {time.time() - t0:.1f} s")
        del L

    def decode_step():
        for B in batches:
            for ly in layers:
                lay = ly["layouts"][ly["cursor"]]
                ly["cursor"] = (ly["cursor"] + 1) % len(ly["layouts"])
                S.stb_gemv(lay, ly["xs"][B], B, ly["ys"][B], False, ly["ws"])

    launches_per_step = len(batches) * len(layers)
    packed_per_step = sum(ly["pm"].packed_bytes for ly in layers) * len(batches)
    algo_per_step = sum(ly["pm"].packed_bytes + 2 * B * ly["spec"].k + 2 * B * ly["spec"].n
                        for ly in layers for B in batches)
    for _ in range(a.warmup):
        decode_step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    # (1) launched one by one from the host
    ev0.record()
    for _ in range(a.steps):
        decode_step()
    ev1.record()
    torch.cuda.synchronize()
    eager_ms_per_step = ev0.elapsed_time(ev1) / a.steps
    # (2) the same K steps captured once in a HIP graph and replayed: the decode loop is launch-bound from the
    #     host side (a launch through the binding costs more host time than the kernel runs), so this is how a
    #     serving loop would issue it.  The timed region is one replay = exactly K steps.
    ms_per_step = eager_ms_per_step
    launch_mode = "stream launches from the host"
    if not a.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for _ in range(a.steps):
                    decode_step()
            graph.replay()                       # untimed replay
            side.synchronize()
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            g0.record(side)
            graph.replay()
            g1.record(side)
            side.synchronize()
        ms_per_step = g0.elapsed_time(g1) / a.steps
        launch_mode = "one HIP graph of the K steps, replayed"
        torch.cuda.current_stream().wait_stream(side)
    value = packed_per_step / (ms_per_step * 1e-3) / 1e9
    launch_us = ms_per_step * 1e3 / launches_per_step
    achieved = (algo_per_step / launches_per_step) / (launch_us * 1e-6) / 1e9
    log(f"decode: {ms_per_step:.4f} ms/step ({launch_mode}; {eager_ms_per_step:.4f} ms/step launched one by one), "
        f"{launch_us:.2f} us/launch, {value:.1f} GB/s packed")

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
        "config": {"workload": "configs[1]: LLaMA-7B MLP linears 11008x4096 + 4096x11008, 2:4 structured binary "
                               "with residual salient plane, decode GEMV at batch 1, 4, 16 (6 launches per step)",
                   "packed_bytes_per_step": packed_per_step,
                   "pool_bytes": int(sum(ly["buf"].numel() for ly in layers)),
                   "launch": launch_mode,
                   "ms_per_step_host_launches": round(eager_ms_per_step, 4)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC_BYTES_PER_LAUNCH,
                     "kernel": "gemv24_kernel (stb_gemv on a tiled 2:4 layout)", "us_per_launch": round(launch_us, 2),
                     "algorithmic_bytes_per_launch": int(algo_per_step / launches_per_step)},
    }

    if not a.no_extra:
        # per-(layer, B) breakdown, same protocol
        breakdown = []
        for ly in layers:
            for B in batches:
                us = timed(torch, lambda r: S.stb_gemv(ly["layouts"][r % len(ly["layouts"])], ly["xs"][B], B,
                                                       ly["ys"][B], False, ly["ws"]), 40)
                breakdown.append(dict(layer=ly["spec"].name, B=B, us=round(us, 2),
                                      packed_gbs=round(ly["pm"].packed_bytes / us / 1e3, 1)))
        log("decode breakdown:", breakdown)
        result["decode_breakdown"] = breakdown
        # streaming-read rate of a plain kernel on a buffer of one layer's size, same rotation over the pool
        ly = layers[0]
        nbytes = ly["pm"].packed_bytes // 16 * 16
        sink = torch.zeros(1024, dtype=torch.int32, device="cuda")
        base = ly["buf"]
        off0 = (-base.data_ptr()) % 256
        stride = (nbytes + 255) // 256 * 256
        ncopy = (base.numel() - off0) // stride
        us = timed(torch, lambda r: S.stb_probe_read(base[off0 + (r % ncopy) * stride:], nbytes, sink), 40)
        result["stream_read_roof"] = {"bytes": nbytes, "us": round(us, 2), "gbs": round(nbytes / us / 1e3, 1),
                                      "note": "plain 128-bit-load read kernel on a buffer of one layer's packed size, "
                                              "same launch-to-launch timing"}
        log("stream read roof:", result["stream_read_roof"])
    for ly in layers:
        del ly["buf"], ly["layouts"]
    torch.cuda.empty_cache()

    if not a.no_extra:
        # the two largest decode layers of workload 5 (B = 1): where the stream is long enough to ramp up
        large = []
        for spec in (WORKLOADS[5]["layers"][4], WORKLOADS[5]["layers"][6]):
            L = make_layer(spec.n, spec.k, spec.seed, spec.salient_kind)
            pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], spec.N, spec.M, spec.region_mode)
            del L
            buf, layouts = build_pool(S, torch, pm, POOL_BYTES)
            ws = pm.new_workspace()
            x = torch.from_numpy(make_x(1, spec.k, spec.seed)).cuda()
            y = torch.empty((1, spec.n), dtype=torch.float16, device="cuda")
            us = timed(torch, lambda r: S.stb_gemv(layouts[r % len(layouts)], x, 1, y, False, ws), 40)
            large.append(dict(layer=spec.name, n=spec.n, k=spec.k, nm=f"{spec.N}:{spec.M}", B=1, us=round(us, 2),
                              packed_mb=round(pm.packed_bytes / 1e6, 1), packed_gbs=round(pm.packed_bytes / us / 1e3, 1),
                              frac_of_hbm_peak=round(pm.packed_bytes / us / 1e3 / HBM_PEAK_GBS, 4)))
            log("decode large:", large[-1])
            del buf, layouts, pm
            torch.cuda.empty_cache()
        result["decode_large"] = large

    # ---------------- prefill leg: workload 4 shapes ----------------
    if not a.no_gemm:
        gemm = []
        # workload 4 (4:8, the dense matrix instruction) and the 2:4 `down` layer of workload 5 (the sparse one)
        for spec, T, reps in ((WORKLOADS[4]["layers"][0], 2048, 10), (WORKLOADS[4]["layers"][1], 8192, 3),
                              (WORKLOADS[5]["layers"][6], 2048, 3)):
            L = make_layer(spec.n, spec.k, spec.seed, spec.salient_kind)
            pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], spec.N, spec.M, spec.region_mode)
            pm.to_device(tiled=True)
            del L
            X = torch.from_numpy(make_x(T, spec.k, spec.seed)).cuda()
            Y = torch.empty((T, spec.n), dtype=torch.float16, device="cuda")
            ws = pm.new_gemm_workspace(T)
            us = timed(torch, lambda r: S.stb_gemm(pm.dev_layout, X, T, Y, False, ws), reps, warm=2)
            flops = 2.0 * T * spec.n * spec.k
            tf = flops / us / 1e6
            case = dict(T=T, n=spec.n, k=spec.k, nm=f"{spec.N}:{spec.M}", us=round(us, 1),
                        tflops=round(tf, 2), frac_of_f16_mfma_peak=round(tf / MFMA_F16_PEAK_TFLOPS, 4))
            # which kernel the library runs
            asked = os.environ.get("STB_GEMM_KERNEL", "")
            dense_name = ("gemm_wide_kernel (v_mfma_f32_32x32x16_f16)" if asked == "dense32"
                          else "gemm_tiled_kernel (v_mfma_f32_16x16x32_f16)")
            case["kernel"] = dense_name
            if (spec.N, spec.M) == (2, 4) and not asked.startswith("d"):
                # the sparse instruction multiplies the kept weights only: 2*T*n*k*N/M flops are executed, and
                # `tflops` (2*T*n*k) is the dense-equivalent rate
                case["kernel"] = ("gemm24_kernel (v_smfmac_f32_16x16x64_f16)" if asked == "sparse16"
                                  else "gemm24_wide_kernel (v_smfmac_f32_32x32x32_f16)")
                case["tflops_kept_weights"] = round(tf * spec.N / spec.M, 2)
                case["frac_of_f16_mfma_peak_kept_weights"] = round(tf * spec.N / spec.M / MFMA_F16_PEAK_TFLOPS, 4)
            gemm.append(case)
            log("gemm:", gemm[-1])
            del pm, X, Y, ws
        # what the matrix instructions themselves sustain on this GPU: one wavefront per SIMD on every compute unit,
        # 32 independent accumulators, alone and with the three vector instructions per MFMA of the kernels' K step
        n_cu = torch.cuda.get_device_properties(0).multi_processor_count
        sink = torch.empty(n_cu * 4096, dtype=torch.uint8, device="cuda")
        steps = 2000
        roof = {}
        for kind, name, flop in ((0, "v_mfma_f32_16x16x32_f16", 16384.0), (1, "v_smfmac_f32_16x16x64_f16", 32768.0),
                                 (2, "v_mfma_f32_32x32x16_f16", 32768.0), (3, "v_smfmac_f32_32x32x32_f16", 65536.0)):
            for valu in (0, 3, 5, 8):
                us = timed(torch, lambda r: S.stb_probe_mfma(kind, valu, steps, n_cu, sink), 3, warm=1)
                ns = us * 1e3 / (steps * 32)
                roof[f"{name}+{valu}valu"] = {"ns_per_instruction_per_simd": round(ns, 2),
                                              "tflops_all_simds": round(flop * 4 * n_cu / ns / 1e3, 1)}
        log("matrix instruction issue roof:", roof)
        best = max((g for g in gemm if g["nm"] != "2:4"), key=lambda g: g["tflops"])
        result["gemm"] = {"cases": gemm,
                          "roofline": {"bound": "mfma", "achieved": best["tflops"], "peak": MFMA_F16_PEAK_TFLOPS,
                                       "unit": "TFLOP/s", "frac": best["frac_of_f16_mfma_peak"], "traffic": None,
                                       "kernel": best["kernel"] + " (stb_gemm), flops = 2*T*n*k executed on the "
                                                 "dequantised tile"},
                          "instruction_issue_roof": roof}

    # ---------------- CPU baseline: the oracle as it stands, on this machine's host cores ----------------
    if not a.no_cpu:
        from oracle import stb_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        ly = layers[0]
        spec, pm = ly["spec"], ly["pm"]
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
        t0 = time.time()
        What = O.unpack(planes, spec.n, spec.k, spec.N, spec.M)
        t_deq = time.time() - t0
        t0 = time.time()
        for B in batches:
            O.matmul(ly["xs"][B].cpu().numpy(), What)
        t_mm = time.time() - t0
        # one decode pass over this layer = len(batches) products; the oracle dequantises once per product
        total = len(batches) * t_deq + t_mm
        result["cpu_baseline"] = {
            "value": round(len(batches) * pm.packed_bytes / total / 1e9, 5), "unit": "GB/s", "cores": int(cores),
            "kind": "oracle",
            "sample": f"layer {spec.name} {spec.n}x{spec.k} only, batches {batches}: numpy dequantisation from the "
                      f"packed bytes ({t_deq:.2f} s, measured once and charged per product) + float64 product "
                      f"({t_mm:.2f} s for the three batches)"}
        log("cpu baseline:", result["cpu_baseline"])

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
