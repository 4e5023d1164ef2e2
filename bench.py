#!/usr/bin/env python3
"""Benchmark of the VQ linear-layer hot path on one MI355X.

A step is one batch-1 vq_gemv call (index unpack -> codebook lookups -> residual / outlier merge ->
scale/bias -> matrix-vector product) on the Llama-2-7B-shaped 11008 x 4096 layer (v=6, k=4096,
12-bit packed indices).  Consecutive steps rotate over distinct device copies of the index stream
whose total size exceeds the 256 MB Infinity Cache, and the timed steps continue the rotation of an
untimed lead-in that has just walked every copy, so every step streams its indices from HBM whatever
--steps is.  `value`, `ms_per_step` and `roofline.achieved` are algorithmic bytes per step over the
time HIP events on the launching stream measure around exactly --steps launches (one graph replay
from 200 steps on, queued single launches below); `roofline.traffic` comes from the tracked
rocprofv3 counter summary under profiles/.  The other layers (residual, outlier columns, batch > 1,
the second target layer with a roofline block of its own), the prefill vq_gemm, vq_dequant,
vq_assign and vq_quantize_columns are timed briefly and reported under "detail".

Prints ONE JSON line.  Inputs are seeded synthetic tensors that stand in for real quantized
checkpoints (same shapes and (v, k) settings; Gaussian tables, uniform indices).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, vendor figure
MFMA_FP16_PEAK_TFLOPS = 2500.0  # dense FP16 matrix-core peak, vendor figure
FP32_VECTOR_PEAK_TFLOPS = 157.3   # published fp32 vector peak (packed FMA on 256 compute units at 2.4 GHz)
LEAD_SECONDS = 0.012            # least duration of the untimed lead-in (host estimate from the warm-up launches)
EAGER_BELOW = 200               # fewer timed steps than this are launched one by one (queued behind the lead-in)
ROTATE_BYTES = 640 << 20        # footprint of the rotated index copies (> 2 x the 256 MB Infinity Cache)

PROFILES = os.path.join(ROOT, "profiles")


def measured_traffic_bytes(cfg):
    """HBM bytes per launch of the headline kernel from the tracked rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE,
    each scaled by what the same counter reads for a 1 GiB device copy), or None when there is no such summary."""
    import re
    path = os.path.join(PROFILES, "gemv_cfg%d_batch1_traffic.txt" % cfg)
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*(\d+)", open(path).read(), re.M)
    return int(m.group(1)) if m else None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", type=int, default=1, help="benchmark configuration of the headline GEMV (1 or 3)")
    ap.add_argument("--no-detail", action="store_true", help="skip the secondary measurements")
    ap.add_argument("--gemm-only", action="store_true", help="only the prefill vq_gemm lines of the detail (for counter runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--copy-kernel", action="store_true",
                    help="also run a plain 1 GiB device copy (counter calibration for rocprofv3 --pmc runs)")
    return ap.parse_args()


class Rotation:
    """R device copies of a layer's index streams (tables, scale and bias are shared)."""

    def __init__(self, vq, layer, min_bytes=ROTATE_BYTES, max_copies=64, min_copies=2):
        import torch
        self.base = vq.DeviceLayer(layer)
        stream_bytes = sum(a.nbytes for a in (layer.idx, layer.idx_res, layer.idx_out) if a is not None)
        copies = max(min_copies, min(max_copies, -(-min_bytes // stream_bytes)))
        self.descs = [self.base.desc]
        self.keep = []
        import ctypes
        for _ in range(copies - 1):
            d = vq.vq_layer_desc()
            ctypes.memmove(ctypes.byref(d), ctypes.byref(self.base.desc), ctypes.sizeof(d))
            for name in ("idx", "idx_res", "idx_out"):
                t = self.base.tensors.get(name)
                if t is not None:
                    c = t.clone()
                    self.keep.append(c)
                    setattr(d, name, c.data_ptr())
            self.descs.append(d)
        torch.cuda.synchronize()
        self.copies = copies


def timed(launch, steps, warmup, use_graph=True, lead=0):
    """Run `warmup` untimed and `steps` timed calls of launch(i).  Returns (wall seconds, event seconds); the event time
    (HIP events on the launching stream around exactly `steps` launches) is the one every reported figure uses.
    The timed launches are i = n .. n + steps - 1 and follow, without a gap, an untimed run of launches 0 .. n - 1,
    n >= max(steps, lead).  With `lead` = the number of index copies that launch(i) rotates over (together more than
    512 MiB), every timed launch reads a copy whose last use lies a full rotation back -- more than twice the 256 MB
    Infinity Cache of other data in between, whatever `steps` is -- and starts on a GPU that is already running.
    Both runs are replays of HIP graphs uploaded beforehand; a few steps are launched one by one instead, queued
    behind the lead-in (a graph replay costs 11-14 us on the GPU's own time line, which twenty steps cannot amortise)."""
    import torch
    stream = torch.cuda.current_stream()
    t0 = time.perf_counter()
    for i in range(warmup):
        launch(i)
    torch.cuda.synchronize()
    # the lead-in also runs long enough for the clocks to settle: measured on the 11008 x 4096 layer, the launches of the
    # first few milliseconds after an idle spell take up to 6 % longer than those of a long run
    per_launch = (time.perf_counter() - t0) / max(warmup, 1) if warmup >= 5 else 50e-6
    n_lead = max(steps, lead, min(4000, int(LEAD_SECONDS / max(per_launch, 2e-6))))
    lead_graph = timed_graph = None
    if use_graph:
        lead_graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        with torch.cuda.graph(lead_graph, stream=side):
            for i in range(n_lead):
                launch(i)
        if steps >= EAGER_BELOW:
            timed_graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(timed_graph, stream=side):
                for i in range(n_lead, n_lead + steps):
                    launch(i)
            timed_graph.replay()       # untimed: uploads the graph
        lead_graph.replay()
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if lead_graph is not None:
        lead_graph.replay()
    else:
        for i in range(n_lead):
            launch(i)
    t0 = time.perf_counter()
    e0.record(stream)
    if timed_graph is not None:
        timed_graph.replay()
    else:
        for i in range(n_lead, n_lead + steps):
            launch(i)
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, e0.elapsed_time(e1) * 1e-3


def bench_gemv(vq, layer, x_np, steps, warmup, use_graph, rotate=True, workspace=False):
    import torch
    rot = Rotation(vq, layer) if rotate else Rotation(vq, layer, min_bytes=0, min_copies=1)
    x = torch.from_numpy(x_np).cuda()
    batch = x.shape[0]
    y = torch.empty((batch, layer.out_features), dtype=torch.float16, device="cuda")
    xp, yp, ldx, ldy = x.data_ptr(), y.data_ptr(), x.stride(0), y.stride(0)
    need = vq.vq_gemv_workspace_bytes(rot.descs[0], batch) if workspace else 0
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")

    def launch(i):
        st = torch.cuda.current_stream().cuda_stream
        if workspace:
            rc = vq.vq_gemv_with_workspace(rot.descs[i % rot.copies], xp, ldx, batch, yp, ldy, ws.data_ptr(), need, st)
        else:
            rc = vq.vq_gemv(rot.descs[i % rot.copies], xp, ldx, batch, yp, ldy, st)
        if rc != 0:
            raise vq.VQError(rc, "vq_gemv")
    wall, ev = timed(launch, steps, warmup, use_graph, lead=rot.copies)
    return dict(wall_s=wall, event_s=ev, copies=rot.copies, y=y)


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the layer shards by output rows; no multi-GPU path is built). "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import vq_synth as s
    import paper_2409_17066_amd as vq

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    vq.load()
    torch.cuda.set_device(0)
    use_graph = not args.no_graph
    if args.gemm_only:
        lines = []
        gemm_lines(vq, s, torch, next(s.config_layers(4))[1], lines)
        print(json.dumps({"detail": lines}))
        return
    cfg = args.config
    spec = s.CONFIGS[cfg]
    _, layer = next(s.config_layers(cfg))
    x_np = s.make_activations(cfg, layer, 1, outlier_gain=spec.get("outlier_gain", 1.0))
    r = bench_gemv(vq, layer, x_np, args.steps, args.warmup, use_graph)
    alg = layer.algorithmic_bytes(1)
    sec = r["event_s"] / args.steps
    gbps = alg / sec / 1e9
    workload = "cfg%d %s %dx%d v%d k%d%s%s batch1 gemv" % (
        cfg, layer.name, layer.out_features, layer.in_features, layer.v, layer.k,
        " res%d" % layer.k_res if layer.k_res else "", " outlier%d" % layer.n_outlier_cols if layer.n_outlier_cols else "")
    # one clock for every figure of the line: HIP events on the launching stream around exactly `steps` launches
    result = {
        "metric": "batch-1 VQ-GEMV effective HBM bandwidth (algorithmic bytes / time)",
        "value": round(gbps, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 6), "us_per_step": round(sec * 1e6, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16 in, f32 accumulate",
        "data": "synthetic (seeded Gaussian tables, uniform indices; stands in for quantized Llama-2 layers)",
        "config": {"workload": workload, "algorithmic_bytes": alg, "index_copies_rotated": r["copies"],
                   "launch": ("hip graph replay" if args.steps >= EAGER_BELOW else "eager launches queued behind a graph lead-in") if use_graph else "eager", "clock": "HIP events on the launching stream",
                   "host_wall_us_per_step": round(r["wall_s"] / args.steps * 1e6, 3)},
        "roofline": {"bound": "hbm", "achieved": round(gbps, 2), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": measured_traffic_bytes(cfg),
                     "kernel_us": round(sec * 1e6, 3)},
    }

    # parity spot check of the timed configuration against the oracle (sampled rows)
    import oracle
    rows = np.unique(np.linspace(0, layer.out_features - 1, 256).astype(np.int32))
    ref = oracle.gemv(layer, x_np, rows=rows)
    full_rms = float(np.sqrt((ref ** 2).mean()))
    err = float(np.abs(r["y"].float().cpu().numpy()[:, rows] - ref).max())
    result["parity"] = {"max_abs_err": err, "tolerance": 1e-2 * full_rms, "ok": bool(err <= 1e-2 * full_rms)}

    if not args.no_cpu_baseline:
        nthreads = oracle.default_threads()
        t_end = time.perf_counter() + args.cpu_seconds
        best, passes = None, 0
        while passes < 3 or time.perf_counter() < t_end:
            t0 = time.perf_counter()
            oracle.gemv(layer, x_np, n_threads=nthreads)
            dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
            passes += 1
            if passes >= 200:
                break
        result["cpu_baseline"] = {"value": round(alg / best / 1e9, 4), "unit": "GB/s", "cores": nthreads, "kind": "oracle",
                                  "sample": "%d full passes of the same layer and activation (best pass %.1f ms)" % (passes, best * 1e3)}

    if args.copy_kernel:
        # a plain copy of known size: reads 1 GiB, writes 1 GiB (what FETCH_SIZE / WRITE_SIZE are scaled by)
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        result["copy_kernel_bytes_each_way"] = a.numel() * 4
    # context, never the headline: the same launches on ONE copy of the indices (they then come from the 256 MB
    # Infinity Cache, not from HBM), and what a plain device-to-device copy of 1 GiB moves per second on this machine
    warm = bench_gemv(vq, layer, x_np, args.steps, args.warmup, use_graph, rotate=False)
    a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    b = torch.empty_like(a)
    b.copy_(a)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * a.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del a, b
    result["context"] = {"cache_warm_us_per_step": round(warm["event_s"] / args.steps * 1e6, 3),
                         "cache_warm_GB/s": round(alg / (warm["event_s"] / args.steps) / 1e9, 1),
                         "device_copy_GB/s_read_plus_write": round(copy_gbps, 1),
                         "achieved_over_device_copy": round(gbps / copy_gbps, 4)}
    if not args.no_detail:
        result["detail"] = detail(vq, s, np, torch, use_graph, skip=(cfg, 1))
    print(json.dumps(result))


def gemm_lines(vq, s, torch, L4, out):
    """The prefill product on the 8192 x 8192, v=8, k=65536 layer at the configuration's token counts, both routes."""
    dl = vq.DeviceLayer(L4)
    for tokens in s.CONFIGS[4]["rows"]:
        X = torch.from_numpy(s.make_activations(4, L4, tokens)).cuda()
        Y = torch.empty((tokens, L4.out_features), dtype=torch.float16, device="cuda")
        flops = 2.0 * tokens * L4.out_features * L4.in_features
        # two routes: weights restored on the fly (no workspace), and restored once into a workspace first
        for route, need in (("on the fly", vq.vq_gemm_workspace_bytes(dl.desc, tokens)),
                            ("restore, then multiply", vq.vq_gemm_fast_workspace_bytes(dl.desc, tokens))):
            ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

            def launch(i):
                rc = vq.vq_gemm(dl.desc, X.data_ptr(), X.stride(0), tokens, Y.data_ptr(), Y.stride(0), ws.data_ptr(), need,
                                torch.cuda.current_stream().cuda_stream)
                if rc != 0:
                    raise vq.VQError(rc, "vq_gemm")
            n = 10
            wall, ev = timed(launch, n, 2, use_graph=False)
            sec = ev / n
            out.append({"op": "vq_gemm", "cfg": 4, "tokens": tokens, "route": route, "workspace_bytes": int(need),
                        "us": round(sec * 1e6, 1), "TFLOP/s": round(flops / sec / 1e12, 1),
                        "frac_mfma_peak": round(flops / sec / 1e12 / MFMA_FP16_PEAK_TFLOPS, 4)})
            del ws
    return dl


def detail(vq, s, np, torch, use_graph, skip):
    """Short timings of the other benchmark layers and entry points."""
    out = []
    steps, warmup = 400, 50
    cfg2_bytes = {}

    def gemv_line(cfg, ordinal, layer, batch):
        spec = s.CONFIGS[cfg]
        x_np = s.make_activations(cfg, layer, batch, layer_ordinal=ordinal, outlier_gain=spec.get("outlier_gain", 1.0))
        r = bench_gemv(vq, layer, x_np, steps, warmup, use_graph)
        sec = r["event_s"] / steps
        alg = layer.algorithmic_bytes(batch)
        cfg2_bytes[layer.name, batch] = alg
        flops = 2.0 * batch * layer.out_features * layer.in_features
        line = {"op": "vq_gemv", "cfg": cfg, "layer": layer.name, "batch": batch, "us": round(sec * 1e6, 3),
                "GB/s": round(alg / sec / 1e9, 1), "frac_hbm_peak": round(alg / sec / 1e9 / HBM_PEAK_GBPS, 4),
                "TFLOP/s": round(flops / sec / 1e12, 2)}
        if batch == 1 and cfg in (1, 3):       # the two layers the target is written for: a roofline block of their own
            line["roofline"] = {"bound": "hbm", "achieved": round(alg / sec / 1e9, 2), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                "frac": round(alg / sec / 1e9 / HBM_PEAK_GBPS, 4), "traffic": measured_traffic_bytes(cfg),
                                "kernel_us": round(sec * 1e6, 3), "algorithmic_bytes": alg}
        if batch > 1:
            # the same call with the matrix cores switched off (VQ_SWITCHES gemv=d: the dot-product kernels on the vector ALUs,
            # batch rows in groups of 4, 2 or 1), and against the larger of the HBM time and the vector-ALU time of its
            # multiply-adds at the published fp32 vector peak
            os.environ["VQ_SWITCHES"] = "gemv=d"
            try:
                rv = bench_gemv(vq, layer, x_np, steps, warmup, use_graph)
            finally:
                del os.environ["VQ_SWITCHES"]
            sec_v = rv["event_s"] / steps
            floor = max(alg / (HBM_PEAK_GBPS * 1e9), flops / (FP32_VECTOR_PEAK_TFLOPS * 1e12))
            line["kernel"] = "matrix cores (default)"
            line["us_vector_alu_kernels"] = round(sec_v * 1e6, 3)
            line["frac_of_max_hbm_valu_time"] = round(floor / sec, 4)
            line["frac_of_max_hbm_valu_time_vector_alu_kernels"] = round(floor / sec_v, 4)
        out.append(line)

    for cfg in (1, 2, 3):
        spec = s.CONFIGS[cfg]
        names = [n for n, _, _ in spec["layers"]]
        if cfg == 2:
            names = ["q", "gate", "down"]              # k, v, o share q's shape; up shares gate's
        for ordinal, layer in s.config_layers(cfg):
            if layer.name not in names:
                continue
            for batch in spec["rows"]:
                if (cfg, batch) == skip:
                    continue
                gemv_line(cfg, ordinal, layer, batch)
            del layer
        if cfg == 2:
            # one decoder layer = q, k, v, o (q's shape) + gate, up (gate's shape) + down: seven GEMV calls
            for batch in spec["rows"]:
                us = {d["layer"]: d["us"] for d in out if d["op"] == "vq_gemv" and d["cfg"] == 2 and d["batch"] == batch}
                total_us = 4 * us["q"] + 2 * us["gate"] + us["down"]
                alg = sum(m * layer_bytes for m, layer_bytes in
                          ((4, cfg2_bytes["q", batch]), (2, cfg2_bytes["gate", batch]), (1, cfg2_bytes["down", batch])))
                out.append({"op": "vq_gemv x7 (whole cfg2 layer: 4 q-shaped, 2 gate-shaped, down; sum of the per-call times)",
                            "cfg": 2, "batch": batch, "us": round(total_us, 2), "GB/s": round(alg / total_us / 1e3, 1),
                            "frac_hbm_peak": round(alg / total_us / 1e3 / HBM_PEAK_GBPS, 4)})
    # the same decoder layer as a chain on one stream: q, k, v in one vq_gemv_multi launch, o, gate and up in one launch,
    # down -- four launches instead of seven, every layer's index streams rotated like the single calls above
    layers2 = {L.name: L for _, L in s.config_layers(2)}
    rots = {n: Rotation(vq, L, min_bytes=ROTATE_BYTES // 4) for n, L in layers2.items()}
    for batch in s.CONFIGS[2]["rows"]:
        xs = {n: torch.from_numpy(s.make_activations(2, layers2[n], batch)).cuda() for n in ("q", "o", "gate", "down")}
        ys = {n: torch.empty((batch, L.out_features), dtype=torch.float16, device="cuda") for n, L in layers2.items()}
        alg = sum(L.algorithmic_bytes(batch) for L in layers2.values())
        for fused in (True, False):
            def chain(i):
                st = torch.cuda.current_stream().cuda_stream
                for group in ((("q", "k", "v"), ("o",), ("gate", "up"), ("down",)) if fused else tuple((n,) for n in layers2)):
                    x = xs[{"k": "q", "v": "q", "up": "gate"}.get(group[0], group[0])]
                    descs = [rots[n].descs[i % rots[n].copies] for n in group]
                    rc = vq.vq_gemv_multi(descs, x.data_ptr(), x.stride(0), batch, [ys[n].data_ptr() for n in group],
                                          [ys[n].stride(0) for n in group], st)
                    if rc != 0:
                        raise vq.VQError(rc, "vq_gemv_multi")
            n_steps = 100
            wall, ev = timed(chain, n_steps, 10, use_graph)
            us = ev / n_steps * 1e6
            out.append({"op": "cfg2 decoder layer as a chain of %d launches (%s)" % (4 if fused else 7,
                                                                                  "qkv and gate+up fused by vq_gemv_multi" if fused else "one vq_gemv per projection"),
                        "cfg": 2, "batch": batch, "us": round(us, 2), "GB/s": round(alg / us / 1e3, 1),
                        "frac_hbm_peak": round(alg / us / 1e3 / HBM_PEAK_GBPS, 4)})
    del rots, xs, ys
    # prefill GEMM and dequant on the 8192 x 8192, v=8, k=65536 layer
    _, L4 = next(s.config_layers(4))
    # (first the decode-sized product on that layer: its 1 MB table stays in L2 and is gathered from there)
    for batch in (1, 4, 16):
        r = bench_gemv(vq, L4, s.make_activations(4, L4, batch), 200, 20, use_graph)
        sec = r["event_s"] / 200
        alg = L4.algorithmic_bytes(batch)
        out.append({"op": "vq_gemv", "cfg": "4 (decode rows on the prefill layer)", "layer": L4.name, "batch": batch, "us": round(sec * 1e6, 3),
                    "GB/s": round(alg / sec / 1e9, 1), "frac_hbm_peak": round(alg / sec / 1e9 / HBM_PEAK_GBPS, 4),
                    "TFLOP/s": round(2.0 * batch * L4.out_features * L4.in_features / sec / 1e12, 2)})
    dl = gemm_lines(vq, s, torch, L4, out)
    # the same two routes on the v = 6 layers (tables in LDS): the headline layer, the 7B attention projection with its
    # 12-bit residual and the 70B-shaped layer with its 8-bit residual and 288 outlier columns, at 512 and 2048 tokens
    for cfg6, name6 in ((1, "up"), (2, "q"), (3, "down70b")):
        _, L6 = next(s.config_layers(cfg6, only=name6))
        dl6 = vq.DeviceLayer(L6)
        for tokens in (512, 2048):
            X = torch.from_numpy(s.make_activations(cfg6, L6, tokens)).cuda()
            Y = torch.empty((tokens, L6.out_features), dtype=torch.float16, device="cuda")
            flops = 2.0 * tokens * L6.out_features * L6.in_features
            for route, need in (("on the fly", 0), ("restore, then multiply", vq.vq_gemm_fast_workspace_bytes(dl6.desc, tokens))):
                ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

                def launch6(i):
                    rc = vq.vq_gemm(dl6.desc, X.data_ptr(), X.stride(0), tokens, Y.data_ptr(), Y.stride(0), ws.data_ptr(), need,
                                    torch.cuda.current_stream().cuda_stream)
                    if rc != 0:
                        raise vq.VQError(rc, "vq_gemm")
                wall, ev = timed(launch6, 10, 2, use_graph=False)
                sec = ev / 10
                out.append({"op": "vq_gemm", "cfg": cfg6, "layer": name6, "tokens": tokens, "route": route, "workspace_bytes": int(need),
                            "us": round(sec * 1e6, 1), "TFLOP/s": round(flops / sec / 1e12, 1),
                            "frac_mfma_peak": round(flops / sec / 1e12 / MFMA_FP16_PEAK_TFLOPS, 4)})
                del ws
        del dl6, L6
    W = torch.empty((L4.out_features, L4.in_features), dtype=torch.float16, device="cuda")

    def launch_dq(i):
        rc = vq.vq_dequant(dl.desc, W.data_ptr(), W.stride(0), torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise vq.VQError(rc, "vq_dequant")
    wall, ev = timed(launch_dq, 20, 3, use_graph=False)
    sec = ev / 20
    moved = W.numel() * 2 + L4.idx.nbytes + L4.codebook.nbytes
    out.append({"op": "vq_dequant", "cfg": 4, "us": round(sec * 1e6, 1), "GB/s": round(moved / sec / 1e9, 1),
                "frac_hbm_peak": round(moved / sec / 1e9 / HBM_PEAK_GBPS, 4)})
    # dequant of the 7B-shaped layer (v=6, k=4096)
    _, L1 = next(s.config_layers(1))
    dl1 = vq.DeviceLayer(L1)
    W1 = torch.empty((L1.out_features, L1.in_features), dtype=torch.float16, device="cuda")

    def launch_dq1(i):
        rc = vq.vq_dequant(dl1.desc, W1.data_ptr(), W1.stride(0), torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise vq.VQError(rc, "vq_dequant")
    wall, ev = timed(launch_dq1, 20, 3, use_graph=False)
    sec = ev / 20
    moved = W1.numel() * 2 + L1.algorithmic_bytes(1)
    out.append({"op": "vq_dequant", "cfg": 1, "us": round(sec * 1e6, 1), "GB/s": round(moved / sec / 1e9, 1),
                "frac_hbm_peak": round(moved / sec / 1e9 / HBM_PEAK_GBPS, 4)})
    del dl1
    # ... and of the same shape in the 2.26-bit setting of Table "Quantization parameters" (v = 12, two 4096-entry tables, 4 codebook
    # groups, 40 outlier columns): one table in LDS at a time
    L12 = s.make_layer(1, "up", L1.out_features, L1.in_features, 12, 4096, 4096, n_outlier_cols=40, v_out=4, k_out=8192, group_vectors=85)
    dl12 = vq.DeviceLayer(L12)

    def launch_dq12(i):
        rc = vq.vq_dequant(dl12.desc, W1.data_ptr(), W1.stride(0), torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise vq.VQError(rc, "vq_dequant")
    wall, ev = timed(launch_dq12, 20, 3, use_graph=False)
    sec = ev / 20
    moved = W1.numel() * 2 + L12.algorithmic_bytes(1)
    out.append({"op": "vq_dequant", "cfg": "1 shape with v12 k4096 + residual k4096, 4 codebook groups, 40 outlier columns", "us": round(sec * 1e6, 1),
                "GB/s": round(moved / sec / 1e9, 1), "frac_hbm_peak": round(moved / sec / 1e9 / HBM_PEAK_GBPS, 4)})
    del dl12, L12, W1
    # encode side: nearest-centroid assignment of the headline layer's 11008 x 683 vectors against its 4096 x 6 table
    Wenc = torch.from_numpy(s.to_fp16(s.normal(77, L1.out_features * L1.in_features, 0.02)).reshape(L1.out_features, L1.in_features)).cuda()
    Cenc = torch.from_numpy(L1.codebook).cuda()
    idx_enc = vq.assign(Wenc, Cenc)

    def launch_assign(i):
        rc = vq.vq_assign(Wenc.data_ptr(), None, Wenc.stride(0), Wenc.shape[0], Wenc.shape[1], Cenc.data_ptr(), 6, 4096,
                          idx_enc.data_ptr(), idx_enc.stride(0), torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise vq.VQError(rc, "vq_assign")
    wall, ev = timed(launch_assign, 3, 1, use_graph=False)
    sec = ev / 3
    pairs = float(L1.out_features) * (L1.in_features // 6) * 4096
    flops = pairs * (3 * 6 + 1)            # per (vector, centroid): v subtractions, v multiply-adds, one compare
    out.append({"op": "vq_assign", "cfg": 1, "ms": round(sec * 1e3, 3), "T pairs/s": round(pairs / sec / 1e12, 3),
                "TFLOP/s": round(flops / sec / 1e12, 1), "bound": "alu",
                "frac_fp32_vector_peak": round(flops / sec / 1e12 / FP32_VECTOR_PEAK_TFLOPS, 4)})
    del Wenc, Cenc, idx_enc
    # the quantizer's column loop (Algorithm 1) on a 4096 x 4096 matrix (the 7B attention projections), v=6, k=4096, blocks
    # of 128 columns, a synthetic Hessian's Cholesky factor in the role of H^-1: the search is the same arithmetic as
    # vq_assign, one column after the other; the end-of-block updates are binary32 matrix products on the matrix cores
    nq = 4096
    Uq = torch.from_numpy(np.ascontiguousarray(np.linalg.cholesky(np.linalg.inv(s.make_hessian(2, nq))).T, dtype=np.float32)).cuda()
    W0q = torch.from_numpy(s.make_weights(2, nq, nq).astype(np.float32)).cuda()
    Cq = torch.from_numpy(next(s.config_layers(1))[1].codebook).cuda()
    Wq = W0q.clone()
    vq.quantize_columns(Wq, Uq, Cq, None, block=128, want_T=False)
    torch.cuda.synchronize()
    best_q = None
    for _ in range(2):
        Wq.copy_(W0q)
        t0 = torch.cuda.Event(enable_timing=True); t1 = torch.cuda.Event(enable_timing=True)
        t0.record()
        vq.quantize_columns(Wq, Uq, Cq, None, block=128, want_T=False)
        t1.record(); torch.cuda.synchronize()
        ms = t0.elapsed_time(t1)
        best_q = ms if best_q is None else min(best_q, ms)
    pairs = float(-(-nq // 6)) * nq * 4096
    flops = pairs * (3 * 6 + 1) + float(nq) * nq * nq              # the searches, and the updates: M N^2 / 2 multiply-adds
    out.append({"op": "vq_quantize_columns", "shape": "4096x4096 v6 k4096, blocks of 128 columns", "ms": round(best_q, 2),
                "TFLOP/s": round(flops / best_q / 1e9, 1), "bound": "alu",
                "frac_fp32_vector_peak": round(flops / best_q / 1e9 / FP32_VECTOR_PEAK_TFLOPS, 4)})
    del Uq, W0q, Wq, Cq
    # the paper's other (v, k) settings on the headline shape (App. "Impact of Vector Length"): tables in LDS, whole-window index loads
    for label, kw in (("v4 k256", dict(v=4, k=256)), ("v4 k256 + residual k256", dict(v=4, k=256, k_res=256)), ("v2 k16", dict(v=2, k=16)),
                      ("v12 k4096", dict(v=12, k=4096)), ("v12 k4096 + residual k4096 (two passes)", dict(v=12, k=4096, k_res=4096)),
                      ("v12 k4096 + residual k4096, 4 codebook groups, 40 outlier columns of v4 k8192 (the 2.26-bit setting of "
                       "Table 'Quantization parameters': nine passes)",
                       dict(v=12, k=4096, k_res=4096, n_outlier_cols=40, v_out=4, k_out=8192, group_vectors=85))):
        Lo = s.make_layer(1, "up", L1.out_features, L1.in_features, **kw)
        r = bench_gemv(vq, Lo, s.make_activations(1, Lo, 1), steps, warmup, use_graph)
        sec = r["event_s"] / steps
        alg = Lo.algorithmic_bytes(1)
        out.append({"op": "vq_gemv", "cfg": "1 shape with " + label, "batch": 1, "us": round(sec * 1e6, 3), "GB/s": round(alg / sec / 1e9, 1),
                    "frac_hbm_peak": round(alg / sec / 1e9 / HBM_PEAK_GBPS, 4)})
        if kw.get("group_vectors"):           # with a workspace: a codebook group per workgroup, then the sum over the groups
            r = bench_gemv(vq, Lo, s.make_activations(1, Lo, 1), steps, warmup, use_graph, workspace=True)
            sec = r["event_s"] / steps
            out.append({"op": "vq_gemv_with_workspace", "cfg": "1 shape with " + label, "batch": 1, "us": round(sec * 1e6, 3),
                        "GB/s": round(alg / sec / 1e9, 1), "frac_hbm_peak": round(alg / sec / 1e9 / HBM_PEAK_GBPS, 4)})
        del Lo
    # the headline shape stored in the paper's own orientation (vectors down the output dimension)
    Ld = s.make_layer(1, "up", L1.out_features, L1.in_features, 6, 4096, orientation=1)
    for batch in (1, 4, 16):
        for with_ws in (False, True):
            if with_ws and not vq.vq_gemv_workspace_bytes(vq.DeviceLayer(Ld).desc, batch):
                continue                    # no kernel would use one for this batch
            r = bench_gemv(vq, Ld, s.make_activations(1, Ld, batch), steps, warmup, use_graph, workspace=with_ws)
            sec = r["event_s"] / steps
            alg = Ld.algorithmic_bytes(batch)
            out.append({"op": "vq_gemv_with_workspace" if with_ws else "vq_gemv",
                        "cfg": "1 with vectors down the output dimension (orientation 1)", "batch": batch,
                        "us": round(sec * 1e6, 3), "GB/s": round(alg / sec / 1e9, 1), "frac_hbm_peak": round(alg / sec / 1e9 / HBM_PEAK_GBPS, 4)})
    del Ld
    # the cfg2 decoder layer stored in that orientation, as a chain on one stream: 4 launches (q+k+v and gate+up through
    # vq_gemv_multi) against 7
    c2 = s.CONFIGS[2]
    layers_d = {name: s.make_layer(2, name, out_f, in_f, c2["v"], c2["k"], c2.get("k_res", 0), layer_ordinal=i, orientation=1)
                for i, (name, out_f, in_f) in enumerate(c2["layers"])}
    rots_d = {n: Rotation(vq, L, min_bytes=ROTATE_BYTES // 4) for n, L in layers_d.items()}
    for batch in (1, 16):
        xs = {n: torch.from_numpy(s.make_activations(2, layers_d[n], batch)).cuda() for n in ("q", "o", "gate", "down")}
        ys = {n: torch.empty((batch, L.out_features), dtype=torch.float16, device="cuda") for n, L in layers_d.items()}
        alg = sum(L.algorithmic_bytes(batch) for L in layers_d.values())
        # single layers get a workspace on loan (column parts on the matrix cores; none is asked for at batch 1)
        need_d = {n: vq.vq_gemv_workspace_bytes(rots_d[n].descs[0], batch) for n in layers_d}
        ws_d = torch.empty(max(max(need_d.values()), 256), dtype=torch.uint8, device="cuda")
        for fused in (True, False):
            def chain_d(i):
                st = torch.cuda.current_stream().cuda_stream
                for group in ((("q", "k", "v"), ("o",), ("gate", "up"), ("down",)) if fused else tuple((n,) for n in layers_d)):
                    x = xs[{"k": "q", "v": "q", "up": "gate"}.get(group[0], group[0])]
                    descs = [rots_d[n].descs[i % rots_d[n].copies] for n in group]
                    if len(group) == 1:
                        n = group[0]
                        rc = vq.vq_gemv_with_workspace(descs[0], x.data_ptr(), x.stride(0), batch, ys[n].data_ptr(), ys[n].stride(0),
                                                       ws_d.data_ptr(), need_d[n], st)
                    else:
                        rc = vq.vq_gemv_multi(descs, x.data_ptr(), x.stride(0), batch, [ys[n].data_ptr() for n in group],
                                              [ys[n].stride(0) for n in group], st)
                    if rc != 0:
                        raise vq.VQError(rc, "vq_gemv_multi")
            wall, ev = timed(chain_d, 100, 10, use_graph)
            us = ev / 100 * 1e6
            out.append({"op": "cfg2 decoder layer in orientation 1 as a chain of %d calls (%ssingle layers through vq_gemv_with_workspace)" % (4 if fused else 7, "q+k+v and gate+up through vq_gemv_multi, " if fused else ""), "cfg": 2, "batch": batch,
                        "us": round(us, 2), "GB/s": round(alg / us / 1e3, 1), "frac_hbm_peak": round(alg / us / 1e3 / HBM_PEAK_GBPS, 4)})
    del rots_d, xs, ys, layers_d, ws_d
    # codebook groups on the headline shape: "group num" 4 and 16 of the paper's parameter table, as group sizes
    # rounded up to 8 vectors
    for group_vectors in (176, 48):
        Lg = s.make_layer(1, "up", L1.out_features, L1.in_features, 6, 4096, group_vectors=group_vectors)
        for batch in (1, 16):
            for with_ws in (False, True):
                r = bench_gemv(vq, Lg, s.make_activations(1, Lg, batch), steps, warmup, use_graph, workspace=with_ws)
                sec = r["event_s"] / steps
                alg = Lg.algorithmic_bytes(batch)
                out.append({"op": "vq_gemv_with_workspace" if with_ws else "vq_gemv", "cfg": "1 with codebook groups", "groups": Lg.n_groups,
                            "group_vectors": group_vectors, "batch": batch, "us": round(sec * 1e6, 3), "GB/s": round(alg / sec / 1e9, 1),
                            "frac_hbm_peak": round(alg / sec / 1e9 / HBM_PEAK_GBPS, 4)})
    return out


if __name__ == "__main__":
    main()
