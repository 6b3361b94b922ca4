#!/usr/bin/env python3
"""Benchmark: one packed encode of the ViT-L/14-336 ragged multi-request batch per step.

Prints ONE JSON line.  A step is one vit_encode_packed call over the whole batch
(64 requests, 260 images, 150 020 tokens) with pixels already resident in HBM.
`roofline` is for the dominant kernel family (the bf16 MFMA matrix products), timed with
HIP events on the launch stream inside the timed region; `cpu_baseline` times the CPU
oracle on a bounded sample of whole images from the same batch.
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

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak
HBM_PEAK_GBS = 8000.0
# HBM-side bytes of all matrix-product launches of one step come from the committed rocprofv3 --pmc summary of the
# workload (FETCH_SIZE and WRITE_SIZE runs, scaled by the copy calibration described there): a profile figure, not
# measured by this script.  The summary names the commit it was taken at; both travel into the JSON line.
TRAFFIC_PROFILES = {"cfg3": "profiles/kernels_cfg3_ragged_hbm_traffic.md"}


def gemm_traffic(workload):
    """(bytes per step, source) parsed from the profile summary of `workload`, or (None, reason)."""
    import re

    rel = TRAFFIC_PROFILES.get(workload)
    if rel is None:
        return None, "no HBM-traffic profile is committed for this workload"
    try:
        text = open(os.path.join(ROOT, rel)).read()
    except OSError:
        return None, f"{rel} is missing"
    m = re.search(r"All matrix-product launches of one step: ([0-9.]+) GB read \+ ([0-9.]+) GB written", text)
    c = re.search(r"Taken at commit ([0-9a-f]{7,40})", text)
    if not m:
        return None, f"{rel} has no matrix-product total"
    return (float(m.group(1)) + float(m.group(2))) * 1e9, f"{rel} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE; taken at commit {c.group(1) if c else 'unknown'})"


def flops(cfg, tile_offsets):
    """Algorithmic FLOPs (2 per multiply-add; LN/softmax/GELU/bias excluded). Returns (total, gemm, attention)."""
    g = cfg["image_size"] // cfg["patch_size"]
    P = g * g
    T = P + cfg["has_cls"]
    K = cfg["channels"] * cfg["patch_size"] ** 2
    D, M = cfg["hidden"], cfg["mlp"]
    L_loc, L_glob = cfg["layers_local"], cfg["layers_global"]
    tpi = np.diff(np.asarray(tile_offsets, dtype=np.int64))
    n_tiles = int(tpi.sum())
    gemm = n_tiles * (2.0 * P * K * D + (L_loc + L_glob) * (2.0 * T * D * 3 * D + 2.0 * T * D * D + 4.0 * T * D * M))
    m = max(cfg["token_merge"], 1)
    d_in, t_out = D * m * m, (T if m == 1 else (g // m) ** 2)  # the projector sees the down-sampled tokens
    for i in range(cfg["proj_layers"]):
        gemm += n_tiles * 2.0 * t_out * d_in * cfg["proj_dims"][i]
        d_in = cfg["proj_dims"][i]
    attn = n_tiles * L_loc * 4.0 * T * T * D + float(sum(L_glob * 4.0 * (n * T) * (n * T) * D for n in tpi))
    return gemm + attn, gemm, attn


def product_flops(cfg, tile_offsets):
    """Algorithmic FLOPs of each matrix-product family of one step (keys as in VitEncoder.profile_read)."""
    g = cfg["image_size"] // cfg["patch_size"]
    P = g * g
    T = P + cfg["has_cls"]
    K = cfg["channels"] * cfg["patch_size"] ** 2
    D, M, L = cfg["hidden"], cfg["mlp"], cfg["layers_local"] + cfg["layers_global"]
    n_tiles = int(np.asarray(tile_offsets)[-1])
    m = max(cfg["token_merge"], 1)
    d_in, t_out, proj = D * m * m, (T if m == 1 else (g // m) ** 2), 0.0
    for i in range(cfg["proj_layers"]):
        proj += n_tiles * 2.0 * t_out * d_in * cfg["proj_dims"][i]
        d_in = cfg["proj_dims"][i]
    rows = float(n_tiles) * T
    return {"gemm_patch": n_tiles * 2.0 * P * K * D, "gemm_qkv": L * 2.0 * rows * D * 3 * D, "gemm_out": L * 2.0 * rows * D * D,
            "gemm_fc1": L * 2.0 * rows * D * M, "gemm_fc2": L * 2.0 * rows * D * M, "gemm_proj": proj}


def cpu_baseline(cfg, weights, px, tile_offsets, n_sample):
    """Oracle (fp32, as it stands) on the first n_sample images of the batch; returns the JSON object."""
    from threadpoolctl import threadpool_info

    from oracle import vit_oracle as O

    w = O.unpack_weights(cfg, weights, np.float32)
    to = np.asarray(tile_offsets[:n_sample + 1])
    t0 = time.perf_counter()
    O.vit_oracle_encode(cfg, w, px[:int(to[-1])], [n_sample], to, dtype=np.float32)
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {
        "value": n_sample / dt, "unit": "images/s", "cores": int(threads), "kind": "oracle",
        "sample": f"first {n_sample} images of the batch, fp32 numpy oracle, {dt:.2f} s wall",
    }


def sweep(args, torch, gen, V):
    """Throughput against images per launch (Sec. 3.2: encode time grows linearly with the batch once the
    device is full) and the config-3 batch under three request packings."""
    cfg, ipr3, to3 = gen.make_workload("cfg3")
    weights = gen.make_weights(cfg, seed=0)
    enc = V.VitEncoder(cfg, weights, device=0)
    px = torch.from_numpy(gen.make_pixels(cfg, 260, seed=1)).cuda()
    T = gen.tokens_per_tile(cfg)

    def timed(n, ipr, label):
        to = np.arange(n + 1, dtype=np.int32)
        n_tok, out_dim, _, _ = enc.query(n, n)
        out = torch.empty((n_tok, out_dim), dtype=torch.bfloat16, device="cuda")
        for _ in range(2):
            enc.encode(px[:n], ipr, to, out=out)
        torch.cuda.synchronize()
        steps = max(3, min(50, int(2000 / max(n, 1))))
        t0 = time.perf_counter()
        for _ in range(steps):
            enc.encode(px[:n], ipr, to, out=out)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        total_f, _, _ = flops(cfg, to)
        print(json.dumps({"sweep": label, "images": n, "requests": int(len(ipr)), "tokens": n * T, "ms_per_launch": ms,
                          "images_per_s": n / (ms * 1e-3), "pct_bf16_peak": 100.0 * total_f / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}))
        return ms

    points = []
    for n in (1, 2, 4, 8, 16, 32, 64, 128, 260):
        points.append((n, timed(n, np.ones(n, dtype=np.int32), "images per launch")))
    # Host side of a small launch: how long the calling thread is busy issuing it, as ~270 kernel launches and as one
    # replay of the recorded sequence (vit_encode_packed_graph).  The device time of the launch is the same either way.
    for n in (1, 8):
        to = np.arange(n + 1, dtype=np.int32)
        n_tok, out_dim, _, _ = enc.query(n, n)
        out = torch.empty((n_tok, out_dim), dtype=torch.bfloat16, device="cuda")
        pxn = px[:n]
        host_us = {}
        for graph in (False, True):
            for _ in range(3):  # (with graph=True: plain, recording, first replay)
                enc.encode(pxn, [n], to, out=out, graph=graph)
            torch.cuda.synchronize()
            ts = []
            for _ in range(20):
                t0 = time.perf_counter()
                enc.encode(pxn, [n], to, out=out, graph=graph)
                ts.append(time.perf_counter() - t0)
                torch.cuda.synchronize()
            host_us[graph] = float(np.median(ts)) * 1e6
        print(json.dumps({"host_time_of_one_call": "plain launches against one graph replay", "images": n,
                          "plain_us": host_us[False], "graph_replay_us": host_us[True]}))
    timed(260, ipr3, "cfg3 as 64 ragged requests")
    timed(260, np.ones(260, dtype=np.int32), "cfg3 as 260 single-image requests")
    timed(260, np.asarray([260], dtype=np.int32), "cfg3 as one request of 260 images")
    enc.close()

    # GPU preprocessing (Sec. 2): Table 1's example, an 896 x 896 image -> 2 x 2 tiles of 448 + a thumbnail
    img = torch.from_numpy(gen.make_image_u8(896, 896, 3, seed=2)).cuda()
    tiles = V.preprocess_tiles(img, 448, 2, 2, True, (0.48, 0.45, 0.41), (0.27, 0.26, 0.28))
    torch.cuda.synchronize()
    reps = 200
    t0 = time.perf_counter()
    for _ in range(reps):
        V.preprocess_tiles(img, 448, 2, 2, True, (0.48, 0.45, 0.41), (0.27, 0.26, 0.28), out=tiles)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / reps * 1e6
    print(json.dumps({"preprocess": "896x896x3 uint8 -> 5 tiles of 448 (fp32)", "us_per_image": us,
                      "images_per_s": 1e6 / us, "gb_per_s": (img.numel() + tiles.numel() * 4) / us / 1e3}))

    # Stage profile -> maximum batch and capacity under a latency SLO (Sec. 4.2), then the two routing
    # policies of Sec. 4.3 on a seeded heavy-tailed request stream, four Image Instances modelled with
    # the latencies just measured.
    from paper_2502_00937_amd import router as R
    from paper_2502_00937_amd import stage_profile as SP

    profile = [SP.ProfilePoint(n, n * T, ms) for n, ms in points]
    for slo in (10.0, 25.0, 50.0, 100.0):
        b = SP.max_batch_under_slo(profile, slo)
        mc = SP.capacity_tokens_per_s(profile, slo, T)
        print(json.dumps({"stage_profile": "max batch under SLO", "slo_ms": slo, "max_images_per_launch": b,
                          "capacity_image_tokens_per_s": mc,
                          "replicas_for_5M_tokens_per_s": SP.replicas(5e6, mc) if mc > 0 else None}))
    lat = lambda images, tiles: SP.latency_at(profile, images)  # noqa: E731
    b50 = max(1, SP.max_batch_under_slo(profile, 50.0))
    for gap in (8.0, 4.0, 3.0):  # mean inter-arrival time in ms; about 4 images per request
        arrivals = gen.make_arrivals(4000, gap, seed=0)
        for policy in ("round_robin_request", "least_image_tokens"):
            r = np.asarray(R.simulate(arrivals, 4, T, lat, b50, policy))
            print(json.dumps({"routing": policy, "instances": 4, "mean_interarrival_ms": gap, "requests": len(arrivals),
                              "images": int(sum(len(t) for _, t in arrivals)), "max_images_per_launch": b50,
                              "encode_latency_ms": {"p50": float(np.percentile(r, 50)), "p90": float(np.percentile(r, 90)),
                                                    "p99": float(np.percentile(r, 99)), "max": float(r.max())}}))


def serve(torch, gen, V):
    """One Image Instance run against the wall clock on a seeded heavy-tailed request stream (Sec. 4.2, 4.3): launches
    of what has arrived, up to the maximum batch under a 50 ms SLO; the encode latency per request beside what
    the event model of `router.simulate` predicts for one instance from the stage profile measured first."""
    from paper_2502_00937_amd import router as R
    from paper_2502_00937_amd import stage_profile as SP
    from paper_2502_00937_amd.image_instance import ImageInstance, percentiles

    cfg, _, _ = gen.make_workload("cfg3")
    enc = V.VitEncoder(cfg, gen.make_weights(cfg, seed=0), device=0)
    T = gen.tokens_per_tile(cfg)
    px = torch.from_numpy(gen.make_pixels(cfg, 128, seed=1)).cuda()
    profile = SP.measure_profile(enc, px, 1, T, (1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128))
    b50 = max(1, min(128, SP.max_batch_under_slo(profile, 50.0)))
    lat = lambda images, tiles: SP.latency_at(profile, images)  # noqa: E731
    inst = ImageInstance(enc, px, max_images=b50)
    for gap in (8.0, 4.0, 2.5):  # mean inter-arrival time in ms; about 4 images per request
        arrivals = gen.make_arrivals(1200, gap, seed=0)
        measured, launches = inst.run_stream(arrivals)
        model = R.simulate(arrivals, 1, T, lat, b50, "least_image_tokens")
        keys = ("p50", "p90", "p99")
        print(json.dumps({"serve": "one Image Instance, real time", "mean_interarrival_ms": gap, "requests": len(arrivals),
                          "images": int(sum(len(t) for _, t in arrivals)), "max_images_per_launch": b50,
                          "launches": len(launches), "mean_images_per_launch": float(np.mean([l[0] for l in launches])),
                          "encode_latency_ms": dict(zip(keys, percentiles(measured)), max=float(max(measured))),
                          "event_model_ms": dict(zip(keys, percentiles(model)), max=float(max(model)))}))
    enc.close()


def vendor_gemm(torch, gen):
    """The vendor library's plain bf16 product C = A W^T (no bias, no epilogue) on the matrix-product shapes of
    one config-3 step, random operands.  Context for `roofline`: what the library reaches on this device for the
    same contraction, without the fused epilogues the encoder's kernels carry.  Not part of the encode path."""
    cfg, ipr, to = gen.make_workload("cfg3")
    m = int(to[-1]) * gen.tokens_per_tile(cfg)
    D, M = cfg["hidden"], cfg["mlp"]
    shapes = [("qkv", 3 * D, D), ("out-proj", D, D), ("fc1", M, D), ("fc2", D, M),
              ("projector 2", cfg["proj_dims"][1], cfg["proj_dims"][0])]
    g = torch.Generator(device="cuda").manual_seed(0)
    for name, n, k in shapes:
        a = (torch.rand((m, k), device="cuda", generator=g) * 2 - 1).to(torch.bfloat16)
        w = ((torch.rand((n, k), device="cuda", generator=g) * 2 - 1) * 0.02).to(torch.bfloat16)
        for _ in range(3):
            c = a @ w.t()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        torch.cuda.synchronize()
        reps = 20
        ev[0].record()
        for _ in range(reps):
            c = a @ w.t()
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1]) / reps
        print(json.dumps({"vendor_gemm": name, "M": m, "N": n, "K": k, "ms": ms, "tflops": 2.0 * m * n * k / ms / 1e9}))
        del a, w, c


def power_trace(args, torch, gen, V):
    """Socket power and per-XCD shader clocks (amd-smi, twice a second) while the workload's encode step runs back to
    back for about six seconds.  Context for every fraction of peak this script prints: the device holds its power
    cap during the step, so its clock, not its issue rate, is what the matrix products run into."""
    import subprocess
    import threading

    cfg, ipr, to = gen.make_workload(args.workload)
    n_images, n_tiles = int(ipr.sum()), int(to[-1])
    enc = V.VitEncoder(cfg, gen.make_weights(cfg, seed=0), device=0)
    px = torch.from_numpy(gen.make_pixels(cfg, n_tiles, seed=1)).cuda()
    n_tok, out_dim, _, _ = enc.query(n_tiles, n_images)
    out = torch.empty((n_tok, out_dim), dtype=torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32, device="cuda")
    samples, stop = [], threading.Event()

    def poll():
        while not stop.is_set():
            try:
                doc = json.loads(subprocess.run(["amd-smi", "metric", "-g", "0", "--power", "--clock", "--json"],
                                                capture_output=True, text=True, timeout=5).stdout)
                g = doc["gpu_data"][0] if isinstance(doc, dict) else doc[0]
                clocks = [g["clock"][k]["clk"]["value"] for k in sorted(g["clock"]) if k.startswith("gfx_")]
                samples.append({"t": time.perf_counter(), "socket_power_w": g["power"]["socket_power"]["value"],
                                "gfx_clock_mhz": clocks})
            except Exception as e:  # the tool is missing or its output changed: report, do not fail the run
                samples.append({"t": time.perf_counter(), "error": repr(e)[:200]})
            stop.wait(0.5)

    for _ in range(2):
        enc.encode(px, ipr, to, out=out)
    torch.cuda.synchronize()
    th = threading.Thread(target=poll, daemon=True)
    t0 = time.perf_counter()
    th.start()
    steps = 0
    while time.perf_counter() - t0 < 6.0:
        enc.encode(px, ipr, to, out=out)
        torch.cuda.synchronize()
        steps += 1
    t1 = time.perf_counter()
    stop.set()
    th.join(timeout=10)
    enc.close()
    busy = [s for s in samples if "error" not in s and t0 + 1.0 <= s["t"] <= t1]  # skip the ramp of the first second
    result = {"power_trace": args.workload, "steps": steps, "ms_per_step": (t1 - t0) / steps * 1e3,
              "samples": len(busy), "errors": [s["error"] for s in samples if "error" in s][:2]}
    if busy:
        pw = [float(s["socket_power_w"]) for s in busy]
        ck = [float(c) for s in busy for c in s["gfx_clock_mhz"]]
        result.update({"socket_power_w": {"mean": sum(pw) / len(pw), "min": min(pw), "max": max(pw)},
                       "gfx_clock_mhz": {"mean": sum(ck) / len(ck), "min": min(ck), "max": max(ck)}})
    print(json.dumps(result))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "cfg6"])
    ap.add_argument("--cpu-sample", type=int, default=12, help="images the CPU oracle encodes (0 = skip)")
    ap.add_argument("--no-kernel-events", action="store_true", help="time the steps without per-kernel events")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line: encode 1, 8, 64 and 260 images of the config-3 model (one JSON "
                         "line per size) and config 3 repacked as 260 single-image requests / one 260-image request")
    ap.add_argument("--serve", action="store_true",
                    help="run one Image Instance in real time on a seeded request stream (three arrival rates, about 20 s) "
                         "and print measured encode latencies beside the event model's")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="time the vendor library's bf16 matrix product (torch.matmul) on the step's shapes: context only")
    ap.add_argument("--power-trace", action="store_true",
                    help="run the workload's step back to back for six seconds while sampling socket power and shader "
                         "clocks with amd-smi; prints one JSON line (context for the fractions of peak)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run five plain 1 GiB device copies and exit (scale reference for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import gen
    import paper_2502_00937_amd as V

    if not torch.cuda.is_available():
        print("bench.py: no HIP device visible; there is no CPU path", file=sys.stderr)
        sys.exit(2)
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": 1 << 30, "bytes_written": 1 << 30, "copies": 5}}))
        return
    if args.vendor_gemm:
        vendor_gemm(torch, gen)
        return
    if args.power_trace:
        power_trace(args, torch, gen, V)
        return
    if args.sweep:
        sweep(args, torch, gen, V)
        return
    if args.serve:
        serve(torch, gen, V)
        return
    cfg, ipr, to = gen.make_workload(args.workload)
    n_images, n_tiles = int(ipr.sum()), int(to[-1])
    T = gen.tokens_per_tile(cfg)
    weights = gen.make_weights(cfg, seed=0)
    px = gen.make_pixels(cfg, n_tiles, seed=1)
    enc = V.VitEncoder(cfg, weights, device=0)
    px_dev = torch.from_numpy(px).cuda()
    n_tok, out_dim, _, _ = enc.query(n_tiles, n_images)
    out = torch.empty((n_tok, out_dim), dtype=torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32,
                      device="cuda")

    for _ in range(args.warmup):
        enc.encode(px_dev, ipr, to, out=out)
    torch.cuda.synchronize()
    if not args.no_kernel_events:
        enc.profile_enable(True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]  # on the launch stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        enc.encode(px_dev, ipr, to, out=out)
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))

    total_f, gemm_f, attn_f = flops(cfg, to)
    result = {
        "metric": "images/sec + encoder tokens/sec (ViT-L/14-336 ragged batch); % bf16 MFMA peak",
        "value": n_images / (ms_per_step * 1e-3),
        "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {
            "workload": {"cfg1": "tiny ViT fp32, 4 images", "cfg2": "ViT-L/14-336 + projector, 8 images",
                         "cfg3": "ViT-L/14-336 + 2-layer projector, ragged batch: 64 requests / 260 images, one launch",
                         "cfg4": "SigLIP-style 384px, 128 images / 591 tiles",
                         "cfg5": "ViT-H/14-560, 32 images x 4 tiles, 32 local + 8 global layers",
                         "cfg6": "6B-class ViT on 448px tiles, 2x2 token down-sampling to 256 tokens per tile, "
                                 "8 images / 36 tiles"}[args.workload],
            "requests": int(len(ipr)), "images": n_images, "tiles": n_tiles, "tokens": int(n_tok),
            "encoder_tokens": n_tiles * T,
            "weights": "seeded N(0, 0.02), bf16-rounded", "pixels": "seeded U[-1,1), resident in HBM",
        },
        "ms_per_step_median": step_ms[len(step_ms) // 2], "ms_per_step_min": step_ms[0],
        "tokens_per_s": n_tiles * T / (ms_per_step * 1e-3),  # encoder tokens; differs from the output only with token_merge
        "output_tokens_per_s": n_tok / (ms_per_step * 1e-3),
        "tiles_per_s": n_tiles / (ms_per_step * 1e-3),
        "tflops": total_f / (ms_per_step * 1e-3) / 1e12,
        "pct_bf16_peak": 100.0 * total_f / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
    }
    if not args.no_kernel_events:
        prof = enc.profile_read()
        enc.profile_enable(False)
        fam_ms = {k: v[0] / args.steps for k, v in prof.items()}
        gemm_ms, gemm_n = prof["gemm"][0] / args.steps, prof["gemm"][1] // args.steps
        achieved = gemm_f / (gemm_ms * 1e-3) / 1e12
        traffic, traffic_source = gemm_traffic(args.workload)
        result["roofline"] = {
            "bound": "mfma", "kernel": "gemm_bf16_dma_kernel (all matrix products of one step; products of fewer than 384 tiles of 256x256, and the short last round of the products one column band wide, run as gemm_bf16_ring_kernel)",
            "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
            # register-only MFMA loop on this device, TFLOP/s: operands random like real data / one constant
            "measured_mfma_ceiling": V.vit_mfma_ceiling(0, 0.1, True),
            "measured_mfma_ceiling_constant_operands": V.vit_mfma_ceiling(0, 0.1, False),
            "traffic": traffic, "traffic_unit": "bytes per step (all launches)", "traffic_source": traffic_source,
            "launches_per_step": int(gemm_n), "ms_per_step": gemm_ms,
            "avg_launch_ms": gemm_ms / max(gemm_n, 1), "flop_per_step": gemm_f,
        }
        result["kernel_ms_per_step"] = fam_ms
        # every matrix product on a line of its own: launches and ms per step, ms per launch, TFLOP/s
        pf = product_flops(cfg, to)
        assert abs(sum(pf.values()) - gemm_f) <= 1e-9 * gemm_f
        result["gemm_products"] = {
            k: {"launches": int(prof[k][1] // args.steps), "ms_per_step": fam_ms[k],
                "ms_per_launch": fam_ms[k] / max(prof[k][1] // args.steps, 1),
                "tflops": pf[k] / (fam_ms[k] * 1e-3) / 1e12 if fam_ms[k] > 0 else None}
            for k in pf}
        att_ms = fam_ms["attention"]
        result["attention_tflops"] = attn_f / (att_ms * 1e-3) / 1e12 if att_ms > 0 else None
        # LayerNorm passes: each reads fp32 [tokens, D] and writes the operand type
        es = 2 if cfg["dtype"] == "bf16" else 4
        ln_n = prof["layernorm"][1] // args.steps
        ln_bytes = ln_n * n_tiles * T * cfg["hidden"] * (4 + es)  # every encoder token, before any down-sampling
        result["layernorm_gbs"] = ln_bytes / (fam_ms["layernorm"] * 1e-3) / 1e9 if fam_ms["layernorm"] > 0 else None
    if not args.no_kernel_events and cfg["dtype"] == "bf16":
        # two more steps, outside the timed region, with the persistent kernel stamping its tiles: microseconds per tile
        # in the k-loop and in the epilogue, and the shader clock the (power-limited) chip held, per matrix product
        enc.profile_tiles_enable(True)
        for _ in range(2):
            enc.encode(px_dev, ipr, to, out=out)
        result["tile_phases"] = {k: {"k_loop_us": v[0], "epilogue_us": v[1], "shader_clock_mhz": v[2], "tiles_stamped": int(v[3])}
                                 for k, v in enc.profile_tiles_read().items()}
        enc.profile_tiles_enable(False)
    enc.close()
    if args.cpu_sample > 0:
        result["cpu_baseline"] = cpu_baseline(cfg, weights, px, to, min(args.cpu_sample, n_images))
    print(json.dumps(result))


if __name__ == "__main__":
    main()
