#!/usr/bin/env python3
"""Bench of the sparse prefill-attention hot path on one MI355X.

One step = one pass of the whole path over one prompt: span table -> tile map (host) -> upload
-> bs_attn_prefill (one launch), with q/k/v already resident in HBM.  Prints ONE JSON line.

  value        useful TFLOP/s of the whole step: 4*d FLOP per unmasked (query, key) pair
  roofline     the attention kernel alone (HIP events around each launch) against the MI355X
               dense bf16 MFMA peak
  cpu_baseline the CPU oracle timed on a bounded sample of the same workload (context only)
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

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2,
                    help="workload family 1..5 (default: the 36K one); 6 = family 4 with non-causal attention "
                         "inside an image and sinks at fixed in-image offsets")
    ap.add_argument("--target-len", type=int, default=None, help="config 5 prompt length")
    ap.add_argument("--map", choices=["packed", "regrouped", "natural"], default="packed",
                    help="tile map layout: natural = query rows and keys in position order; regrouped = text "
                         "rows in query tiles of their own (BS_MAP_REGROUP_ROWS); packed = that plus compact "
                         "key tiles of text and sink keys for the sparse classes (BS_MAP_PACK_KEYS)")
    ap.add_argument("--window", type=int, default=0, help="sliding window of the layer (0 = none)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--sink-mode", default="paper10", choices=["paper10", "prefix"])
    ap.add_argument("--all-dense", action="store_true", help="run the same prompt with every head Dense")
    ap.add_argument("--no-dense-leg", action="store_true", help="skip the all-Dense comparison run")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true",
                    help="skip the 36K-300K sweep (class map and all-Dense on the stress prompts at four lengths and "
                         "on the 128K and 300K model-shaped prompts) that the default run adds to its JSON line")
    ap.add_argument("--sweep-steps", type=int, default=3, help="timed launches per sweep entry and leg")
    ap.add_argument("--cpu-seconds", type=float, default=40.0, help="target CPU time of the oracle sample")
    ap.add_argument("--characterize", action="store_true",
                    help="time the offline prompt-level characterisation (Alg. 1: the kernel under the dense "
                         "mask and the three sparse masks for every head + error reduction) instead of the "
                         "prefill step; prints its own JSON line")
    ap.add_argument("--alpha", type=float, default=0.1, help="NMSE threshold of --characterize")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a kernel of known HBM traffic, "
                         "used to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


class HipEvents:
    """Raw hipEvent_t pairs on the process's HIP runtime, for timing the attention kernel alone
    on the stream it is launched on."""

    def __init__(self):
        import ctypes
        self.ct = ctypes
        self.hip = ctypes.CDLL("libamdhip64.so")   # resolves to the copy the process already loaded
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        e = self.ct.c_void_p()
        rc = self.hip.hipEventCreate(self.ct.byref(e))
        assert rc == 0, f"hipEventCreate failed ({rc})"
        return e

    def elapsed_ms(self, a, b):
        self.hip.hipEventSynchronize(b)
        ms = self.ct.c_float()
        rc = self.hip.hipEventElapsedTime(self.ct.byref(ms), a, b)
        assert rc == 0, f"hipEventElapsedTime failed ({rc})"
        return float(ms.value)

    def destroy(self, e):
        self.hip.hipEventDestroy(e)


# HBM-side traffic of one attention launch (read + written past the L2s, where they meet the fabric: the
# 256 MB memory-side cache sits behind that point), from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this bench with the packed tile map, each counter scaled by its reading for a 1 GiB copy.  These are
# figures of earlier profiled runs of the same command, NOT read in this run; the JSON says so.
# Keyed by workload and row order of the map -> (bytes, summary under profiles/).
MEASURED_TRAFFIC = {
    ("cfg2-qwen2vl7b-36k/paper10/seed0", "packed"): (4.82e9, "profiles/attn_prefill_bf16_d128_cfg2_36k.md"),
    ("cfg3-qwen25vl32b-128k/paper10/seed0", "packed"): (62.8e9, "profiles/attn_prefill_bf16_d128_128k_300k.md"),
    ("cfg4-gemma3-27b-300k/paper10/seed0", "packed"): (374.4e9, "profiles/attn_prefill_bf16_d128_128k_300k.md"),
    ("cfg5-stress-307200/paper10/seed0", "packed"): (174.5e9, "profiles/attn_prefill_bf16_d128_128k_300k.md"),
}


def class_totals(tm, head_class):
    """Sum the per-class tile-map statistics over the heads."""
    tot = {"visited": 0, "full": 0, "partial": 0, "allowed_pairs": 0}
    per_class = [tm.stats(c) for c in range(4)]
    for c in head_class:
        for k in tot:
            tot[k] += per_class[int(c)][k]
    return tot, per_class


def timed_steps(bs, torch, p, q, k, v, out, steps, warmup, hev, flags):
    """Returns (wall ms per step, mean attention-kernel ms, mean device ms of the whole call
    incl. map upload and the tile-pack pre-pass, mean host ms of the tile-map build, mean host ms
    inside the attention call (work-unit planning, staging, launches), last tile map)."""
    dt = bs.BS_BF16 if p.dtype == "bf16" else bs.BS_F32
    stream = torch.cuda.current_stream()
    keep = []
    build_s = []
    call_s = []
    ev = []

    def step(record):
        t0 = time.perf_counter()
        tm = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, 128, 64, flags=flags,
                                 sink_offsets=p.sink_offsets or None, window=p.window)
        t1 = time.perf_counter()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        k0, k1 = (hev.create(), hev.create()) if record else (None, None)
        e0.record(stream)
        bs.bs_attn_prefill_ex(q, k, v, out, tm, dt, p.n_q_heads, p.gqa_group, p.head_dim, p.scale,
                              stream.cuda_stream, k0.value if k0 else None, k1.value if k1 else None)
        e1.record(stream)
        t2 = time.perf_counter()
        keep[:] = [tm]   # the previous map is destroyed here; its device blocks go back to the library's cache
        if record:
            build_s.append(t1 - t0)
            call_s.append(t2 - t1)
            ev.append((e0, e1, k0, k1))

    for _ in range(warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(True)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    call_ms = sum(a.elapsed_time(b) for a, b, _, _ in ev) / len(ev)
    kern_ms = sum(hev.elapsed_ms(c, d) for _, _, c, d in ev) / len(ev)
    for _, _, c, d in ev:
        hev.destroy(c)
        hev.destroy(d)
    return wall * 1e3, kern_ms, call_ms, 1e3 * sum(build_s) / len(build_s), 1e3 * sum(call_s) / len(call_s), keep[-1]


def sampled_pairs(head_class, rows, imgid, issink, img_bidir=False, window=0):
    """Allowed pairs of the given query rows summed over the heads (the oracle's own enumeration)."""
    import oracle
    per_class = {c: oracle.pair_count_rows(c, imgid, issink, rows, img_bidir, window) for c in set(int(x) for x in head_class)}
    return sum(per_class[int(c)] for c in head_class)


def cpu_baseline(p, q, k, v, target_seconds):
    """Time the oracle as it stands on a bounded sample of rows of this workload."""
    import numpy as np

    import oracle

    imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len, p.sink_offsets)
    qn, kn, vn = (t.float().cpu().numpy() for t in (q, k, v))
    rng = np.random.default_rng(123)
    # pairs a row costs: count allowed keys per sampled row from the oracle's own predicate
    # via its tile-free mask would be O(L) per row; instead time first, count after.
    n_rows = 8
    rows = np.sort(rng.choice(p.seq_len, size=n_rows, replace=False)).astype(np.int32)
    t0 = time.perf_counter()
    oracle.attention(qn, kn, vn, p.head_class, imgid, issink, p.scale, rows, p.img_bidir, p.window)
    t_probe = time.perf_counter() - t0
    n_rows = int(max(8, min(p.seq_len, n_rows * target_seconds / max(t_probe, 1e-3))))
    rows = np.sort(rng.choice(p.seq_len, size=n_rows, replace=False)).astype(np.int32)
    t0 = time.perf_counter()
    oracle.attention(qn, kn, vn, p.head_class, imgid, issink, p.scale, rows, p.img_bidir, p.window)
    t = time.perf_counter() - t0
    # allowed pairs of the sampled rows, summed over heads (enumeration, outside the timed part)
    pairs = sampled_pairs(p.head_class, rows, imgid, issink, p.img_bidir, p.window)
    flops = 4.0 * p.head_dim * pairs
    return {"value": flops / t / 1e12, "unit": "TFLOP/s (useful, fp64 oracle)", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": round(t, 2),
            "sample": f"{n_rows} random query rows x all {p.n_q_heads} heads of the same prompt "
                      f"({pairs} unmasked pairs)"}


def characterize_bench(args, bs, torch, p, q, k, v, flags):
    """Alg. 1 on the GPU for all heads of one layer of the workload; one step = one whole call
    (four tile maps, four attention launches, three error reductions, decision, read-back)."""
    import numpy as np

    dt = bs.BS_BF16 if p.dtype == "bf16" else bs.BS_F32
    st = torch.cuda.current_stream().cuda_stream
    call = lambda: bs.bs_characterize_prompt(q, k, v, p.spans, p.seq_len, p.sink_len, dt, p.n_q_heads, p.gqa_group,
                                              p.head_dim, p.scale, args.alpha, flags, st, p.sink_offsets or None, p.window)
    for _ in range(args.warmup):
        call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        head_type, nmse = call()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    # the error reduction alone: reads two outputs once
    a, b = torch.randn_like(q), torch.randn_like(q)
    sums = torch.empty((p.n_q_heads, 2), dtype=torch.float64, device=q.device)
    n = p.seq_len * p.head_dim
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for i in range(args.warmup + args.steps):
        j = i - args.warmup
        if j >= 0:
            ev[j][0].record()
        bs.bs_head_sq_error(a, b, dt, p.n_q_heads, n, sums, st)
        if j >= 0:
            ev[j][1].record()
    torch.cuda.synchronize()
    red_ms = sum(x.elapsed_time(y) for x, y in ev) / len(ev)   # includes the 1-workgroup clearing kernel
    red_bytes = 2 * p.n_q_heads * n * (2 if p.dtype == "bf16" else 4)
    # attention work of the four runs
    pairs = []
    for c in range(4):
        tm = bs.bs_build_tilemap(p.spans, p.seq_len, np.full(p.n_q_heads, c, np.uint8), p.sink_len, 128, 64, flags=flags,
                                 sink_offsets=p.sink_offsets or None, window=p.window)
        pairs.append(tm.stats(c)["allowed_pairs"] * p.n_q_heads)
    flop = 4.0 * p.head_dim * sum(pairs)
    res = {
        "metric": "prompt-level characterisation (Alg. 1), all heads of one layer",
        "value": round(ms, 4), "unit": "ms per prompt and layer (host wall clock, call returns results)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": p.dtype, "data": "synthetic",
        "config": {"workload": p.name, "seq_len": p.seq_len, "n_q_heads": p.n_q_heads, "n_kv_heads": p.n_kv_heads,
                   "head_dim": p.head_dim, "n_images": int(len(p.spans)), "map": args.map, "alpha": args.alpha,
                   "values": "random (bench tensors): every sparse mask is expected to fail"},
        "head_types": {nm: int((head_type == c).sum()) for c, nm in enumerate(("dense", "sink", "intra", "intra_sink"))},
        "nmse_median_per_mask": [float(np.median(nmse[m])) for m in range(3)],
        "useful_tflops_whole_call": round(flop / (ms * 1e-3) / 1e12, 2),
        "unmasked_pairs_per_mask": pairs,
        "roofline": {"bound": "hbm", "kernel": "head_sq_error<%s>" % p.dtype, "achieved": round(red_bytes / (red_ms * 1e-3) / 1e9, 1),
                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(red_bytes / (red_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                     "traffic": None, "bytes_per_launch": red_bytes, "avg_launch_ms": round(red_ms, 4)},
    }
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = characterize_cpu_baseline(p, q, k, v, pairs, args.cpu_seconds)
    print(json.dumps(res))


def characterize_cpu_baseline(p, q, k, v, pairs_per_mask, target_seconds):
    """The oracle's attention under the four masks on a sample of rows, extrapolated to the prompt."""
    import numpy as np

    import oracle

    imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len, p.sink_offsets)
    qn, kn, vn = (t.float().cpu().numpy() for t in (q, k, v))
    rng = np.random.default_rng(321)
    n_rows = 4
    total, spent, done = 0.0, 0.0, 0
    for attempt in range(2):
        rows = np.sort(rng.choice(p.seq_len, size=n_rows, replace=False)).astype(np.int32)
        total, spent = 0.0, 0.0
        for c in range(4):
            hc = np.full(p.n_q_heads, c, np.uint8)
            t0 = time.perf_counter()
            oracle.attention(qn, kn, vn, hc, imgid, issink, p.scale, rows, p.img_bidir, p.window)
            t = time.perf_counter() - t0
            spent += t
            total += t * pairs_per_mask[c] / max(1, sampled_pairs(hc, rows, imgid, issink, p.img_bidir, p.window))
        done = n_rows
        if attempt == 0:
            n_rows = int(max(4, min(p.seq_len, n_rows * target_seconds / max(spent, 1e-3))))
    return {"value": round(total * 1e3, 1), "unit": "ms per prompt and layer (extrapolated, attention of the four masks only)",
            "cores": oracle.num_threads(), "kind": "oracle", "seconds": round(spent, 2),
            "sample": f"{done} random query rows x all {p.n_q_heads} heads x 4 masks, scaled by unmasked pairs"}


def reused_map_steps(bs, torch, p, q, k, v, out, steps, flags):
    """A model's prefill reuses ONE tile map of the prompt for all its layers and binds it to each layer's
    class vector (bs_tilemap_rebind).  Times `steps` such layer calls queued back to back, alternating between
    the workload's class vector and a rotated copy (so that every call plans and uploads new work units).
    Returns (wall ms per layer, host ms per layer spent in rebind + bs_attn_prefill while the launches queue
    up, the same host time with the device idle before every call: a single call's host latency)."""
    import numpy as np
    dt = bs.BS_BF16 if p.dtype == "bf16" else bs.BS_F32
    st = torch.cuda.current_stream().cuda_stream
    tm = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, 128, 64, flags=flags,
                             sink_offsets=p.sink_offsets or None, window=p.window)
    vecs = [p.head_class, np.roll(p.head_class, p.gqa_group)]   # same classes per KV group count, other heads
    for i in range(2):
        tm.rebind(vecs[i % 2])
        bs.bs_attn_prefill(q, k, v, out, tm, dt, p.n_q_heads, p.gqa_group, p.head_dim, p.scale, st)
    torch.cuda.synchronize()
    host = 0.0
    t0 = time.perf_counter()
    for i in range(steps):
        h0 = time.perf_counter()
        tm.rebind(vecs[i % 2])
        bs.bs_attn_prefill(q, k, v, out, tm, dt, p.n_q_heads, p.gqa_group, p.head_dim, p.scale, st)
        host += time.perf_counter() - h0
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    idle = 0.0
    for i in range(steps):
        h0 = time.perf_counter()
        tm.rebind(vecs[i % 2])
        bs.bs_attn_prefill(q, k, v, out, tm, dt, p.n_q_heads, p.gqa_group, p.head_dim, p.scale, st)
        idle += time.perf_counter() - h0
        torch.cuda.synchronize()
    return 1e3 * wall / steps, 1e3 * host / steps, 1e3 * idle / steps


def measure_workload(bs, torch, W, p, seed, steps, warmup, hev, flags):
    """Class map and all-Dense on one prompt: kernel ms of both, speed-up, the skipped-tile prediction,
    useful TFLOP/s and the fraction of the bf16 MFMA peak (attention kernel alone, HIP events)."""
    q, k, v = W.make_qkv(p, seed, "cuda:0")
    out = torch.empty_like(q)
    wall, kern, call, build, host_call, tm = timed_steps(bs, torch, p, q, k, v, out, steps, warmup, hev, flags)
    tot, _ = class_totals(tm, p.head_class)
    pd = p.all_dense()
    d_wall, d_kern, d_call, _, _, d_tm = timed_steps(bs, torch, pd, q, k, v, out, steps, 1, hev, flags)
    d_tot, _ = class_totals(d_tm, pd.head_class)
    useful = 4.0 * p.head_dim * tot["allowed_pairs"]
    d_useful = 4.0 * p.head_dim * d_tot["allowed_pairs"]
    tf = useful / (kern * 1e-3) / 1e12
    res = {"workload": p.name, "seq_len": p.seq_len, "n_images": int(len(p.spans)),
           "heads": "%d/%d" % (p.n_q_heads, p.n_kv_heads), "steps": steps,
           "kernel_ms": round(kern, 3), "device_ms_per_call": round(call, 3), "ms_per_step": round(wall, 3),
           "all_dense_kernel_ms": round(d_kern, 3), "speedup_kernel": round(d_kern / kern, 3),
           "predicted_speedup_from_tiles": round(d_tot["visited"] / tot["visited"], 3),
           "skipped_tile_fraction": round(1.0 - tot["visited"] / d_tot["visited"], 4),
           "useful_tflops": round(tf, 1), "frac": round(tf / PEAK_BF16_TFLOPS, 4),
           "frac_with_prepass": round(useful / (call * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
           "all_dense_tflops": round(d_useful / (d_kern * 1e-3) / 1e12, 1),
           "all_dense_frac": round(d_useful / (d_kern * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
           "tilemap_build_host_ms": round(build, 3), "attn_call_host_ms": round(host_call, 3)}
    del q, k, v, out
    torch.cuda.empty_cache()
    return res


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2507_09071_amd as bs
    import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    bs.load_library()

    p = W.config(args.config, args.seed, args.sink_mode, args.target_len)
    if args.all_dense:
        p = p.all_dense()
    if args.window:
        from dataclasses import replace
        p = replace(p, window=args.window, name=p.name + "/window%d" % args.window)
    q, k, v = W.make_qkv(p, args.seed, "cuda:0")
    out = torch.empty_like(q)
    hev = HipEvents()
    if args.calibrate_copy:
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    flags = {"natural": 0, "regrouped": bs.BS_MAP_REGROUP_ROWS, "packed": bs.BS_MAP_PACK_KEYS}[args.map]
    if p.img_bidir:
        flags |= bs.BS_MAP_BIDIR_IMAGES
    order = args.map
    if args.characterize:
        del out
        characterize_bench(args, bs, torch, p, q, k, v, flags)
        return
    wall_ms, kern_ms, call_ms, build_ms, host_call_ms, tm = timed_steps(bs, torch, p, q, k, v, out, args.steps, args.warmup, hev, flags)
    tot, per_class = class_totals(tm, p.head_class)
    d = p.head_dim
    useful_flop = 4.0 * d * tot["allowed_pairs"]
    executed_flop = 4.0 * d * 128 * 64 * tot["visited"]
    esize = 2 if p.dtype == "bf16" else 4
    plan = tm.pair_plan(p.gqa_group) if p.dtype == "bf16" else None
    # K and V^T tile bytes the attention kernel requests from L2: one pair of tiles per step of a
    # work unit (bf16: two items share the stream), else per visited tile
    kv_steps = plan["unit_tiles"] if plan else tot["visited"]
    kv_stream_bytes = kv_steps * 2 * 64 * d * esize
    min_bytes = (2 * p.n_q_heads + 2 * p.n_kv_heads) * p.seq_len * d * esize

    dense = None
    if not args.all_dense and not args.no_dense_leg:
        pd = p.all_dense()
        dsteps = max(3, min(args.steps, 10))
        d_wall, d_kern, d_call, _, _, d_tm = timed_steps(bs, torch, pd, q, k, v, out, dsteps, 1, hev, flags)
        d_tot, _ = class_totals(d_tm, pd.head_class)
        dense = {"ms_per_step": round(d_wall, 4), "kernel_ms": round(d_kern, 4), "steps": dsteps,
                 "visited_tiles": d_tot["visited"],
                 "useful_tflops": round(4.0 * d * d_tot["allowed_pairs"] / (d_kern * 1e-3) / 1e12, 2),
                 "speedup_kernel": round(d_kern / kern_ms, 3),
                 "speedup_device_call": round(d_call / call_ms, 3),     # pre-pass included on both sides
                 "speedup_step": round(d_wall / wall_ms, 3),
                 "predicted_speedup_from_tiles": round(d_tot["visited"] / tot["visited"], 3)}
    reuse_wall, reuse_host, reuse_idle = reused_map_steps(bs, torch, p, q, k, v, out, args.steps, flags)

    achieved = useful_flop / (kern_ms * 1e-3) / 1e12
    traffic, traffic_file = MEASURED_TRAFFIC.get((p.name, order), (None, None))
    res = {
        "metric": "attn prefill ms + useful TFLOP/s (MFMA util), speedup vs all-Dense @36K-300K",
        "value": round(useful_flop / (wall_ms * 1e-3) / 1e12, 3),
        "unit": "TFLOP/s useful (4*d FLOP per unmasked pair), whole step",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": p.dtype, "data": "synthetic",
        "config": {"workload": p.name, "seq_len": p.seq_len, "n_q_heads": p.n_q_heads,
                   "n_kv_heads": p.n_kv_heads, "head_dim": d, "n_images": int(len(p.spans)),
                   "sink_mode": args.sink_mode if not p.sink_offsets else "%d in-image offsets" % len(p.sink_offsets),
                   "image_attention": "bidirectional" if p.img_bidir else "causal", "window": p.window,
                   "seed": args.seed, "map": order,
                   "head_classes": {n: int((p.head_class == c).sum()) for c, n in enumerate(W.CLASS_NAMES)}},
        "kernel_ms": round(kern_ms, 4),
        "device_ms_per_call": round(call_ms, 4),
        "tilemap_build_host_ms": round(build_ms, 4),
        "attn_call_host_ms": round(host_call_ms, 4),
        "reused_map": {"what": "one tile map of the prompt, re-bound to another class vector before every call (a layer of "
                               "a model): no map build, the work units are planned and uploaded per call",
                       "ms_per_layer": round(reuse_wall, 4), "host_ms_per_layer_queued": round(reuse_host, 4),
                       "host_ms_per_layer_device_idle": round(reuse_idle, 4),
                       "useful_tflops": round(useful_flop / (reuse_wall * 1e-3) / 1e12, 2)},
        "executed_tflops": round(executed_flop / (kern_ms * 1e-3) / 1e12, 2),
        "kv_stream_gbs": round(kv_stream_bytes / (kern_ms * 1e-3) / 1e9, 1),
        "min_hbm_gbs": round(min_bytes / (kern_ms * 1e-3) / 1e9, 1),
        "work_units": plan,
        "tiles": {"visited": tot["visited"], "full": tot["full"], "partial": tot["partial"],
                  "unmasked_pairs": tot["allowed_pairs"],
                  "useful_over_executed": round(useful_flop / executed_flop, 4)},
        "all_dense": dense,
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": traffic,
                     "traffic_source": (traffic_file + " (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; not measured in this run)") if traffic is not None else None,
                     "kernel": "attn_prefill_%s<%d>" % (p.dtype, d),
                     "flop_per_launch": useful_flop, "avg_launch_ms": round(kern_ms, 4),
                     # the same useful FLOP over the device time of the whole call: the K / V^T tile-pack
                     # pre-pass that every bf16 call runs (two HBM-bound kernels) counted in
                     "frac_with_prepass": round(useful_flop / (call_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                     "device_ms_per_call": round(call_ms, 4)},
    }
    del q, k, v, out
    torch.cuda.empty_cache()
    if not args.no_sweep and args.config == 2 and not args.all_dense and not args.window and p.dtype == "bf16":
        # the 36K-300K range of the metric: the stress prompts at their four lengths, then the
        # 128K and 300K model-shaped prompts; same kernel, same map layout, few launches each
        sweep = []
        for cfg, target in [(5, L) for L in W.STRESS_LENGTHS] + [(3, None), (4, None)]:
            ps = W.config(cfg, args.seed, args.sink_mode, target)
            sweep.append(measure_workload(bs, torch, W, ps, args.seed, args.sweep_steps, 1, hev, flags))
            print("sweep", json.dumps(sweep[-1]), file=sys.stderr, flush=True)
        res["sweep"] = sweep
    if not args.no_cpu_baseline:
        q, k, v = W.make_qkv(p, args.seed, "cuda:0")
        res["cpu_baseline"] = cpu_baseline(p, q, k, v, args.cpu_seconds)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
