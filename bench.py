#!/usr/bin/env python3
"""Benchmark of the compression hot path on one MI355X.

A "step" is one synchronisation round of the whole hot path over one batch of synthetic input:
qsl_compress for the R workers (form m + Delta, Top_k select, QSGD quantise, bit-pack, error-memory
update, payload bit counts) followed by qsl_aggregate of the R messages into the dense update.
Inputs (a fresh Delta[R, d] per step, the carried error memory) are resident in HBM before the timed
region starts.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published peak
ALGO_BYTES_PER_COORD = 12       # read m, read Delta, write m': what the method itself must move
PROFILES = os.path.join(ROOT, "profiles")


def kernel_source_digest():
    """sha256 over the kernel sources: a counter summary under profiles/ names the digest it was taken with."""
    import hashlib
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_1906_02367_amd", "csrc")
    for name in sorted(os.listdir(src)):
        with open(os.path.join(src, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def measured_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` from the rocprofv3 counter summary profiles/<kernel>_<workload>_hbm_traffic.txt
    (FETCH_SIZE and WRITE_SIZE runs, scaled by a device copy of known size), if that summary was taken with the kernel
    sources as they are now; else None and the reason."""
    import re
    path = os.path.join(PROFILES, f"{kernel}_{workload}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None, "no counter summary for this kernel and workload under profiles/"
    text = open(path).read()
    dig = re.search(r"kernel_source_sha256:\s*([0-9a-f]+)", text)
    tot = re.search(r"traffic_bytes_per_launch:\s*([0-9]+)", text)
    if not dig or not tot:
        return None, f"{os.path.basename(path)} has no digest or total"
    if dig.group(1) != kernel_source_digest():
        return None, f"{os.path.basename(path)} was taken with other kernel sources ({dig.group(1)})"
    return int(tot.group(1)), f"profiles/{os.path.basename(path)}"


def gpu_state():
    """Clock levels and power of the first AMD GPU as the driver's sysfs files show them (plain file reads:
    nothing is executed); None if they are not there."""
    import glob

    def read(path):
        try:
            with open(path) as f:
                return f.read().strip()
        except OSError:
            return None

    for dev in sorted(glob.glob("/sys/class/drm/card[0-9]*/device")):
        if read(os.path.join(dev, "vendor")) != "0x1002":
            continue
        out = {}
        for name in ("pp_dpm_sclk", "pp_dpm_mclk", "pp_dpm_fclk"):
            txt = read(os.path.join(dev, name))
            if txt:
                cur = [ln.strip() for ln in txt.splitlines() if ln.strip().endswith("*")]
                out[name] = cur[0] if cur else txt.splitlines()[-1].strip()
        for hw in glob.glob(os.path.join(dev, "hwmon", "hwmon*")):
            for name in ("power1_average", "power1_input", "power1_cap"):
                txt = read(os.path.join(hw, name))
                if txt and txt.isdigit():
                    out[name + "_W"] = int(txt) / 1e6
        if out:
            return out
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration 1..5 (2 = headline); 6 = the paper's own per-tensor rule on ResNet-50's tensor table; "
                         "7, 8 = every coordinate kept with index-free messages (EF-signSGD, EF-QSGD as this operator)")
    ap.add_argument("--workers", type=int, default=0,
                    help="override the configuration's R (R = 1 is the deployment shape: one worker per GPU); "
                         "not the headline line")
    ap.add_argument("--from-models", action="store_true",
                    help="time qsl_compress_diff (Delta = x - xhat formed on the fly; the fresh buffers act as the "
                         "local models) instead of qsl_compress; not the headline line")
    ap.add_argument("--standalone-update", action="store_true",
                    help="the error memory is written by the stand-alone qsl_error_update (compress writes a copy that is "
                         "thrown away): times that entry point inside the round; not the headline line")
    ap.add_argument("--aggregate-messages", default="",
                    help="comma-separated message counts (at most 64): after the timed rounds, also time qsl_aggregate alone "
                         "on that many messages of this workload (master line of Algorithm 1 with many workers); an extra "
                         "object in the JSON line, not part of `value`")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="do not bracket the streaming kernel with HIP events (diagnostic: the roofline entry is then empty)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rounds", type=int, default=5)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a kernel of known traffic, to scale rocprofv3 counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the R workers are a batch on one device); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    state = gpu_state()
    import numpy as np
    import torch
    from paper_1906_02367_amd import binding as B
    from paper_1906_02367_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = W.config(args.config, R=args.workers) if args.workers else W.config(args.config)
    q = B.from_workload(wl, device=dev)
    R, d = wl.R, wl.d
    total = args.steps + args.warmup

    # inputs resident in HBM: one fresh Delta per step, generated on the device from a fixed seed
    gen = W.TorchDeltas(wl, dev)
    n_buf = total if total * R * d * 4 <= 120e9 else max(2, int(120e9 // (R * d * 4)))
    deltas = [gen(t) for t in range(n_buf)]
    m = torch.zeros(R, d, dtype=torch.float32, device=dev)
    msg = q.new_msg(R)
    msg_bits = torch.zeros(R, dtype=torch.int64, device=dev)
    x = torch.zeros(d, dtype=torch.float32, device=dev)       # the master's parameter vector
    torch.cuda.synchronize()

    m_copy = torch.empty_like(m) if args.standalone_update else None

    def compress(t):
        if args.from_models:
            q.compress_diff(m, x, deltas[t % n_buf], m, 0, t, msg, msg_bits)
        elif args.standalone_update:
            q.compress(m, deltas[t % n_buf], m_copy, 0, t, msg, msg_bits)
            q.error_update(m, deltas[t % n_buf], msg)
        else:
            q.compress(m, deltas[t % n_buf], m, 0, t, msg, msg_bits)

    def step(t):
        compress(t)
        q.aggregate(msg, x, -1.0 / R, accumulate=True)     # x <- x - (1/R) sum_r g^(r)

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)                       # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for t in range(args.warmup):
        step(t)
    torch.cuda.synchronize()
    q.timing_enable(not args.no_kernel_timing)
    t0 = time.perf_counter()
    for t in range(args.warmup, total):
        step(t)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    stream_ms, launches = q.timing_read()
    q.timing_enable(False)
    assert q.device_status() == B.OK
    elapsed = t1 - t0
    # a second, separate pass: every round bracketed by events on the stream the library launches on
    ev = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(3)) for _ in range(args.steps)]
    for i, (e0, ec, e1) in enumerate(ev):
        e0.record()
        compress(total + i)
        ec.record()
        q.aggregate(msg, x, -1.0 / R, accumulate=True)
        e1.record()
    torch.cuda.synchronize()
    per_round = sorted(e0.elapsed_time(e1) for e0, ec, e1 in ev)
    per_compress = sorted(e0.elapsed_time(ec) for e0, ec, e1 in ev)
    assert q.device_status() == B.OK
    state_after = gpu_state()
    # for scale: the same traffic shape (two [R, d] reads, one [R, d] write) through PyTorch's own elementwise add
    ref_out = torch.empty_like(m)
    for _ in range(3):
        torch.add(m, deltas[0], out=ref_out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        torch.add(m, deltas[0], out=ref_out)
    e1.record()
    torch.cuda.synchronize()
    ref_us = e0.elapsed_time(e1) * 100.0
    del ref_out
    coords_per_s = R * d * args.steps / elapsed
    units = q.debug_units()
    bits = msg_bits.cpu().numpy()

    avg_stream_s = stream_ms / 1e3 / max(1, launches)
    algo_bytes = ALGO_BYTES_PER_COORD * R * d + (4 * d if args.from_models else 0)     # + one read of x
    achieved = algo_bytes / avg_stream_s / 1e9 if launches else None
    kernel = "k_dense_norm" if wl.dense else "k_stream"
    plain = not (args.from_models or args.workers or args.standalone_update)
    traffic, traffic_source = measured_traffic(kernel, wl.name) if plain else (None, "only the plain entry point is profiled")
    roofline = {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": (achieved / HBM_PEAK_GBS) if achieved else None,
                "traffic": traffic, "traffic_source": traffic_source,
                "avg_launch_us": avg_stream_s * 1e6, "launches": launches,
                "algorithmic_bytes_per_launch": algo_bytes}
    # the whole compress call (every kernel from the sample to the packed message) on the same accounting; an operator
    # that keeps every coordinate reads v once more and writes m' in its second pass: 20 bytes per coordinate
    step_bytes = (20 if wl.dense else ALGO_BYTES_PER_COORD) * R * d
    compress_ms = per_compress[len(per_compress) // 2]
    compress_call = {"median_ms": compress_ms, "min_ms": per_compress[0], "algorithmic_bytes": step_bytes,
                     "GB/s": step_bytes / compress_ms / 1e6, "frac": step_bytes / compress_ms / 1e6 / HBM_PEAK_GBS}

    aggregate_scaling = None
    if args.aggregate_messages:
        counts = sorted({int(c) for c in args.aggregate_messages.split(",")})
        n_max = counts[-1]
        qa = B.from_workload(wl, max_workers=n_max, device=dev)
        many = qa.new_msg(n_max)
        ma = torch.empty_like(m)
        for b in range((n_max + R - 1) // R):              # workers b R .. b R + R - 1: their own inputs and random words
            n = min(R, n_max - b * R)
            ma.zero_()
            qa.compress(ma[:n], deltas[b % n_buf][:n], ma[:n], b * R, 0, many[b * R:b * R + n])
        torch.cuda.synchronize()
        entries = [int(v) for v in many[:, :4].contiguous().view(torch.int32)[:, 0].cpu()]
        xa = torch.zeros(d, dtype=torch.float32, device=dev)
        aggregate_scaling = []
        for n in counts:
            for _ in range(3):
                qa.aggregate(many[:n], xa, -1.0 / n, accumulate=True)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                qa.aggregate(many[:n], xa, -1.0 / n, accumulate=True)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1000.0 / 20
            tot = sum(entries[:n]) if not wl.dense else n * d
            aggregate_scaling.append({"messages": n, "entries": tot, "us": us, "ns_per_entry": us * 1000.0 / max(1, tot)})
        assert qa.device_status() == B.OK
        del qa, many, ma, xa

    cpu = None
    if not args.no_cpu_baseline:
        from concurrent.futures import ThreadPoolExecutor
        from oracle import oracle as O
        op = O.OracleOp(wl.d, wl.seg_offset, wl.seg_k, wl.s, wl.sparsifier, wl.quantizer, wl.seed, dense=wl.dense)
        try:
            cores = len(os.sched_getaffinity(0))
        except AttributeError:
            cores = os.cpu_count() or 1
        threads = max(1, min(R, cores, int(os.environ.get("OMP_NUM_THREADS", cores))))
        m_host = np.zeros((R, d), dtype=np.float32)
        cpu_t, cpu_coords = 0.0, 0
        x_now = x.cpu().numpy()
        for t in range(args.cpu_rounds):
            d_host = deltas[t % n_buf].cpu().numpy()
            if args.from_models:
                d_host = np.subtract(x_now[None, :], d_host, dtype=np.float32)
            c0 = time.perf_counter()
            with ThreadPoolExecutor(max_workers=threads) as ex:
                res = list(ex.map(lambda r: op.compress(m_host[r], d_host[r], r, t), range(R)))
            msgs = np.stack([x["msg"] for x in res])
            op.aggregate(msgs, 1.0 / R)
            cpu_t += time.perf_counter() - c0
            cpu_coords += R * d
            m_host = np.stack([x["m_out"] for x in res])
        cpu = {"value": cpu_coords / cpu_t, "unit": "coords/s", "cores": threads, "kind": "oracle",
               "sample": f"{args.cpu_rounds} full sync rounds of the same workload (R={R}, d={d}), one oracle "
                         f"thread per worker, compress + aggregate"}

    line = {
        "metric": "compressed coords/sec, Top-k+QSGD+err-update+aggregate" if args.config == 2 else
                  f"compressed coords/sec, {wl.name}",
        "value": coords_per_s, "unit": "coords/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "R": R, "d": d, "k": int(wl.K), "s": wl.s, "segments": wl.L,
                   "sparsifier": ["top_k", "rand_k"][wl.sparsifier],
                   "quantizer": ["qsgd", "sign_l1", "sign_l2", "fp32", "qsgd_scaled", "sign_l3", "sign_l4"][wl.quantizer],
                   "format": "index-free" if wl.dense else "indices + codes",
                   "error_update": "stand-alone qsl_error_update" if args.standalone_update else "fused",
                   "fresh_delta_buffers": n_buf, "delta": "x - xhat on the fly" if args.from_models else "given",
                   "paths": {"fast": int((units[:, 0] == 0).sum()), "general": int((units[:, 0] == 1).sum()),
                             "fallback": int((units[:, 0] == 2).sum()), "one_block": int((units[:, 0] == 3).sum()),
                             "all_kept": int((units[:, 0] == 4).sum())},
                   "max_candidates": int(units[:, 1].max()), "mean_msg_bits": float(bits.mean())},
        "algorithmic_GBps_whole_step": step_bytes / (R * d) * coords_per_s / 1e9,
        "compress_call": compress_call,
        "per_round_ms": {"median": per_round[len(per_round) // 2], "min": per_round[0], "max": per_round[-1],
                         "note": "separate pass after the timed region, HIP events around each round"},
        "gpu_state": {"before": state, "after": state_after, "kernel_source_sha256": kernel_source_digest()},
        "stream_reference": {"what": "torch.add(m, delta, out=...) on the same [R, d] arrays: 2 reads + 1 write per coordinate",
                             "us": ref_us, "GB/s": ALGO_BYTES_PER_COORD * R * d / ref_us / 1e3},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    if aggregate_scaling is not None:
        line["aggregate_scaling"] = aggregate_scaling
    print(json.dumps(line))


if __name__ == "__main__":
    main()
