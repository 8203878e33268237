#!/usr/bin/env python3
"""Benchmark of the SGPRS stage computation on one MI355X.

A "step" is one pass of the whole hot path -- all six ResNet18 stages -- over
one batch of synthetic input already resident in HBM.  The headline workload
is the batch-64 bf16 (fp32 accumulate) forward on one partition of all CUs;
`value` is images/s.  The same run also reports, in the one JSON line:

  roofline      the dominant kernel (the convolution kernel instantiation with
                the largest total time): algorithmic FLOP / measured duration
                against the dense bf16 MFMA peak
  cpu_baseline  the fp64 oracle timed on the host cores on a bounded sample
  stages        per-stage time, FLOP/s, GB/s and fraction of the per-kernel
                roofline max(FLOP/peak, bytes/HBM peak)
  batch1_fp32   six-stage latency of the fp32 batch-1 network (median / max)
  cu_sweep      time and speed-up of six isolated operators on CU masks
                8..256 (fp32 and bf16), with the oracle's host time beside it
  multi_tenant  eight bf16 instances on an 8 x 32-CU pool, issued concurrently

Only one GPU is used; --gpus above 1 is refused.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16 = 2500.0e12   # dense bf16 MFMA, FLOP/s
PEAK_F32 = 157.3e12     # fp32 MFMA
PEAK_HBM = 8.0e12       # bytes/s


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Hip:
    """Just enough of the HIP runtime for event timing on a given stream."""

    def __init__(self):
        self.l = ctypes.CDLL("libamdhip64.so")

    def event(self):
        e = ctypes.c_void_p()
        assert self.l.hipEventCreate(ctypes.byref(e)) == 0
        return e

    def record(self, e, stream):
        assert self.l.hipEventRecord(e, ctypes.c_void_p(stream)) == 0

    def elapsed_ms(self, a, b):
        assert self.l.hipEventSynchronize(b) == 0
        ms = ctypes.c_float()
        assert self.l.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
        return ms.value


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--no-extras", action="store_true", help="skip batch-1, CU sweep and multi-tenant legs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle CPU baseline")
    ap.add_argument("--cpu-sample", type=int, default=64, help="images of the batch the oracle is timed on")
    ap.add_argument("--periodic-only", action="store_true", help="only the periodic-task scheduler experiment")
    ap.add_argument("--batch-sweep-only", action="store_true", help="only the bf16 throughput at batches 1..32")
    ap.add_argument("--probes-only", action="store_true", help="only the sustained MFMA and load-path probes")
    ap.add_argument("--pool-scaling-only", default=None, metavar="N[,N...]",
                    help="only the eight-instance throughput on pools of N equal partitions (for tracing which kernels "
                         "run beside which), e.g. 8 or 4,8")
    ap.add_argument("--pool-rounds", type=int, default=150, help="rounds of eight inferences per pool in that leg")
    ap.add_argument("--multi-tenant-only", action="store_true",
                    help="only the eight-instance leg on the 8 x 32-CU pool (stage by stage, static executor with and "
                         "without the busy-partition gate, sweeps over partitions in use and over the gate)")
    ap.add_argument("--membound-only", action="store_true",
                    help="run only the memory-bound operator leg (for profiling it); prints its own JSON line")
    ap.add_argument("--copy-calib", action="store_true",
                    help="also run one plain 256 MiB copy (bn_relu with scale 1, shift 0 on non-negative data), "
                         "the known-size kernel that HBM traffic counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (the stage computation has no multi-GPU "
                 "part); run with --gpus 1")

    import torch

    import paper_2406_09425_amd as S
    from workloads import BN_EPS, SWEEP_OPS, make_bn, make_conv_weight, make_input, make_resnet18_params

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    hip = Hip()
    total_cus = S.Pool(1, 8).info()["total_cus"]
    pool = S.Pool(1, total_cus)
    stream = pool.stream(0)

    def nhwc(x, tdt):
        return torch.from_numpy(np.ascontiguousarray(x.transpose(0, 2, 3, 1))).to(tdt).cuda().contiguous()

    def copy_calibration():
        nel = 128 << 20  # 128 Mi bf16 elements = 256 MiB read + 256 MiB written
        src = torch.ones(nel, dtype=torch.bfloat16, device="cuda")
        dst = torch.empty_like(src)
        one = torch.ones(64, dtype=torch.float32, device="cuda")
        zero = torch.zeros(64, dtype=torch.float32, device="cuda")
        S.sgprs_bn_relu(S.SGPRS_BF16, nel // 64, 64, src.data_ptr(), one.data_ptr(), zero.data_ptr(), dst.data_ptr(),
                        pool, 0)
        pool.sync()

    if args.probes_only:
        print(json.dumps(dict(sustained_mfma=leg_mfma_probe(S, hip, torch, pool, stream, total_cus),
                              sustained_load_to_lds=leg_load_probe(S, hip, torch, pool, stream, total_cus))), flush=True)
        pool.destroy()
        return

    if args.pool_scaling_only:
        parts = tuple(int(v) for v in args.pool_scaling_only.split(","))
        print(json.dumps(dict(pool_scaling=leg_pool_scaling(S, torch, total_cus, nhwc, rounds=args.pool_rounds, partitions=parts))),
              flush=True)
        pool.destroy()
        return

    if args.batch_sweep_only:
        print(json.dumps(dict(batch_sweep_bf16=leg_batch_sweep(S, hip, torch, pool, stream, nhwc))), flush=True)
        pool.destroy()
        return

    if args.periodic_only:
        print(json.dumps(dict(periodic_tasks=leg_periodic(S, hip, torch, total_cus, nhwc))), flush=True)
        pool.destroy()
        return

    if args.multi_tenant_only:
        print(json.dumps(dict(multi_tenant=leg_multi_tenant(S, hip, torch, total_cus, nhwc))), flush=True)
        pool.destroy()
        return

    if args.membound_only:
        if args.copy_calib:
            copy_calibration()
        print(json.dumps(dict(memory_bound_ops=leg_membound(S, hip, torch, pool, stream, reps=6))), flush=True)
        pool.destroy()
        return

    # ------------------------------------------------------------ headline
    n = args.batch
    params = make_resnet18_params(4, 0, bf16=True)
    x_host = make_input(4, 0, (n, 3, 224, 224), bf16=True)
    task = S.Task(params, S.SGPRS_BF16, n, BN_EPS)
    xd = nhwc(x_host, torch.bfloat16)
    logits = torch.empty((n, 1000), dtype=torch.float32, device="cuda")

    def step():
        task.run(n, xd.data_ptr(), logits.data_ptr(), pool, 0)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize(); pool.sync()
    e0, e1 = hip.event(), hip.event()
    t0 = time.perf_counter()
    hip.record(e0, stream)
    for _ in range(args.steps):
        step()
    hip.record(e1, stream)
    pool.sync(); torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = hip.elapsed_ms(e0, e1)
    ms_per_step = wall * 1e3 / args.steps
    value = n * args.steps / wall
    log(f"headline: {value:.0f} img/s, {ms_per_step:.3f} ms/step (events: {ev_ms / args.steps:.3f} ms/step)")

    if args.copy_calib:
        copy_calibration()

    # ------------------------------------------------------------ per-kernel profile
    task.set_profiling(True)
    agg = {}      # kernel name -> [time_s, flops, bytes, launches]
    stages = []
    prof_steps = min(args.steps, 100)
    per_stage = [dict(ms=0.0, flops=0.0, bytes=0.0, roof_s=0.0) for _ in range(6)]
    for _ in range(prof_steps):
        step()
        pool.sync()
        for j in range(6):
            for r in task.kernel_times(j):
                a = agg.setdefault((r["name"], r["kind"]), [0.0, 0.0, 0.0, 0])
                a[0] += r["ms"] * 1e-3; a[1] += r["flops"]; a[2] += r["bytes"]; a[3] += 1
                ps = per_stage[j]
                ps["ms"] += r["ms"]; ps["flops"] += r["flops"]; ps["bytes"] += r["bytes"]
                ps["roof_s"] += max(r["flops"] / PEAK_BF16, r["bytes"] / PEAK_HBM)
    # Per-kernel times are start..stop of each dispatch (both events ride on the
    # kernel's own packet), i.e. the kernel alone, as a profiler's kernel trace
    # reports it.  Gaps between kernels are not in them; what the unprofiled
    # step spends outside kernels is reported as gap_us_per_step.
    launches = sum(v[3] for v in agg.values()) / prof_steps
    sum_prof_us = sum(v[0] for v in agg.values()) / prof_steps * 1e6
    gap_us = ev_ms / args.steps * 1e3 - sum_prof_us

    for j, ps in enumerate(per_stage):
        t_s = max(ps["ms"] * 1e-3 / prof_steps, 1e-7)
        stages.append(dict(stage=j, ms=round(t_s * 1e3, 4),
                           images_per_s=round(n / t_s, 1),
                           tflops=round(ps["flops"] / prof_steps / t_s / 1e12, 2),
                           mfma_frac=round(ps["flops"] / prof_steps / t_s / PEAK_BF16, 4),
                           gb_per_s=round(ps["bytes"] / prof_steps / t_s / 1e9, 1),
                           roofline_frac=round(ps["roof_s"] / prof_steps / t_s, 4)))
    kernels = []
    for (name, kind), (t_s, fl, by, cnt) in sorted(agg.items(), key=lambda kv: -kv[1][0]):
        kernels.append(dict(kernel=name, launches_per_step=cnt // prof_steps, avg_us=round(t_s / cnt * 1e6, 2),
                            tflops=round(fl / t_s / 1e12, 2), gb_per_s=round(by / t_s / 1e9, 1)))
    dom_key = max((k for k in agg if k[1] in (0, 8, 10, 11, 12)), key=lambda k: agg[k][0])
    dt_s, dfl, dby, dcnt = agg[dom_key]
    traffic = None
    tr_file = os.path.join(ROOT, "profiles", "resnet18_b64_bf16_hbm_traffic.txt")
    if n == 64 and os.path.exists(tr_file):  # measured once with rocprofv3 --pmc, see profiles/
        tot, disp = 0.0, 0   # a kernel launched at several grid sizes has several rows: dispatch-weighted mean
        for line in open(tr_file):
            if dom_key[0] in line:
                f = line.split()
                tot += int(f[-3]) * (float(f[-2]) + float(f[-1])) * 1e6
                disp += int(f[-3])
        if disp:
            traffic = round(tot / disp)
    roofline = dict(bound="mfma", kernel=dom_key[0], achieved=round(dfl / dt_s / 1e12, 2), peak=PEAK_BF16 / 1e12,
                    unit="TFLOP/s", frac=round(dfl / dt_s / PEAK_BF16, 4), traffic=traffic,
                    avg_launch_us=round(dt_s / dcnt * 1e6, 2), launches_per_step=dcnt // prof_steps,
                    flop_per_launch=round(dfl / dcnt, 1), algorithmic_bytes_per_launch=round(dby / dcnt, 1),
                    kernel_us_per_step=round(sum_prof_us, 1), gap_us_per_step=round(gap_us, 1),
                    launches_all_kernels=round(launches))
    conv_t = sum(v[0] for k, v in agg.items() if k[1] in (0, 1, 2, 8, 9, 10, 11, 12))
    conv_fl = sum(v[1] for k, v in agg.items() if k[1] in (0, 1, 8, 9, 10, 11, 12))
    conv_all = dict(tflops=round(conv_fl / conv_t / 1e12, 2), mfma_frac=round(conv_fl / conv_t / PEAK_BF16, 4),
                    us_per_step=round(conv_t / prof_steps * 1e6, 1))
    task.set_profiling(False)
    log("roofline:", json.dumps(roofline))
    log("conv total:", json.dumps(conv_all))
    for s in stages:
        log("stage", json.dumps(s))
    for k in kernels:
        log("kernel", json.dumps(k))

    # ------------------------------------------------------------ CPU baseline (oracle)
    cpu = None
    if not args.no_cpu:
        import oracle
        ns = max(1, min(args.cpu_sample, n))
        t1 = time.perf_counter()
        ref = oracle.resnet18(params, BN_EPS, x_host[:ns])
        dt = time.perf_counter() - t1
        got = logits[:ns].cpu().numpy().astype(np.float64)
        err = float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))
        cpu = dict(value=round(ns / dt, 3), unit="images/s", cores=oracle.max_threads(), kind="oracle",
                   sample=(f"all {ns} images" if ns == n else f"first {ns} images") +
                          f" of the batch-{n} workload, fp64 direct loops, {dt:.1f} s",
                   gpu_vs_oracle_max_rel_err=err,
                   argmax_equal=bool(np.array_equal(np.argmax(got, 1), np.argmax(ref, 1))))
        log("cpu_baseline:", json.dumps(cpu))
    task.destroy()

    out = {
        "metric": "resnet18_images_per_s", "value": round(value, 1), "unit": "images/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"ResNet18 forward, batch {n}, bf16 storage / fp32 accumulate, 3x224x224 ~N(0,1), "
                               f"six stages on one partition of all {total_cus} CUs",
                   "batch": n, "partition_cus": total_cus},
        "roofline": roofline, "cpu_baseline": cpu, "conv_all": conv_all, "stages": stages, "kernels": kernels,
    }

    if not args.no_extras:
        # sustained matrix-core rate of this chip (instruction mix of the conv inner loop, no global traffic)
        out["roofline"]["sustained_mfma"] = leg_mfma_probe(S, hip, torch, pool, stream, total_cus)
        rnd = out["roofline"]["sustained_mfma"]["random_data"]["tflops"]
        out["roofline"]["frac_of_sustained_random_data"] = round(roofline["achieved"] / rnd, 4)
        out["conv_all"]["frac_of_sustained_random_data"] = round(conv_all["tflops"] / rnd, 4)
        out["roofline"]["sustained_load_to_lds"] = leg_load_probe(S, hip, torch, pool, stream, total_cus)
        out["periodic_tasks"] = leg_periodic(S, hip, torch, total_cus, nhwc)
        out["batch1_fp32"] = leg_batch1(S, hip, pool, stream, nhwc, torch, total_cus)
        out["batch_sweep_bf16"] = leg_batch_sweep(S, hip, torch, pool, stream, nhwc)
        out["cu_sweep"] = leg_sweep(S, hip, torch, total_cus, nhwc, with_cpu=not args.no_cpu)
        out["multi_tenant"] = leg_multi_tenant(S, hip, torch, total_cus, nhwc)
        out["pool_scaling"] = leg_pool_scaling(S, torch, total_cus, nhwc)
        out["memory_bound_ops"] = leg_membound(S, hip, torch, pool, stream)
        out["oversubscribed_pool"] = leg_oversubscribed(S, torch, total_cus, nhwc, headline_ips=value)
    pool.destroy()
    print(json.dumps(out), flush=True)


def leg_batch1(S, hip, pool, stream, nhwc, torch, total_cus, runs=100):
    """Six-stage latency of the fp32 batch-1 network; max over runs = WCET."""
    from workloads import BN_EPS, STAGE_IO, make_input, make_resnet18_params
    params = make_resnet18_params(1, 0)
    x = make_input(1, 0, (1, 3, 224, 224))
    res = {}
    for dtype, tdt, name in ((S.SGPRS_F32, torch.float32, "fp32"), (S.SGPRS_BF16, torch.bfloat16, "bf16")):
        task = S.Task(params, dtype, 1, BN_EPS)
        xd = nhwc(x, tdt)
        lg = torch.empty((1, 1000), dtype=torch.float32, device="cuda")
        ev = [hip.event() for _ in range(7)]
        per = [[] for _ in range(6)]
        whole = []
        for it in range(runs + 10):
            for j in range(6):
                hip.record(ev[j], stream)
                src = xd.data_ptr() if j == 0 else task.stage_output(j - 1)
                dst = lg.data_ptr() if j == 5 else task.stage_output(j)
                task.stage_run(j, 1, src, dst, pool, 0)
            hip.record(ev[6], stream)
            pool.sync()
            if it >= 10:
                for j in range(6):
                    per[j].append(hip.elapsed_ms(ev[j], ev[j + 1]))
                whole.append(hip.elapsed_ms(ev[0], ev[6]))
        # back-to-back whole-network throughput (no per-stage events)
        e0, e1 = hip.event(), hip.event()
        hip.record(e0, stream)
        for _ in range(runs):
            task.run(1, xd.data_ptr(), lg.data_ptr(), pool, 0)
        hip.record(e1, stream)
        pool.sync()
        thr_ms = hip.elapsed_ms(e0, e1) / runs
        res[name] = dict(stage_ms_median=[round(statistics.median(p), 4) for p in per],
                         stage_ms_max=[round(max(p), 4) for p in per],
                         net_ms_median=round(statistics.median(whole), 4), net_ms_max=round(max(whole), 4),
                         back_to_back_ms=round(thr_ms, 4), images_per_s=round(1e3 / thr_ms, 1))
        log("batch1", name, json.dumps(res[name]))
        task.destroy()
    return res


def leg_batch_sweep(S, hip, torch, pool, stream, nhwc, batches=(1, 2, 4, 8, 16, 32), runs=200):
    """bf16 whole-network throughput at batch sizes below the headline's, on the whole chip, through
    sgprs_task_run (graph replay), back to back on one stream."""
    from workloads import BN_EPS, make_input, make_resnet18_params
    params = make_resnet18_params(4, 0, bf16=True)
    res = {}
    for n in batches:
        task = S.Task(params, S.SGPRS_BF16, n, BN_EPS)
        xd = nhwc(make_input(4, 0, (n, 3, 224, 224), bf16=True), torch.bfloat16)
        lg = torch.empty((n, 1000), dtype=torch.float32, device="cuda")
        for _ in range(20):
            task.run(n, xd.data_ptr(), lg.data_ptr(), pool, 0)
        e0, e1 = hip.event(), hip.event()
        hip.record(e0, stream)
        for _ in range(runs):
            task.run(n, xd.data_ptr(), lg.data_ptr(), pool, 0)
        hip.record(e1, stream)
        pool.sync()
        ms = hip.elapsed_ms(e0, e1) / runs
        res[str(n)] = dict(ms_per_step=round(ms, 4), images_per_s=round(n * 1e3 / ms, 1),
                           tflops=round(3.628e9 * n / (ms * 1e-3) / 1e12, 1))
        log("batch_sweep", n, json.dumps(res[str(n)]))
        task.destroy()
    return res


def leg_sweep(S, hip, torch, total_cus, nhwc, with_cpu=True, reps=200):
    """Six isolated operators on CU masks 8..total; speed-up relative to 8 CUs."""
    from workloads import BN_EPS, make_bn, make_conv_weight, make_input
    cu_list = [c for c in (8, 16, 32, 64, 128, 256) if c <= total_cus]
    res = {}
    oracle_ms = {}
    if with_cpu:
        import oracle
        x = make_input(2, 0, (1, 256, 14, 14)); w = make_conv_weight(2, 0, 1, 256, 256, 3)
        xs = make_input(2, 1, (1, 3, 224, 224)); wsx = make_conv_weight(2, 1, 1, 64, 3, 7)
        xm = make_input(2, 2, (1, 64, 112, 112)); xb = make_input(2, 3, (1, 128, 28, 28))
        g, b, m, v = make_bn(2, 3, 1, 128)
        xa = make_input(2, 4, (1, 512, 7, 7)); xf = make_input(2, 5, (1, 512, 7, 7))
        wf = make_conv_weight(2, 5, 1, 1000, 512, 1)[:, :, 0, 0]

        def tm(f):
            ts = []
            for _ in range(5):
                t = time.perf_counter(); f(); ts.append(time.perf_counter() - t)
            return round(statistics.median(ts) * 1e3, 4)
        oracle_ms = {
            "conv3x3_256": tm(lambda: oracle.conv2d(x, w, 1, 1)),
            "conv7x7_stem": tm(lambda: oracle.conv2d(xs, wsx, 2, 3)),
            "maxpool": tm(lambda: oracle.maxpool2d(xm)),
            "bn_relu": tm(lambda: oracle.relu(oracle.bn(xb, g, b, m, v, BN_EPS))),
            "add": tm(lambda: oracle.add(xa, xa)),
            "avgpool_fc": tm(lambda: oracle.fc(oracle.global_avgpool(xf), wf, None)),
        }
    for dtype, tdt, dname in ((S.SGPRS_F32, torch.float32, "fp32"), (S.SGPRS_BF16, torch.bfloat16, "bf16")):
        bf = dtype == S.SGPRS_BF16
        es = 2 if bf else 4
        # operands, built once
        x = nhwc(make_input(2, 0, (1, 256, 14, 14), bf16=bf), tdt)
        d3 = S.ConvDesc(1, 14, 14, 256, 256, 3, 3, 1, 1, dtype, 1)
        w3 = torch.from_numpy(S.sgprs_pack_conv_weights(d3, make_conv_weight(2, 0, 1, 256, 256, 3, bf16=bf))).cuda()
        xs = nhwc(make_input(2, 1, (1, 3, 224, 224), bf16=bf), tdt)
        d7 = S.ConvDesc(1, 224, 224, 3, 64, 7, 7, 2, 3, dtype, 1)
        w7 = torch.from_numpy(S.sgprs_pack_conv_weights(d7, make_conv_weight(2, 1, 1, 64, 3, 7, bf16=bf))).cuda()
        ones = torch.ones(1024, dtype=torch.float32, device="cuda")
        zeros = torch.zeros(1024, dtype=torch.float32, device="cuda")
        y3 = torch.empty((1, 14, 14, 256), dtype=tdt, device="cuda")
        y7 = torch.empty((1, 112, 112, 64), dtype=tdt, device="cuda")
        xm = nhwc(make_input(2, 2, (1, 64, 112, 112), bf16=bf), tdt)
        ym = torch.empty((1, 56, 56, 64), dtype=tdt, device="cuda")
        xb = nhwc(make_input(2, 3, (1, 128, 28, 28), bf16=bf), tdt)
        yb = torch.empty_like(xb)
        xa = nhwc(make_input(2, 4, (1, 512, 7, 7), bf16=bf), tdt)
        ya = torch.empty_like(xa)
        wf = torch.from_numpy(make_conv_weight(2, 5, 1, 1000, 512, 1, bf16=bf)[:, :, 0, 0].copy()).to(tdt).cuda()
        yf = torch.empty((1, 1000), dtype=torch.float32, device="cuda")
        wsf = torch.empty(512, dtype=torch.float32, device="cuda")
        work = {  # algorithmic FLOP, bytes
            "conv3x3_256": (2.0 * 196 * 256 * 2304, (196 * 256 * 2 + 256 * 2304) * es),
            "conv7x7_stem": (2.0 * 12544 * 64 * 147, (3 * 224 * 224 + 64 * 147 + 12544 * 64) * es),
            "maxpool": (0.0, (64 * 112 * 112 + 64 * 56 * 56) * es),
            "bn_relu": (2.0 * 100352, 2 * 100352 * es),
            "add": (25088.0, 3 * 25088 * es),
            "avgpool_fc": (2.0 * 512 * 1000, (25088 + 512000) * es + 4000),
        }
        res[dname] = {k: {"cus": cu_list, "us": [], "speedup_vs_8": [], "tflops": [], "gb_per_s": [],
                          "flop": work[k][0], "bytes": work[k][1], "oracle_host_ms": oracle_ms.get(k)}
                      for k in work}
        for cus in cu_list:
            pool = S.Pool(1, cus)
            st = pool.stream(0)
            wsb = max(S.sgprs_conv2d_workspace(d3, cus), 16)
            ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
            ops = {
                "conv3x3_256": lambda: S.sgprs_conv2d(d3, x.data_ptr(), w3.data_ptr(), ones.data_ptr(),
                                                      zeros.data_ptr(), None, y3.data_ptr(), ws.data_ptr(), wsb,
                                                      pool, 0),
                "conv7x7_stem": lambda: S.sgprs_conv2d(d7, xs.data_ptr(), w7.data_ptr(), ones.data_ptr(),
                                                       zeros.data_ptr(), None, y7.data_ptr(), None, 0, pool, 0),
                "maxpool": lambda: S.sgprs_maxpool2d(dtype, 1, 112, 112, 64, xm.data_ptr(), ym.data_ptr(), pool, 0),
                "bn_relu": lambda: S.sgprs_bn_relu(dtype, 784, 128, xb.data_ptr(), ones.data_ptr(),
                                                   zeros.data_ptr(), yb.data_ptr(), pool, 0),
                "add": lambda: S.sgprs_add_relu(dtype, 25088, xa.data_ptr(), xa.data_ptr(), ya.data_ptr(), False,
                                                pool, 0),
                "avgpool_fc": lambda: S.sgprs_avgpool_fc(dtype, 1, 49, 512, 1000, xa.data_ptr(), wf.data_ptr(), None,
                                                         yf.data_ptr(), wsf.data_ptr(), pool, 0),
            }
            for name, f in ops.items():
                for _ in range(10):
                    f()
                pool.sync()
                e0, e1 = hip.event(), hip.event()
                hip.record(e0, st)
                for _ in range(reps):
                    f()
                hip.record(e1, st)
                pool.sync()
                us = hip.elapsed_ms(e0, e1) * 1e3 / reps
                r = res[dname][name]
                r["us"].append(round(us, 3))
                r["tflops"].append(round(work[name][0] / us / 1e6, 3))
                r["gb_per_s"].append(round(work[name][1] / us / 1e3, 2))
            pool.destroy()
        for name, r in res[dname].items():
            r["speedup_vs_8"] = [round(r["us"][0] / u, 2) for u in r["us"]]
            log("sweep", dname, name, "us", r["us"], "speedup", r["speedup_vs_8"])
    return res


def leg_mfma_probe(S, hip, torch, pool, stream, total_cus, steps=4000, reps=5):
    """What the matrix cores sustain on this chip with the conv kernel's inner-loop instruction mix
    (LDS fragment reads + MFMA 32x32x16 bf16, 8 wavefronts per CU, no global memory traffic), with
    constant and with pseudo-random operands: under dense MFMA load the shader clock settles well
    below its 2.4 GHz maximum, and lower still when the operand bits toggle."""
    out = torch.zeros(3, dtype=torch.int64, device="cuda")
    res = {}
    for name, rnd in (("constant_data", False), ("random_data", True)):
        pool.mfma_probe(0, rnd, 200, out.data_ptr())
        pool.sync()
        e0, e1 = hip.event(), hip.event()
        hip.record(e0, stream)
        for _ in range(reps):
            pool.mfma_probe(0, rnd, steps, out.data_ptr())
        hip.record(e1, stream)
        pool.sync()
        sec = hip.elapsed_ms(e0, e1) * 1e-3 / reps
        ticks, clocks, _ = (int(v) for v in out.cpu().tolist())
        mfmas_per_simd = steps * 18 * 4 * 2                       # two wavefronts per SIMD
        flops = 2.0 * 32 * 32 * 16 * steps * 18 * 4 * 8 * total_cus
        res[name] = dict(tflops=round(flops / sec / 1e12, 1), shader_ghz=round(clocks / (ticks / 100e6) / 1e9, 3),
                         mfma_pipe_busy=round(mfmas_per_simd * 32 / clocks, 3),
                         frac_of_published_peak=round(flops / sec / PEAK_BF16, 4))
        log("mfma_probe", name, json.dumps(res[name]))
    return res


def leg_load_probe(S, hip, torch, pool, stream, total_cus, iters=2048, reps=3):
    """What the load path of the convolution kernels sustains (16-byte buffer loads straight into
    LDS, 8 wavefronts per CU, 64 KiB in flight per CU): every workgroup cycles through its own region;
    the regions together fit the L2s (16 MiB), the memory-side cache (64 MiB) or neither (1 GiB)."""
    buf = torch.ones(256 << 20, dtype=torch.int32, device="cuda")  # 1 GiB
    out = torch.zeros(total_cus, dtype=torch.int32, device="cuda")
    res = {}
    for name, region in (("l2_resident_64KiB_regions", 64 << 10), ("beyond_l2_256KiB_regions", 256 << 10),
                         ("beyond_caches_4MiB_regions", 4 << 20)):
        nbytes = min(buf.numel() * 4, region * total_cus)
        pool.load_probe(0, buf.data_ptr(), nbytes, region, 64, out.data_ptr())
        pool.sync()
        e0, e1 = hip.event(), hip.event()
        hip.record(e0, stream)
        for _ in range(reps):
            pool.load_probe(0, buf.data_ptr(), nbytes, region, iters, out.data_ptr())
        hip.record(e1, stream)
        pool.sync()
        sec = hip.elapsed_ms(e0, e1) * 1e-3 / reps
        moved = float(total_cus) * iters * 65536
        assert int(out.min()) == 16384 and int(out.max()) == 16384
        res[name] = dict(tb_per_s=round(moved / sec / 1e12, 2), gb_per_s_per_cu=round(moved / sec / 1e9 / total_cus, 1))
        log("load_probe", name, json.dumps(res[name]))
    return res


def leg_membound(S, hip, torch, pool, stream, reps=100):
    """Bandwidth kernels at batch-64 sizes, bf16, on the full-GPU partition.  Each launch works on its
    own buffers out of a rotating set larger than the 256 MB last-level cache, so the bytes really
    come from and go to HBM.  GB/s = algorithmic bytes / time."""
    dt, tdt, es = S.SGPRS_BF16, torch.bfloat16, 2
    res = {}

    def timed(name, nbytes, make, run):
        sets = [make() for _ in range(max(2, int(700e6 // nbytes) + 1))]
        for k in range(min(reps, 30)):  # long enough for the chip to settle in its loaded state
            run(sets[k % len(sets)])
        pool.sync()
        e0, e1 = hip.event(), hip.event()
        hip.record(e0, stream)
        for k in range(reps):
            run(sets[k % len(sets)])
        hip.record(e1, stream)
        pool.sync()
        us = hip.elapsed_ms(e0, e1) * 1e3 / reps
        res[name] = dict(us=round(us, 2), mbytes=round(nbytes / 1e6, 1), gb_per_s=round(nbytes / us / 1e3, 1),
                         hbm_frac=round(nbytes / us / 1e3 / (PEAK_HBM / 1e9), 3), buffer_sets=len(sets))
        log("membound", name, json.dumps(res[name]))

    n = 64
    timed("maxpool3x3s2 64x(112x112x64)", (n * 112 * 112 * 64 + n * 56 * 56 * 64) * es,
          lambda: (torch.randn((n, 112, 112, 64), device="cuda").to(tdt), torch.empty((n, 56, 56, 64), dtype=tdt, device="cuda")),
          lambda b: S.sgprs_maxpool2d(dt, n, 112, 112, 64, b[0].data_ptr(), b[1].data_ptr(), pool, 0))
    sc = torch.ones(128, dtype=torch.float32, device="cuda"); sh = torch.zeros(128, dtype=torch.float32, device="cuda")
    npx = 1024 * 28 * 28
    timed("bn_relu 1024x(28x28x128)", 2 * npx * 128 * es,
          lambda: (torch.randn((npx, 128), device="cuda").to(tdt), torch.empty((npx, 128), dtype=tdt, device="cuda")),
          lambda b: S.sgprs_bn_relu(dt, npx, 128, b[0].data_ptr(), sc.data_ptr(), sh.data_ptr(), b[1].data_ptr(), pool, 0))
    cnt = 4096 * 512 * 7 * 7
    timed("add_relu 4096x(7x7x512)", 3 * cnt * es,
          lambda: (torch.randn(cnt, device="cuda").to(tdt), torch.randn(cnt, device="cuda").to(tdt), torch.empty(cnt, dtype=tdt, device="cuda")),
          lambda b: S.sgprs_add_relu(dt, cnt, b[0].data_ptr(), b[1].data_ptr(), b[2].data_ptr(), True, pool, 0))
    # avg-pool + FC at a size beyond the caches (4096 images: 205 MB of activations per call; the 1 MB of
    # weights and the pooled vectors stay in the L2) and at the headline's batch of 64 (3.2 MB: two
    # dependent launches, bound by their latency, not by bandwidth: reported as such)
    wfc = (torch.randn((1000, 512), device="cuda") * 0.05).to(tdt)
    bfc = torch.zeros(1000, dtype=torch.float32, device="cuda")
    # the average pool alone (the memory-bound half; the FC at 4096 images is a 4096 x 512 x 1000 GEMM)
    timed("global_avgpool 4096x(7x7x512)", 4096 * 49 * 512 * es + 4096 * 512 * 4,
          lambda: (torch.randn((4096, 49, 512), device="cuda").to(tdt), torch.empty((4096, 512), dtype=torch.float32, device="cuda")),
          lambda b: S.sgprs_global_avgpool(dt, 4096, 49, 512, b[0].data_ptr(), b[1].data_ptr(), pool, 0))
    for nimg in (4096, 64):
        ws = torch.empty(nimg * 512, dtype=torch.float32, device="cuda")
        nbytes = nimg * 49 * 512 * es + 1000 * 512 * es + nimg * 1000 * 4
        timed(f"avgpool_fc {nimg}x(7x7x512) -> 1000", nbytes,
              lambda: (torch.randn((nimg, 49, 512), device="cuda").to(tdt), torch.empty((nimg, 1000), dtype=torch.float32, device="cuda")),
              lambda b: S.sgprs_avgpool_fc(dt, nimg, 49, 512, 1000, b[0].data_ptr(), wfc.data_ptr(), bfc.data_ptr(), b[1].data_ptr(),
                                           ws.data_ptr(), pool, 0))
    return res


def leg_oversubscribed(S, torch, total_cus, nhwc, headline_ips, rounds=300):
    """Two bf16 instances on a pool of two partitions that BOTH span all CUs (an
    over-subscribed context pool): the tails, prologues and idle CUs of one
    instance's kernels are filled by the other's workgroups.  Measured with two
    batch-64 instances (twice the headline's work per round) and with two batch-32
    instances (the headline's 64 images per round, as two halves)."""
    import numpy as np
    from workloads import BN_EPS, make_input, make_resnet18_params
    n_p = 2
    words = S.Pool(1, total_cus).mask(0)
    pool = S.Pool(n_p, 0, masks=np.stack([words] * n_p))
    res = []
    for n in (64, 32):
        tasks, xs, lgs = [], [], []
        for i in range(n_p):
            tasks.append(S.Task(make_resnet18_params(4, 0, bf16=True), S.SGPRS_BF16, n, BN_EPS))
            xs.append(nhwc(make_input(4, i, (n, 3, 224, 224), bf16=True), torch.bfloat16))
            lgs.append(torch.empty((n, 1000), dtype=torch.float32, device="cuda"))

        def issue_all():
            for j in range(6):
                for i in range(n_p):
                    src = xs[i].data_ptr() if j == 0 else tasks[i].stage_output(j - 1)
                    dst = lgs[i].data_ptr() if j == 5 else tasks[i].stage_output(j)
                    tasks[i].stage_run(j, n, src, dst, pool, i)

        for _ in range(50):
            issue_all()
        pool.sync()
        t0 = time.perf_counter()
        for _ in range(rounds):
            issue_all()
        pool.sync()
        dt = (time.perf_counter() - t0) / rounds
        ips = n_p * n / dt
        for t in tasks:
            t.destroy()
        res.append(dict(instances=n_p, batch=n, partitions="2 x all CUs", ms_per_round=round(dt * 1e3, 4),
                        aggregate_images_per_s=round(ips, 1), vs_single_partition=round(ips / headline_ips, 3)))
    pool.destroy()
    return res


def leg_periodic(S, hip, torch, total_cus, nhwc, n_list=(128, 256, 320, 384, 448, 512, 576), levels=(1.0, 1.5, 2.0),
                 shapes=((2, 4, 2), (4, 1, 4)), fps=32.0, duration=0.5):
    """'Simulation Results' in kind: N identical periodic ResNet18 tasks (bf16, batch 1, six stages,
    deadline = period = 1/32 s, releases spread evenly over the period) under the SGPRS scheduler
    (sgprs_sched_run_periodic), at over-subscription levels 1.0 / 1.5 / 2.0 (CUs of all contexts /
    CUs of the GPU), on two pool shapes: the paper's two contexts with four lanes each (two for
    high-priority stages, two for the others), and four contexts with one lane each.  The third
    number of a shape is the run loop's limit on lanes busy at once: CU-masked streams that take
    turns on the hardware's dispatch pipes slow each other down, and with eight lanes carrying
    10-50 us stages a limit of two measured best (6.7 k FPS against 5.6 k with three, 4.6 k with
    four and 4.4 k with none).  Stage WCETs are measured first, on one lane with the rest of the GPU idle
    (the paper's offline phase).  Reported: total FPS and deadline miss rate against the number of
    tasks, and the pivot point (the largest N without a miss)."""
    from workloads import BN_EPS, make_input, make_resnet18_params
    period = 1.0 / fps
    n_max = max(n_list)
    params = make_resnet18_params(3, 0, bf16=True)
    tasks = [S.Task(params, S.SGPRS_BF16, 1, BN_EPS) for _ in range(n_max)]
    x = nhwc(make_input(3, 0, (1, 3, 224, 224), bf16=True), torch.bfloat16)
    lgs = [torch.empty((1, 1000), dtype=torch.float32, device="cuda") for _ in range(n_max)]
    out = []
    for (n_ctx, lanes, max_busy) in shapes:
        res = {}
        for level in levels:
            cus = min(total_cus, int(round(total_cus / n_ctx * level)) // 8 * 8)
            base = S.Pool(n_ctx, cus, flags=S.SGPRS_POOL_OVERSUBSCRIBE if n_ctx * cus > total_cus else 0)
            masks = np.stack([base.mask(c) for c in range(n_ctx) for _ in range(lanes)])
            base.destroy()
            pool = S.Pool(n_ctx * lanes, 0, masks=masks)
            # offline phase: per-stage WCET on one lane, alone
            stream = pool.stream(0)
            ev = [hip.event() for _ in range(7)]
            per = [[] for _ in range(6)]
            for it in range(40):
                for j in range(6):
                    hip.record(ev[j], stream)
                    src = x.data_ptr() if j == 0 else tasks[0].stage_output(j - 1)
                    dst = lgs[0].data_ptr() if j == 5 else tasks[0].stage_output(j)
                    tasks[0].stage_run(j, 1, src, dst, pool, 0)
                hip.record(ev[6], stream)
                pool.sync()
                if it >= 10:
                    for j in range(6):
                        per[j].append(hip.elapsed_ms(ev[j], ev[j + 1]) * 1e-3)
            wcet = [max(p) for p in per]
            rows, pivot = [], 0
            for n in n_list:
                sch = S.Sched(n_ctx, lanes)
                sch.set_max_busy(max_busy)
                for _ in range(n):
                    sch.add_task(wcet, period, period)
                rep = sch.run_periodic(pool, tasks[:n], [x.data_ptr()] * n, [l.data_ptr() for l in lgs[:n]], 1, duration,
                                       offsets=[i * period / n for i in range(n)])
                pool.sync()
                sch.destroy()
                rows.append(dict(n_tasks=n, total_fps=round(rep["fps"], 1), dmr=round(rep["dmr"], 4), dropped=rep["dropped"],
                                 jobs_missed=rep["jobs_missed"], releases=rep["releases"],
                                 mean_response_ms=round(rep["mean_response_s"] * 1e3, 3),
                                 max_response_ms=round(rep["max_response_s"] * 1e3, 3)))
                if all(r["dmr"] == 0.0 for r in rows):
                    pivot = n
                log("periodic", f"{n_ctx}x{lanes} os={level}", json.dumps(rows[-1]))
            res[f"SGPRS_{level}"] = dict(cus_per_context=cus, stage_wcet_us=[round(w * 1e6, 1) for w in wcet], pivot_tasks=pivot,
                                         points=rows)
            pool.destroy()
        out.append(dict(contexts=n_ctx, lanes_per_context=lanes, max_busy_lanes=max_busy, results=res))
    for t in tasks:
        t.destroy()
    return dict(task_fps=fps, duration_s=duration, pools=out)


def leg_pool_scaling(S, torch, total_cus, nhwc, instances=8, rounds=150, partitions=(1, 2, 3, 4, 8)):
    """Eight bf16 batch-1 instances spread round-robin over pools of 1, 2, 3, 4 and 8 equal
    partitions (the paper's question: how does throughput grow with the number of contexts?).
    Every instance is issued with sgprs_task_run from one host thread, i.e. replayed as a HIP
    graph after its second run: one host call per inference."""
    from workloads import BN_EPS, make_input, make_resnet18_params
    tasks, xs, lgs = [], [], []
    for i in range(instances):
        tasks.append(S.Task(make_resnet18_params(3, i, bf16=True), S.SGPRS_BF16, 1, BN_EPS))
        xs.append(nhwc(make_input(3, i, (1, 3, 224, 224), bf16=True), torch.bfloat16))
        lgs.append(torch.empty((1, 1000), dtype=torch.float32, device="cuda"))
    res = []
    for n_p in partitions:
        cus = total_cus // n_p // 8 * 8
        pool = S.Pool(n_p, cus)

        def issue():
            for i in range(instances):
                tasks[i].run(1, xs[i].data_ptr(), lgs[i].data_ptr(), pool, i % n_p)

        for _ in range(20):
            issue()
        pool.sync()
        t0 = time.perf_counter()
        for _ in range(rounds):
            issue()
        t1 = time.perf_counter()
        pool.sync()
        t2 = time.perf_counter()
        res.append(dict(partitions=n_p, partition_cus=cus, images_per_s=round(instances * rounds / (t2 - t0), 1),
                        us_per_round=round((t2 - t0) / rounds * 1e6, 1), host_issue_us_per_round=round((t1 - t0) / rounds * 1e6, 1)))
        log("pool_scaling", json.dumps(res[-1]))
        pool.destroy()
    for t in tasks:
        t.destroy()
    return res


def leg_multi_tenant(S, hip, torch, total_cus, nhwc, n_p=8, rounds=100):
    """Eight bf16 instances, each pinned to its own 32-CU partition (a static
    instance->partition assignment, i.e. pure spatial partitioning), stages of
    all instances issued round-robin from one host thread."""
    from workloads import BN_EPS, make_input, make_resnet18_params
    pool = S.Pool(n_p, total_cus // n_p)
    tasks, xs, lgs = [], [], []
    for i in range(n_p):
        tasks.append(S.Task(make_resnet18_params(3, i, bf16=True), S.SGPRS_BF16, 1, BN_EPS))
        xs.append(nhwc(make_input(3, i, (1, 3, 224, 224), bf16=True), torch.bfloat16))
        lgs.append(torch.empty((1, 1000), dtype=torch.float32, device="cuda"))

    def issue_all(ev=None):
        for j in range(6):
            for i in range(n_p):
                if ev is not None:
                    hip.record(ev[i][j], pool.stream(i))
                src = xs[i].data_ptr() if j == 0 else tasks[i].stage_output(j - 1)
                dst = lgs[i].data_ptr() if j == 5 else tasks[i].stage_output(j)
                tasks[i].stage_run(j, 1, src, dst, pool, i)
        if ev is not None:
            for i in range(n_p):
                hip.record(ev[i][6], pool.stream(i))

    for _ in range(5):
        issue_all()
    pool.sync()
    ev = [[hip.event() for _ in range(7)] for _ in range(n_p)]
    lat = [[[] for _ in range(6)] for _ in range(n_p)]
    for _ in range(10):
        issue_all(ev)
        pool.sync()
        for i in range(n_p):
            for j in range(6):
                lat[i][j].append(hip.elapsed_ms(ev[i][j], ev[i][j + 1]))
    t0 = time.perf_counter()
    for _ in range(rounds):
        issue_all()
    pool.sync()
    dt = time.perf_counter() - t0
    conc = n_p * rounds / dt
    # the same eight tasks on the same eight partitions through the library's static executor, which
    # keeps at most four partitions busy at once (and without that gate, for comparison)
    ptrs = ([x.data_ptr() for x in xs], [l.data_ptr() for l in lgs])
    pool.run_static(tasks, ptrs[0], ptrs[1], 1, list(range(n_p)), 20, 4)
    gated = n_p * rounds / pool.run_static(tasks, ptrs[0], ptrs[1], 1, list(range(n_p)), rounds, 4)
    ungated = n_p * rounds / pool.run_static(tasks, ptrs[0], ptrs[1], 1, list(range(n_p)), rounds, 0)
    # Where the collapse sets in: the same eight tasks pinned to the first k of the eight partitions
    # (the other queues exist but stay idle), no gate; and all eight partitions with the gate at m.
    busy_sweep = []
    for k in range(1, n_p + 1):
        ips = n_p * rounds / pool.run_static(tasks, ptrs[0], ptrs[1], 1, [i % k for i in range(n_p)], rounds, 0)
        busy_sweep.append(dict(partitions_in_use=k, images_per_s=round(ips, 1)))
    gate_sweep = []
    for m in range(1, n_p + 1):
        ips = n_p * rounds / pool.run_static(tasks, ptrs[0], ptrs[1], 1, list(range(n_p)), rounds, m)
        gate_sweep.append(dict(max_busy=m, images_per_s=round(ips, 1)))
    # context: the same eight images back to back on one full-GPU partition
    full = S.Pool(1, total_cus)
    t0 = time.perf_counter()
    for _ in range(rounds):
        for i in range(n_p):
            tasks[i].run(1, xs[i].data_ptr(), lgs[i].data_ptr(), full, 0)
    full.sync()
    serial = n_p * rounds / (time.perf_counter() - t0)
    out = dict(instances=n_p, partition_cus=total_cus // n_p, aggregate_images_per_s=round(conc, 1),
               run_static_max_4_busy_images_per_s=round(gated, 1), run_static_no_gate_images_per_s=round(ungated, 1),
               serial_full_gpu_images_per_s=round(serial, 1), issue="one host thread, round-robin over instances",
               no_gate_by_partitions_in_use=busy_sweep, all_partitions_by_gate=gate_sweep,
               stage_latency_ms_median=[[round(statistics.median(l), 4) for l in inst] for inst in lat])
    log("multi_tenant", json.dumps({k: v for k, v in out.items() if k != "stage_latency_ms_median"}))
    for t in tasks:
        t.destroy()
    full.destroy(); pool.destroy()
    return out


if __name__ == "__main__":
    main()
