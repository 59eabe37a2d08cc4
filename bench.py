#!/usr/bin/env python3
"""Benchmark of the fused-DAG hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4|cfg3|cfg2|fam:<family>[x<members>][@<batch>]] [--swap-requests R]

A step is one pass of the whole launch schedule (input staging, every member's convolutions,
pooling, FC) over one synthetic batch that is already resident in HBM.  Prints ONE JSON line:
fused-DAG images/s (each image goes through every member), the roofline of the dominant kernel
measured with HIP events on the launch stream, the CPU oracle timed on this machine's cores, and the
fused-vs-separate throughput, memory and swap-latency comparison.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOADS = {
    "cfg2": dict(desc="2x ResNet-18 fused, bf16, batch 1x3x224x224", fams=["resnet18"] * 2, batch=1),
    "cfg3": dict(desc="ResNet-50 + MobileNetV2 + VGG-16 fused, bf16, batch 8x3x224x224", fams=["resnet50", "mobilenetv2", "vgg16"], batch=8),
    "cfg4": dict(desc="8x ResNet-50 fused (grouped conv GEMMs), bf16, batch 32x3x224x224", fams=["resnet50"] * 8, batch=32),
}
# Members that keep fp32 activations: with synthetic He-normal weights MobileNetV2 amplifies bf16 storage
# rounding about twentyfold (the CPU oracle's own bf16-storage mode sits 2e-2 from its fp32 mode), so bf16
# storage cannot meet the 1e-2 bar; its convolutions still run on the bf16 matrix cores (hi/lo split).
# MobileNetV3-Large behaves the same way (the oracle's bf16-storage mode sits 2e-2 ... 9e-2 from its fp32 mode).
WIDE = {"mobilenetv2", "mobilenet_v3_large"}
PEAK_MFMA_BF16 = 2500.0  # TFLOP/s dense
PEAK_HBM = 8000.0        # GB/s


def workload(name, families):
    """A named configuration, or `fam:<family>[x<members>][@<batch>]`: identical members of one family."""
    if name in WORKLOADS:
        return WORKLOADS[name]
    m = re.fullmatch(r"fam:([a-z0-9_]+?)(?:x(\d+))?(?:@(\d+))?", name)
    if not m or m.group(1) not in families:
        sys.exit("unknown workload %r: one of %s or fam:<family>[x<members>][@<batch>] with a family of "
                 "workloads/zoo.py" % (name, ", ".join(sorted(WORKLOADS))))
    fam, n, b = m.group(1), int(m.group(2) or 1), int(m.group(3) or 32)
    if not (1 <= n <= 64 and 1 <= b <= 1024):
        sys.exit("fam: workloads take 1..64 members and a batch of 1..1024")
    shape = families[fam]()   # the family's own input size (299 for Inception v3, 384 for EfficientNetV2-S, ...)
    return dict(desc="%dx %s fused, bf16, batch %dx%dx%dx%d" % (n, fam, b, shape.in_c, shape.in_h, shape.in_w), fams=[fam] * n, batch=b)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg4",
                    help="cfg4 | cfg3 | cfg2, or fam:<family>[x<members>][@<batch>] for identical members of one "
                         "family of workloads/zoo.py (e.g. fam:densenet121x4@32)")
    ap.add_argument("--swap-requests", type=int, default=1000, help="requests of the swap-churn stream that are replayed (the stream has 1000)")
    ap.add_argument("--launch-table", default=None, metavar="FILE",
                    help="also write the per-launch roofline table (every launch beside its own roofline ceiling) as markdown")
    ap.add_argument("--member-chunks", type=int, default=2,
                    help="fi_build_opts.member_chunks of the timed DAG: the early, activation-heavy levels run for one chunk of a lane's "
                         "members after the other (smaller activation arena, more launches); 0 = every level for all members together")
    ap.add_argument("--no-extras", action="store_true", help="skip separate-DAG, swap and CPU legs")
    ap.add_argument("--serial-lanes", action="store_true",
                    help="issue every launch on the caller's stream (no concurrent lanes): the condition the per-kernel "
                         "roofline is measured in, for profiler runs that should show the same durations")
    ap.add_argument("--separate-stem", action="store_true",
                    help="fi_build_opts.separate_stem of the timed DAG: the first convolution with the general kernel and the max-pool "
                         "behind it as a launch of its own (the same bits; for an A/B timing of the stem launch on one box)")
    ap.add_argument("--probe-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a kernel of known traffic, to calibrate rocprofv3 counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py runs on ONE GPU (member models are independent, so more GPUs would each take "
              "a subset of members with its own arena and schedule, no collective); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2410_21120_amd as fi
    from workloads import gen, zoo

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    fi.lib()
    wl = workload(a.workload, zoo.FAMILIES)
    B = wl["batch"]
    stream = torch.cuda.current_stream().cuda_stream
    alloc = fi.TorchAllocators("cuda:0")

    members = []
    for i, fam in enumerate(wl["fams"]):
        m = zoo.FAMILIES[fam]()
        members.append((m, gen.make_blob(m, 1000 + i), "f32" if fam in WIDE else None))

    def make_dag(mem, **kw):
        specs, keep = [], []
        for m, blob, act in mem:
            s, k = fi.make_spec(m, blob.ctypes.data, blob.nbytes, act_dtype=act)
            specs.append(s)
            keep.append((k, blob))
        return fi.Dag(specs, B, alloc, keepalive=keep, **kw)

    m0 = members[0][0]
    # one input feeds every member: they must agree on its shape, and the buffer handed over must hold it
    assert all((m.in_c, m.in_h, m.in_w) == (m0.in_c, m0.in_h, m0.in_w) for m, _, _ in members), "members disagree on the input shape"
    x = gen.make_input(7, B, m0.in_c, m0.in_h, m0.in_w, "normal", "bf16")
    xin = torch.from_numpy(gen.to_nhwc_storage(x, "bf16").view(np.int16)).cuda()
    assert xin.numel() == B * m0.in_h * m0.in_w * m0.in_c
    check_buffers = lambda d: (xin.numel() * xin.element_size() == B * d.query().input_image_bytes and
                               all(o.numel() * 4 == B * mi.output_row_bytes for mi, o in zip(d.members(), outs)))
    outs = [torch.zeros((B, m.layers[-1].cout), dtype=torch.float32, device="cuda:0") for m, _, _ in members]
    optr = [o.data_ptr() for o in outs]

    if a.probe_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        src.fill_(1)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- fused DAG: timed region ------------------------------------------------------------
    t0 = time.perf_counter()
    dag = make_dag(members, serial_lanes=a.serial_lanes, member_chunks=a.member_chunks, separate_stem=a.separate_stem)
    t_build = time.perf_counter() - t0
    torch.cuda.empty_cache()
    free0 = torch.cuda.mem_get_info()[0]
    t0 = time.perf_counter()
    dag.load(stream)
    torch.cuda.synchronize()
    t_load = time.perf_counter() - t0
    hbm_delta = free0 - torch.cuda.mem_get_info()[0]   # what the device reports (allocator granularity included)
    q = dag.query()
    assert check_buffers(dag), "input / output buffers do not have the sizes the handle reads and writes"
    for _ in range(a.warmup):
        dag.run(xin.data_ptr(), B, optr, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        dag.run(xin.data_ptr(), B, optr, stream)
    torch.cuda.synchronize()
    fused_ms = (time.perf_counter() - t0) * 1e3 / a.steps
    # per-step distribution: an event pair on the caller's stream around every step (lanes fork from
    # and join that stream, so the pair brackets the whole schedule)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(a.steps)]
    for e0, e1 in evs:
        e0.record()
        dag.run(xin.data_ptr(), B, optr, stream)
        e1.record()
    torch.cuda.synchronize()
    step_ms = np.array([e0.elapsed_time(e1) for e0, e1 in evs])

    # ---- per-launch HIP-event timing on the streams the launches go to -------------------------
    # fi_timeline issues the step exactly as fi_run does (lanes concurrent) with an event after every
    # launch on its own stream.  Launch i spans [end of the previous launch on that stream, its own end].
    # Launches of one kernel on different lanes overlap, so a kernel's rate is its algorithmic work
    # divided by the time during which at least one of its launches was running (the union of its
    # intervals): never more than the chip delivered, and an underestimate whenever a different
    # kernel shared the chip during that time.
    launches = dag.launches()
    prof_iters = max(3, min(10, a.steps))
    per_kernel = {}
    def kname(L):   # one name per kernel template: the chains of two and of three are one kernel (chain_mfma_kernel)
        n = L.name.decode()
        return "conv_chain" if n.startswith("conv_chain") else n
    for L in launches:
        k = per_kernel.setdefault(kname(L), dict(launches=0, ms=0.0, busy_ms=0.0, flops=0.0, bytes=0.0))
        k["launches"] += 1
        k["flops"] += 2.0 * L.macs_per_image * B
        k["bytes"] += float(L.bytes_per_image) * B + L.weight_bytes
    per_launch_span = [0.0] * len(launches)
    for _ in range(prof_iters):
        tb, te = dag.timeline(xin.data_ptr(), B, optr, stream)
        spans = {}
        for i, (L, b, e) in enumerate(zip(launches, tb, te)):
            per_launch_span[i] += (e - b) / prof_iters
            per_kernel[kname(L)]["ms"] += (e - b) / prof_iters
            spans.setdefault(kname(L), []).append((b, e))
        for n, iv in spans.items():
            iv.sort()
            busy, hi = 0.0, -1.0
            for b, e in iv:
                if e > hi:
                    busy += e - max(b, hi)
                    hi = e
            per_kernel[n]["busy_ms"] += busy / prof_iters
    dom_name = max((n for n in per_kernel if n.startswith("conv_")), key=lambda n: per_kernel[n]["busy_ms"],
                   default=max(per_kernel, key=lambda n: per_kernel[n]["busy_ms"]))
    dom = per_kernel[dom_name]
    mfma = [v for n, v in per_kernel.items() if n.startswith("conv_")]
    mfma_flops = sum(v["flops"] for v in mfma)
    # the roofline that binds this kernel's algorithmic work: matrix cores or HBM
    t_mfma = dom["flops"] / (PEAK_MFMA_BF16 * 1e12)
    t_hbm = dom["bytes"] / (PEAK_HBM * 1e9)
    if t_mfma >= t_hbm:
        achieved = dom["flops"] / (dom["busy_ms"] * 1e-3) / 1e12
        roofline = dict(bound="mfma", achieved=achieved, peak=PEAK_MFMA_BF16, unit="TFLOP/s", frac=achieved / PEAK_MFMA_BF16)
    else:
        achieved = dom["bytes"] / (dom["busy_ms"] * 1e-3) / 1e9
        roofline = dict(bound="hbm", achieved=achieved, peak=PEAK_HBM, unit="GB/s", frac=achieved / PEAK_HBM)
    roofline.update(kernel=dom_name, launches_per_step=dom["launches"], avg_launch_ms=dom["ms"] / dom["launches"],
                    busy_ms_per_step=dom["busy_ms"], concurrent_lanes=q.n_lanes,
                    flops_per_step=dom["flops"], bytes_per_step=dom["bytes"],
                    timing="HIP events after every launch on the stream it is issued to, in the schedule the timed region runs; "
                           "achieved = algorithmic work of all launches of the kernel / time at least one of them was running",
                    algorithmic_bytes_per_launch=dom["bytes"] / dom["launches"])
    tr = counter_traffic(dom_name, a.workload)
    roofline["traffic"] = tr["bytes_per_launch"] if tr else None   # HBM bytes per launch from the counters
    roofline["traffic_detail"] = tr
    # ---- every launch beside its own roofline ceiling ------------------------------------------
    # alone_ms: the launch with the chip to itself (fi_profile: one stream, an event between launches).
    # span_ms: the launch in the schedule the timed region runs (its lane's stream; other lanes share the chip).
    alone = np.zeros(len(launches))
    for _ in range(prof_iters):
        alone += np.array(dag.profile(xin.data_ptr(), B, optr, stream)) / prof_iters
    nodes = dag.nodes()
    per_launch = []
    for i, L in enumerate(launches):
        flops = 2.0 * L.macs_per_image * B
        nbytes = float(L.bytes_per_image) * B + L.weight_bytes
        t_m, t_h = flops / (PEAK_MFMA_BF16 * 1e12) * 1e3, nbytes / (PEAK_HBM * 1e9) * 1e3   # ms at either roof
        row = dict(launch=i, level=L.level, lane=L.lane, kernel=L.name.decode(), problems=L.n_problems,
                   gflop=round(flops / 1e9, 2), mbytes=round(nbytes / 1e6, 2), flop_per_byte=round(flops / max(nbytes, 1.0), 1),
                   bound="mfma" if t_m >= t_h else "hbm", roof_ms=round(max(t_m, t_h), 5),
                   alone_ms=round(float(alone[i]), 5), span_ms=round(per_launch_span[i], 5),
                   frac_alone=round(max(t_m, t_h) / max(float(alone[i]), 1e-9), 3))
        if L.first_node >= 0:
            nd = nodes[L.first_node]
            row["out"] = "%dx%dx%d" % (nd.out_h, nd.out_w, nd.out_c)
        per_launch.append(row)
    kernels = {n: dict(launches=v["launches"], ms=round(v["ms"], 4), busy_ms=round(v["busy_ms"], 4),
                       tflops=round(v["flops"] / (v["busy_ms"] * 1e-3) / 1e12, 2) if v["flops"] else 0.0,
                       gbps=round(v["bytes"] / (v["busy_ms"] * 1e-3) / 1e9, 1)) for n, v in per_kernel.items()}
    res = {
        "metric": "fused-DAG images/sec + MFMA util; peak HBM and swap latency vs per-model",
        "value": B / (fused_ms * 1e-3), "unit": "images/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": fused_ms, "ms_per_step_median": float(np.median(step_ms)), "ms_per_step_p95": float(np.percentile(step_ms, 95)),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl["desc"], "members": len(members), "batch": B,
                   "model_inferences_per_s": B * len(members) / (fused_ms * 1e-3)},
        "roofline": roofline,
        # every dense (matrix-core) FLOP of the step over the whole step time
        "mfma_util_all_dense": mfma_flops / (fused_ms * 1e-3) / 1e12 / PEAK_MFMA_BF16,
        "kernels": kernels,
        # sum over launches of each launch's own roofline floor (no reuse between launches), and what the launches take alone
        "roofline_floor_ms": round(sum(r["roof_ms"] for r in per_launch), 4),
        "sum_alone_ms": round(sum(r["alone_ms"] for r in per_launch), 4),
        "per_launch": per_launch,
        # the paper's own figures, for context only: another machine, framework-level, another metric
        "paper_context": {"speedup_up_to_pct": 14.0, "memory_reduction_up_to_pct": 17.0,
                          "hardware": "AMD Threadripper 5955WX + NVIDIA RTX 4090",
                          "note": "end-to-end time and peak memory of load + 100 iterations per model of pretrained torchvision models, fused "
                                  "against the same models initialised and run one by one in one process; not comparable with the figures here"},
        "dag": dict(nodes=q.n_nodes, levels=q.n_levels, launches=q.n_launches, device_allocs=q.n_device_allocs,
                    h2d_copies=q.n_h2d_copies, arena_bytes=q.arena_bytes, act_bytes=q.act_bytes,
                    lanes=q.n_lanes, device_bytes=q.device_bytes, device_bytes_mem_get_info=hbm_delta, build_ms=t_build * 1e3, load_ms=t_load * 1e3,
                    load_gbps=q.arena_bytes / t_load / 1e9),
    }
    dag.unload()
    dag.destroy()
    if a.launch_table:
        write_launch_table(a.launch_table, wl["desc"], res, " ".join(sys.argv))

    if not a.no_extras:
        # ---- the same members as n single-model DAGs ("without fusion") -----------------------
        singles = [make_dag([mb]) for mb in members]
        torch.cuda.empty_cache()
        free0 = torch.cuda.mem_get_info()[0]
        for d in singles:
            d.load(stream)
        torch.cuda.synchronize()
        sep_delta = free0 - torch.cuda.mem_get_info()[0]
        sq = [d.query() for d in singles]

        def run_sep():
            for d, p in zip(singles, optr):
                d.run(xin.data_ptr(), B, [p], stream)
        for _ in range(a.warmup):
            run_sep()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            run_sep()
        torch.cuda.synchronize()
        sep_ms = (time.perf_counter() - t0) * 1e3 / a.steps
        # second variant: every single-model handle on a stream of its own
        side = [torch.cuda.Stream() for _ in singles]

        def run_sep_streams():
            for d, p, st in zip(singles, optr, side):
                d.run(xin.data_ptr(), B, [p], st.cuda_stream)
        for _ in range(a.warmup):
            run_sep_streams()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            run_sep_streams()
        torch.cuda.synchronize()
        sep_streams_ms = (time.perf_counter() - t0) * 1e3 / a.steps
        res["fused_vs_separate"] = dict(
            fused_ms=fused_ms, separate_ms=sep_ms, speedup=sep_ms / fused_ms,
            separate_on_own_streams_ms=sep_streams_ms, speedup_vs_own_streams=sep_streams_ms / fused_ms,
            hbm_mem_get_info_fused=hbm_delta, hbm_mem_get_info_separate_resident=sep_delta,
            launches_fused=q.n_launches, launches_separate=sum(s.n_launches for s in sq),
            hbm_bytes_fused=q.device_bytes, hbm_bytes_separate_resident=sum(s.device_bytes for s in sq),
            hbm_bytes_separate_sequential=max(s.device_bytes for s in sq),
            device_allocs_fused=1, device_allocs_separate=len(singles))
        for d in singles:
            d.unload()
            d.destroy()
        res["swap"] = swap_churn(fi, torch, gen, zoo, alloc, stream, a.swap_requests)
        sw = res["swap"]
        # "fused" and "per_model" both load with FI_LOAD_AUTO (a handle that is loaded once copies its members straight out of
        # the repository's pinned blobs; the literal one-copy mode, also reported, pays a host gather per request first)
        sw["fused_vs_per_model"] = {k: sw["fused"][k] / sw["per_model"][k] for k in ("p50_ms", "p95_ms", "p99_ms")}
        res["serving"] = serving(fi, torch, gen, zoo, alloc, stream)
        res["cpu_baseline"] = cpu_baseline(members[0], x, len(members))
    print(json.dumps(res))


# HBM traffic of the dominant kernel from rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE; KiB per dispatch,
# summed over the kernel's launches of one step and scaled by what the same counters read for a
# 1 GiB device-to-device copy).  The figures belong to one exact set of sources: when any of them
# has changed since the counters were taken the entry no longer applies and traffic is null.
COUNTERS = {
    "sources_sha256": "9b606115b84689c62433e6363bdfe3f1430ba51e1bd7c0343ffe29c13a4932da",
    "workload": "cfg4",
    "fetch_scale": 2.0, "write_scale": 1.0,
    "kernels": {   # kernel name -> launches and KiB per step
        "conv_chain": {"launches_per_step": 20, "fetch_kib_per_step": 1454594.1, "write_kib_per_step": 2579447.5},
        "conv_mfma_128x128": {"launches_per_step": 38, "fetch_kib_per_step": 1098184.7, "write_kib_per_step": 1618214.0},
        "conv_mfma_128x64": {"launches_per_step": 4, "fetch_kib_per_step": 50694.5, "write_kib_per_step": 100352.0},
        "conv_mfma_256x128": {"launches_per_step": 24, "fetch_kib_per_step": 613750.8, "write_kib_per_step": 376320.0},
    },
}


def sources_sha256():
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2410_21120_amd", "csrc")
    for f in ("fi_internal.h", "fi_device.h", "fi_plan.cpp", "fi_api.cpp", "fi_kernels.hip", "fi_chain.hip", "fi_stem.hip"):
        with open(os.path.join(csrc, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def counter_traffic(kernel, workload):
    c = COUNTERS
    k = c["kernels"].get(kernel)
    if not c["sources_sha256"] or k is None or c["workload"] != workload or c["sources_sha256"] != sources_sha256():
        return None
    n = k["launches_per_step"]
    fetch, write = k["fetch_kib_per_step"] * c["fetch_scale"] * 1024.0 / n, k["write_kib_per_step"] * c["write_scale"] * 1024.0 / n
    return dict(bytes_per_launch=fetch + write, fetch_bytes_per_launch=fetch, write_bytes_per_launch=write,
                source="a stored rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of these exact sources (not measured in this run), "
                       "scaled by a 1 GiB copy probe")


def write_launch_table(path, desc, res, cmd):
    """Markdown table: every launch of the step beside the roofline that bounds it."""
    rows = res["per_launch"]
    with open(path, "w") as fh:
        fh.write("# Per-launch roofline table: %s\n\n" % desc)
        fh.write("Command: `python %s`\n\n" % cmd)
        fh.write("Each launch's algorithmic work (flops; input + output + residual activations and weights once) against the\n"
                 "roof that binds it (2.5 PFLOP/s dense bf16 MFMA, 8 TB/s HBM).  `alone`: the launch with the chip to itself\n"
                 "(one stream, HIP events between launches); `span`: in the schedule the timed region runs (lanes concurrent).\n"
                 "`frac` = roof time / alone time.\n\n")
        fh.write("step %.3f ms; sum of per-launch roofline floors %.3f ms; sum of launches alone %.3f ms; dense flops over the step: %.1f %% of the MFMA peak\n\n"
                 % (res["ms_per_step"], res["roofline_floor_ms"], res["sum_alone_ms"], 100 * res["mfma_util_all_dense"]))
        fh.write("| # | level | lane | kernel | n | out (HxWxC) | GFLOP | MB | flop/B | bound | roof ms | alone ms | span ms | frac |\n")
        fh.write("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|\n")
        for r in rows:
            fh.write("| %d | %d | %d | %s | %d | %s | %.1f | %.1f | %.0f | %s | %.4f | %.4f | %.4f | %.2f |\n" % (
                r["launch"], r["level"], r["lane"], r["kernel"], r["problems"], r.get("out", "-"), r["gflop"], r["mbytes"], r["flop_per_byte"],
                r["bound"], r["roof_ms"], r["alone_ms"], r["span_ms"], r["frac_alone"]))


def serving(fi, torch, gen, zoo, alloc, stream, seconds=1.0):
    """Request aggregation (Section IV, Manager): single-image requests for four resident models arrive as a
    seeded Poisson stream; the library's server gathers, per model, what arrived while the device was busy into
    the next pass of the model's lane.  Open loop at several rates, against the capacity of serving every request in
    a pass of its own, and against four single-model handles with a server each."""
    import numpy as np
    fams = ["resnet18", "resnet50", "mobilenetv2", "vgg16"]
    B = 8
    specs, keep = [], []
    for i, fam in enumerate(fams):
        m = zoo.FAMILIES[fam]()
        blob = gen.make_blob(m, 1000 + i)
        sp, k = fi.make_spec(m, blob.ctypes.data, blob.nbytes, act_dtype="f32" if fam in WIDE else None)
        specs.append(sp)
        keep.append((k, blob))
    dag = fi.Dag(specs, B, alloc, keepalive=keep, per_member_inputs=True)
    dag.load(stream)
    imgs = [torch.from_numpy(gen.to_nhwc_storage(gen.make_input(70 + j, 1, 3, 224, 224, "normal", "bf16"), "bf16").view(np.int16)).cuda() for j in range(4)]
    n = len(fams)
    one = torch.zeros((1, 1000), dtype=torch.float32, device="cuda:0")
    torch.cuda.synchronize()
    # capacity without aggregation: every request is a pass of its own (one member, one image)
    alone_ms = []
    for m in range(n):
        ins = [imgs[0].data_ptr() if k == m else 0 for k in range(n)]
        outs = [one.data_ptr() if k == m else 0 for k in range(n)]
        nb = [1 if k == m else 0 for k in range(n)]
        for _ in range(3):
            dag.run_batches(ins, nb, outs, stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(20):
            dag.run_batches(ins, nb, outs, stream)
        torch.cuda.synchronize()
        alone_ms.append((time.perf_counter() - t0) * 1e3 / 20)
    out = dict(models=fams, max_batch=B, one_request_per_pass_ms=[round(v, 4) for v in alone_ms],
               one_request_per_pass_capacity_rps=1e3 / (sum(alone_ms) / n), rates=[])
    rng = np.random.default_rng(2024)
    for rate in (1000.0, 4000.0, 16000.0, 32000.0):
        n_req = int(rate * seconds)
        gaps = rng.exponential(1.0 / rate, n_req)
        who = rng.integers(0, n, n_req)
        outs = torch.zeros((n_req, 1000), dtype=torch.float32, device="cuda:0")
        base, row = outs.data_ptr(), 4000
        torch.cuda.synchronize()
        srv = fi.Server(dag)
        tickets = []
        t0 = time.perf_counter()
        due = 0.0
        for r in range(n_req):
            due += gaps[r]
            while time.perf_counter() - t0 < due:   # open loop: arrivals do not wait for the server
                pass
            tickets.append(srv.submit(int(who[r]), imgs[r & 3].data_ptr(), base + r * row))
        t_sub = time.perf_counter() - t0
        srv.wait(tickets[-1])
        for t in tickets[-64:]:
            srv.wait(t)
        t_all = time.perf_counter() - t0
        st = srv.stats()
        srv.stop()
        out["rates"].append(dict(offered_rps=rate, submitted_rps=n_req / t_sub, served_rps=n_req / t_all, requests=n_req, passes=int(st.passes),
                                 mean_images_per_pass=st.mean_images_per_pass, max_images_per_pass=int(st.max_images_per_pass),
                                 mean_latency_ms=st.mean_latency_ms, max_latency_ms=st.max_latency_ms, lanes_busy=st.busy_ms / (t_all * 1e3)))
    dag.unload()
    dag.destroy()
    # the same stream against four single-model handles, each behind a server (worker thread and stream) of its own
    singles = []
    for sp, kp in zip(specs, keep):
        d1 = fi.Dag([sp], B, alloc, keepalive=[kp], per_member_inputs=True)
        d1.load(stream)
        singles.append(d1)
    torch.cuda.synchronize()
    rate = 32000.0
    n_req = int(rate * seconds)
    rng = np.random.default_rng(2024)
    for earlier in (1000.0, 4000.0, 16000.0):   # skip the draws of the loop above: the same arrivals as its 32 k/s run (beyond capacity: served_rps is the capacity)
        rng.exponential(1.0, int(earlier * seconds)); rng.integers(0, n, int(earlier * seconds))
    gaps = rng.exponential(1.0 / rate, n_req)
    who = rng.integers(0, n, n_req)
    outs = torch.zeros((n_req, 1000), dtype=torch.float32, device="cuda:0")
    base, row = outs.data_ptr(), 4000
    torch.cuda.synchronize()
    servers = [fi.Server(d1) for d1 in singles]
    tickets = []
    t0 = time.perf_counter()
    due = 0.0
    for r in range(n_req):
        due += gaps[r]
        while time.perf_counter() - t0 < due:
            pass
        m = int(who[r])
        tickets.append((m, servers[m].submit(0, imgs[r & 3].data_ptr(), base + r * row)))
    t_sub = time.perf_counter() - t0
    for m, t in tickets[-256:]:
        servers[m].wait(t)
    t_all = time.perf_counter() - t0
    sts = [sv.stats() for sv in servers]
    for sv in servers:
        sv.stop()
    for d1 in singles:
        d1.unload()
        d1.destroy()
    served = sum(int(st.requests) for st in sts)
    out["per_model_servers"] = dict(offered_rps=rate, submitted_rps=n_req / t_sub, served_rps=n_req / t_all, requests=served,
                                    passes=[int(st.passes) for st in sts], mean_images_per_pass=[st.mean_images_per_pass for st in sts],
                                    mean_latency_ms=sum(st.mean_latency_ms * st.requests for st in sts) / max(served, 1),
                                    max_latency_ms=max(st.max_latency_ms for st in sts))
    return out


def swap_churn(fi, torch, gen, zoo, alloc, stream, n_req):
    """Configuration 5: pool of 16 packed models in pinned memory; per request build, load, run, unload a
    4-member DAG (fused) versus four single-member DAGs (per-model).  Closed loop over the seeded stream."""
    import numpy as np
    fams = ["resnet18", "resnet50", "mobilenetv2", "vgg16"]
    pool = []
    for i in range(16):
        fam = fams[i // 4]
        m = zoo.FAMILIES[fam]()
        blob = gen.make_blob(m, 1000 + i)
        act = "f32" if fam in WIDE else None
        spec, keep = fi.make_spec(m, blob.ctypes.data, blob.nbytes, act_dtype=act)
        n = fi.fi_model_packed_size(spec)
        packed = torch.empty(n, dtype=torch.uint8, pin_memory=True)
        fi.fi_model_pack(spec, packed.data_ptr(), n)
        pool.append((m, act, packed))
    xs = [torch.from_numpy(gen.to_nhwc_storage(gen.make_input(7 + j, 8, 3, 224, 224, "normal", "bf16"), "bf16").view(np.int16)).cuda()
          for j in range(2)]
    outs = [torch.zeros((8, 1000), dtype=torch.float32, device="cuda:0") for _ in range(4)]
    reqs = gen.request_stream(2024, 1000, 16, 4, 50.0, 2)[:n_req]

    def serve(member_ids, bi, out_ptrs, load_mode):
        specs, keep = [], []
        for mi in member_ids:
            m, act, packed = pool[mi]
            s, k = fi.make_spec(m, packed.data_ptr(), packed.numel(), act_dtype=act, packed=True)
            specs.append(s)
            keep.append(k)
        d = fi.Dag(specs, 8, alloc, keepalive=keep, load_mode=load_mode)
        d.load(stream)
        d.run(xs[bi].data_ptr(), 8, out_ptrs, stream)
        torch.cuda.synchronize()
        nbytes = d.query().arena_bytes
        d.unload()
        d.destroy()
        return nbytes

    lat = {"fused": [], "fused_one_copy": [], "fused_per_model_copies": [], "per_model": []}
    arena = []
    serve(reqs[0][1], 0, [o.data_ptr() for o in outs], fi.FI_LOAD_ONE_COPY)  # warm the allocators
    for _, members, bi in reqs:
        t0 = time.perf_counter()
        serve(members, bi, [o.data_ptr() for o in outs], fi.FI_LOAD_AUTO)   # the library's choice: no gather for a handle that is loaded once
        lat["fused"].append(time.perf_counter() - t0)
        t0 = time.perf_counter()
        arena.append(serve(members, bi, [o.data_ptr() for o in outs], fi.FI_LOAD_ONE_COPY))
        lat["fused_one_copy"].append(time.perf_counter() - t0)
        t0 = time.perf_counter()
        serve(members, bi, [o.data_ptr() for o in outs], fi.FI_LOAD_PER_MODEL)
        lat["fused_per_model_copies"].append(time.perf_counter() - t0)
        t0 = time.perf_counter()
        for slot, mi in enumerate(members):
            serve([mi], bi, [outs[slot].data_ptr()], fi.FI_LOAD_AUTO)
        lat["per_model"].append(time.perf_counter() - t0)
    # incremental (Section V, individual model swaps in a DAG): one resident handle; members that
    # leave are replaced in place by those that arrive, the ones that stay are not touched.
    def spec_of(mi):
        m, act, packed = pool[mi]
        return fi.make_spec(m, packed.data_ptr(), packed.numel(), act_dtype=act, packed=True)

    cur = list(reqs[0][1])
    sk = [spec_of(mi) for mi in cur]
    res_dag = fi.Dag([a for a, _ in sk], 8, alloc, keepalive=[b for _, b in sk], load_mode=fi.FI_LOAD_PER_MODEL,
                     swap_headroom_bytes=3 << 29)
    res_dag.load(stream)
    torch.cuda.synchronize()
    inc_lat, swapped, moved, fallbacks = [], 0, 0, 0
    for _, members, bi in reqs:
        t0 = time.perf_counter()
        arriving = [mi for mi in members if mi not in cur]
        for slot in range(4):
            if cur[slot] in members:
                continue
            mi = arriving.pop()
            spec, keep = spec_of(mi)
            try:
                res_dag.swap_model(slot, spec, stream, keepalive=keep)
                moved += res_dag.query().last_h2d_bytes
            except fi.FiError:
                fallbacks += 1      # does not fit the resident allocation: rebuild from scratch
                cur[slot] = mi
                res_dag.unload()
                res_dag.destroy()
                sk = [spec_of(c) for c in cur]
                res_dag = fi.Dag([a for a, _ in sk], 8, alloc, keepalive=[b for _, b in sk], load_mode=fi.FI_LOAD_PER_MODEL,
                                 swap_headroom_bytes=3 << 29)
                res_dag.load(stream)
            cur[slot] = mi
            swapped += 1
        res_dag.run(xs[bi].data_ptr(), 8, [o.data_ptr() for o in outs], stream)
        torch.cuda.synchronize()
        inc_lat.append(time.perf_counter() - t0)
    res_dag.unload()
    res_dag.destroy()
    lat["resident_dag_member_swaps"] = inc_lat

    # open loop: requests arrive at the stream's own (Poisson, 50/s) times and queue behind each other
    open_lat = []
    t_start = time.perf_counter()
    for t_arr, members, bi in reqs[:250]:   # the first 250 arrivals (5 s of the stream)
        now = time.perf_counter() - t_start
        if now < t_arr - reqs[0][0]:
            time.sleep(t_arr - reqs[0][0] - now)
        serve(members, bi, [o.data_ptr() for o in outs], fi.FI_LOAD_PER_MODEL)
        open_lat.append(time.perf_counter() - t_start - (t_arr - reqs[0][0]))
    lat["fused_per_model_copies_open_loop_50rps"] = open_lat
    # ---- manager batching + round-robin scheduler over the whole pool (Section IV) ----------------
    # The 16 models do not get the device at once: batches of at most a quarter of the pool's footprint,
    # 20 iterations per DAG, 2 rounds; fused batches with and without the overlapped load, against one
    # model per DAG ("without fusion": same scheduler, 16 batches).
    all_specs = [spec_of(mi) for mi in range(16)]
    rr_specs, rr_keep = [a for a, _ in all_specs], [b for _, b in all_specs]
    rr_opts = fi.make_opts(8, alloc, load_mode=fi.FI_LOAD_PER_MODEL)
    rr_outs = [torch.zeros((8, 1000), dtype=torch.float32, device="cuda:0") for _ in range(16)]
    rr_ptrs = [o.data_ptr() for o in rr_outs]
    whole = fi.fi_footprint(rr_specs, rr_opts).device_bytes
    largest = max(fi.fi_footprint([sp], rr_opts).device_bytes for sp in rr_specs)
    budget = max(whole // 4, largest)
    group_of, n_groups = fi.fi_partition(rr_specs, rr_opts, budget)
    rr = {"budget_bytes": budget, "pool_bytes": whole, "batches": n_groups, "iterations": 20, "rounds": 2}
    for name, grp, ng, ov in (("fused_overlapped_load", group_of, n_groups, True), ("fused", group_of, n_groups, False),
                              ("one_model_per_dag", list(range(16)), 16, False), ("one_model_per_dag_overlapped_load", list(range(16)), 16, True)):
        torch.cuda.synchronize()
        st = fi.fi_round_robin(rr_specs, rr_opts, grp, ng, 20, 2, ov, xs[0].data_ptr(), 8, rr_ptrs, stream)
        rr[name] = dict(total_ms=st.total_ms, run_ms=st.run_ms, swap_ms=st.swap_ms, build_ms=st.build_ms,
                        peak_device_bytes=st.peak_device_bytes, loads=st.n_loads, runs=st.n_runs)
    del rr_keep

    out = {"requests": len(reqs), "mean_arena_mb": float(np.mean(arena)) / 1e6, "round_robin": rr,
           "member_swaps": dict(swaps=swapped, per_request=swapped / len(reqs), mean_h2d_mb_per_request=moved / len(reqs) / 1e6,
                                rebuild_fallbacks=fallbacks)}
    for k, v in lat.items():
        v = np.array(v) * 1e3
        out[k] = dict(p50_ms=float(np.percentile(v, 50)), p95_ms=float(np.percentile(v, 95)),
                      p99_ms=float(np.percentile(v, 99)), mean_ms=float(v.mean()))
    return out


def cpu_baseline(member, x, n_members):
    """The CPU oracle as it stands, on this machine's cores: independent (model, image) units of the same
    single-threaded code, one per thread.  Sample: eight rounds of one-image ResNet-50 forward passes (about 15 s)."""
    import oracle
    m, blob, _ = member
    cores = min(16, os.cpu_count() or 1)
    units = [(m, blob, x[(i % x.shape[0]):(i % x.shape[0]) + 1], False) for i in range(8 * cores)]
    oracle.lib()
    t0 = time.perf_counter()
    oracle.run_models_parallel(units, threads=cores)
    dt = time.perf_counter() - t0
    model_inf_per_s = len(units) / dt
    cpu = "unknown"
    try:
        with open("/proc/cpuinfo") as fh:
            cpu = next((l.split(":", 1)[1].strip() for l in fh if l.startswith("model name")), cpu)
    except OSError:
        pass
    return dict(value=model_inf_per_s / n_members, unit="images/s", cores=cores, kind="oracle",
                model_inferences_per_s=model_inf_per_s, per_thread_model_inferences_per_s=model_inf_per_s / cores,
                cpu=cpu, nproc=os.cpu_count(),
                sample=f"{len(units)} single-image {m.name} forward passes on {cores} threads ({dt:.1f} s); "
                       f"images/s = model-inferences/s / {n_members} members")


if __name__ == "__main__":
    main()
