#!/usr/bin/env python3
"""Benchmark of the fused-DAG hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4|cfg3|cfg2] [--swap-requests R]

A step is one pass of the whole launch schedule (input staging, every member's convolutions,
pooling, FC) over one synthetic batch that is already resident in HBM.  Prints ONE JSON line:
fused-DAG images/s (each image goes through every member), the roofline of the dominant kernel
measured with HIP events on the launch stream, the CPU oracle timed on this machine's cores, and the
fused-vs-separate throughput, memory and swap-latency comparison.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOADS = {
    "cfg2": dict(desc="2x ResNet-18 fused, bf16, batch 1x3x224x224", fams=["resnet18"] * 2, batch=1),
    "cfg3": dict(desc="ResNet-50 + MobileNetV2 + VGG-16 fused, bf16, batch 8x3x224x224", fams=["resnet50", "mobilenetv2", "vgg16"], batch=8),
    "cfg4": dict(desc="8x ResNet-50 fused (grouped conv GEMMs), bf16, batch 32x3x224x224", fams=["resnet50"] * 8, batch=32),
}
WIDE = {"mobilenetv2"}  # members that keep fp32 activations (tolerance derivation)
PEAK_MFMA_BF16 = 2500.0  # TFLOP/s dense
PEAK_HBM = 8000.0        # GB/s


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg4", choices=sorted(WORKLOADS))
    ap.add_argument("--swap-requests", type=int, default=200)
    ap.add_argument("--no-extras", action="store_true", help="skip separate-DAG, swap and CPU legs")
    ap.add_argument("--serial-lanes", action="store_true",
                    help="issue every launch on the caller's stream (no concurrent lanes): the condition the per-kernel "
                         "roofline is measured in, for profiler runs that should show the same durations")
    ap.add_argument("--probe-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a kernel of known traffic, to calibrate rocprofv3 counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (member models shard across GPUs without any collective; "
              "see DESIGN.md); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2410_21120_amd as fi
    from workloads import gen, zoo

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    fi.lib()
    wl = WORKLOADS[a.workload]
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

    x = gen.make_input(7, B, 3, 224, 224, "normal", "bf16")
    xin = torch.from_numpy(gen.to_nhwc_storage(x, "bf16").view(np.int16)).cuda()
    outs = [torch.zeros((B, 1000), dtype=torch.float32, device="cuda:0") for _ in members]
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
    dag = make_dag(members, serial_lanes=a.serial_lanes)
    t_build = time.perf_counter() - t0
    t0 = time.perf_counter()
    dag.load(stream)
    torch.cuda.synchronize()
    t_load = time.perf_counter() - t0
    q = dag.query()
    for _ in range(a.warmup):
        dag.run(xin.data_ptr(), B, optr, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        dag.run(xin.data_ptr(), B, optr, stream)
    torch.cuda.synchronize()
    fused_ms = (time.perf_counter() - t0) * 1e3 / a.steps

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
    for L in launches:
        k = per_kernel.setdefault(L.name.decode(), dict(launches=0, ms=0.0, busy_ms=0.0, flops=0.0, bytes=0.0))
        k["launches"] += 1
        k["flops"] += 2.0 * L.macs_per_image * B
        k["bytes"] += float(L.bytes_per_image) * B + L.weight_bytes
    for _ in range(prof_iters):
        tb, te = dag.timeline(xin.data_ptr(), B, optr, stream)
        spans = {}
        for L, b, e in zip(launches, tb, te):
            per_kernel[L.name.decode()]["ms"] += (e - b) / prof_iters
            spans.setdefault(L.name.decode(), []).append((b, e))
        for n, iv in spans.items():
            iv.sort()
            busy, hi = 0.0, -1.0
            for b, e in iv:
                if e > hi:
                    busy += e - max(b, hi)
                    hi = e
            per_kernel[n]["busy_ms"] += busy / prof_iters
    dom_name = max((n for n in per_kernel if n.startswith("conv_mfma")), key=lambda n: per_kernel[n]["busy_ms"],
                   default=max(per_kernel, key=lambda n: per_kernel[n]["busy_ms"]))
    dom = per_kernel[dom_name]
    mfma = [v for n, v in per_kernel.items() if n.startswith("conv_mfma")]
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
    kernels = {n: dict(launches=v["launches"], ms=round(v["ms"], 4), busy_ms=round(v["busy_ms"], 4),
                       tflops=round(v["flops"] / (v["busy_ms"] * 1e-3) / 1e12, 2) if v["flops"] else 0.0,
                       gbps=round(v["bytes"] / (v["busy_ms"] * 1e-3) / 1e9, 1)) for n, v in per_kernel.items()}
    res = {
        "metric": "fused-DAG images/sec + MFMA util; peak HBM and swap latency vs per-model",
        "value": B / (fused_ms * 1e-3), "unit": "images/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": fused_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl["desc"], "members": len(members), "batch": B,
                   "model_inferences_per_s": B * len(members) / (fused_ms * 1e-3)},
        "roofline": roofline,
        # every dense (matrix-core) FLOP of the step over the whole step time
        "mfma_util_all_dense": mfma_flops / (fused_ms * 1e-3) / 1e12 / PEAK_MFMA_BF16,
        "kernels": kernels,
        "dag": dict(nodes=q.n_nodes, levels=q.n_levels, launches=q.n_launches, device_allocs=q.n_device_allocs,
                    h2d_copies=q.n_h2d_copies, arena_bytes=q.arena_bytes, act_bytes=q.act_bytes,
                    lanes=q.n_lanes, device_bytes=q.device_bytes, build_ms=t_build * 1e3, load_ms=t_load * 1e3,
                    load_gbps=q.arena_bytes / t_load / 1e9),
    }
    dag.unload()
    dag.destroy()

    if not a.no_extras:
        # ---- the same members as n single-model DAGs ("without fusion") -----------------------
        singles = [make_dag([mb]) for mb in members]
        for d in singles:
            d.load(stream)
        torch.cuda.synchronize()
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
        res["fused_vs_separate"] = dict(
            fused_ms=fused_ms, separate_ms=sep_ms, speedup=sep_ms / fused_ms,
            launches_fused=q.n_launches, launches_separate=sum(s.n_launches for s in sq),
            hbm_bytes_fused=q.device_bytes, hbm_bytes_separate_resident=sum(s.device_bytes for s in sq),
            hbm_bytes_separate_sequential=max(s.device_bytes for s in sq),
            device_allocs_fused=1, device_allocs_separate=len(singles))
        for d in singles:
            d.unload()
            d.destroy()
        res["swap"] = swap_churn(fi, torch, gen, zoo, alloc, stream, a.swap_requests)
        res["cpu_baseline"] = cpu_baseline(members[0], x, len(members))
    print(json.dumps(res))


# HBM traffic of the dominant kernel from rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE; KiB per dispatch,
# summed over the kernel's launches of one step and scaled by what the same counters read for a
# 1 GiB device-to-device copy).  The figures belong to one exact set of sources: when any of them
# has changed since the counters were taken the entry no longer applies and traffic is null.
COUNTERS = {
    "sources_sha256": "a6c038937873f348a8b0ab510529c57301e36c1c1b4ca5d606a8520c753c4ada",
    "workload": "cfg4",
    "kernel": "conv_mfma_128x128",
    "launches_per_step": 54,
    "fetch_kib_per_step": 2889688.4, "write_kib_per_step": 3976448.0,
    "fetch_scale": 2.0, "write_scale": 1.0,
}


def sources_sha256():
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2410_21120_amd", "csrc")
    for f in ("fi_internal.h", "fi_plan.cpp", "fi_api.cpp", "fi_kernels.hip"):
        with open(os.path.join(csrc, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def counter_traffic(kernel, workload):
    c = COUNTERS
    if not c["sources_sha256"] or c["kernel"] != kernel or c["workload"] != workload or c["sources_sha256"] != sources_sha256():
        return None
    per_launch = (c["fetch_kib_per_step"] * c["fetch_scale"] + c["write_kib_per_step"] * c["write_scale"]) * 1024.0 / c["launches_per_step"]
    return dict(bytes_per_launch=per_launch, fetch_bytes_per_launch=c["fetch_kib_per_step"] * c["fetch_scale"] * 1024.0 / c["launches_per_step"],
                write_bytes_per_launch=c["write_kib_per_step"] * c["write_scale"] * 1024.0 / c["launches_per_step"],
                source="rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a 1 GiB copy probe")


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

    lat = {"fused_one_copy": [], "fused_per_model_copies": [], "per_model": []}
    arena = []
    serve(reqs[0][1], 0, [o.data_ptr() for o in outs], fi.FI_LOAD_ONE_COPY)  # warm the allocators
    for _, members, bi in reqs:
        t0 = time.perf_counter()
        arena.append(serve(members, bi, [o.data_ptr() for o in outs], fi.FI_LOAD_ONE_COPY))
        lat["fused_one_copy"].append(time.perf_counter() - t0)
        t0 = time.perf_counter()
        serve(members, bi, [o.data_ptr() for o in outs], fi.FI_LOAD_PER_MODEL)
        lat["fused_per_model_copies"].append(time.perf_counter() - t0)
        t0 = time.perf_counter()
        for slot, mi in enumerate(members):
            serve([mi], bi, [outs[slot].data_ptr()], fi.FI_LOAD_ONE_COPY)
        lat["per_model"].append(time.perf_counter() - t0)
    out = {"requests": len(reqs), "mean_arena_mb": float(np.mean(arena)) / 1e6}
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
    return dict(value=model_inf_per_s / n_members, unit="images/s", cores=cores, kind="oracle",
                model_inferences_per_s=model_inf_per_s,
                sample=f"{len(units)} single-image {m.name} forward passes on {cores} threads ({dt:.1f} s); "
                       f"images/s = model-inferences/s / {n_members} members")


if __name__ == "__main__":
    main()
