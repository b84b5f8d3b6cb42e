#!/usr/bin/env python3
"""Benchmark of the ENEC codec hot path on one MI355X.

Workload (default, `--workload config2`): the synthetic 7B-style decoder layer (nine bf16 tensors,
404.8 MB), resident in HBM.  One step = compress every tensor of the workload, then decompress every
tensor (every row of the hot path).  Throughput counts uncompressed bytes, as the paper does (Sec. VI-B).
The tensors of a pass go to the library's batch entry points, one call per (n, m) tuple and per sixteen
tensors, which is one kernel launch each.

Other workloads: config1 (one 1024x4096 matrix), config3 (edge-case mix, one 64M-element tensor),
config3b (the same blocks as four per-category tensors), config4 (32 tensors of 8192x28672, 15 GB, the
largest single-GPU configuration), config5 (8 layers of 8192x8192 + 8192x28672, resident in HBM for the
headline figures; the offload scenario over PCIe is measured beside them, outside the timed steps).

Prints ONE JSON line.  `value` is the whole-step throughput: uncompressed bytes through the codec
(compress pass + decompress pass) per second.  `compress_GBps` / `decompress_GBps` are the two
passes alone, from HIP events on the launch stream inside the same timed region.
"""
import argparse
import hashlib
import json
import os
import sys
import threading
import time
import zlib

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "decompress & compress GB/s (uncompressed bf16) + compression ratio, 1 MI355X"
HBM_PEAK_GBPS = 8000.0
WORKLOADS = ["config1", "config2", "config3", "config3b", "config4", "config5"]

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE in two runs, each scaled by
# what the same counter reads for enec_copy of known size); figures and commands are in
# profiles/codec_kernels_config2_hbm_traffic.md.  A figure is reported only while the kernel sources still
# hash to what they were when it was measured, and only for the workload it was measured on; else null.
MEASURED_TRAFFIC = {
    "kernel_sources_sha256": "2b9e048caf862dc139eed311f676362c928a25bdaf8f7238c6f8e1fa06dcd19b",
    "bytes_per_launch": {
        "config2": {"enec::compress_kernel<4,2>": 714768173, "enec::decompress_kernel<4,2>": 713773370},
    },
}


def kernel_sources_sha256():
    """Hash of the library's sources with // comments, blank lines and indentation taken out (no string literal of these
    files holds "//"), so that a reworded comment does not retire a measurement."""
    csrc = os.path.join(ROOT, "paper_2604_03298_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".hpp")):
            with open(os.path.join(csrc, name), "r", encoding="utf-8") as f:
                lines = [ln.split("//", 1)[0].strip() for ln in f]
            h.update(name.encode() + b"\0" + "\n".join(ln for ln in lines if ln).encode())
    return h.hexdigest()


def load_workload(name, torch, np, workloads):
    """-> (label, names, device tensors of int16 bit patterns, host arrays or None when drawn on the GPU)"""
    def dev(a):
        return torch.from_numpy(a.view(np.int16)).cuda()
    if name == "config1":
        host = [("matrix", workloads.config1())]
        label = "config1: 1024x4096 N(0,0.02^2)"
    elif name == "config2":
        host = list(workloads.config2())
        label = "config2: 7B-style decoder layer, q/k/v/o 4096x4096, gate/up 4096x11008, down 11008x4096, 2 norm vectors"
    elif name == "config3":
        host = [("mix", workloads.config3()[0])]
        label = "config3: edge-case mix, 4096 blocks of 16384 (zero / constant / Student-t / random bits), one tensor"
    elif name == "config3b":
        host = list(zip(["zero", "constant", "student_t", "random_bits"], workloads.config3_by_category()))
        label = "config3b: the blocks of the edge-case mix as four per-category tensors of 16M elements"
    elif name == "config4":
        srcs = [workloads.config4_device(torch, i) for i in range(32)]
        return ("config4: 32 tensors 8192x28672, N(0, s_t^2), s_t log-uniform in [0.003, 0.03], drawn on the GPU",
                [f"t{i:02d}" for i in range(32)], srcs, None)
    else:
        spec = workloads.config5_spec()
        srcs = [workloads.config5_device(torch, i, spec) for i in range(len(spec))]
        return ("config5: 8 layers of 8192x8192 + 8192x28672, N(0, 0.015^2), drawn on the GPU",
                [f"l{i // 2}_{'attn' if i % 2 == 0 else 'ffn'}" for i in range(len(spec))], srcs, None)
    return label, [n for n, _ in host], [dev(w) for _, w in host], [w for _, w in host]


def cpu_baseline(np, samples, budget_s=6.0):
    """The oracle as it stands, timed on this machine's host cores: compress + decompress of the sample
    tensors, once on one thread and once on one thread per core (each thread whole tensors; ctypes drops
    the GIL).  samples: list of (bit patterns, tuple).  -> the cpu_baseline object"""
    from oracle import enec_oracle

    def one(w, prm):
        B = enec_oracle.default_block(w.size)
        rc, s = enec_oracle.compress(w, prm, B)
        rc2, d = enec_oracle.decompress(s, w.size)
        assert rc == 0 and rc2 == 0
        return 2 * 2 * w.size                     # bytes of bf16 through compress and through decompress

    def leg(threads):
        done = [0] * threads
        stop = time.perf_counter() + budget_s

        def work(t):
            i = t
            while time.perf_counter() < stop:
                w, prm = samples[i % len(samples)]
                done[t] += one(w, prm)
                i += threads
        t0 = time.perf_counter()
        ths = [threading.Thread(target=work, args=(t,)) for t in range(threads)]
        for th in ths:
            th.start()
        for th in ths:
            th.join()
        wall = time.perf_counter() - t0
        return sum(done) / wall / 1e9, sum(done), wall

    cores = min(16, len(os.sched_getaffinity(0)))       # a one-GPU job's share of the box, whatever the affinity mask shows
    one(*samples[0])                                   # builds / loads the oracle outside the timing
    g1, b1, w1 = leg(1)
    gN, bN, wN = leg(cores)
    return {"value": round(gN, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{len(samples)} tensors of the workload ({sum(w.size for w, _ in samples) * 2 / 1e6:.0f} MB of bf16), "
                      f"compress + decompress of whole tensors, one thread per core for {wN:.1f} s "
                      f"({bN / 2e6:.0f} MB of bf16 through the codec)",
            "single_thread": {"value": round(g1, 4), "unit": "GB/s", "cores": 1, "seconds": round(w1, 1)}}


def offload_scenario(torch, np, enec, srcs, streams, reps=3):
    """Configuration 5's transport: the compressed streams in pinned host memory go over PCIe on one HIP
    stream and are decoded on another (the library's pipeline, double-buffered staging), against copying the
    uncompressed bf16 from pinned host memory.  Outputs are checked after the pipelined runs."""
    host_c = [torch.empty(s.numel(), dtype=torch.uint8).pin_memory() for s in streams]
    for h, s in zip(host_c, streams):
        h.copy_(s)
    host_raw = [torch.empty(s.numel(), dtype=torch.int16).pin_memory() for s in srcs]
    for h, s in zip(host_raw, srcs):
        h.copy_(s)
    torch.cuda.synchronize()
    copy_s, dec_s = torch.cuda.Stream(), torch.cuda.Stream()
    staging = torch.empty(2 * ((max(h.numel() for h in host_c) + 255) & ~255), dtype=torch.uint8, device="cuda")
    backs = [torch.zeros_like(s) for s in srcs]
    plain_dst = [torch.zeros_like(s) for s in srcs]
    pipe = enec.Pipeline(1, dec_s, copy_s, staging)

    def pipelined():
        rc = pipe.prefetch_from_host(0, host_c, backs)
        assert rc == 0, enec.strerror(rc)
        dec_s.synchronize()

    def plain():
        with torch.cuda.stream(copy_s):
            for d, h in zip(plain_dst, host_raw):
                d.copy_(h, non_blocking=True)
        copy_s.synchronize()

    res = {}
    for name, fn in (("compressed_copy_plus_decompress", pipelined), ("uncompressed_copy", plain)):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            t0 = time.perf_counter()
            fn()
            ts.append(time.perf_counter() - t0)
        res[name + "_ms"] = round(1e3 * float(np.median(ts)), 3)
    assert all(torch.equal(b, s) for b, s in zip(backs, srcs)), "offload pipeline output is not bit-exact"
    pipe.close()
    raw = 2 * sum(s.numel() for s in srcs)
    res["effective_weights_GBps_compressed"] = round(raw / res["compressed_copy_plus_decompress_ms"] / 1e6, 1)
    res["effective_weights_GBps_uncompressed"] = round(raw / res["uncompressed_copy_ms"] / 1e6, 1)
    res["speedup"] = round(res["uncompressed_copy_ms"] / res["compressed_copy_plus_decompress_ms"], 3)
    res["pcie_inclusive"] = True
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="config2", choices=WORKLOADS)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the brief fp16 / fp32 / joint-search / per-block / offload measurements")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1")

    import numpy as np
    import torch
    from paper_2604_03298_amd import enec, workloads

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    enec.lib()
    torch.cuda.set_device(0)

    # ---- inputs: resident in HBM before anything is timed ------------------------------------
    wl_name, names, srcs, host = load_workload(args.workload, torch, np, workloads)
    nt = len(srcs)
    n_el = [s.numel() for s in srcs]
    raw_bytes = 2 * sum(n_el)
    ws = enec.new_workspace(sum(n_el))
    params = enec.tune_batch(srcs, ws)                              # library tuner, outside the timed steps
    tune_info = None
    if args.workload == "config2":
        # what tuning costs, reported beside the headline (the paper tunes offline): all exponents one tensor
        # at a time, a sample of every 16th chunk of 4096 elements, and all exponents with one wait per layer
        tune_info = {}
        for key, fn in (("all_exponents", lambda: [enec.tune(s, ws) for s in srcs]),
                        ("every_16th_chunk", lambda: [enec.tune_sampled(s, 16, ws) for s in srcs]),
                        ("all_exponents_batched", lambda: enec.tune_batch(srcs, ws))):
            torch.cuda.synchronize()
            tt = time.perf_counter()
            got = fn()
            tune_info[key] = {"ms_for_the_layer": round((time.perf_counter() - tt) * 1e3, 3),
                              "same_tuples_as_all_exponents": got == params}
    outs = [torch.zeros(enec.compress_bound(n), dtype=torch.uint8, device="cuda") for n in n_el]
    backs = [torch.zeros_like(s) for s in srcs]
    sizes = torch.zeros(nt, dtype=torch.int64, device="cuda")

    # tensors that share (n, m) go into one library call of at most sixteen tensors (= one kernel launch)
    by_tuple = {}
    for i in range(nt):
        by_tuple.setdefault((params[i][1], params[i][2]), []).append(i)
    groups = [g[c:c + 16] for g in by_tuple.values() for c in range(0, len(g), 16)]
    ng = len(groups)
    calls = groups

    def compress_all(ev=None):
        if ev:
            ev[0].record()
        for gi, g in enumerate(calls):
            rc = enec.compress_batch([srcs[i] for i in g], [params[i] for i in g], [outs[i] for i in g], ws,
                                     out_bytes=[sizes[i:i + 1] for i in g])
            assert rc == 0, enec.strerror(rc)
            if ev:
                ev[gi + 1].record()

    compress_all()
    torch.cuda.synchronize()
    stream_bytes = [int(v) for v in sizes.cpu()]
    assert all(v > 0 for v in stream_bytes)
    headers = [outs[i][:64].cpu().numpy().tobytes() for i in range(nt)]
    ditems = [enec.make_decompress_items([outs[i] for i in g], [headers[i] for i in g], [backs[i] for i in g])
              for g in calls]

    def decompress_all(ev=None):
        if ev:
            ev[0].record()
        for gi, g in enumerate(calls):
            rc = enec.decompress_batch(None, None, None, items=ditems[gi][0])
            assert rc == 0, enec.strerror(rc)
            if ev:
                ev[gi + 1].record()

    decompress_all()
    torch.cuda.synchronize()
    for i in range(nt):
        assert torch.equal(backs[i], srcs[i]), f"round trip of {names[i]} is not bit-exact"

    def new_events():
        return [torch.cuda.Event(enable_timing=True) for _ in range(ng + 1)]

    evc = [new_events() for _ in range(args.steps)]
    evd = [new_events() for _ in range(args.steps)]

    for _ in range(args.warmup):
        compress_all()
        decompress_all()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        compress_all(evc[k])
        decompress_all(evd[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = 2 * raw_bytes / (ms_per_step * 1e-3) / 1e9

    # per-launch durations from the events recorded inside the timed region (one launch per group)
    dur_c = np.array([[evc[k][gi].elapsed_time(evc[k][gi + 1]) for gi in range(ng)] for k in range(args.steps)])
    dur_d = np.array([[evd[k][gi].elapsed_time(evd[k][gi + 1]) for gi in range(ng)] for k in range(args.steps)])
    pass_c = np.array([evc[k][0].elapsed_time(evc[k][ng]) for k in range(args.steps)])
    pass_d = np.array([evd[k][0].elapsed_time(evd[k][ng]) for k in range(args.steps)])
    comp_gbps = raw_bytes / (np.median(pass_c) * 1e-3) / 1e9
    decomp_gbps = raw_bytes / (np.median(pass_d) * 1e-3) / 1e9

    # ---- roofline of the dominant kernel ------------------------------------------------
    # algorithmic bytes of one launch = for each of its tensors the bf16 data (2 bytes/element) plus
    # the whole stream (sign/mantissa plane, mask, packed planes, offset table, header), each read
    # or written once
    kern = {}
    for gi, g in enumerate(groups):
        m, a = params[g[0]][2], params[g[0]][1] - params[g[0]][2]
        moved = sum(2 * n_el[i] + stream_bytes[i] for i in g)
        for kind, dur in (("compress", dur_c), ("decompress", dur_d)):
            e = kern.setdefault(f"enec::{kind}_kernel<{m},{a}>", dict(ms=0.0, bytes=0, launches=0, tensors=0))
            e["ms"] += float(dur[:, gi].sum())
            e["bytes"] += moved * args.steps
            e["launches"] += args.steps
            e["tensors"] += len(g)
    dom = max(kern, key=lambda k: kern[k]["ms"])
    gd = kern[dom]
    achieved = gd["bytes"] / (gd["ms"] * 1e-3) / 1e9
    traffic = None
    if MEASURED_TRAFFIC["kernel_sources_sha256"] == kernel_sources_sha256():
        traffic = MEASURED_TRAFFIC["bytes_per_launch"].get(args.workload, {}).get(dom)
    roofline = {
        "kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBPS, 4),
        "timing": "HIP events around each launch on the launch stream, inside the timed steps (includes the launch gap; "
                  "rocprofv3's begin-to-end kernel time in profiles/ is 3-5 % shorter)",
        "avg_launch_us": round(gd["ms"] * 1e3 / gd["launches"], 2),
        "algorithmic_bytes_per_launch": gd["bytes"] // gd["launches"],
        "traffic": traffic,
    }
    per_kernel = {k: {"GBps_moved": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1),
                      "frac_of_hbm_peak": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                      "avg_launch_us": round(v["ms"] * 1e3 / v["launches"], 2), "launches": v["launches"],
                      "tensors_per_step": v["tensors"]}
                  for k, v in sorted(kern.items())}
    moved_total = raw_bytes + sum(stream_bytes)

    # practical ceiling: the library's plain 128-bit copy on the workload's largest tensor
    big = max(range(nt), key=lambda i: n_el[i])
    cp_src, cp_dst = srcs[big].view(torch.uint8), backs[big].view(torch.uint8)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        enec.copy(cp_dst, cp_src)
    e0.record()
    for _ in range(10):
        enec.copy(cp_dst, cp_src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbps = 2 * cp_src.numel() * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9

    # ---- the CPU oracle timed beside it (a baseline, not the target) ----------------------
    cpu = None
    if not args.no_cpu_baseline:
        # a bounded sample of the same workload: its tensors, largest first, at most 2^25 elements of each
        order = sorted(range(nt), key=lambda j: -n_el[j])[:16]
        samples = []
        for j in order:
            w = host[j] if host is not None else srcs[j][:1 << 25].cpu().numpy().view(np.uint16)
            samples.append((np.ascontiguousarray(w[:1 << 25]), params[j]))
        cpu = cpu_baseline(np, samples)

    # ---- measured briefly beside the headline, outside the timed steps -----------------------------------
    extra = None
    if not args.no_extra:
        try:
            import report
            extra = {}
            if args.workload == "config2":
                # the other element formats and the joint (m, L) search: the same seven matrix shapes,
                # N(0, 0.02^2) drawn on the GPU; bf16 with Eq. 4's group-length search
                shapes = [(r, c) for _, r, c, _ in workloads.config2_spec() if r > 1]
                for key, tdt, code, lengths in (("fp16", torch.float16, enec.FP16, None), ("fp32", torch.float32, enec.FP32, None),
                                                ("bf16_joint_m_L", torch.bfloat16, enec.BF16, (8, 16, 32))):
                    t = [workloads.gpu_gaussian(torch, r, c, 0.02, 6000 + i, tdt) for i, (r, c) in enumerate(shapes)]
                    res = report.run_group(torch, enec, key, t, reps=5, dtype=code, lengths=lengths)[0]
                    extra[key] = {k: res[k] for k in ("params", "compression_ratio", "compress_GBps", "decompress_GBps",
                                                      "compress_frac_of_hbm_peak", "decompress_frac_of_hbm_peak")}
                    del t
                    torch.cuda.empty_cache()
            if args.workload in ("config2", "config3"):
                # the same tensors with one tuple per data block instead of one per tensor
                res = report.run_per_block(torch, enec, "bf16_tuple_per_block", srcs, reps=5)
                extra["bf16_tuple_per_block"] = {k: res[k] for k in ("compression_ratio", "compress_GBps", "decompress_GBps",
                                                                     "compress_frac_of_hbm_peak", "decompress_frac_of_hbm_peak")}
            if args.workload == "config5":
                extra["offload"] = offload_scenario(torch, np, enec, srcs, [outs[i][:stream_bytes[i]] for i in range(nt)])
        except Exception as exc:          # the headline line must not depend on this
            extra = {"error": repr(exc)}

    ratio = raw_bytes / sum(stream_bytes)
    cfg = {"workload": wl_name, "tensors": nt, "uncompressed_bytes": raw_bytes, "block_size": 16384,
           "params": sorted({tuple(p) for p in params}) if nt > 9 else {names[i]: list(params[i]) for i in range(nt)},
           "launches_per_pass": ng}
    if host is not None:
        cfg["input_crc32"] = {names[i]: zlib.crc32(host[i].tobytes()) for i in range(nt)}
        # ties the timed streams to the oracle's: tests/test_gpu_parity.py compares these streams byte for byte
        cfg["stream_crc32"] = {names[i]: zlib.crc32(outs[i][:stream_bytes[i]].cpu().numpy().tobytes()) for i in range(nt)}
    else:
        cfg["input_crc32"] = {names[0]: zlib.crc32(srcs[0].cpu().numpy().tobytes())}
    line = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": cfg,
        "compress_GBps": round(comp_gbps, 1), "decompress_GBps": round(decomp_gbps, 1),
        "compress_frac_of_hbm_peak": round(moved_total / (np.median(pass_c) * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "decompress_frac_of_hbm_peak": round(moved_total / (np.median(pass_d) * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "compression_ratio": round(ratio, 4),
        "compress_ms": round(float(np.median(pass_c)), 4), "decompress_ms": round(float(np.median(pass_d)), 4),
        "copy_kernel_GBps_moved": round(copy_gbps, 1),
        "roofline": roofline, "kernels": per_kernel, "cpu_baseline": cpu, "tuner": tune_info, "other_measurements": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
