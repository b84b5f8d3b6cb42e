#!/usr/bin/env python3
"""Benchmark of the ENEC codec hot path on one MI355X.

Workload (default): the synthetic 7B-style decoder layer (nine bf16 tensors, 404.8 MB), resident
in HBM.  One step = compress all nine tensors, then decompress all nine (every row of the hot
path).  Throughput counts uncompressed bytes, as the paper does (Sec. VI-B).
The tensors of a pass go to the library's batch entry points, one call per (n, m) tuple, which
is one kernel launch each.

Prints ONE JSON line.  `value` is the whole-step throughput: uncompressed bytes through the codec
(compress pass + decompress pass) per second.  `compress_GBps` / `decompress_GBps` are the two
passes alone, from HIP events on the launch stream inside the same timed region.
"""
import argparse
import json
import os
import sys
import time
import zlib

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "decompress & compress GB/s (uncompressed bf16) + compression ratio, 1 MI355X"
HBM_PEAK_GBPS = 8000.0

# HBM bytes per launch measured with rocprofv3 --pmc on this workload (FETCH_SIZE and WRITE_SIZE in
# two runs, each scaled by what the same counter reads for enec_copy of known size); the figures
# and the commands are in profiles/codec_kernels_config2_hbm_traffic.md.  They apply to the default
# workload only; another workload reports null.
MEASURED_TRAFFIC_BYTES = {
    "config2": {"enec::compress_kernel<4,2>": 717855233, "enec::decompress_kernel<4,2>": 713721026},
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="config2", choices=["config1", "config2"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the brief fp16 / fp32 / joint-search measurements")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1")

    import numpy as np
    import torch
    from paper_2604_03298_amd import enec, workloads

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    enec.lib()
    torch.cuda.set_device(0)

    # ---- inputs: generated on the host, resident in HBM before anything is timed --------
    if args.workload == "config2":
        host = list(workloads.config2())
        wl_name = "config2: 7B-style decoder layer, q/k/v/o 4096x4096, gate/up 4096x11008, down 11008x4096, 2 norm vectors"
    else:
        host = [("matrix", workloads.config1())]
        wl_name = "config1: 1024x4096 N(0,0.02^2)"
    names = [n for n, _ in host]
    srcs = [torch.from_numpy(w.view(np.int16)).cuda() for _, w in host]
    n_el = [w.size for _, w in host]
    raw_bytes = 2 * sum(n_el)
    ws = enec.new_workspace(sum(n_el))
    params = [enec.tune(s, ws) for s in srcs]                      # library tuner, outside the timed steps
    # what tuning costs, reported beside the headline (the paper tunes offline): all exponents, and a
    # sample of every 16th chunk of 4096 elements
    tune_info = {}
    for key, fn in (("all_exponents", lambda s: enec.tune(s, ws)), ("every_16th_chunk", lambda s: enec.tune_sampled(s, 16, ws))):
        torch.cuda.synchronize()
        tt = time.perf_counter()
        got = [fn(s) for s in srcs]
        tune_info[key] = {"ms_for_the_layer": round((time.perf_counter() - tt) * 1e3, 3),
                          "same_tuples_as_all_exponents": got == params}
    torch.cuda.synchronize()
    tt = time.perf_counter()
    got = enec.tune_batch(srcs, ws)                                  # one wait for the stream instead of nine
    tune_info["all_exponents_batched"] = {"ms_for_the_layer": round((time.perf_counter() - tt) * 1e3, 3),
                                          "same_tuples_as_all_exponents": got == params}
    outs = [torch.zeros(enec.compress_bound(n), dtype=torch.uint8, device="cuda") for n in n_el]
    backs = [torch.zeros_like(s) for s in srcs]
    sizes = torch.zeros(len(srcs), dtype=torch.int64, device="cuda")
    nt = len(srcs)

    # tensors that share (n, m) go into one library call (= one kernel launch)
    groups = {}
    for i in range(nt):
        groups.setdefault((params[i][1], params[i][2]), []).append(i)
    groups = list(groups.values())
    ng = len(groups)

    def compress_all(ev=None):
        if ev:
            ev[0].record()
        for gi, g in enumerate(groups):
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
              for g in groups]

    def decompress_all(ev=None):
        if ev:
            ev[0].record()
        for gi, g in enumerate(groups):
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
            kern[f"enec::{kind}_kernel<{m},{a}>"] = dict(
                ms=float(dur[:, gi].sum()), bytes=moved * args.steps, launches=args.steps,
                tensors=[names[i] for i in g])
    dom = max(kern, key=lambda k: kern[k]["ms"])
    gd = kern[dom]
    achieved = gd["bytes"] / (gd["ms"] * 1e-3) / 1e9
    roofline = {
        "kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBPS, 4),
        "avg_launch_us": round(gd["ms"] * 1e3 / gd["launches"], 2),
        "algorithmic_bytes_per_launch": gd["bytes"] // gd["launches"],
        "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload, {}).get(dom),
    }
    per_kernel = {k: {"GBps_moved": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1),
                      "frac_of_hbm_peak": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                      "avg_launch_us": round(v["ms"] * 1e3 / v["launches"], 2), "launches": v["launches"],
                      "tensors_per_launch": len(v["tensors"])}
                  for k, v in sorted(kern.items())}
    moved_total = raw_bytes + sum(stream_bytes)

    # practical ceiling: the library's plain 128-bit copy on a buffer of the layer's size
    cp_src, cp_dst = srcs[4].view(torch.uint8), backs[4].view(torch.uint8)
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
        from oracle import enec_oracle
        done_bytes, t_cpu, i = 0, 0.0, 0
        order = sorted(range(nt), key=lambda j: -n_el[j])
        while t_cpu < 12.0 and i < 40 * nt:
            j = order[i % nt]
            w = host[j][1]
            B = enec_oracle.default_block(w.size)
            ts = time.perf_counter()
            rc, s = enec_oracle.compress(w, params[j], B)
            rc2, d = enec_oracle.decompress(s, w.size)
            t_cpu += time.perf_counter() - ts
            assert rc == 0 and rc2 == 0
            done_bytes += 2 * 2 * w.size
            i += 1
        cpu = {"value": round(done_bytes / t_cpu / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"{i} tensors of the same layer, largest first, compress + decompress each, "
                         f"{done_bytes / 2e6:.0f} MB of bf16, {t_cpu:.1f} s of CPU time"}

    # ---- the other element formats and the joint (m, L) search, measured briefly beside the headline -----
    # (same seven matrix shapes, N(0, 0.02^2) drawn on the GPU; bf16 with Eq. 4's group-length search)
    extra = None
    if args.workload == "config2" and not args.no_extra:
        try:
            import report
            shapes = [(r, c) for _, r, c, _ in workloads.config2_spec() if r > 1]
            extra = {}
            for key, tdt, code, lengths in (("fp16", torch.float16, enec.FP16, None), ("fp32", torch.float32, enec.FP32, None),
                                            ("bf16_joint_m_L", torch.bfloat16, enec.BF16, (8, 16, 32))):
                t = [workloads.gpu_gaussian(torch, r, c, 0.02, 6000 + i, tdt) for i, (r, c) in enumerate(shapes)]
                res = report.run_group(torch, enec, key, t, reps=5, dtype=code, lengths=lengths)[0]
                extra[key] = {k: res[k] for k in ("params", "compression_ratio", "compress_GBps", "decompress_GBps",
                                                  "compress_frac_of_hbm_peak", "decompress_frac_of_hbm_peak")}
                del t
                torch.cuda.empty_cache()
            # the headline layer itself with one tuple per data block instead of one per tensor
            res = report.run_per_block(torch, enec, "bf16_tuple_per_block", srcs, reps=5)
            extra["bf16_tuple_per_block"] = {k: res[k] for k in ("compression_ratio", "compress_GBps", "decompress_GBps",
                                                                 "compress_frac_of_hbm_peak", "decompress_frac_of_hbm_peak")}
        except Exception as exc:          # the headline line must not depend on this
            extra = {"error": repr(exc)}

    ratio = raw_bytes / sum(stream_bytes)
    line = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": wl_name, "tensors": nt, "uncompressed_bytes": raw_bytes,
                   "block_size": 16384, "params": {names[i]: list(params[i]) for i in range(nt)},
                   "input_crc32": {names[i]: zlib.crc32(host[i][1].tobytes()) for i in range(nt)}},
        "compress_GBps": round(comp_gbps, 1), "decompress_GBps": round(decomp_gbps, 1),
        "compress_frac_of_hbm_peak": round(moved_total / (np.median(pass_c) * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "decompress_frac_of_hbm_peak": round(moved_total / (np.median(pass_d) * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "compression_ratio": round(ratio, 4),
        "compress_ms": round(float(np.median(pass_c)), 4), "decompress_ms": round(float(np.median(pass_d)), 4),
        "copy_kernel_GBps_moved": round(copy_gbps, 1),
        "roofline": roofline, "kernels": per_kernel, "cpu_baseline": cpu, "tuner": tune_info, "other_formats": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
