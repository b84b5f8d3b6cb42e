"""Runs the codec on all five synthetic configurations on one MI355X and prints one JSON line per
configuration (throughput on uncompressed bytes, ratio, fraction of the 8 TB/s HBM peak in bytes
moved).  `python report.py [--configs 1,2,2j,2p,3a,3p,3b,4,4p,5,fp16,fp32]`.
2j is configuration 2 tuned with the group length searched together with m (Eq. 4); 2p, 3p and 4p are configuration 2,
configuration 3a and four tensors of configuration 4 with one tuple per data block; the last two are the
seven matrix shapes of configuration 2 as fp16 / fp32 tensors, N(0, 0.02^2).

Tensors of configurations 1-3 come from the seeded numpy generators of `workloads.py` (the ones the
parity tests use); configurations 4 and 5 (15 GB / 4.8 GB of bf16) are drawn on the GPU with a
seeded torch generator, same shapes and standard deviations.  Every run checks on the device that
decompress(compress(x)) == x bit for bit.
"""
from __future__ import annotations

import argparse
import json
import time

import numpy as np

HBM_PEAK = 8000.0


def _events(torch, n):
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def run_group(torch, enec, name, srcs, reps=5, dtype=0, lengths=None):
    """Tune, compress (batched), decompress (batched), verify; returns a dict of results."""
    n_el = [s.numel() for s in srcs]
    raw = srcs[0].element_size() * sum(n_el)
    ws = enec.new_workspace(sum(n_el))
    params = [enec.tune(s, ws, dtype=dtype, lengths=lengths) for s in srcs]
    outs = [torch.empty(enec.compress_bound(n, dtype=dtype), dtype=torch.uint8, device="cuda") for n in n_el]
    sizes = torch.zeros(len(srcs), dtype=torch.int64, device="cuda")
    szl = [sizes[i:i + 1] for i in range(len(srcs))]
    chunks = [list(range(i, min(i + 16, len(srcs)))) for i in range(0, len(srcs), 16)]

    def comp():
        for c in chunks:
            rc = enec.compress_batch([srcs[i] for i in c], [params[i] for i in c], [outs[i] for i in c], ws,
                                     out_bytes=[szl[i] for i in c], dtype=dtype)
            assert rc == 0, enec.strerror(rc)

    comp()
    torch.cuda.synchronize()
    stream_bytes = [int(v) for v in sizes.cpu()]
    assert all(v > 0 for v in stream_bytes), "range error"
    hdrs = [outs[i][:64].cpu().numpy().tobytes() for i in range(len(srcs))]
    backs = [torch.empty_like(s) for s in srcs]
    items = [enec.make_decompress_items([outs[i] for i in c], [hdrs[i] for i in c], [backs[i] for i in c])
             for c in chunks]

    def decomp():
        for it in items:
            rc = enec.decompress_batch(None, None, None, items=it[0])
            assert rc == 0, enec.strerror(rc)

    decomp()
    torch.cuda.synchronize()
    assert all(torch.equal(b, s) for b, s in zip(backs, srcs)), "round trip is not bit-exact"
    # all repetitions are queued back to back (no host synchronisation in between, which would add the
    # latency of a launch into an idle GPU to every pass); events bracket each pass on the stream
    evs = [_events(torch, 3) for _ in range(reps)]
    comp(); decomp()
    for e in evs:
        e[0].record(); comp(); e[1].record(); decomp(); e[2].record()
    torch.cuda.synchronize()
    tc = float(np.median([e[0].elapsed_time(e[1]) for e in evs]))
    td = float(np.median([e[1].elapsed_time(e[2]) for e in evs]))
    moved = raw + sum(stream_bytes)
    return {
        "config": name, "tensors": len(srcs), "uncompressed_bytes": raw, "compression_ratio": round(raw / sum(stream_bytes), 4),
        "params": sorted({tuple(p) for p in params}),
        "compress_ms": round(tc, 4), "decompress_ms": round(td, 4),
        "compress_GBps": round(raw / tc / 1e6, 1), "decompress_GBps": round(raw / td / 1e6, 1),
        "compress_frac_of_hbm_peak": round(moved / tc / 1e6 / HBM_PEAK, 4),
        "decompress_frac_of_hbm_peak": round(moved / td / 1e6 / HBM_PEAK, 4),
        "roundtrip_bit_exact": True,
    }, (outs, stream_bytes, hdrs, backs)


def run_per_block(torch, enec, name, srcs, reps=5, dtype=0):
    """The same measurement for streams with one tuple per data block (all tensors in one batched call)."""
    n_el = [s.numel() for s in srcs]
    raw = srcs[0].element_size() * sum(n_el)
    ws = enec.new_workspace(sum(n_el), block_size=min(enec.default_block_size(n) for n in n_el))
    outs = [torch.empty(enec.compress_bound_per_block(n, dtype=dtype), dtype=torch.uint8, device="cuda") for n in n_el]
    sizes = torch.zeros(len(srcs), dtype=torch.int64, device="cuda")
    szl = [sizes[i:i + 1] for i in range(len(srcs))]

    def comp():
        rc = enec.compress_per_block_batch(srcs, outs, ws, out_bytes=szl, dtype=dtype)
        assert rc == 0, enec.strerror(rc)

    comp()
    torch.cuda.synchronize()
    stream_bytes = [int(v) for v in sizes.cpu()]
    assert all(v > 0 for v in stream_bytes)
    hdrs = [o[:64].cpu().numpy().tobytes() for o in outs]
    backs = [torch.empty_like(s) for s in srcs]
    items = enec.make_decompress_items(outs, hdrs, backs)

    def decomp():
        rc = enec.decompress_batch(None, None, None, items=items[0])
        assert rc == 0, enec.strerror(rc)

    decomp()
    torch.cuda.synchronize()
    assert all(torch.equal(b, s) for b, s in zip(backs, srcs)), "round trip is not bit-exact"
    evs = [_events(torch, 3) for _ in range(reps)]
    comp(); decomp()
    for e in evs:
        e[0].record(); comp(); e[1].record(); decomp(); e[2].record()
    torch.cuda.synchronize()
    tc = float(np.median([e[0].elapsed_time(e[1]) for e in evs]))
    td = float(np.median([e[1].elapsed_time(e[2]) for e in evs]))
    moved = raw + sum(stream_bytes)
    return {
        "config": name, "tensors": len(srcs), "uncompressed_bytes": raw, "compression_ratio": round(raw / sum(stream_bytes), 4),
        "params": "one tuple per data block",
        "compress_ms": round(tc, 4), "decompress_ms": round(td, 4),
        "compress_GBps": round(raw / tc / 1e6, 1), "decompress_GBps": round(raw / td / 1e6, 1),
        "compress_frac_of_hbm_peak": round(moved / tc / 1e6 / HBM_PEAK, 4),
        "decompress_frac_of_hbm_peak": round(moved / td / 1e6 / HBM_PEAK, 4),
        "roundtrip_bit_exact": True,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="1,2,2j,2p,3a,3p,3b,4,4p,5,fp16,fp32")
    args = ap.parse_args()
    want = args.configs.split(",")
    import torch
    from paper_2604_03298_amd import enec, workloads as W
    assert torch.cuda.is_available()
    enec.lib()

    def dev(a):
        return torch.from_numpy(a.view(np.int16)).cuda()

    if "1" in want:
        print(json.dumps(run_group(torch, enec, "1: 1024x4096 N(0,0.02^2)", [dev(W.config1())], reps=20)[0]), flush=True)
    if "2" in want:
        print(json.dumps(run_group(torch, enec, "2: 7B-style decoder layer", [dev(w) for _, w in W.config2()], reps=20)[0]), flush=True)
    if "2j" in want:      # the same layer with Eq. 4's joint search of (m, L) instead of the paper's L = 16
        print(json.dumps(run_group(torch, enec, "2j: 7B-style decoder layer, group length searched with m",
                                   [dev(w) for _, w in W.config2()], reps=20, lengths=(8, 16, 32))[0]), flush=True)
    if "3a" in want:
        print(json.dumps(run_group(torch, enec, "3a: edge-case mix, one tensor", [dev(W.config3()[0])], reps=10)[0]), flush=True)
    if "3p" in want:      # the same tensor with one tuple per data block
        print(json.dumps(run_per_block(torch, enec, "3p: edge-case mix, one tensor, one tuple per data block",
                                       [dev(W.config3()[0])], reps=10)), flush=True)
    if "2p" in want:
        print(json.dumps(run_per_block(torch, enec, "2p: 7B-style decoder layer, one tuple per data block",
                                       [dev(w) for _, w in W.config2()], reps=20)), flush=True)
    if "3b" in want:
        for c, t in enumerate(W.config3_by_category()):
            name = ["zero blocks", "constant blocks", "Student-t blocks", "random 16-bit patterns"][c]
            print(json.dumps(run_group(torch, enec, f"3b: {name}", [dev(t)], reps=10)[0]), flush=True)
    if "4" in want:
        srcs = [W.config4_device(torch, i) for i in range(32)]
        print(json.dumps(run_group(torch, enec, "4: 32 tensors 8192x28672", srcs, reps=3)[0]), flush=True)
        del srcs
        torch.cuda.empty_cache()
    if "4p" in want:      # four of these tensors (1.9 GB) with one tuple per data block
        srcs = [W.config4_device(torch, i) for i in range(4)]
        print(json.dumps(run_per_block(torch, enec, "4p: 4 tensors 8192x28672, one tuple per data block", srcs, reps=5)), flush=True)
        del srcs
        torch.cuda.empty_cache()
    if "5" in want:
        srcs = [W.config5_device(torch, i) for i in range(16)]
        res, (outs, stream_bytes, hdrs, backs) = run_group(torch, enec, "5: 8 layers 8192x8192 + 8192x28672 (HBM resident)", srcs, reps=3)
        import bench
        res["offload"] = bench.offload_scenario(torch, np, enec, srcs, [o[:b] for o, b in zip(outs, stream_bytes)])
        print(json.dumps(res), flush=True)
        del srcs, outs, backs
        torch.cuda.empty_cache()
    for key, tdt, code in (("fp16", torch.float16, enec.FP16), ("fp32", torch.float32, enec.FP32)):
        if key in want:
            shapes = [(r, c) for name, r, c, _ in W.config2_spec() if r > 1 and c > 1]
            srcs = [W.gpu_gaussian(torch, r, c, 0.02, 6000 + i, tdt) for i, (r, c) in enumerate(shapes)]
            print(json.dumps(run_group(torch, enec, f"{key}: the seven matrices of configuration 2 as {key}, N(0,0.02^2)",
                                       srcs, reps=20, dtype=code)[0]), flush=True)
            del srcs
            torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
