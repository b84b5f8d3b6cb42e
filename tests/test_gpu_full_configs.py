"""All five configurations at full size, every tensor: the library's streams against the CPU oracle's, byte for byte,
in the launch configuration bench.py times (batched launches of up to sixteen tensors), and both decoders on them.

Configurations 4 and 5 (15 GB and 4.8 GB of bf16) are drawn on the GPU with the seeded generator bench.py uses and
reach the oracle through a device-to-host copy, one tensor per worker thread at a time; the oracle's streams go back
to the device, where they are compared.  The oracle legs run in a thread pool (ctypes and numpy drop the GIL).
Bit-exact: byte and integer work only.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from paper_2604_03298_amd import workloads as W

pytestmark = pytest.mark.gpu

WORKERS = 12        # the GPU machine gives a one-GPU job sixteen cores


@pytest.fixture(scope="module")
def dev():
    import torch
    from paper_2604_03298_amd import enec
    assert torch.cuda.is_available(), "these tests need the MI355X"
    enec.lib()
    return torch, enec


def oracle_leg(oracle, w, B=16384):
    """What one worker does for one tensor: tuple, stream, and the oracle's own round trip."""
    prm = oracle.tune(w)
    rc, s = oracle.compress(w, prm, B)
    assert rc == oracle.OK
    rc, d = oracle.decompress(s, w.size)
    assert rc == oracle.OK and np.array_equal(d, w)
    return prm, s


def check_batched(torch, enec, oracle, srcs, label, chunk=16):
    """srcs: device tensors (int16 bit patterns).  Oracle streams for all of them (thread pool), then the
    library's batched compression and batched decompression exactly as bench.py launches them."""
    n = len(srcs)
    with ThreadPoolExecutor(WORKERS) as pool:
        legs = list(pool.map(lambda s: oracle_leg(oracle, s.cpu().numpy().view(np.uint16)), srcs))
    params = [p for p, _ in legs]
    refs = [torch.from_numpy(s).cuda() for _, s in legs]
    del legs
    ws = enec.new_workspace(sum(s.numel() for s in srcs))
    # the library's tuner sees the same exponents
    assert enec.tune_batch(srcs, ws) == params, label
    outs = [torch.full((enec.compress_bound(s.numel()),), 0xA5, dtype=torch.uint8, device="cuda") for s in srcs]
    sizes = torch.zeros(n, dtype=torch.int64, device="cuda")
    for c0 in range(0, n, chunk):
        c = range(c0, min(n, c0 + chunk))
        rc = enec.compress_batch([srcs[i] for i in c], [params[i] for i in c], [outs[i] for i in c], ws,
                                 out_bytes=[sizes[i:i + 1] for i in c])
        assert rc == enec.OK, enec.strerror(rc)
    torch.cuda.synchronize()
    got = [int(v) for v in sizes.cpu()]
    for i in range(n):
        assert got[i] == refs[i].numel(), f"{label}[{i}]: size {got[i]} vs oracle {refs[i].numel()}"
        assert torch.equal(outs[i][:got[i]], refs[i]), f"{label}[{i}]: compressed stream differs from the oracle's"
    # the library decodes the oracle's streams, again batched (the oracle has decoded them itself, and the
    # library's streams are those bytes)
    backs = [torch.full_like(s, 0x5A5A) for s in srcs]
    hdrs = [r[:64].cpu().numpy().tobytes() for r in refs]
    for c0 in range(0, n, chunk):
        c = range(c0, min(n, c0 + chunk))
        rc = enec.decompress_batch([refs[i] for i in c], [hdrs[i] for i in c], [backs[i] for i in c])
        assert rc == enec.OK, enec.strerror(rc)
    torch.cuda.synchronize()
    for i in range(n):
        assert torch.equal(backs[i], srcs[i]), f"{label}[{i}]: library decompress(oracle stream) != input"
    return params, refs


@pytest.mark.parametrize("half", [0, 1])
def test_config4_all_32_tensors(dev, oracle, half):
    """The large-layer stream, sixteen tensors of 8192 x 28672 per launch as bench.py --workload config4 runs it."""
    torch, enec = dev
    srcs = [W.config4_device(torch, i) for i in range(16 * half, 16 * half + 16)]
    params, _ = check_batched(torch, enec, oracle, srcs, f"config4[{16 * half}..]")
    assert all(p[3] == 16 and p[2] == 3 and p[1] in (6, 7) for p in params), params


def test_config4_uses_both_kernel_instances():
    """sigma log-uniform in [0.003, 0.03] puts tensors on both sides of the n = 6 / n = 7 boundary: the two
    halves above exercise compress_kernel<3,3> and <3,4> (and the two decompress instances) at full size."""
    std = [W.config4_std(i) for i in range(32)]
    assert min(std) < 0.006 and max(std) > 0.02


def test_config5_all_16_tensors(dev, oracle):
    torch, enec = dev
    srcs = [W.config5_device(torch, i) for i in range(16)]
    check_batched(torch, enec, oracle, srcs, "config5")


def test_config3b_four_tensors_full_size(dev, oracle):
    """The edge-case mix by category, four tensors of 16M elements: width-0 planes (all-zero blocks), a constant,
    heavy tails, and random bit patterns where every group takes the full width."""
    torch, enec = dev
    parts = W.config3_by_category()
    assert [p.size for p in parts] == [1 << 24] * 4
    srcs = [torch.from_numpy(p.view(np.int16)).cuda() for p in parts]
    params, refs = check_batched(torch, enec, oracle, srcs, "config3b")
    assert params[0] == (0, 1, 0, 16) and params[3][1] == 8, params
    ratio = [2 * parts[i].size / refs[i].numel() for i in range(4)]
    assert ratio[0] > 1.98 and 0.99 < ratio[3] < 1.0, ratio
