"""The decompression pipelines (enec_pipeline_*): the offload scenario of configuration 5 and the layer-wise
overlap with a consumer, through the C ABI, against the oracle and against the inputs."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from paper_2604_03298_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    import torch
    from paper_2604_03298_amd import enec
    assert torch.cuda.is_available(), "these tests need the MI355X"
    enec.lib()
    return torch, enec


def compress_all(torch, enec, srcs):
    ws = enec.new_workspace(sum(s.numel() for s in srcs))
    params = enec.tune_batch(srcs, ws)
    outs = [torch.empty(enec.compress_bound(s.numel()), dtype=torch.uint8, device="cuda") for s in srcs]
    sizes = torch.zeros(len(srcs), dtype=torch.int64, device="cuda")
    for c0 in range(0, len(srcs), 16):
        c = range(c0, min(len(srcs), c0 + 16))
        rc = enec.compress_batch([srcs[i] for i in c], [params[i] for i in c], [outs[i] for i in c], ws,
                                 out_bytes=[sizes[i:i + 1] for i in c])
        assert rc == enec.OK, enec.strerror(rc)
    torch.cuda.synchronize()
    nbytes = [int(v) for v in sizes.cpu()]
    assert all(v > 0 for v in nbytes)
    return params, [o[:b] for o, b in zip(outs, nbytes)]


def test_config5_offload_pipeline_against_oracle_and_inputs(dev, oracle):
    """Configuration 5 as the library runs it: sixteen streams in pinned host memory, copied over PCIe on one HIP
    stream and decoded on another, double-buffered.  The streams in host memory must be the oracle's, every
    decoded tensor must be its input, and the recorded timeline must show the copy of stream i + 1 running while
    stream i is decoded."""
    torch, enec = dev
    srcs = [W.config5_device(torch, i) for i in range(16)]
    params, streams = compress_all(torch, enec, srcs)
    host = [torch.empty(s.numel(), dtype=torch.uint8).pin_memory() for s in streams]
    for h, s in zip(host, streams):
        h.copy_(s)
    torch.cuda.synchronize()

    def oracle_stream(i):
        w = srcs[i].cpu().numpy().view(np.uint16)
        assert oracle.tune(w) == params[i]
        rc, s = oracle.compress(w, params[i], 16384)
        assert rc == oracle.OK
        return np.array_equal(s, host[i].numpy())
    with ThreadPoolExecutor(12) as pool:
        same = list(pool.map(oracle_stream, range(16)))
    assert all(same), same

    copy_s, dec_s = torch.cuda.Stream(), torch.cuda.Stream()
    staging = torch.empty(2 * ((max(h.numel() for h in host) + 255) & ~255), dtype=torch.uint8, device="cuda")
    backs = [torch.full_like(s, 0x5A5A) for s in srcs]
    pipe = enec.Pipeline(1, dec_s, copy_s, staging, trace=True)
    rc = pipe.prefetch_from_host(0, host, backs)
    assert rc == enec.OK, enec.strerror(rc)
    assert pipe.acquire(0) == enec.OK                      # the current stream waits for the last decode
    torch.cuda.synchronize()
    for i in range(16):
        assert torch.equal(backs[i], srcs[i]), f"tensor {i}: offload pipeline output != input"
    t = pipe.trace()
    assert t.shape == (16, 4)
    for i in range(16):
        assert t[i, 0] <= t[i, 1] <= t[i, 2] + 0.01 and t[i, 2] <= t[i, 3], (i, t[i])     # copy, then decode, of one stream
    # overlap: the copy of stream i + 1 starts before the decoding of stream i has ended (every pair, but one
    # is enough to prove the two streams run side by side), and a copy never waits for the decode before it
    overlapped = [bool(t[i + 1, 0] < t[i, 3]) for i in range(15)]
    assert sum(overlapped) >= 12, (overlapped, t)
    # double buffering: the copy of stream i + 2 reuses the half stream i was decoded from
    for i in range(14):
        assert t[i + 2, 0] >= t[i, 3] - 1e-3, (i, t[i], t[i + 2])
    # a second pass through the same pipeline object and staging buffer, outputs cleared in between
    for b in backs:
        b.fill_(0x5A5A)
    assert pipe.prefetch_from_host(0, host[:5], backs[:5]) == enec.OK
    assert pipe.acquire(0) == enec.OK
    torch.cuda.synchronize()
    assert all(torch.equal(backs[i], srcs[i]) for i in range(5))
    assert pipe.trace().shape == (5, 4)
    # a stream larger than half the staging buffer is refused before anything is enqueued
    small = enec.Pipeline(1, dec_s, copy_s, staging[:1 << 20])
    assert small.prefetch_from_host(0, host[:1], backs[:1]) == enec.E_CAPACITY
    small.close()
    pipe.close()


def test_layer_wise_prefetch_overlaps_a_consumer(dev, oracle):
    """Six layers of three matrices, compressed streams resident in HBM, two weight slots: layer k + 1 is
    decompressed on a side stream into the other slot while a stand-in consumer (matrix products with layer
    k's weights) runs on the main stream.  Every product must equal the one computed from the original
    weights, i.e. the consumer never saw a half-written or stale slot."""
    torch, enec = dev
    layers, shapes = 6, [(2048, 2048), (2048, 5504), (5504, 2048)]
    host_w = [[W.gaussian(r * c, 0.02, 900 + 10 * k + j) for j, (r, c) in enumerate(shapes)] for k in range(layers)]
    srcs = [[torch.from_numpy(w.view(np.int16)).cuda() for w in lw] for lw in host_w]
    flat = [s for ls in srcs for s in ls]
    params, streams = compress_all(torch, enec, flat)
    # the streams the pipeline reads are the oracle's
    for i in (0, 7, 17):
        w = flat[i].cpu().numpy().view(np.uint16)
        rc, s = oracle.compress(w, params[i], 16384)
        assert rc == oracle.OK and np.array_equal(s, streams[i].cpu().numpy()), i
    hdrs = [s[:64].cpu().numpy().tobytes() for s in streams]
    slots = [[torch.full((r * c,), 0x5A5A, dtype=torch.int16, device="cuda") for r, c in shapes] for _ in range(2)]
    items = [enec.make_decompress_items(streams[3 * k:3 * k + 3], hdrs[3 * k:3 * k + 3], slots[k % 2])
             for k in range(layers)]
    x = torch.randn(64, 2048, device="cuda", dtype=torch.bfloat16)

    def consume(ws):         # ws: three int16 tensors holding bf16 bit patterns
        a, b, c = [w.view(torch.bfloat16).view(r, cc) for w, (r, cc) in zip(ws, shapes)]
        return ((x @ a) @ b) @ c

    want = [consume(srcs[k]).clone() for k in range(layers)]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    main = torch.cuda.current_stream()
    pipe = enec.Pipeline(2, side, trace=True)
    got = []
    side.wait_stream(main)
    assert pipe.prefetch(0, items[0][0]) == enec.OK
    for k in range(layers):
        if k + 1 < layers:
            assert pipe.prefetch((k + 1) % 2, items[k + 1][0]) == enec.OK
        assert pipe.acquire(k % 2, main) == enec.OK
        got.append(consume(slots[k % 2]))
        assert pipe.release(k % 2, main) == enec.OK
    torch.cuda.synchronize()
    for k in range(layers):
        assert torch.equal(got[k], want[k]), f"layer {k}: consumer saw other weights than the original ones"
    t = pipe.trace()
    assert t.shape == (layers, 4) and (t[:, 0] == -1).all() and (t[:, 2] <= t[:, 3]).all()
    pipe.close()
