"""The codec calls can be captured into a HIP graph and replayed (serving loops do that): no allocation, no
memset, no synchronisation happens inside enec_compress_batch / enec_decompress_batch once the occupancy
figures are cached.  Every replay is checked against the eager result, with eager work between replays."""
import numpy as np
import pytest

from paper_2604_03298_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_compress_and_decompress_replay_from_a_graph(oracle):
    import torch
    from paper_2604_03298_amd import enec
    enec.lib()
    tensors = [W.gaussian(20 * 16384 + 77, 0.02, 91), W.gaussian(5 * 16384, 0.02, 92), W.gaussian(3000, 0.3, 93)]
    params = [oracle.tune(t) for t in tensors]
    want = [oracle.compress(t, p, oracle.default_block(t.size))[1] for t, p in zip(tensors, params)]
    srcs = [torch.from_numpy(t.view(np.int16)).cuda() for t in tensors]
    outs = [torch.zeros(enec.compress_bound(t.size), dtype=torch.uint8, device="cuda") for t in tensors]
    backs = [torch.zeros_like(s) for s in srcs]
    sizes = [torch.zeros(1, dtype=torch.int64, device="cuda") for _ in tensors]
    ws = enec.new_workspace(sum(t.size for t in tensors))
    hdrs = [w[:64].tobytes() for w in want]
    items, keep = enec.make_decompress_items(outs, hdrs, backs)

    def step():
        assert enec.compress_batch(srcs, params, outs, ws, out_bytes=sizes) == 0
        assert enec.decompress_batch(None, None, None, items=items) == 0

    step()                                  # eager: fills the occupancy cache, gives the expected state
    torch.cuda.synchronize()
    for i, t in enumerate(tensors):
        assert int(sizes[i]) == want[i].size and np.array_equal(outs[i][:want[i].size].cpu().numpy(), want[i])
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        step()
        graph.capture_end()
    torch.cuda.synchronize()
    for replay in range(4):
        for o, b, s in zip(outs, backs, sizes):
            o.zero_()
            b.zero_()
            s.zero_()
        if replay % 2:
            step()                          # the program's own eager work between replays
            for o, b in zip(outs, backs):
                o.zero_()
                b.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, t in enumerate(tensors):
            assert int(sizes[i]) == want[i].size, (replay, i)
            assert np.array_equal(outs[i][:want[i].size].cpu().numpy(), want[i]), (replay, i)
            assert np.array_equal(backs[i].cpu().numpy().view(np.uint16), t), (replay, i)


def test_one_tuple_per_block_replays_from_a_graph(oracle):
    """The per-block call clears its look-back words with a fill kernel (no memset), so it can be captured too."""
    import torch
    from paper_2604_03298_amd import enec
    enec.lib()
    rng = np.random.default_rng(5)
    # 262 data blocks, one workgroup each (no multiple of the eight ticket counters), the last one ragged
    t = np.concatenate([W.gaussian(256 * 16384, 0.02, 1), np.zeros(16384, np.uint16),
                        rng.integers(0, 65536, 16384).astype(np.uint16), W.gaussian(3 * 16384 + 55, 0.2, 2)])
    want = oracle.compress_per_block(t, 16384)[1]
    src = torch.from_numpy(t.view(np.int16)).cuda()
    out = torch.zeros(enec.compress_bound_per_block(t.size), dtype=torch.uint8, device="cuda")
    back = torch.zeros_like(src)
    size = torch.zeros(1, dtype=torch.int64, device="cuda")
    ws = enec.new_workspace(t.size)
    hdr = want[:64].tobytes()

    def step():
        assert enec.compress_per_block(src, out, ws, out_bytes=size) == 0
        assert enec.decompress_with_header(out, hdr, back) == 0

    step()
    torch.cuda.synchronize()
    assert int(size) == want.size and np.array_equal(out[:want.size].cpu().numpy(), want)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        step()
        graph.capture_end()
    torch.cuda.synchronize()
    for replay in range(4):
        out.zero_(); back.zero_(); size.zero_()
        if replay % 2:
            step()
            out.zero_(); back.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert int(size) == want.size, replay
        assert np.array_equal(out[:want.size].cpu().numpy(), want), replay
        assert np.array_equal(back.cpu().numpy().view(np.uint16), t), replay
