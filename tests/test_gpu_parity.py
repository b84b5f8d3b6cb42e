"""GPU parity: libenec (through its C ABI) against the CPU oracle, byte for byte.

The compressed stream is a pure function of (input, params, block size), so the GPU
stream must equal the oracle's stream exactly, and both decompressors must give back
the input bit for bit.  Integer / byte work only: the bar is bit-exact everywhere.
"""
import numpy as np
import pytest

from paper_2604_03298_amd import workloads as W

pytestmark = pytest.mark.gpu

STATE_AT = 1024 + 16 * 2048     # workspace: control records, sixteen histogram slots, then the scan state



@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2604_03298_amd import enec
    assert torch.cuda.is_available(), "these tests need the MI355X"
    enec.lib()      # raises if libenec.so is missing: there is no fallback

    class G:
        pass
    g = G()
    g.torch, g.enec = torch, enec
    g.ws = enec.new_workspace(1 << 28)
    g.size_pinned = torch.zeros(1, dtype=torch.int64).pin_memory()

    def to_dev(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda() if a.size else \
            torch.empty(8, dtype=torch.int16, device="cuda")

    def compress(w, params, B=0, src=None):
        src = to_dev(w) if src is None else src
        cap = enec.compress_bound(w.size, block_size=B)
        out = torch.full((cap + 64,), 0xA5, dtype=torch.uint8, device="cuda")   # poison
        g.size_pinned.fill_(-1)
        rc = enec.compress(src, params, out, g.ws, block_size=B, out_bytes=g.size_pinned, n_elems=w.size)
        torch.cuda.synchronize()
        return rc, out.cpu().numpy(), int(g.size_pinned.item()), cap

    def decompress(stream, n, with_header=True):
        buf = torch.from_numpy(np.ascontiguousarray(stream)).cuda()
        out = torch.full((max(n, 8),), 0x5A5A, dtype=torch.int16, device="cuda")
        if with_header:
            rc = enec.decompress_with_header(buf, stream[:64].tobytes(), out, n_elems=n)
        else:
            rc = enec.decompress(buf, out, n_elems=n)
        torch.cuda.synchronize()
        return rc, out.cpu().numpy().view(np.uint16)[:n]

    g.to_dev, g.compress, g.decompress = to_dev, compress, decompress
    return g


def check_both_ways(gpu, oracle, w, params, B=0, label=""):
    Bo = B if B else oracle.default_block(w.size)
    rc_o, s_o = oracle.compress(w, params, Bo)
    assert rc_o == oracle.OK, label
    rc, out, nbytes, cap = gpu.compress(w, params, B)
    assert rc == 0, label
    assert nbytes == s_o.size, f"{label}: size {nbytes} vs oracle {s_o.size}"
    assert np.array_equal(out[:nbytes], s_o), f"{label}: compressed stream differs from the oracle's"
    assert (out[cap:] == 0xA5).all(), f"{label}: wrote past the bound"
    rc, d = gpu.decompress(s_o, w.size)                     # GPU decodes the oracle's stream
    assert rc == 0 and np.array_equal(d, w), f"{label}: GPU decompress(oracle stream) != input"
    rc_d, d_o = oracle.decompress(out[:nbytes], w.size)     # oracle decodes the GPU's stream
    assert rc_d == 0 and np.array_equal(d_o, w), label
    return s_o


def in_window_tensor(rng, b, n, size, quiet_frac=0.6, m=0):
    lo, hi = max(0, b - (1 << (n - 1)) + 1), min(255, b + (1 << (n - 1)))
    x = rng.integers(lo, hi + 1, size=size).astype(np.uint16)
    groups = size // 16
    quiet = np.nonzero(rng.random(groups) < quiet_frac)[0]
    small = max(1, min(1 << m, 1 << (n - 1), b - lo + 1))
    for g in quiet:
        x[g * 16:(g + 1) * 16] = b - rng.integers(0, small, size=16)
    return ((rng.integers(0, 2, size=size).astype(np.uint16) << 15) | (x << 7)
            | rng.integers(0, 128, size=size).astype(np.uint16)).astype(np.uint16)


def test_config1_full(gpu, oracle):
    w = W.config1()
    params = oracle.tune(w)
    s = check_both_ways(gpu, oracle, w, params, 16384, "config1")
    assert 1.33 < 2 * w.size / s.size < 1.40


@pytest.mark.parametrize("n", range(1, 9))
def test_every_width_pair(gpu, oracle, n):
    rng = np.random.default_rng(900 + n)
    for m in range(0, n + 1):
        for B, size in [(2048, 3 * 2048 + 517), (16384, 2 * 16384 + 4099)]:
            w = in_window_tensor(rng, 128, n, size, m=m)
            check_both_ways(gpu, oracle, w, (128, n, m, 16), B, f"n={n} m={m} B={B}")


@pytest.mark.parametrize("B", [2048, 4096, 8192, 16384, 32768])
def test_block_sizes(gpu, oracle, B):
    w = W.gaussian(7 * B + 1234, 0.02, 31 + B)
    check_both_ways(gpu, oracle, w, oracle.tune(w), B, f"B={B}")
    w = W.gaussian(3 * B, 0.02, 32 + B)                     # no ragged tail
    check_both_ways(gpu, oracle, w, oracle.tune(w), B, f"B={B} exact")


@pytest.mark.parametrize("n_elems", [0, 1, 7, 8, 15, 16, 17, 2047, 2048, 2049, 16383, 16384, 16385, 50001])
def test_ragged_and_tiny(gpu, oracle, n_elems):
    w = W.gaussian(n_elems, 0.02, 2000 + n_elems) if n_elems else np.zeros(0, np.uint16)
    assert gpu.enec.default_block_size(n_elems) == oracle.default_block(n_elems)
    check_both_ways(gpu, oracle, w, oracle.tune(w), 0, f"n_elems={n_elems}")


def test_window_at_the_ends_of_the_exponent_range(gpu, oracle):
    rng = np.random.default_rng(5)
    for (b, n, m) in [(3, 6, 2), (0, 1, 0), (0, 4, 1), (250, 6, 3), (255, 3, 1), (255, 8, 4),
                      (0, 8, 3), (127, 8, 4), (128, 8, 0), (100, 8, 8), (31, 6, 3), (223, 6, 3),
                      (30, 6, 3), (224, 6, 3)]:
        w = in_window_tensor(rng, b, n, 2 * 16384 + 77, m=m)
        check_both_ways(gpu, oracle, w, (b, n, m, 16), 16384, f"b={b} n={n} m={m}")


def test_config2_reduced_and_norm_vectors(gpu, oracle):
    for name, w in W.config2(hidden=1024, ffn=2752):
        check_both_ways(gpu, oracle, w, oracle.tune(w), 0, name)


def test_config3_edge_mix(gpu, oracle):
    w, cat = W.config3(n_blocks=256)
    p = oracle.tune(w)
    check_both_ways(gpu, oracle, w, p, 16384, "mix")
    for c, t in enumerate(W.config3_by_category(n_blocks=256)):
        check_both_ways(gpu, oracle, t, oracle.tune(t), 16384, f"category {c}")


def test_special_bit_patterns(gpu, oracle):
    specials = np.array([0x0000, 0x8000, 0x7F80, 0xFF80, 0x7FC0, 0xFFFF, 0x7F81, 0x0001, 0x807F,
                         0x0080, 0x3F80, 0xBF80], np.uint16)
    w = np.tile(specials, 5000)
    check_both_ways(gpu, oracle, w, oracle.tune(w), 0, "specials")
    w = np.full(40000, 0xFFFF, np.uint16)
    check_both_ways(gpu, oracle, w, oracle.tune(w), 0, "all ones")


def test_range_error_is_reported_in_the_header(gpu, oracle):
    w = W.gaussian(5 * 16384, 0.02, 77)
    for params in [(122, 3, 1, 16), (3, 4, 2, 16), (250, 5, 2, 16)]:
        rc_o, s_o = oracle.compress(w, params, 16384)
        assert rc_o == oracle.E_RANGE
        rc, out, nbytes, cap = gpu.compress(w, params, 16384)
        assert rc == 0 and nbytes == 0
        assert np.array_equal(out[:64], s_o[:64])
        info = gpu.enec.stream_info(out[:64])
        assert info["status"] == gpu.enec.E_RANGE and info["total_bytes"] == 0
        rc, d = gpu.decompress(out, w.size)
        assert rc == gpu.enec.E_FORMAT
    # a single offending element in the last block is enough
    w = W.gaussian(3 * 16384, 0.02, 78)
    p = oracle.tune(w)
    w[-1] = 0x7F80
    assert gpu.compress(w, p, 16384)[2] == 0


def test_workspace_is_reusable_and_results_are_deterministic(gpu, oracle):
    big = W.gaussian(300 * 16384 + 5, 0.02, 81)
    small = W.gaussian(3 * 16384, 0.01, 82)
    pb, ps = oracle.tune(big), oracle.tune(small)
    sb, ss = oracle.compress(big, pb, 16384)[1], oracle.compress(small, ps, 16384)[1]
    src_b, src_s = gpu.to_dev(big), gpu.to_dev(small)
    for i in range(6):
        rc, out, nbytes, _ = gpu.compress(big, pb, 16384, src=src_b)
        assert rc == 0 and nbytes == sb.size and np.array_equal(out[:nbytes], sb), f"run {i}"
        rc, out, nbytes, _ = gpu.compress(small, ps, 16384, src=src_s)
        assert rc == 0 and nbytes == ss.size and np.array_equal(out[:nbytes], ss), f"run {i}"
    # the ticket counter of every class has come back to the base the next call will read; nobody gave up
    ws_host = gpu.ws.cpu().numpy()
    ctl = ws_host[:1024].view(np.uint32).reshape(8, 32)
    assert (ctl[:, 0] == ctl[:, 1]).all()
    assert len(set(ctl[:, 2].tolist())) == 1
    assert ctl[0, 4] == 0 and ctl[0, 5] == 0
    # every group accumulator (the first ninth of the state words) is back to zero
    words = ws_host[STATE_AT:STATE_AT + (ws_host.size - STATE_AT) // 8 * 8].view(np.uint64)
    assert (words[:words.size // 9] == 0).all()


def _test_library_compress(enec, src, n, params, out, ws, size):
    """enec_compress of libenec_test.so (the library built with ENEC_TEST_HOOKS: it reads ENEC_SPIN_LIMIT)."""
    import ctypes as C
    import os
    path = os.path.join(os.path.dirname(enec.LIB_PATH), "libenec_test.so")
    assert os.path.exists(path), "build libenec_test.so with `python -m paper_2604_03298_amd.build`"
    L = C.CDLL(path)
    L.enec_compress.restype = C.c_int
    L.enec_compress.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_uint32, C.POINTER(enec.Params), C.c_void_p,
                                C.c_size_t, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    return L.enec_compress(src.data_ptr(), n, 0, 0, C.byref(enec.Params(*params)), out.data_ptr(), out.numel(),
                           size.data_ptr(), ws.data_ptr(), ws.numel(), None)


def test_dirty_workspace_ends_in_a_status_not_in_a_hang(gpu, oracle, monkeypatch):
    """A workspace left dirty (a process died in the middle of a call) must not hang the scan: the
    waits are bounded and the stream header then says ENEC_E_HIP.  The bound is shortened through
    the test build of the library so that the kernel gives up after microseconds."""
    torch, enec = gpu.torch, gpu.enec
    w = W.gaussian(400 * 16384, 0.02, 83)               # more than 256 blocks: the scan goes through group words
    p = oracle.tune(w)
    src = gpu.to_dev(w)
    ws = enec.new_workspace(w.size)
    words = ws[STATE_AT:STATE_AT + (ws.numel() - STATE_AT) // 8 * 8].view(torch.int64)
    words[:words.numel() // 9] = 100 << 48            # accumulators claim 100 blocks too many: no group ever completes
    out = torch.zeros(enec.compress_bound(w.size), dtype=torch.uint8, device="cuda")
    size = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    monkeypatch.setenv("ENEC_SPIN_LIMIT", "200")
    assert _test_library_compress(enec, src, w.size, p, out, ws, size) == 0
    torch.cuda.synchronize()
    monkeypatch.delenv("ENEC_SPIN_LIMIT")
    info = enec.stream_info(out[:64].cpu().numpy())
    assert info["status"] == enec.E_HIP and info["total_bytes"] == 0 and int(size.item()) == 0
    enec.workspace_init(ws)                              # the documented way out
    assert enec.compress(src, p, out, ws, out_bytes=size) == 0
    torch.cuda.synchronize()
    s_o = oracle.compress(w, p, 16384)[1]
    assert int(size.item()) == s_o.size and np.array_equal(out[:s_o.size].cpu().numpy(), s_o)


def test_a_wait_given_up_anywhere_shows_in_the_header(gpu, oracle, monkeypatch):
    """With a bound of one poll, blocks in the middle of a tensor give up on predecessors that publish a moment
    later, while the last block may find everything in place.  Whoever gives up leaves a mark that the writer of
    the header sees: a run ends either with status 0 and the oracle's stream, or with ENEC_E_HIP and size 0,
    never with status 0 and a misplaced payload.  (Every kernel exits normally; nothing hangs or faults.)"""
    torch, enec = gpu.torch, gpu.enec
    w = W.gaussian(2000 * 16384 + 77, 0.02, 84)
    p = oracle.tune(w)
    s_o = oracle.compress(w, p, 16384)[1]
    ref = torch.from_numpy(s_o).cuda()
    src = gpu.to_dev(w)
    ws = enec.new_workspace(w.size)
    out = torch.zeros(enec.compress_bound(w.size), dtype=torch.uint8, device="cuda")
    size = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    monkeypatch.setenv("ENEC_SPIN_LIMIT", "1")
    outcomes = []
    for _ in range(8):
        out.zero_()
        assert _test_library_compress(enec, src, w.size, p, out, ws, size) == 0
        torch.cuda.synchronize()
        info = enec.stream_info(out[:64].cpu().numpy())
        if info["status"] == 0:
            assert int(size.item()) == s_o.size and torch.equal(out[:s_o.size], ref)
        else:
            assert info["status"] == enec.E_HIP and info["total_bytes"] == 0 and int(size.item()) == 0
            enec.workspace_init(ws)        # a call that gave up may leave accumulators behind
            torch.cuda.synchronize()
        outcomes.append(info["status"])
    monkeypatch.delenv("ENEC_SPIN_LIMIT")
    # and the ordinary library on the same workspace afterwards
    enec.workspace_init(ws)
    assert enec.compress(src, p, out, ws, out_bytes=size) == 0
    torch.cuda.synchronize()
    assert int(size.item()) == s_o.size and torch.equal(out[:s_o.size], ref), outcomes


def test_back_to_back_calls_without_sync(gpu, oracle):
    torch, enec = gpu.torch, gpu.enec
    tensors = [W.gaussian(n, 0.02, 90 + i) for i, n in enumerate([70000, 16384 * 40, 4096, 16384 * 9 + 1])]
    params = [oracle.tune(t) for t in tensors]
    srcs = [gpu.to_dev(t) for t in tensors]
    outs = [torch.zeros(enec.compress_bound(t.size), dtype=torch.uint8, device="cuda") for t in tensors]
    sizes = torch.zeros(len(tensors), dtype=torch.int64, device="cuda")
    for i, t in enumerate(tensors):
        assert enec.compress(srcs[i], params[i], outs[i], gpu.ws, out_bytes=sizes[i:i + 1], n_elems=t.size) == 0
    torch.cuda.synchronize()
    for i, t in enumerate(tensors):
        s_o = oracle.compress(t, params[i], oracle.default_block(t.size))[1]
        assert int(sizes[i]) == s_o.size
        assert np.array_equal(outs[i].cpu().numpy()[:s_o.size], s_o)
    # and decompress all of them back to back
    backs = [torch.zeros(max(t.size, 8), dtype=torch.int16, device="cuda") for t in tensors]
    for i, t in enumerate(tensors):
        hdr = outs[i][:64].cpu().numpy()
        assert enec.decompress_with_header(outs[i], hdr.tobytes(), backs[i], n_elems=t.size) == 0
    torch.cuda.synchronize()
    for i, t in enumerate(tensors):
        assert np.array_equal(backs[i].cpu().numpy().view(np.uint16)[:t.size], t)


def test_random_shapes_and_parameters(gpu, oracle):
    rng = np.random.default_rng(2024)
    for case in range(40):
        B = int(rng.choice([2048, 4096, 8192, 16384, 32768]))
        size = int(rng.integers(1, 12 * B))
        n = int(rng.integers(1, 9))
        m = int(rng.integers(0, n + 1))
        half = 1 << (n - 1)
        b = int(rng.integers(0, 256)) if n == 8 else int(rng.integers(max(0, half - 1), 256 - half + 1))
        if case % 5 == 0:                        # windows that touch the ends of the exponent range
            b = int(rng.choice([0, 1, 254, 255]))
        w = in_window_tensor(rng, b, n, size, quiet_frac=float(rng.random()), m=m)
        check_both_ways(gpu, oracle, w, (b, n, m, 16), B, f"case {case}: B={B} size={size} b={b} n={n} m={m}")


def test_config3_full_size(gpu, oracle):
    w, cat = W.config3()
    check_both_ways(gpu, oracle, w, oracle.tune(w), 16384, "config3 mix, 64M elements")


def test_two_streams_two_workspaces(gpu, oracle):
    torch, enec = gpu.torch, gpu.enec
    tensors = [W.gaussian(16384 * 200 + 3, 0.02, 700), W.gaussian(16384 * 150 + 11, 0.01, 701)]
    params = [oracle.tune(t) for t in tensors]
    refs = [oracle.compress(t, p, 16384)[1] for t, p in zip(tensors, params)]
    srcs = [gpu.to_dev(t) for t in tensors]
    outs = [torch.zeros(enec.compress_bound(t.size), dtype=torch.uint8, device="cuda") for t in tensors]
    backs = [torch.zeros(t.size, dtype=torch.int16, device="cuda") for t in tensors]
    wss = [enec.new_workspace(t.size) for t in tensors]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(5):
        for i in range(2):
            assert enec.compress(srcs[i], params[i], outs[i], wss[i], stream=streams[i]) == 0
        for i in range(2):
            assert enec.decompress_with_header(outs[i], refs[i][:64].tobytes(), backs[i], stream=streams[i]) == 0
        torch.cuda.synchronize()
        for i in range(2):
            assert np.array_equal(outs[i].cpu().numpy()[:refs[i].size], refs[i]), (rep, i)
            assert np.array_equal(backs[i].cpu().numpy().view(np.uint16), tensors[i]), (rep, i)


def test_two_full_grids_at_once(gpu, oracle, monkeypatch):
    """Two compressions whose persistent grids each fill the device run on two streams: the device cannot hold
    both grids, workgroups of either kernel start late.  Every block is drawn from a ticket counter, so a late
    workgroup never owns a block that running ones wait for.  (The wait bound is lowered so that a regression
    would end in a header status within milliseconds instead of seconds.)"""
    torch, enec = gpu.torch, gpu.enec
    monkeypatch.setenv("ENEC_SPIN_LIMIT", "20000")
    tensors = [W.gaussian(16384 * 1500 + 3, 0.02, 710), W.gaussian(16384 * 1300 + 11, 0.01, 711)]
    params = [oracle.tune(t) for t in tensors]
    refs = [oracle.compress(t, p, 16384)[1] for t, p in zip(tensors, params)]
    srcs = [gpu.to_dev(t) for t in tensors]
    outs = [torch.zeros(enec.compress_bound(t.size), dtype=torch.uint8, device="cuda") for t in tensors]
    wss = [enec.new_workspace(t.size) for t in tensors]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(4):
        for _ in range(3):                       # several launches per stream keep both queues busy
            for i in range(2):
                assert enec.compress(srcs[i], params[i], outs[i], wss[i], stream=streams[i]) == 0
        torch.cuda.synchronize()
        for i in range(2):
            got = outs[i][:refs[i].size].cpu().numpy()
            assert enec.stream_info(got[:64])["status"] == 0, (rep, i)
            assert np.array_equal(got, refs[i]), (rep, i)


def test_batch_entry_points(gpu, oracle):
    torch, enec = gpu.torch, gpu.enec
    rng = np.random.default_rng(123)
    # tensors of several shapes and parameter tuples, empty and single-block ones included
    tensors = [W.gaussian(16384 * 70 + 9, 0.02, 301), W.norm_vector(4096, 27), W.gaussian(16384 * 3, 0.02, 302),
               W.gaussian(40000, 0.3, 303), np.zeros(0, np.uint16), W.norm_vector(4096, 28),
               in_window_tensor(rng, 128, 8, 16384 * 5 + 1, m=4), W.gaussian(16384 * 33 + 100, 0.02, 304),
               np.zeros(50000, np.uint16), W.gaussian(2049, 0.02, 305)]
    params = [oracle.tune(t) for t in tensors]
    params[6] = (128, 8, 4, 16)
    srcs = [gpu.to_dev(t) for t in tensors]
    outs = [torch.full((enec.compress_bound(t.size),), 0x5A, dtype=torch.uint8, device="cuda") for t in tensors]
    sizes = [torch.zeros(1, dtype=torch.int64, device="cuda") for _ in tensors]
    total = sum(t.size for t in tensors)
    ws = enec.new_workspace(total)
    class Shim:          # compress_batch takes numel() from the tensor: empty tensors are padded on the device
        def __init__(self, t, n): self.t, self.n = t, n
        def data_ptr(self): return self.t.data_ptr()
        def numel(self): return self.n
    shims = [Shim(srcs[i], tensors[i].size) for i in range(len(tensors))]
    for rep in range(3):
        assert enec.compress_batch(shims, params, outs, ws, out_bytes=sizes) == 0
        torch.cuda.synchronize()
        for i, t in enumerate(tensors):
            s_o = oracle.compress(t, params[i], oracle.default_block(t.size))[1]
            assert int(sizes[i]) == s_o.size, (rep, i)
            assert np.array_equal(outs[i].cpu().numpy()[:s_o.size], s_o), (rep, i)
    backs = [torch.full((max(t.size, 8),), 0x1111, dtype=torch.int16, device="cuda") for t in tensors]
    hdrs = [outs[i][:64].cpu().numpy().tobytes() for i in range(len(tensors))]
    bshims = [Shim(backs[i], tensors[i].size) for i in range(len(tensors))]
    assert enec.decompress_batch(outs, hdrs, bshims) == 0
    torch.cuda.synchronize()
    for i, t in enumerate(tensors):
        assert np.array_equal(backs[i].cpu().numpy().view(np.uint16)[:t.size], t), i
    # one item with a range error does not disturb the others
    bad_params = list(params)
    bad_params[2] = (122, 3, 1, 16)
    assert enec.compress_batch(shims, bad_params, outs, ws, out_bytes=sizes) == 0
    torch.cuda.synchronize()
    assert int(sizes[2]) == 0 and enec.stream_info(outs[2][:64].cpu().numpy())["status"] == enec.E_RANGE
    for i in (0, 3, 7):
        s_o = oracle.compress(tensors[i], params[i], oracle.default_block(tensors[i].size))[1]
        assert np.array_equal(outs[i].cpu().numpy()[:s_o.size], s_o), i
    # more than 16 tensors of one kind: several launches
    many = [W.gaussian(16384 + 7 * j, 0.02, 400 + j) for j in range(20)]
    msrc = [gpu.to_dev(t) for t in many]
    mout = [torch.zeros(enec.compress_bound(t.size), dtype=torch.uint8, device="cuda") for t in many]
    msz = [torch.zeros(1, dtype=torch.int64, device="cuda") for _ in many]
    assert enec.compress_batch(msrc, [(122, 6, 3, 16)] * 20, mout, ws, out_bytes=msz) == 0
    torch.cuda.synchronize()
    for j, t in enumerate(many):
        s_o = oracle.compress(t, (122, 6, 3, 16), 16384)[1]
        assert int(msz[j]) == s_o.size and np.array_equal(mout[j].cpu().numpy()[:s_o.size], s_o), j


def test_decompress_variants_and_header_mismatch(gpu, oracle):
    w = W.gaussian(5 * 16384 + 3, 0.02, 99)
    p = oracle.tune(w)
    s = oracle.compress(w, p, 16384)[1]
    rc, d = gpu.decompress(s, w.size, with_header=False)          # reads the header itself
    assert rc == 0 and np.array_equal(d, w)
    assert gpu.decompress(s, w.size + 1)[0] == gpu.enec.E_FORMAT
    bad = s.copy(); bad[0] = ord("X")
    assert gpu.decompress(bad, w.size, with_header=False)[0] == gpu.enec.E_FORMAT
    # a host header that does not match the device stream: the kernel must write nothing
    other = oracle.compress(w, (p[0], 8, 4, 16), 16384)[1]
    torch, enec = gpu.torch, gpu.enec
    buf = torch.from_numpy(other).cuda()
    out = torch.full((w.size,), 0x5A5A, dtype=torch.int16, device="cuda")
    assert enec.decompress_with_header(buf, s[:64].tobytes(), out, n_elems=w.size) == 0
    torch.cuda.synchronize()
    assert (out.cpu().numpy() == 0x5A5A).all()
    # a header that claims more bytes than the buffer holds is refused on the host
    assert enec.decompress_with_header(torch.from_numpy(s).cuda(), other[:64].tobytes(), out,
                                       n_elems=w.size) == enec.E_FORMAT


def test_damaged_offset_table_skips_blocks_and_stays_in_bounds(gpu, oracle):
    """Offsets come from the stream: entries that point outside it, go backwards, are misaligned or imply an
    impossible size make the kernel leave that block's output alone; the other blocks are exact and nothing
    outside the output tensor is written."""
    torch, enec = gpu.torch, gpu.enec
    B = 16384
    w = W.gaussian(12 * B + 1000, 0.02, 98)
    s = oracle.compress(w, oracle.tune(w), B)[1]
    nb = 13
    table = s[64:64 + 8 * (nb + 1)].view("<u8").copy()
    damaged = {}
    for k, how in ((2, "huge"), (5, "backwards"), (8, "misaligned"), (10, "too_long")):
        t = table.copy()
        if how == "huge":
            t[k] = np.uint64(1) << np.uint64(40)
        elif how == "backwards":
            t[k + 1] = t[k] - np.uint64(16)
        elif how == "misaligned":
            t[k] += np.uint64(8)
        else:
            t[k + 1] = t[k] + np.uint64(4 * B)
        damaged[how] = (k, t)
    # the undamaged stream leaves the status word alone (device memory and pinned host memory)
    for status in (torch.zeros(1, dtype=torch.int32, device="cuda"), torch.zeros(1, dtype=torch.int32).pin_memory()):
        out = torch.full((w.size,), 0x5A5A, dtype=torch.int16, device="cuda")
        assert enec.decompress_with_header(torch.from_numpy(s).cuda(), s[:64].tobytes(), out, status=status) == 0
        torch.cuda.synchronize()
        assert int(status.item()) == 0 and np.array_equal(out.cpu().numpy().view(np.uint16), w)
    for how, (k, t) in damaged.items():
        bad = s.copy()
        bad[64:64 + 8 * (nb + 1)] = t.view(np.uint8)
        buf = torch.from_numpy(bad).cuda()
        out = torch.full((w.size + 64,), 0x5A5A, dtype=torch.int16, device="cuda")
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        assert enec.decompress_with_header(buf, bad[:64].tobytes(), out, n_elems=w.size, status=status) == 0
        torch.cuda.synchronize()
        assert int(status.item()) == enec.E_FORMAT, how          # the caller is told that blocks were skipped
        got = out.cpu().numpy().view(np.uint16)
        assert (got[w.size:] == 0x5A5A).all(), how
        # entry k starts block k and ends block k - 1; entry k + 1 ends block k and starts block k + 1
        touched = {k, k - 1} if how in ("huge", "misaligned") else {k, k + 1}
        for blk in range(nb):
            seg = slice(blk * B, min(w.size, (blk + 1) * B))
            if blk in touched:
                assert (got[seg] == 0x5A5A).all() or np.array_equal(got[seg], w[seg]), (how, blk)
            else:
                assert np.array_equal(got[seg], w[seg]), (how, blk)
        assert any((got[blk * B:min(w.size, (blk + 1) * B)] == 0x5A5A).all() for blk in touched), how


def test_tuner_matches_oracle(gpu, oracle):
    cases = [W.config1(), W.gaussian(100003, 0.003, 5), np.zeros(70000, np.uint16),
             np.full(33333, 0x3D12, np.uint16), W.config3(n_blocks=64)[0],
             W.layer_matrix(512, 1376, 24), W.norm_vector(4096, 27), W.gaussian(5, 0.02, 1)]
    for i, w in enumerate(cases):
        params, hist = gpu.enec.tune(gpu.to_dev(w), gpu.ws, want_histogram=True)
        assert np.array_equal(hist, oracle.histogram(w)), f"case {i}"
        assert params == oracle.tune(w), f"case {i}"
    # params = None: tune inside enec_compress
    w = cases[0]
    torch, enec = gpu.torch, gpu.enec
    out = torch.zeros(enec.compress_bound(w.size), dtype=torch.uint8, device="cuda")
    assert enec.compress(gpu.to_dev(w), None, out, gpu.ws, out_bytes=gpu.size_pinned) == 0
    torch.cuda.synchronize()
    s_o = oracle.compress(w, oracle.tune(w), 16384)[1]
    assert np.array_equal(out.cpu().numpy()[:s_o.size], s_o)


def test_host_argument_errors_on_device_pointers(gpu):
    torch, enec = gpu.torch, gpu.enec
    src = torch.zeros(16384, dtype=torch.int16, device="cuda")
    out = torch.zeros(enec.compress_bound(16384), dtype=torch.uint8, device="cuda")
    assert enec.compress(src, (122, 6, 3, 16), out[:1000], gpu.ws) == enec.E_CAPACITY
    assert enec.compress(src, (122, 6, 3, 16), out, gpu.ws, block_size=3000) == enec.E_BLOCK
    assert enec.compress(src, (122, 9, 3, 16), out, gpu.ws) == enec.E_PARAMS
    assert enec.compress(src, (122, 6, 3, 12), out, gpu.ws) == enec.E_PARAMS
    assert enec.compress(src[1:], (122, 6, 3, 16), out, gpu.ws, n_elems=100) == enec.E_ARG   # misaligned
    pageable = torch.zeros(1, dtype=torch.int64)
    assert enec.compress(src, (122, 6, 3, 16), out, gpu.ws, out_bytes=pageable) == enec.E_ARG


def test_full_size_layer_and_large_tensor(gpu, oracle):
    # configuration 2 at full size (the benchmark workload), whole streams compared
    for name, w in W.config2():
        check_both_ways(gpu, oracle, w, oracle.tune(w), 0, name)
    # one tensor of the large-layer stream (8192 x 28672)
    w = W.config4_tensor(0)
    check_both_ways(gpu, oracle, w, oracle.tune(w), 16384, "config4[0]")


def test_tensor_beyond_4_gib_sampled_against_the_oracle(gpu, oracle):
    """2.6e9 elements (5.2 GB of bf16): element and byte offsets beyond 32 bits.  The round trip is compared
    on the device; blocks sampled along the tensor are recompressed by the oracle one group of blocks at a
    time, and their payloads must be the bytes the library wrote at the offsets its table gives."""
    torch, enec = gpu.torch, gpu.enec
    from paper_2604_03298_amd.workloads import gpu_gaussian
    rows, cols = 90000, 28672 + 231          # not a multiple of the block size: ragged tail
    src = gpu_gaussian(torch, rows, cols, 0.02, 4242)
    n = src.numel()
    assert 2 * n > (1 << 32)
    ws = enec.new_workspace(n)
    prm = enec.tune(src, ws)
    out = torch.empty(enec.compress_bound(n), dtype=torch.uint8, device="cuda")
    size = torch.zeros(1, dtype=torch.int64, device="cuda")
    assert enec.compress(src, prm, out, ws, out_bytes=size) == 0
    torch.cuda.synchronize()
    total = int(size.item())
    assert 0 < total < 2 * n
    back = torch.empty_like(src)
    assert enec.decompress_with_header(out, out[:64].cpu().numpy().tobytes(), back) == 0
    torch.cuda.synchronize()
    assert torch.equal(back, src)
    del back
    B = 16384
    nb = (n + B - 1) // B
    base = oracle.payload_base(n, B)
    table = out[64:64 + 8 * (nb + 1)].cpu().numpy().view("<u8")
    assert table[0] == 0 and int(table[nb]) + base == total and (np.diff(table.astype(np.int64)) > 0).all()
    for k0 in (0, 1234, nb // 2, (1 << 32) // (2 * B) + 5, nb - 3):           # incl. the blocks around byte 2^32 and the tail
        cnt = min(3, nb - k0)
        w = src[k0 * B:min(n, (k0 + cnt) * B)].cpu().numpy().view(np.uint16)
        rc, s = oracle.compress(w, prm, B)
        assert rc == 0
        ob = oracle.payload_base(w.size, B)
        got = out[base + int(table[k0]):base + int(table[k0 + cnt])].cpu().numpy()
        assert got.size == s.size - ob and np.array_equal(got, s[ob:]), k0


def test_batches_with_single_block_tensors(gpu, oracle):
    """A layer's tiny tensors (one data block each, tuples of their own) beside matrices, in one batch call, with
    status words for the decoder: same streams as the oracle's, same round trip, also when the calls are repeated
    back to back without synchronisation, and also when the batch has only tiny tensors or none."""
    torch, enec = gpu.torch, gpu.enec
    tensors = [W.layer_matrix(512, 1376, 24), W.norm_vector(4096, 27), W.layer_matrix(1376, 512, 26),
               W.norm_vector(4096, 28), W.gaussian(3000, 0.5, 29), W.gaussian(16384, 0.02, 30)]
    params = [oracle.tune(t) for t in tensors]
    assert len({p[:3] for p in params}) >= 3
    refs = [oracle.compress(t, p, oracle.default_block(t.size))[1] for t, p in zip(tensors, params)]
    srcs = [gpu.to_dev(t) for t in tensors]
    for pick in (list(range(6)), [1, 3, 4], [0, 2]):
        outs = [torch.full((enec.compress_bound(tensors[i].size),), 0xA5, dtype=torch.uint8, device="cuda") for i in pick]
        sizes = torch.zeros(len(pick), dtype=torch.int64, device="cuda")
        for rep in range(3):
            rc = enec.compress_batch([srcs[i] for i in pick], [params[i] for i in pick], outs, gpu.ws,
                                     out_bytes=[sizes[j:j + 1] for j in range(len(pick))])
            assert rc == 0, enec.strerror(rc)
        torch.cuda.synchronize()
        for j, i in enumerate(pick):
            assert int(sizes[j]) == refs[i].size, (pick, i)
            assert np.array_equal(outs[j].cpu().numpy()[:refs[i].size], refs[i]), (pick, i)
        backs = [torch.full((tensors[i].size,), 0x5A5A, dtype=torch.int16, device="cuda") for i in pick]
        status = [torch.zeros(1, dtype=torch.int32, device="cuda") for _ in pick]
        for rep in range(3):
            rc = enec.decompress_batch(outs, [refs[i][:64] for i in pick], backs, statuses=status)
            assert rc == 0, enec.strerror(rc)
        torch.cuda.synchronize()
        for j, i in enumerate(pick):
            assert int(status[j].item()) == 0
            assert np.array_equal(backs[j].cpu().numpy().view(np.uint16), tensors[i]), (pick, i)


def test_header_mismatch_sets_the_status_word(gpu, oracle):
    torch, enec = gpu.torch, gpu.enec
    w = W.gaussian(5 * 16384, 0.02, 97)
    s = oracle.compress(w, oracle.tune(w), 16384)[1]
    other = s.copy()
    other[24] ^= 1                                   # a header with another b: valid in itself, not the stream's
    out = torch.full((w.size,), 0x5A5A, dtype=torch.int16, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert enec.decompress_with_header(torch.from_numpy(s).cuda(), other[:64].tobytes(), out, status=status) == 0
    torch.cuda.synchronize()
    assert int(status.item()) == enec.E_FORMAT and (out == 0x5A5A).all()
