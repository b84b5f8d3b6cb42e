"""GPU parity for fp16 and fp32 tensors: libenec (through its C ABI) against the CPU oracle, byte for byte."""
import numpy as np
import pytest

from paper_2604_03298_amd import workloads as W

pytestmark = pytest.mark.gpu

BF16, FP16, FP32 = 0, 1, 2
WORD = {BF16: np.uint16, FP16: np.uint16, FP32: np.uint32}


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
    g.ws = enec.new_workspace(1 << 26)
    g.size_pinned = torch.zeros(1, dtype=torch.int64).pin_memory()

    def to_dev(w, dtype):
        view = np.int32 if dtype == FP32 else np.int16
        if w.size == 0:
            return torch.empty(8, dtype=torch.int32 if dtype == FP32 else torch.int16, device="cuda")
        return torch.from_numpy(np.ascontiguousarray(w).view(view)).cuda()

    def compress(w, params, dtype, B=0):
        src = to_dev(w, dtype)
        cap = enec.compress_bound(w.size, dtype=dtype, block_size=B)
        out = torch.full((cap + 64,), 0xA5, dtype=torch.uint8, device="cuda")   # poison
        g.size_pinned.fill_(-1)
        rc = enec.compress(src, params, out, g.ws, block_size=B, out_bytes=g.size_pinned, n_elems=w.size, dtype=dtype)
        torch.cuda.synchronize()
        return rc, out.cpu().numpy(), int(g.size_pinned.item()), cap

    def decompress(stream, n, dtype, with_header=True):
        buf = torch.from_numpy(np.ascontiguousarray(stream)).cuda()
        if dtype == FP32:
            out = torch.full((max(n, 8),), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
        else:
            out = torch.full((max(n, 8),), 0x5A5A, dtype=torch.int16, device="cuda")
        if with_header:
            rc = enec.decompress_with_header(buf, stream[:64].tobytes(), out, n_elems=n)
        else:
            rc = enec.decompress(buf, out, n_elems=n)
        torch.cuda.synchronize()
        return rc, out.cpu().numpy().view(WORD[dtype])[:n], out.cpu().numpy().view(WORD[dtype])[n:]

    g.to_dev, g.compress, g.decompress = to_dev, compress, decompress
    return g


def check_both_ways(gpu, oracle, w, params, dtype, B=0, label=""):
    Bo = B if B else oracle.default_block(w.size)
    rc_o, s_o = oracle.compress(w, params, Bo, dtype=dtype)
    assert rc_o == oracle.OK, label
    rc, out, nbytes, cap = gpu.compress(w, params, dtype, B)
    assert rc == 0, label
    assert nbytes == s_o.size, f"{label}: size {nbytes} vs oracle {s_o.size}"
    bad = np.nonzero(out[:nbytes] != s_o)[0]
    assert bad.size == 0, f"{label}: compressed stream differs from the oracle's, first at byte {bad[:4]}"
    assert (out[cap:] == 0xA5).all(), f"{label}: wrote past the bound"
    rc, d, rest = gpu.decompress(s_o, w.size, dtype)         # GPU decodes the oracle's stream
    assert rc == 0 and np.array_equal(d, w), f"{label}: GPU decompress(oracle stream) != input"
    assert (rest == (0x5A5A5A5A if dtype == FP32 else 0x5A5A)).all(), f"{label}: wrote past the tensor"
    rc_d, d_o = oracle.decompress(out[:nbytes], w.size)      # oracle decodes the GPU's stream
    assert rc_d == 0 and np.array_equal(d_o, w), label
    return s_o


def in_window_words(rng, b, n, size, dtype, quiet_frac=0.6, m=0):
    """Random words whose exponents lie inside the window of (b, n); a share of the groups only uses m bits."""
    E = 5 if dtype == FP16 else 8
    top = (1 << E) - 1
    lo, hi = (0, top) if n == E else (max(0, b - (1 << (n - 1)) + 1), min(top, b + (1 << (n - 1))))
    x = rng.integers(lo, hi + 1, size=size).astype(np.uint32)
    groups = size // 16
    small = max(1, min(1 << m, 1 << (n - 1), b - lo + 1))
    for g in np.nonzero(rng.random(groups) < quiet_frac)[0]:
        x[g * 16:(g + 1) * 16] = b - rng.integers(0, small, size=16)
    sign = rng.integers(0, 2, size=size).astype(np.uint32)
    if dtype == FP16:
        return ((sign << 15) | (x << 10) | rng.integers(0, 1 << 10, size=size).astype(np.uint32)).astype(np.uint16)
    return ((sign << 31) | (x << 23) | rng.integers(0, 1 << 23, size=size).astype(np.uint32)).astype(np.uint32)


@pytest.mark.parametrize("dtype", [FP16, FP32])
def test_gaussian_weights(gpu, oracle, dtype):
    gen = W.gaussian_fp16 if dtype == FP16 else W.gaussian_fp32
    w = gen(1024 * 1024 + 12345, 0.02, 7)
    params = oracle.tune(w, dtype)
    s = check_both_ways(gpu, oracle, w, params, dtype, 16384, f"gaussian dtype {dtype}")
    ratio = w.nbytes / s.size
    assert (1.08 < ratio < 1.14) if dtype == FP16 else (1.14 < ratio < 1.18)
    # the device tuner agrees with the oracle's
    assert gpu.enec.tune(gpu.to_dev(w, dtype), gpu.ws, dtype=dtype) == params


@pytest.mark.parametrize("n", range(1, 6))
def test_fp16_every_width_pair(gpu, oracle, n):
    rng = np.random.default_rng(1900 + n)
    for m in range(0, n + 1):
        for b in (3, 15, 29):
            for B, size in [(2048, 3 * 2048 + 517), (16384, 2 * 16384 + 4099)]:
                w = in_window_words(rng, b, n, size, FP16, m=m)
                check_both_ways(gpu, oracle, w, (b, n, m, 16), FP16, B, f"fp16 b={b} n={n} m={m} B={B}")


@pytest.mark.parametrize("n", range(1, 9))
def test_fp32_every_width_pair(gpu, oracle, n):
    rng = np.random.default_rng(2900 + n)
    for m in range(0, n + 1):
        B, size = [(2048, 3 * 2048 + 517), (16384, 2 * 16384 + 4099)][(n + m) % 2]
        for b in (128, 2, 253):
            w = in_window_words(rng, b, n, size, FP32, m=m)
            check_both_ways(gpu, oracle, w, (b, n, m, 16), FP32, B, f"fp32 b={b} n={n} m={m} B={B}")


@pytest.mark.parametrize("dtype", [FP16, FP32])
@pytest.mark.parametrize("B", [2048, 4096, 8192, 16384, 32768])
def test_block_sizes(gpu, oracle, dtype, B):
    gen = W.gaussian_fp16 if dtype == FP16 else W.gaussian_fp32
    w = gen(5 * B + 1234, 0.02, 31 + B)
    check_both_ways(gpu, oracle, w, oracle.tune(w, dtype), dtype, B, f"dtype {dtype} B={B}")
    w = gen(3 * B, 0.02, 32 + B)
    check_both_ways(gpu, oracle, w, oracle.tune(w, dtype), dtype, B, f"dtype {dtype} B={B} exact")


@pytest.mark.parametrize("dtype", [FP16, FP32])
@pytest.mark.parametrize("n_elems", [0, 1, 3, 4, 7, 8, 9, 15, 16, 17, 2047, 2048, 2049, 16383, 16385, 50001])
def test_ragged_and_tiny(gpu, oracle, dtype, n_elems):
    gen = W.gaussian_fp16 if dtype == FP16 else W.gaussian_fp32
    w = gen(n_elems, 0.02, 2000 + n_elems) if n_elems else np.zeros(0, WORD[dtype])
    params = oracle.tune(w, dtype)
    check_both_ways(gpu, oracle, w, params, dtype, 0, f"dtype {dtype} n_elems={n_elems}")


def test_fp16_all_bit_patterns(gpu, oracle):
    w = np.arange(65536, dtype=np.uint16)
    np.random.default_rng(4).shuffle(w)
    w = np.concatenate([w, w[::-1], w[:777]])
    for prm in [(15, 5, 3, 16), (0, 5, 0, 16), (31, 5, 5, 16)]:
        check_both_ways(gpu, oracle, w, prm, FP16, 4096, f"fp16 all patterns {prm}")


def test_fp32_special_values(gpu, oracle):
    vals = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-45, -1e-45, 3.4e38, 1.17549435e-38], np.float32)
    w = np.concatenate([vals.view(np.uint32), np.array([0x7FC12345, 0xFFFFFFFF, 0x00000001, 0x807FFFFF], np.uint32)])
    w = np.tile(w, 3000)
    check_both_ways(gpu, oracle, w, oracle.tune(w, FP32), FP32, 0, "fp32 specials")


@pytest.mark.parametrize("dtype", [FP16, FP32])
def test_range_error(gpu, oracle, dtype):
    if dtype == FP16:
        b, n, m, L = 10, 4, 2, 16
        w = in_window_words(np.random.default_rng(77), b, n, 40000, FP16, m=m)
    else:
        w = W.gaussian_fp32(40000, 0.02, 77).copy()
        b, n, m, L = oracle.tune(w, dtype)
        assert n < 8
    shift = 10 if dtype == FP16 else 23
    emask = (31 if dtype == FP16 else 255) << shift
    w[33333] = (w[33333] & ~WORD[dtype](emask)) | WORD[dtype](min(b + (1 << (n - 1)) + 1, 30) << shift)
    rc_o, s_o = oracle.compress(w, (b, n, m, L), 16384, dtype=dtype)
    assert rc_o == oracle.E_RANGE
    rc, out, nbytes, cap = gpu.compress(w, (b, n, m, L), dtype, 16384)
    assert rc == 0 and nbytes == 0
    assert np.array_equal(out[:64], s_o[:64])          # header with status 6 and total 0
    info = gpu.enec.stream_info(out[:64])
    assert info["status"] == gpu.enec.E_RANGE and info["total_bytes"] == 0 and info["dtype"] == dtype


def test_batches_and_dtype_dispatch(gpu, oracle):
    """A batch of fp32 tensors with two different tuples; decompress_batch with streams of all three dtypes."""
    torch, enec = gpu.torch, gpu.enec
    t32 = [W.gaussian_fp32(70000, 0.02, 1), W.gaussian_fp32(16384 * 3, 0.5, 2), W.gaussian_fp32(1000, 0.02, 3),
           np.zeros(0, np.uint32), W.gaussian_fp32(40000, 0.001, 4)]
    prm = [oracle.tune(t, FP32) for t in t32]
    srcs = [gpu.to_dev(t, FP32) for t in t32]
    outs = [torch.zeros(enec.compress_bound(t.size, dtype=FP32), dtype=torch.uint8, device="cuda") for t in t32]
    sizes = torch.zeros(len(t32), dtype=torch.int64, device="cuda")
    items = [s if t.size else s[:0] for s, t in zip(srcs, t32)]
    assert enec.compress_batch(items, prm, outs, gpu.ws, out_bytes=[sizes[i:i + 1] for i in range(len(t32))], dtype=FP32) == 0
    torch.cuda.synchronize()
    streams = []
    for i, t in enumerate(t32):
        rc, s = oracle.compress(t, prm[i], oracle.default_block(t.size), dtype=FP32)
        assert rc == 0 and int(sizes[i]) == s.size and np.array_equal(outs[i][:s.size].cpu().numpy(), s), i
        streams.append(s)
    # mixed decompress batch
    h = W.gaussian_fp16(50000, 0.02, 9)
    bf = W.gaussian(50000, 0.02, 10)
    extra = [(h, FP16, oracle.compress(h, oracle.tune(h, FP16), 16384, dtype=FP16)[1]),
             (bf, BF16, oracle.compress(bf, oracle.tune(bf), 16384)[1])]
    bufs, hdrs, backs, want = [], [], [], []
    for t, s in list(zip(t32, streams)) + [(e[0], e[2]) for e in extra]:
        if t.size == 0:
            continue
        bufs.append(torch.from_numpy(s).cuda())
        hdrs.append(s[:64].tobytes())
        backs.append(torch.zeros(t.size, dtype=torch.int32 if t.dtype == np.uint32 else torch.int16, device="cuda"))
        want.append(t)
    assert enec.decompress_batch(bufs, hdrs, backs) == 0
    torch.cuda.synchronize()
    for b, t in zip(backs, want):
        assert np.array_equal(b.cpu().numpy().view(t.dtype), t)


def test_decompress_without_host_header_and_wrong_size(gpu, oracle):
    w = W.gaussian_fp32(30000, 0.02, 5)
    rc, s = oracle.compress(w, oracle.tune(w, FP32), 16384, dtype=FP32)
    rc, d, _ = gpu.decompress(s, w.size, FP32, with_header=False)
    assert rc == 0 and np.array_equal(d, w)
    buf = gpu.torch.from_numpy(s).cuda()
    out = gpu.torch.zeros(w.size, dtype=gpu.torch.int32, device="cuda")
    assert gpu.enec.decompress(buf, out, n_elems=w.size - 1) == gpu.enec.E_FORMAT
    assert gpu.enec.decompress(buf[:s.size - 16], out, n_elems=w.size) == gpu.enec.E_FORMAT


def test_fp32_tensor_beyond_4_gib(gpu, oracle):
    """1.3e9 fp32 elements (5.2 GB): the region of lower halves alone exceeds 2^31 bytes, offsets exceed 2^32."""
    torch, enec = gpu.torch, gpu.enec
    from paper_2604_03298_amd.workloads import gpu_gaussian
    src = gpu_gaussian(torch, 45000, 28672 + 231, 0.02, 4343, torch.float32)
    n = src.numel()
    assert 4 * n > (1 << 32)
    ws = enec.new_workspace(n)
    prm = enec.tune(src, ws, dtype=FP32)
    out = torch.empty(enec.compress_bound(n, dtype=FP32), dtype=torch.uint8, device="cuda")
    size = torch.zeros(1, dtype=torch.int64, device="cuda")
    assert enec.compress(src, prm, out, ws, out_bytes=size, dtype=FP32) == 0
    torch.cuda.synchronize()
    back = torch.empty_like(src)
    assert enec.decompress_with_header(out, out[:64].cpu().numpy().tobytes(), back) == 0
    torch.cuda.synchronize()
    assert torch.equal(back, src)
    del back
    B = 16384
    nb = (n + B - 1) // B
    te, base = oracle.table_end(n, B), oracle.payload_base(n, B, FP32)
    assert int(size.item()) > base
    table = out[64:64 + 8 * (nb + 1)].cpu().numpy().view("<u8")
    for k0 in (0, nb // 2, nb - 2):
        cnt = min(2, nb - k0)
        w = src[k0 * B:min(n, (k0 + cnt) * B)].cpu().numpy().view(np.uint32)
        rc, s = oracle.compress(w, prm, B, dtype=FP32)
        assert rc == 0
        ob = oracle.payload_base(w.size, B, FP32)
        got = out[base + int(table[k0]):base + int(table[k0 + cnt])].cpu().numpy()
        assert np.array_equal(got, s[ob:]), k0
        tail = out[te + 2 * k0 * B:te + 2 * (k0 * B + w.size)].cpu().numpy()
        assert np.array_equal(tail.view("<u2"), (w & 0xFFFF).astype(np.uint16)), k0
