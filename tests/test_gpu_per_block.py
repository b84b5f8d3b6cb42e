"""GPU parity for streams with one tuple per data block: libenec (through its C ABI) against the CPU oracle,
byte for byte in both directions; every decision (b, n by Eq. 1-3 in integers, m by Eq. 4 in IEEE double)
is taken by the kernel and by the oracle in the same precision, so the tuples must be identical."""
import numpy as np
import pytest

from paper_2604_03298_amd import workloads as W
from test_gpu_dtypes import gpu, BF16, FP16, FP32, WORD  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def _compress(gpu, w, dtype, B=0, L=0):
    torch, enec = gpu.torch, gpu.enec
    src = gpu.to_dev(w, dtype)
    cap = enec.compress_bound_per_block(w.size, dtype=dtype, block_size=B)
    out = torch.full((cap + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    gpu.size_pinned.fill_(-1)
    rc = enec.compress_per_block(src, out, gpu.ws, block_size=B, out_bytes=gpu.size_pinned, n_elems=w.size, dtype=dtype,
                                 group_length=L)
    torch.cuda.synchronize()
    return rc, out.cpu().numpy(), int(gpu.size_pinned.item()), cap


def _check(gpu, oracle, w, dtype, B=0, label="", L=0):
    Bo = B if B else oracle.default_block(w.size)
    rc_o, s_o = oracle.compress_per_block(w, Bo, dtype, L if L else 16)
    assert rc_o == oracle.OK, label
    rc, out, nbytes, cap = _compress(gpu, w, dtype, B, L)
    assert rc == 0, label
    assert nbytes == s_o.size, f"{label}: size {nbytes} vs oracle {s_o.size}"
    bad = np.nonzero(out[:nbytes] != s_o)[0]
    assert bad.size == 0, f"{label}: stream differs from the oracle's, first at byte {bad[:4]}"
    assert (out[cap:] == 0xA5).all(), f"{label}: wrote past the bound"
    for with_header in (True, False):
        rc, d, rest = gpu.decompress(s_o, w.size, dtype, with_header)
        assert rc == 0 and np.array_equal(d, w), f"{label}: GPU decompress(oracle stream) != input"
        assert (rest == (0x5A5A5A5A if dtype == FP32 else 0x5A5A)).all(), f"{label}: wrote past the tensor"
    return s_o


def _mixed16(n_blocks, B, seed, dtype=BF16):
    rng = np.random.default_rng(seed)
    out = np.empty(n_blocks * B, np.uint16)
    gen = W.gaussian if dtype == BF16 else W.gaussian_fp16
    for k in range(n_blocks):
        kind = int(rng.integers(0, 5))
        blk = out[k * B:(k + 1) * B]
        if kind == 0:
            blk[:] = 0
        elif kind == 1:
            blk[:] = gen(1, 0.02, seed + k)[0]
        elif kind == 2:
            blk[:] = gen(B, 0.02 * 2.0 ** (k % 7 - 3), seed + k)
        elif kind == 3:
            blk[:] = rng.integers(0, 65536, B)
        else:       # a quiet block with a few outliers
            blk[:] = gen(B, 0.01, seed + k)
            blk[rng.integers(0, B, 5)] = rng.integers(0, 65536, 5)
    return out


@pytest.mark.parametrize("B", [2048, 4096, 16384, 32768])
def test_bf16_mixed_blocks(gpu, oracle, B):
    w = _mixed16(19, B, 100 + B)
    _check(gpu, oracle, w, BF16, B, f"B={B}")
    _check(gpu, oracle, w[:w.size - B // 2 - 3], BF16, B, f"B={B} ragged")
    _check(gpu, oracle, w[:B + 1], BF16, B, f"B={B} one element in the last block")


def test_config3_blocks_and_ratio(gpu, oracle):
    w, cat = W.config3(n_blocks=256)
    s = _check(gpu, oracle, w, BF16, 16384, "config 3a, 256 blocks")
    tuples = oracle.block_tuples(s)
    assert all(tuples[k] == (0, 1, 0) for k in range(256) if cat[k] == 0)
    assert all(tuples[k][1] == 1 for k in range(256) if cat[k] == 1)
    assert all(tuples[k][1] == 8 for k in range(256) if cat[k] == 3)
    one = oracle.compress(w, oracle.tune(w), 16384)[1]
    assert s.size < 0.85 * one.size          # one tuple for the tensor cannot adapt to the mix


def test_fp16_and_fp32(gpu, oracle):
    for B in (2048, 16384):
        w = _mixed16(9, B, 7 + B, FP16)
        _check(gpu, oracle, w, FP16, B, f"fp16 B={B}")
        _check(gpu, oracle, w[:w.size - 1234], FP16, B, f"fp16 B={B} ragged")
        parts = [W.gaussian_fp32(B * 2, 0.02, 1), np.zeros(B, np.uint32), W.gaussian_fp32(B, 300.0, 2),
                 np.random.default_rng(B).integers(0, 2**32, B, dtype=np.uint64).astype(np.uint32),
                 W.gaussian_fp32(B * 2 - 77, 1e-4, 3)]
        _check(gpu, oracle, np.concatenate(parts), FP32, B, f"fp32 B={B}")


def test_degenerate_tensors(gpu, oracle):
    for dt in (BF16, FP16, FP32):
        word = WORD[dt]
        _check(gpu, oracle, np.zeros(0, word), dt, 0, "empty")
        _check(gpu, oracle, np.array([0x3C01], word), dt, 0, "one element")
        _check(gpu, oracle, np.zeros(5000, word), dt, 0, "zeros")
        top = 0xFFFFFFFF if dt == FP32 else 0xFFFF
        _check(gpu, oracle, np.full(4097, top, word), dt, 2048, "all ones")
    rng = np.random.default_rng(5)
    _check(gpu, oracle, rng.integers(0, 65536, 16384 * 3 + 5).astype(np.uint16), BF16, 0, "noise")
    # exponents 0 and 255 in one block: the window is the whole range
    w = W.gaussian(16384, 0.02, 6)
    w[3], w[9000] = 0x0001, 0x7F80
    _check(gpu, oracle, w, BF16, 0, "extremes")


def test_oracle_reads_the_gpu_stream_and_many_blocks(gpu, oracle):
    """More blocks than the device holds workgroups at once: the look-back crosses many windows."""
    w = _mixed16(3000, 2048, 77)
    s = _check(gpu, oracle, w, BF16, 2048, "3000 blocks")
    rc, d = oracle.decompress(s, w.size)
    assert rc == oracle.OK and np.array_equal(d, w)


def test_workspace_shared_with_the_one_tuple_path(gpu, oracle):
    """Both kinds of call use the same workspace one after the other."""
    w = _mixed16(40, 4096, 9)
    prm = oracle.tune(w)
    for _ in range(2):
        _check(gpu, oracle, w, BF16, 4096, "per block")
        rc, out, nbytes, cap = gpu.compress(w, prm, BF16, 4096)
        assert rc == 0 and np.array_equal(out[:nbytes], oracle.compress(w, prm, 4096)[1])


def test_batch_decompress_mixes_both_kinds(gpu, oracle):
    torch, enec = gpu.torch, gpu.enec
    ws = [_mixed16(5, 2048, 1), W.gaussian(30000, 0.02, 2), _mixed16(3, 16384, 3), W.gaussian(2048 * 4, 0.02, 4)]
    streams = [oracle.compress_per_block(ws[0], 2048)[1], oracle.compress(ws[1], oracle.tune(ws[1]), 16384)[1],
               oracle.compress_per_block(ws[2], 16384)[1], oracle.compress(ws[3], oracle.tune(ws[3]), 2048)[1]]
    bufs = [torch.from_numpy(s).cuda() for s in streams]
    outs = [torch.full((w.size,), 0x5A5A, dtype=torch.int16, device="cuda") for w in ws]
    assert enec.decompress_batch(bufs, [s[:64].tobytes() for s in streams], outs) == 0
    torch.cuda.synchronize()
    for w, o in zip(ws, outs):
        assert np.array_equal(o.cpu().numpy().view(np.uint16), w)


def test_damaged_tuples_and_offsets_skip_blocks(gpu, oracle):
    """A tuple or table entry that cannot be right makes the kernel leave that block alone."""
    B = 2048
    w = _mixed16(8, B, 21)
    s = oracle.compress_per_block(w, B)[1]
    at = oracle.table_end(w.size, B)
    for what in ("n zero", "m above n", "n above 8", "offset"):
        bad = s.copy()
        k = 3
        if what == "n zero":
            bad[at + 4 * k + 1] = 0
        elif what == "m above n":
            bad[at + 4 * k + 2] = bad[at + 4 * k + 1] + 1
        elif what == "n above 8":
            bad[at + 4 * k + 1] = 9
        else:
            bad[64 + 8 * k:64 + 8 * k + 8] = np.frombuffer(np.uint64(1 << 40).tobytes(), np.uint8)
        rc, d, rest = gpu.decompress(bad, w.size, BF16)
        assert rc == 0 and (rest == 0x5A5A).all()
        # the status word tells the caller that blocks were left undecoded
        torch, enec = gpu.torch, gpu.enec
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        back = torch.full((w.size,), 0x5A5A, dtype=torch.int16, device="cuda")
        assert enec.decompress_with_header(torch.from_numpy(bad).cuda(), bad[:64].tobytes(), back, status=status) == 0
        torch.cuda.synchronize()
        assert int(status.item()) == enec.E_FORMAT, what
        touched = {k, k - 1} if what == "offset" else {k}
        for j in range(8):
            blk = d[j * B:(j + 1) * B]
            if j in touched:
                assert (blk == 0x5A5A).all(), (what, j)
            else:
                assert np.array_equal(blk, w[j * B:(j + 1) * B]), (what, j)


def test_host_checks(gpu):
    torch, enec = gpu.torch, gpu.enec
    src = torch.zeros(4096, dtype=torch.int16, device="cuda")
    out = torch.zeros(enec.compress_bound_per_block(4096), dtype=torch.uint8, device="cuda")
    assert enec.compress_per_block(src, out[:100], gpu.ws) == enec.E_CAPACITY
    assert enec.compress_per_block(src, out, gpu.ws, block_size=3000) == enec.E_BLOCK
    assert enec.compress_per_block(src, out, gpu.ws, dtype=7) == enec.E_DTYPE
    assert enec.compress_per_block(src, out, gpu.ws[:1024 + 16 * 2048]) == enec.E_CAPACITY
    assert enec.compress_bound_per_block(4096, BF16, 2048) == enec.compress_bound(4096, BF16, 2048) + 16


def test_configuration_3_at_full_size(gpu, oracle):
    """All 4096 data blocks of the edge-case mix (134 MB), the launch the report times: the whole stream against the oracle's."""
    w, cat = W.config3()
    rc_o, s_o = oracle.compress_per_block(w, 16384)
    assert rc_o == oracle.OK
    rc, out, nbytes, cap = _compress(gpu, w, BF16, 16384)
    assert rc == 0 and nbytes == s_o.size
    assert np.array_equal(out[:nbytes], s_o)
    rc, d, rest = gpu.decompress(s_o, w.size, BF16)
    assert rc == 0 and np.array_equal(d, w)


def test_repeated_and_back_to_back_calls_give_the_same_bytes(gpu, oracle):
    """The look-back must not depend on timing: the same stream 60 times, calls queued without synchronisation,
    two tensors alternating on one workspace."""
    torch, enec = gpu.torch, gpu.enec
    ws_a, ws_b = _mixed16(300, 2048, 31), _mixed16(37, 16384, 32)
    want = [oracle.compress_per_block(w, B)[1] for w, B in ((ws_a, 2048), (ws_b, 16384))]
    srcs = [gpu.to_dev(w, BF16) for w in (ws_a, ws_b)]
    outs = [[torch.zeros(enec.compress_bound_per_block(w.size, block_size=B) + 64, dtype=torch.uint8, device="cuda")
             for _ in range(30)] for w, B in ((ws_a, 2048), (ws_b, 16384))]
    for rep in range(30):
        assert enec.compress_per_block(srcs[0], outs[0][rep], gpu.ws, block_size=2048) == 0
        assert enec.compress_per_block(srcs[1], outs[1][rep], gpu.ws, block_size=16384) == 0
    torch.cuda.synchronize()
    for t in range(2):
        for rep in range(30):
            got = outs[t][rep].cpu().numpy()
            assert np.array_equal(got[:want[t].size], want[t]), (t, rep)


def test_two_streams_two_workspaces(gpu, oracle):
    torch, enec = gpu.torch, gpu.enec
    w1, w2 = _mixed16(64, 16384, 41), _mixed16(64, 16384, 42)
    want = [oracle.compress_per_block(w, 16384)[1] for w in (w1, w2)]
    srcs = [gpu.to_dev(w, BF16) for w in (w1, w2)]
    outs = [torch.zeros(enec.compress_bound_per_block(w.size), dtype=torch.uint8, device="cuda") for w in (w1, w2)]
    wss = [enec.new_workspace(w.size) for w in (w1, w2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(5):
        for i in range(2):
            with torch.cuda.stream(streams[i]):
                assert enec.compress_per_block(srcs[i], outs[i], wss[i], stream=streams[i]) == 0
    torch.cuda.synchronize()
    for i in range(2):
        assert np.array_equal(outs[i].cpu().numpy()[:want[i].size], want[i]), i


@pytest.mark.parametrize("L", [8, 32])
def test_group_lengths_8_and_32(gpu, oracle, L):
    """Blocks coded with groups of 8 or 32 elements (the search is the same, the records differ)."""
    for B in ((2048, 16384) if L == 8 else (4096, 16384, 32768)):
        w = _mixed16(11, B, 500 + B + L)
        _check(gpu, oracle, w, BF16, B, f"L={L} B={B}", L)
        _check(gpu, oracle, w[:w.size - B // 3 - 1], BF16, B, f"L={L} B={B} ragged", L)
    # blocks of two scales: Eq. 4 gives them another m at L = 32 than at L = 16, so the kernel's search must use
    # the length the block is coded with
    two = np.concatenate([np.concatenate([W.gaussian(2048, 0.02, 10 + i), W.gaussian(2048, 0.005, 20 + i)]) for i in range(5)])
    s_two = _check(gpu, oracle, two, BF16, 4096, f"L={L} two scales", L)
    if L == 32:
        assert any(t[2] != oracle.tune(two[k * 4096:(k + 1) * 4096])[2] for k, t in enumerate(oracle.block_tuples(s_two)))
    w = _mixed16(7, 16384, 77 + L, FP16)
    _check(gpu, oracle, w, FP16, 16384, f"fp16 L={L}", L)
    parts = [W.gaussian_fp32(16384 * 2, 0.02, 1), np.zeros(16384, np.uint32), W.gaussian_fp32(16384 + 99, 300.0, 2)]
    _check(gpu, oracle, np.concatenate(parts), FP32, 16384, f"fp32 L={L}", L)
    torch, enec = gpu.torch, gpu.enec
    src = torch.zeros(4096, dtype=torch.int16, device="cuda")
    out = torch.zeros(enec.compress_bound_per_block(4096), dtype=torch.uint8, device="cuda")
    assert enec.compress_per_block(src, out, gpu.ws, block_size=2048, group_length=32) == enec.E_PARAMS
    assert enec.compress_per_block(src, out, gpu.ws, block_size=2048, group_length=12) == enec.E_PARAMS


def test_tensor_beyond_4_gib_sampled_against_the_oracle(gpu, oracle):
    """2.6e9 elements (5.2 GB of bf16), 158 000 data blocks with one tuple each: element and byte offsets beyond
    32 bits, a look-back over many windows.  The round trip is compared on the device; blocks sampled along the
    tensor are recompressed by the oracle, tuples and payloads must be what the library wrote."""
    torch, enec = gpu.torch, gpu.enec
    from paper_2604_03298_amd.workloads import gpu_gaussian
    rows, cols = 90000, 28672 + 231          # not a multiple of the block size: ragged tail
    src = gpu_gaussian(torch, rows, cols, 0.02, 4343)
    n = src.numel()
    assert 2 * n > (1 << 32)
    B = 16384
    nb = (n + B - 1) // B
    src[5 * B:6 * B] = 0                      # a block of zeros and a block of noise among the weights
    src[(nb // 2) * B:(nb // 2 + 1) * B] = torch.randint(-32768, 32767, (B,), dtype=torch.int16, device="cuda",
                                                         generator=torch.Generator(device="cuda").manual_seed(1))
    ws = enec.new_workspace(n)
    out = torch.empty(enec.compress_bound_per_block(n), dtype=torch.uint8, device="cuda")
    size = torch.zeros(1, dtype=torch.int64, device="cuda")
    assert enec.compress_per_block(src, out, ws, out_bytes=size) == 0
    torch.cuda.synchronize()
    total = int(size.item())
    assert 0 < total < 2 * n
    back = torch.empty_like(src)
    assert enec.decompress_with_header(out, out[:64].cpu().numpy().tobytes(), back) == 0
    torch.cuda.synchronize()
    assert torch.equal(back, src)
    del back
    base = oracle.payload_base_pb(n, B)
    at = oracle.table_end(n, B)
    table = out[64:64 + 8 * (nb + 1)].cpu().numpy().view("<u8")
    tuples = out[at:at + 4 * nb].cpu().numpy().reshape(nb, 4)
    assert table[0] == 0 and int(table[nb]) + base == total and (np.diff(table.astype(np.int64)) > 0).all()
    assert (tuples[:, 3] == 0).all()
    for k in (0, 5, 1234, nb // 2, (1 << 32) // (2 * B) + 5, nb - 2, nb - 1):      # incl. byte 2^32 and the ragged tail
        w = src[k * B:min(n, (k + 1) * B)].cpu().numpy().view(np.uint16)
        b, n_, m, _ = oracle.tune(w)
        assert tuple(int(v) for v in tuples[k, :3]) == (b, n_, m), k
        rc, s = oracle.compress(w, (b, n_, m, 16), B)
        assert rc == 0
        ob = oracle.payload_base(w.size, B)
        got = out[base + int(table[k]):base + int(table[k + 1])].cpu().numpy()
        assert got.size == s.size - ob and np.array_equal(got, s[ob:]), k
    assert tuple(int(v) for v in tuples[5, :3]) == (0, 1, 0)


@pytest.mark.parametrize("L", [8, 16, 32])
def test_a_few_hundred_blocks_all_formats(gpu, oracle, L):
    """More data blocks than ticket counters and a count that is no multiple of eight, a ragged last block; every
    element format and group length."""
    B = 16384
    w = _mixed16(261, B, 900 + L)
    _check(gpu, oracle, w[:w.size - 77], BF16, B, f"bf16 L={L}", L)
    h = _mixed16(258, B, 950 + L, FP16)
    _check(gpu, oracle, h, FP16, B, f"fp16 L={L}", L)
    f = np.concatenate([W.gaussian_fp32(200 * B, 0.02, 1), np.zeros(B, np.uint32), W.gaussian_fp32(58 * B + 5, 3.0, 2)])
    _check(gpu, oracle, f, FP32, B, f"fp32 L={L}", L)


def test_the_largest_block_size(gpu, oracle):
    w = _mixed16(131, 32768, 77)
    _check(gpu, oracle, w, BF16, 32768, "B=32768, 131 blocks")
    _check(gpu, oracle, w, BF16, 32768, "B=32768, 131 blocks, L=32", 32)


@pytest.mark.parametrize("span", [64, 65, 80, 100, 127, 128, 129, 200, 256])
def test_blocks_whose_exponents_spread_over_many_values(gpu, oracle, span):
    """Exponents uniform over `span` consecutive values: from 65 values on the kernel searches (b, n) with the
    incremental form of Eq. 3's cost, and Eq. 1 gives n = 7 for central b when the spread allows it."""
    B = 16384
    rng = np.random.default_rng(span)
    blocks = []
    for k in range(6):
        lo = int(rng.integers(0, 257 - span))
        e = rng.integers(lo, lo + span, B).astype(np.uint16)
        if k == 1:        # the same spread, most elements on one value
            e[rng.random(B) < 0.9] = lo + span // 3
        if k == 2:        # only the two ends and a few values in between
            e = np.where(rng.random(B) < 0.5, lo, lo + span - 1).astype(np.uint16)
            e[:16] = rng.integers(lo, lo + span, 16)
        blocks.append((rng.integers(0, 2, B).astype(np.uint16) << 15) | (e << 7) | rng.integers(0, 128, B).astype(np.uint16))
    w = np.concatenate(blocks)
    _check(gpu, oracle, w, BF16, B, f"bf16 span={span}")
    f = (w.astype(np.uint32) << 16) | rng.integers(0, 65536, w.size).astype(np.uint32)
    _check(gpu, oracle, f, FP32, B, f"fp32 span={span}")


def _batch(gpu, ws_list, dtype, Bs=None, L=0, workspace=None):
    """enec_compress_per_block_batch on the tensors of ws_list; returns rc and, per tensor, (stream bytes, size, bound)."""
    torch, enec = gpu.torch, gpu.enec
    srcs = [gpu.to_dev(w, dtype) for w in ws_list]
    caps = [enec.compress_bound_per_block(w.size, dtype=dtype, block_size=(Bs[i] if Bs else 0)) for i, w in enumerate(ws_list)]
    outs = [torch.full((c + 64,), 0xA5, dtype=torch.uint8, device="cuda") for c in caps]
    sizes = torch.full((len(ws_list),), -1, dtype=torch.int64, device="cuda")
    items_n = [w.size for w in ws_list]
    # the binding takes numel() of the tensors: empty tensors travel as 8-element dummies, so pass views of the right length
    srcs = [s[:n] for s, n in zip(srcs, items_n)]
    rc = enec.compress_per_block_batch(srcs, outs, gpu.ws if workspace is None else workspace,
                                       out_bytes=[sizes[i:i + 1] for i in range(len(ws_list))], dtype=dtype,
                                       block_sizes=Bs, group_length=L)
    torch.cuda.synchronize()
    return rc, [(o.cpu().numpy(), int(s), c) for o, s, c in zip(outs, sizes.cpu(), caps)]


@pytest.mark.parametrize("L", [8, 16, 32])
def test_batch_of_tensors_equals_the_oracle_tensor_by_tensor(gpu, oracle, L):
    """Several tensors in one call: different lengths (one block, many blocks, a ragged tail, empty), two block
    sizes (two launches) and more than 16 tensors of one block size (a launch holds 16); every stream is the
    oracle's, byte for byte, and nothing is written past a tensor's bound."""
    B = 16384
    ws_list = [_mixed16(37, B, 1), _mixed16(1, B, 2)[:5000], _mixed16(300, B, 3)[:300 * B - 77], np.zeros(0, np.uint16),
               _mixed16(9, 4096, 4), W.gaussian(8 * B, 0.02, 5), _mixed16(2, 4096, 6)[:4097]]
    ws_list += [_mixed16(1 + (i % 3), B, 10 + i) for i in range(17)]
    Bs = [B, B, B, B, 4096, B, 4096] + [B] * 17
    rc, res = _batch(gpu, ws_list, BF16, Bs, L)
    assert rc == 0
    for i, (w, (out, nbytes, cap)) in enumerate(zip(ws_list, res)):
        rc_o, s_o = oracle.compress_per_block(w, Bs[i], BF16, L)
        assert rc_o == oracle.OK
        assert nbytes == s_o.size, f"tensor {i}: size {nbytes} vs oracle {s_o.size}"
        assert np.array_equal(out[:nbytes], s_o), f"tensor {i}: stream differs from the oracle's"
        assert (out[cap:] == 0xA5).all(), f"tensor {i}: wrote past the bound"


def test_batch_default_block_sizes_and_other_formats(gpu, oracle):
    """Block size 0 = each tensor's default (small tensors get smaller blocks, hence a launch of their own); fp16 and
    fp32 batches."""
    ws_list = [W.gaussian(100000, 0.02, 1), W.gaussian(4096, 0.5, 2), W.gaussian(3000, 0.02, 3), W.gaussian(70000, 0.1, 4)]
    rc, res = _batch(gpu, ws_list, BF16)
    assert rc == 0
    for w, (out, nbytes, cap) in zip(ws_list, res):
        rc_o, s_o = oracle.compress_per_block(w, oracle.default_block(w.size), BF16, 16)
        assert rc_o == oracle.OK and nbytes == s_o.size and np.array_equal(out[:nbytes], s_o)
    hs = [_mixed16(5, 16384, 31, FP16), _mixed16(3, 16384, 32, FP16)[:40000]]
    rc, res = _batch(gpu, hs, FP16, [16384, 16384])
    assert rc == 0
    for w, (out, nbytes, cap) in zip(hs, res):
        rc_o, s_o = oracle.compress_per_block(w, 16384, FP16, 16)
        assert rc_o == oracle.OK and nbytes == s_o.size and np.array_equal(out[:nbytes], s_o)
    fs = [W.gaussian_fp32(5 * 16384 + 3, 0.02, 1), W.gaussian_fp32(16384, 3.0, 2)]
    rc, res = _batch(gpu, fs, FP32, [16384, 16384])
    assert rc == 0
    for w, (out, nbytes, cap) in zip(fs, res):
        rc_o, s_o = oracle.compress_per_block(w, 16384, FP32, 16)
        assert rc_o == oracle.OK and nbytes == s_o.size and np.array_equal(out[:nbytes], s_o)


def test_batch_host_checks(gpu):
    torch, enec = gpu.torch, gpu.enec
    w = gpu.to_dev(W.gaussian(16384 * 4, 0.02, 1), BF16)
    good = torch.empty(enec.compress_bound_per_block(w.numel()), dtype=torch.uint8, device="cuda")
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    assert enec.compress_per_block_batch([w, w], [good, small], gpu.ws) == 5          # capacity: nothing is enqueued
    assert enec.compress_per_block_batch([w], [good], gpu.ws, block_sizes=[3000]) == 3    # block size
    assert enec.compress_per_block_batch([w], [good], gpu.ws, block_sizes=[2048], group_length=32) == 4   # L does not fit
    tiny_ws = torch.zeros(enec.workspace_bytes(2048) // 8, dtype=torch.int64, device="cuda")
    big = gpu.to_dev(W.gaussian(16384 * 4096, 0.02, 2), BF16)
    out = torch.empty(enec.compress_bound_per_block(big.numel()), dtype=torch.uint8, device="cuda")
    assert enec.compress_per_block_batch([big], [out], tiny_ws) == 5                  # workspace too small
    assert enec.compress_per_block_batch([], [], gpu.ws) == 0


def test_batch_decompress_of_many_per_block_streams(gpu, oracle):
    """More than 16 streams with one tuple per block in one decompress call (a launch holds 16), a second block size,
    an empty tensor and one damaged stream: its status word alone is set, its damaged block alone is left undecoded."""
    torch, enec = gpu.torch, gpu.enec
    B = 4096
    ws = [_mixed16(1 + (i * 7) % 13, B, 60 + i)[:(1 + (i * 7) % 13) * B - (i % 3) * 11] for i in range(19)]
    ws += [_mixed16(3, 16384, 90), np.zeros(0, np.uint16)]
    Bs = [B] * 19 + [16384, 16384]
    streams = [oracle.compress_per_block(w, b)[1] for w, b in zip(ws, Bs)]
    bad = 7
    at = oracle.table_end(ws[bad].size, B)
    streams[bad] = streams[bad].copy()
    streams[bad][at + 4 * 2 + 1] = 0                      # n = 0 in the tuple of block 2
    bufs = [torch.from_numpy(s).cuda() for s in streams]
    outs = [torch.full((max(w.size, 8),), 0x5A5A, dtype=torch.int16, device="cuda")[:w.size] for w in ws]
    statuses = [torch.zeros(1, dtype=torch.int32, device="cuda") for _ in ws]
    assert enec.decompress_batch(bufs, [s[:64].tobytes() for s in streams], outs, statuses=statuses) == 0
    torch.cuda.synchronize()
    for i, (w, o) in enumerate(zip(ws, outs)):
        got = o.cpu().numpy().view(np.uint16)
        if i == bad:
            assert int(statuses[i].item()) == enec.E_FORMAT
            assert (got[2 * B:3 * B] == 0x5A5A).all()
            assert np.array_equal(got[:2 * B], w[:2 * B]) and np.array_equal(got[3 * B:], w[3 * B:])
        else:
            assert int(statuses[i].item()) == 0, i
            assert np.array_equal(got, w), i
