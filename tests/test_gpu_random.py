"""GPU parity on seeded random cases: element format, group length, block size, tensor length, the spread and shape
of the exponent distribution and (for one tuple per tensor) the tuple itself are drawn at random; every stream must be
the oracle's byte for byte and decode to the input.  The fixed cases of the other files aim at known edges; these
sweep the combinations in between."""
import numpy as np
import pytest

from test_gpu_dtypes import gpu, BF16, FP16, FP32  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu

BLOCKS = (2048, 4096, 8192, 16384, 32768)


def _words(rng, dtype, e):
    n = e.size
    e = e.astype(np.uint32)
    sign = rng.integers(0, 2, n).astype(np.uint32)
    if dtype == BF16:
        return ((sign << 15) | (e << 7) | rng.integers(0, 128, n).astype(np.uint32)).astype(np.uint16)
    if dtype == FP16:
        return ((sign << 15) | (e << 10) | rng.integers(0, 1024, n).astype(np.uint32)).astype(np.uint16)
    return ((sign << 31) | (e << 23) | rng.integers(0, 1 << 23, n).astype(np.uint32)).astype(np.uint32)


def _exponents(rng, E, n):
    """n exponents out of a random window of the 2^E values: uniform, concentrated, the two ends, or one value
    with a few strays."""
    span = int(rng.integers(1, (1 << E) + 1))
    lo = int(rng.integers(0, (1 << E) - span + 1))
    kind = int(rng.integers(0, 4))
    if kind == 0:
        return rng.integers(lo, lo + span, n)
    if kind == 1:
        return np.clip(np.rint(rng.normal(lo + span / 2, max(span / 8, 0.5), n)), lo, lo + span - 1).astype(np.int64)
    if kind == 2:
        return np.where(rng.random(n) < rng.random(), lo, lo + span - 1)
    e = np.full(n, lo + span // 2)
    if n:
        e[rng.integers(0, n, 8)] = rng.integers(lo, lo + span, 8)
    return e


def _dev(torch, w, dtype):
    if w.size == 0:
        return torch.empty(8, dtype=torch.int32 if dtype == FP32 else torch.int16, device="cuda")[:0]
    return torch.from_numpy(np.ascontiguousarray(w).view(np.int32 if dtype == FP32 else np.int16)).cuda()


def test_random_tensors_one_tuple_per_tensor(gpu, oracle):
    torch, enec = gpu.torch, gpu.enec
    rng = np.random.default_rng(2024)
    same = ranged = 0
    for case in range(250):
        dtype = int(rng.choice([BF16, BF16, FP16, FP32]))
        E = 5 if dtype == FP16 else 8
        L = int(rng.choice([8, 16, 32]))
        B = int(rng.choice([b for b in BLOCKS if 128 * L <= b <= 2048 * L]))
        n_el = int(rng.integers(1, 24 * B))
        w = _words(rng, dtype, _exponents(rng, E, n_el))
        if rng.random() < 0.7:
            b, n, m, _ = oracle.tune(w, dtype)
            if rng.random() < 0.5:
                m = int(rng.integers(0, n + 1))
        else:       # any valid tuple, windows that miss exponents included
            n = int(rng.integers(1, E + 1))
            m = int(rng.integers(0, n + 1))
            b = int(rng.integers(0, 1 << E))
        prm = (b, n, m, L)
        rc_o, s_o = oracle.compress(w, prm, B, dtype=dtype)
        src = _dev(torch, w, dtype)
        out = torch.zeros(enec.compress_bound(n_el, dtype=dtype, block_size=B), dtype=torch.uint8, device="cuda")
        size = torch.zeros(1, dtype=torch.int64, device="cuda")
        assert enec.compress(src, prm, out, gpu.ws, block_size=B, out_bytes=size, n_elems=n_el, dtype=dtype) == 0
        torch.cuda.synchronize()
        status = int(out[28:32].cpu().numpy().view(np.uint32)[0])
        label = f"case {case}: dtype {dtype} L {L} B {B} n {n_el} tuple {prm}"
        if rc_o == oracle.E_RANGE:
            assert status == enec.E_RANGE and int(size.item()) == 0, label
            ranged += 1
            continue
        assert rc_o == oracle.OK and status == 0, label
        nbytes = int(size.item())
        assert nbytes == s_o.size and np.array_equal(out[:nbytes].cpu().numpy(), s_o), label
        back = torch.zeros_like(src)
        assert enec.decompress(out[:nbytes], back, n_elems=n_el) == 0
        torch.cuda.synchronize()
        assert torch.equal(back, src), label
        same += 1
    assert same > 100 and ranged > 10          # both outcomes were exercised


def test_random_batches_one_tuple_per_block(gpu, oracle):
    torch, enec = gpu.torch, gpu.enec
    rng = np.random.default_rng(2025)
    for case in range(40):
        dtype = int(rng.choice([BF16, BF16, FP16, FP32]))
        E = 5 if dtype == FP16 else 8
        L = int(rng.choice([8, 16, 32]))
        count = int(rng.integers(1, 36))
        Bs, ws = [], []
        for _ in range(count):
            B = int(rng.choice([b for b in BLOCKS if 128 * L <= b <= 2048 * L]))
            blocks = int(rng.integers(0, 6))
            parts = [_words(rng, dtype, _exponents(rng, E, B)) for _ in range(blocks)]
            tail = int(rng.integers(0, B)) if rng.random() < 0.6 else 0       # a ragged last block, or an empty tensor
            if tail:
                parts.append(_words(rng, dtype, _exponents(rng, E, tail)))
            ws.append(np.concatenate(parts) if parts else np.zeros(0, np.uint32 if dtype == FP32 else np.uint16))
            Bs.append(B)
        srcs = [_dev(torch, w, dtype) for w in ws]
        caps = [enec.compress_bound_per_block(w.size, dtype=dtype, block_size=b) for w, b in zip(ws, Bs)]
        outs = [torch.full((c + 16,), 0xA5, dtype=torch.uint8, device="cuda") for c in caps]
        sizes = torch.zeros(count, dtype=torch.int64, device="cuda")
        rc = enec.compress_per_block_batch(srcs, outs, gpu.ws, out_bytes=[sizes[i:i + 1] for i in range(count)],
                                           dtype=dtype, block_sizes=Bs, group_length=L)
        torch.cuda.synchronize()
        assert rc == 0, case
        got_sizes = sizes.cpu().numpy()
        streams = []
        for i, (w, b) in enumerate(zip(ws, Bs)):
            rc_o, s_o = oracle.compress_per_block(w, b, dtype, L)
            got = outs[i].cpu().numpy()
            label = f"case {case} tensor {i}: dtype {dtype} L {L} B {b} n {w.size}"
            assert rc_o == oracle.OK and got_sizes[i] == s_o.size and np.array_equal(got[:s_o.size], s_o), label
            assert (got[caps[i]:] == 0xA5).all(), label
            streams.append(s_o)
        backs = [torch.full((max(w.size, 8),), 0x5A, dtype=torch.int32 if dtype == FP32 else torch.int16, device="cuda")[:w.size]
                 for w in ws]
        rc = enec.decompress_batch([o[:max(s.size, 64)] for o, s in zip(outs, streams)], [s[:64].tobytes() for s in streams], backs)
        torch.cuda.synchronize()
        assert rc == 0, case
        for i, w in enumerate(ws):
            assert np.array_equal(backs[i].cpu().numpy().view(w.dtype), w), (case, i)
