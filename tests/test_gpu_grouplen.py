"""GPU parity for group lengths 8 and 32 (Eq. 4 searches the length together with m): libenec against the
CPU oracle, byte for byte, all three element formats."""
import numpy as np
import pytest

from paper_2604_03298_amd import workloads as W
from test_gpu_dtypes import gpu, check_both_ways, in_window_words, BF16, FP16, FP32, WORD   # noqa: F401

pytestmark = pytest.mark.gpu


def bf16_window(rng, b, n, size, m):
    w32 = in_window_words(rng, b, n, size, FP32, m=m)
    return (w32 >> 16).astype(np.uint16)


@pytest.mark.parametrize("L", [8, 32])
@pytest.mark.parametrize("n", range(1, 9))
def test_bf16_every_width_pair(gpu, oracle, L, n):
    rng = np.random.default_rng(3000 + 10 * L + n)
    for m in range(0, n + 1):
        for B, size in [(4096, 3 * 4096 + 517), (16384, 2 * 16384 + 4099)]:
            w = bf16_window(rng, 128, n, size, m)
            check_both_ways(gpu, oracle, w, (128, n, m, L), BF16, B, f"bf16 L={L} n={n} m={m} B={B}")


@pytest.mark.parametrize("L", [8, 32])
@pytest.mark.parametrize("n", range(1, 6))
def test_fp16_every_width_pair(gpu, oracle, L, n):
    rng = np.random.default_rng(4000 + 10 * L + n)
    for m in range(0, n + 1):
        B, size = [(4096, 3 * 4096 + 517), (16384, 2 * 16384 + 4099)][(n + m) % 2]
        w = in_window_words(rng, 14, n, size, FP16, m=m)
        check_both_ways(gpu, oracle, w, (14, n, m, L), FP16, B, f"fp16 L={L} n={n} m={m} B={B}")


@pytest.mark.parametrize("L", [8, 32])
@pytest.mark.parametrize("n", range(1, 9))
def test_fp32_every_width_pair(gpu, oracle, L, n):
    rng = np.random.default_rng(5000 + 10 * L + n)
    for m in range(0, n + 1):
        B, size = [(4096, 3 * 4096 + 517), (16384, 2 * 16384 + 4099)][(n + m) % 2]
        w = in_window_words(rng, 128, n, size, FP32, m=m)
        check_both_ways(gpu, oracle, w, (128, n, m, L), FP32, B, f"fp32 L={L} n={n} m={m} B={B}")


@pytest.mark.parametrize("L,B", [(8, 2048), (8, 4096), (8, 8192), (8, 16384), (32, 4096), (32, 8192), (32, 16384), (32, 32768)])
def test_block_sizes(gpu, oracle, L, B):
    w = W.gaussian(5 * B + 1234, 0.02, 31 + B + L)
    b, n, m, _ = oracle.tune(w)
    check_both_ways(gpu, oracle, w, (b, n, m, L), BF16, B, f"L={L} B={B}")


@pytest.mark.parametrize("L", [8, 32])
@pytest.mark.parametrize("n_elems", [0, 1, 7, 8, 9, 31, 32, 33, 4095, 4097, 16383, 16385, 50001])
def test_ragged_and_tiny(gpu, oracle, L, n_elems):
    w = W.gaussian(n_elems, 0.02, 2000 + n_elems) if n_elems else np.zeros(0, np.uint16)
    b, n, m, _ = oracle.tune(w)
    B = max(oracle.default_block(n_elems), 4096) if L == 32 else oracle.default_block(n_elems)
    check_both_ways(gpu, oracle, w, (b, n, m, L), BF16, B, f"L={L} n_elems={n_elems}")


def test_joint_tuner_and_ratio_gain(gpu, oracle):
    """The device tuner with Eq. 4's joint search agrees with the oracle's and picks L = 8 on Gaussian weights,
    which compresses a little better than the paper's L = 16."""
    w = W.config1()
    src = gpu.to_dev(w, BF16)
    p16 = gpu.enec.tune(src, gpu.ws)
    pj = gpu.enec.tune(src, gpu.ws, lengths=(8, 16, 32))
    assert p16 == oracle.tune(w) and pj == oracle.tune(w, lengths=(8, 16, 32)) and pj[3] == 8
    s16 = check_both_ways(gpu, oracle, w, p16, BF16, 16384, "config1 L=16")
    s8 = check_both_ways(gpu, oracle, w, pj, BF16, 16384, "config1 joint")
    assert s8.size < s16.size


def test_joint_tuner_respects_the_block_size(gpu, oracle):
    """A tensor shorter than 4096 elements is compressed with blocks of 2048, which do not admit L = 32."""
    w = np.full(3000, 0x3F80, np.uint16)                 # a constant tensor: Eq. 4 prefers the longest group
    src = gpu.to_dev(w, BF16)
    assert oracle.tune(w, lengths=(8, 16, 32))[3] == 32
    prm = gpu.enec.tune(src, gpu.ws, lengths=(8, 16, 32))
    assert prm[3] == 16 and prm == oracle.tune(w, lengths=(8, 16))
    check_both_ways(gpu, oracle, w, prm, BF16, 0, "short constant tensor")


def test_invalid_combinations_are_refused(gpu):
    torch, enec = gpu.torch, gpu.enec
    src = torch.zeros(1 << 16, dtype=torch.int16, device="cuda")
    out = torch.zeros(enec.compress_bound(1 << 16), dtype=torch.uint8, device="cuda")
    assert enec.compress(src, (122, 6, 3, 32), out, gpu.ws, block_size=2048) == enec.E_PARAMS    # mask < 16 bytes
    assert enec.compress(src, (122, 6, 3, 8), out, gpu.ws, block_size=32768) == enec.E_PARAMS    # > 64 mask words
    assert enec.compress(src, (122, 6, 3, 12), out, gpu.ws) == enec.E_PARAMS


def test_mixed_batch(gpu, oracle):
    """One call with tensors of different group lengths: one launch per (m, n - m, L)."""
    torch, enec = gpu.torch, gpu.enec
    ts = [W.gaussian(70000, 0.02, 1), W.gaussian(16384 * 3, 0.02, 2), W.gaussian(40000, 0.02, 3)]
    prm = []
    for t, L in zip(ts, (8, 16, 32)):
        b, n, m, _ = oracle.tune(t)
        prm.append((b, n, m, L))
    srcs = [gpu.to_dev(t, BF16) for t in ts]
    outs = [torch.zeros(enec.compress_bound(t.size), dtype=torch.uint8, device="cuda") for t in ts]
    sizes = torch.zeros(3, dtype=torch.int64, device="cuda")
    assert enec.compress_batch(srcs, prm, outs, gpu.ws, out_bytes=[sizes[i:i + 1] for i in range(3)]) == 0
    torch.cuda.synchronize()
    want = [oracle.compress(t, p, 16384)[1] for t, p in zip(ts, prm)]
    for i in range(3):
        assert int(sizes[i]) == want[i].size and np.array_equal(outs[i][:want[i].size].cpu().numpy(), want[i]), i
    backs = [torch.zeros_like(s) for s in srcs]
    assert enec.decompress_batch(outs, [w[:64].tobytes() for w in want], backs) == 0
    torch.cuda.synchronize()
    for b, t in zip(backs, ts):
        assert np.array_equal(b.cpu().numpy().view(np.uint16), t)
