"""GPU parity of the sampled tuner and of compression with its fall-back, against the CPU oracle."""
import numpy as np
import pytest

from paper_2604_03298_amd import workloads as W
from test_gpu_dtypes import gpu, BF16, FP16, FP32, WORD  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def _cases():
    yield BF16, W.gaussian(4096 * 37 + 1234, 0.02, 1)
    yield BF16, W.gaussian(4096 * 3 - 5, 0.02, 2)
    yield BF16, W.gaussian(7, 0.02, 3)
    yield BF16, W.gaussian(4096 * 64 + 3, 0.003, 4)
    yield FP16, W.gaussian_fp16(4096 * 21 + 77, 0.02, 5)
    yield FP32, W.gaussian_fp32(4096 * 19 + 2, 0.02, 6)
    yield FP32, W.gaussian_fp32(4096 * 4 + 1, 0.02, 7)


def test_sampled_histogram_and_tuple_match_the_oracle(gpu, oracle):
    for i, (dt, w) in enumerate(_cases()):
        src = gpu.to_dev(w, dt)[:w.size]
        for every in (1, 2, 3, 5, 16, 1000):
            prm, hist = gpu.enec.tune_sampled(src, every, gpu.ws, dtype=dt, want_histogram=True)
            picked = oracle.sample(w, every, dt)
            assert np.array_equal(hist, oracle.histogram(picked, dt)), (i, every)
            assert prm == oracle.tune(picked, dt), (i, every)


def test_compress_sampled_with_and_without_fall_back(gpu, oracle):
    torch, enec = gpu.torch, gpu.enec
    for dt, w, where, big in ((BF16, W.gaussian(4096 * 40 + 11, 0.02, 8), 4096 * 3 + 9, 0x7F00),
                              (FP16, W.gaussian_fp16(4096 * 33, 0.02, 9), 4096 * 5 + 1, 0x7BFF),
                              (FP32, W.gaussian_fp32(4096 * 17 + 100, 0.02, 10), 4096 * 7, 0x7F000001)):
        for planted in (False, True):
            v = w.copy()
            if planted:
                v[where] = big
            for every in (1, 4):
                used_o, rc_o, s_o = oracle.compress_sampled(v, every, 16384, dt)
                assert rc_o == oracle.OK
                src = gpu.to_dev(v, dt)
                cap = enec.compress_bound(v.size, dtype=dt)
                out = torch.full((cap + 64,), 0xA5, dtype=torch.uint8, device="cuda")
                rc, used = enec.compress_sampled(src, every, out, gpu.ws, dtype=dt)
                assert rc == 0 and used == used_o, (dt, planted, every)
                got = out.cpu().numpy()
                assert np.array_equal(got[:s_o.size], s_o), (dt, planted, every)
                assert (got[cap:] == 0xA5).all()
                # with every = 4 chunk 3, 5 and 7 are outside the sample, so the planted value forces the fall-back
                if planted and every == 4:
                    assert used[1] == (5 if dt == FP16 else 8)
                back = gpu.decompress(got[:s_o.size], v.size, dt)
                assert back[0] == 0 and np.array_equal(back[1], v)


def test_every_zero_is_an_argument_error(gpu):
    src = gpu.to_dev(W.gaussian(4096, 0.02, 1), BF16)
    p = gpu.enec.Params()
    import ctypes as C
    rc = gpu.enec.lib().enec_tune_sampled(C.c_void_p(src.data_ptr()), 4096, 0, 0, C.byref(p), None,
                                          C.c_void_p(gpu.ws.data_ptr()), gpu.ws.numel(), None)
    assert rc == gpu.enec.E_ARG


def test_batched_tuner_matches_the_oracle(gpu, oracle):
    """Twenty tensors (two rounds of sixteen slots), one empty: histograms and tuples against the oracle's, for all
    exponents and for a sample; enec_compress_batch tunes the tensors it gets without a tuple the same way."""
    torch, enec = gpu.torch, gpu.enec
    ws = [W.gaussian(4096 * (3 + 2 * i) + 17 * i, 0.005 * (1 + i % 5), 100 + i) for i in range(19)]
    ws.insert(7, np.zeros(0, np.uint16))
    srcs = [gpu.to_dev(w, BF16)[:w.size] for w in ws]
    for every in (1, 3):
        prm, hist = enec.tune_batch(srcs, gpu.ws, every=every, want_histograms=True)
        for i, w in enumerate(ws):
            picked = oracle.sample(w, every)
            assert np.array_equal(hist[i], oracle.histogram(picked)), (every, i)
            assert prm[i] == oracle.tune(picked), (every, i)
    f = [W.gaussian_fp32(5000 + 4096 * i, 0.02, i) for i in range(3)]
    prm = enec.tune_batch([gpu.to_dev(w, FP32) for w in f], gpu.ws, dtype=FP32)
    assert prm == [oracle.tune(w, FP32) for w in f]
    some = [w for w in ws if w.size][:5]
    dev = [gpu.to_dev(w, BF16) for w in some]
    outs = [torch.zeros(enec.compress_bound(w.size), dtype=torch.uint8, device="cuda") for w in some]
    assert enec.compress_batch(dev, [None] * len(some), outs, gpu.ws) == 0
    torch.cuda.synchronize()
    for w, o in zip(some, outs):
        want = oracle.compress(w, oracle.tune(w), oracle.default_block(w.size))[1]
        assert np.array_equal(o.cpu().numpy()[:want.size], want)
