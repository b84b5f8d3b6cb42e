"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and its pure host functions agree with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

from conftest import ROOT
from paper_2604_03298_amd import workloads as W


@pytest.fixture(scope="module")
def enec():
    from paper_2604_03298_amd import enec as E
    if not os.path.exists(E.LIB_PATH):
        from paper_2604_03298_amd import build
        build.build()
    E.lib()
    return E


def test_library_exports_every_declared_symbol(enec):
    text = open(os.path.join(ROOT, "include", "enec.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(enec_[a-z_0-9]+)\s*\(", text))
    assert declared == set(enec.EXPORTS), declared ^ set(enec.EXPORTS)
    lib = ctypes.CDLL(enec.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_version_and_strerror(enec):
    assert enec.version() == 1
    msgs = {enec.strerror(i) for i in range(9)}
    assert len(msgs) == 9 and enec.strerror(99) == "unknown status"


def test_bounds_and_block_sizes_match_oracle(enec, oracle):
    for n in [0, 1, 100, 2047, 2048, 2049, 4096, 5000, 16383, 16384, 16385, 1 << 20, (1 << 26) + 3]:
        assert enec.default_block_size(n) == oracle.default_block(n)
        for B in [2048, 4096, 8192, 16384, 32768]:
            assert enec.compress_bound(n, block_size=B) == oracle.compress_bound(n, B)
        assert enec.compress_bound(n) == oracle.compress_bound(n, oracle.default_block(n))
        assert enec.workspace_bytes(n) >= 1024 + 16 * 2048 + 8 * max(1, oracle.num_blocks(n, oracle.default_block(n)))
        assert enec.workspace_bytes(n) % 256 == 0
        for dt in (1, 2):                     # fp16, fp32
            for B in [2048, 16384]:
                assert enec.compress_bound(n, dtype=dt, block_size=B) == oracle.compress_bound(n, B, dt)
                assert enec.compress_bound_per_block(n, dtype=dt, block_size=B) == oracle.compress_bound_pb(n, B, dt)
    assert enec.compress_bound(100, block_size=3000) == 0
    assert enec.compress_bound(100, dtype=3) == 0
    assert enec.workspace_bytes(100, block_size=1000) == 0


def test_host_tuner_matches_oracle(enec, oracle, ref):
    rng = np.random.default_rng(17)
    hists = [oracle.histogram(W.config1()), oracle.histogram(W.gaussian(100000, 0.3, 2)),
             oracle.histogram(np.zeros(100, np.uint16)), np.zeros(256, np.uint64),
             oracle.histogram(W.config3(n_blocks=16)[0]),
             oracle.histogram(W.norm_vector(4096, 27))]
    for _ in range(200):
        h = np.zeros(256, np.uint64)
        lo = int(rng.integers(0, 250)); width = int(rng.integers(1, 256 - lo))
        idx = rng.integers(lo, lo + width, size=int(rng.integers(1, 40)))
        h[idx] = rng.integers(1, 1 << int(rng.integers(1, 40)), size=idx.size).astype(np.uint64)
        hists.append(h)
    for h in hists:
        assert enec.tune_histogram(h) == oracle.tune_hist(h)[0]
    for h in hists[:20]:
        assert enec.tune_histogram(h) == ref.tune_hist([int(v) for v in h])[0]
    # fp16: 32 exponent values, Eq. 1's width capped at 5
    for _ in range(200):
        h = np.zeros(256, np.uint64)
        lo = int(rng.integers(0, 31)); width = int(rng.integers(1, 33 - lo))
        idx = rng.integers(lo, lo + width, size=int(rng.integers(1, 12)))
        h[idx] = rng.integers(1, 1 << int(rng.integers(1, 40)), size=idx.size).astype(np.uint64)
        assert enec.tune_histogram(h, dtype=1) == oracle.tune_hist(h, 5)[0]
    with pytest.raises(Exception):
        enec.tune_histogram(hists[0], dtype=7)
    # Eq. 4 with the group length searched together with m
    for h in hists[:60]:
        for lengths in ((8, 16, 32), (16,), (8,), (16, 32)):
            assert enec.tune_histogram(h, lengths=lengths) == oracle.tune_hist_groups(h, 8, lengths)[0]
    with pytest.raises(Exception):
        enec.tune_histogram(hists[0], lengths=(4,))
    # the library drops the lengths the block size does not admit (128 L <= B <= 2048 L): L = 32 needs B >= 4096,
    # L = 8 needs B <= 16384, and 16 stands in when nothing is left
    for h in hists[:30]:
        assert enec.tune_histogram(h, lengths=(8, 16, 32), block_size=2048) == oracle.tune_hist_groups(h, 8, (8, 16))[0]
        assert enec.tune_histogram(h, lengths=(8, 16, 32), block_size=32768) == oracle.tune_hist_groups(h, 8, (16, 32))[0]
        assert enec.tune_histogram(h, lengths=(8,), block_size=32768) == oracle.tune_hist(h)[0]
        assert enec.tune_histogram(h, lengths=(32,), block_size=2048) == oracle.tune_hist(h)[0]
    with pytest.raises(Exception):
        enec.tune_histogram(hists[0], lengths=(8, 16), block_size=3000)


def test_stream_info_parses_oracle_headers(enec, oracle):
    w = W.gaussian(40000, 0.02, 3)
    p = oracle.tune(w)
    rc, s = oracle.compress(w, p, 16384)
    info = enec.stream_info(s[:64])
    assert info == dict(rc=0, params=p, n_elems=w.size, block_size=16384, total_bytes=s.size,
                        dtype=0, status=0, per_block=False)
    bad = s[:64].copy(); bad[1] = 0
    assert enec.stream_info(bad)["rc"] == enec.E_FORMAT
    bad = s[:64].copy(); bad[4] = 2
    assert enec.stream_info(bad)["rc"] == enec.E_FORMAT


def test_null_and_misaligned_arguments_are_rejected_on_the_host(enec):
    L = enec.lib()
    p = enec.Params(122, 6, 3, 16)
    fake = ctypes.c_void_p(0x1000)       # never dereferenced: every call below fails its checks first
    odd = ctypes.c_void_p(0x1008)
    assert L.enec_compress(None, 10, 0, 0, ctypes.byref(p), fake, 1 << 20, None, fake, 1 << 20, None) == enec.E_ARG
    assert L.enec_compress(fake, 10, 0, 0, ctypes.byref(p), None, 1 << 20, None, fake, 1 << 20, None) == enec.E_ARG
    assert L.enec_compress(fake, 10, 0, 0, ctypes.byref(p), fake, 1 << 20, None, None, 1 << 20, None) == enec.E_ARG
    assert L.enec_compress(odd, 10, 0, 0, ctypes.byref(p), fake, 1 << 20, None, fake, 1 << 20, None) == enec.E_ARG
    assert L.enec_compress(fake, 10, 5, 0, ctypes.byref(p), fake, 1 << 20, None, fake, 1 << 20, None) == enec.E_DTYPE
    assert L.enec_compress(fake, 10, 0, 1000, ctypes.byref(p), fake, 1 << 20, None, fake, 1 << 20, None) == enec.E_BLOCK
    assert L.enec_compress(fake, 10, 0, 0, ctypes.byref(p), fake, 10, None, fake, 1 << 20, None) == enec.E_CAPACITY
    assert L.enec_compress(fake, 10, 0, 0, ctypes.byref(p), fake, 1 << 20, None, fake, 16, None) == enec.E_CAPACITY
    assert L.enec_compress(fake, 1 << 35, 0, 0, ctypes.byref(p), fake, 1 << 20, None, fake, 1 << 20, None) == enec.E_ARG
    for bad in [(122, 0, 0, 16), (122, 9, 3, 16), (122, 6, 7, 16), (122, 6, 3, 32)]:
        q = enec.Params(*bad)
        assert L.enec_compress(fake, 10, 0, 0, ctypes.byref(q), fake, 1 << 20, None, fake, 1 << 20, None) == enec.E_PARAMS
    hdr = (ctypes.c_uint8 * 64)()
    assert L.enec_decompress_with_header(fake, 1 << 20, hdr, fake, 10, None, None) == enec.E_FORMAT
    assert L.enec_decompress_with_header(None, 1 << 20, hdr, fake, 10, None, None) == enec.E_ARG
    assert L.enec_decompress_with_header(fake, 1 << 20, None, fake, 10, None, None) == enec.E_ARG
    assert L.enec_decompress(fake, 10, fake, 10, None) == enec.E_FORMAT
    assert L.enec_workspace_init(None, 16, None) == enec.E_ARG
    assert L.enec_workspace_init(fake, 17, None) == enec.E_ARG
    assert L.enec_copy(fake, odd, 16, None) == enec.E_ARG
    assert L.enec_tune_histogram(None, 0, ctypes.byref(p)) == enec.E_ARG
    assert L.enec_tune_sampled(fake, 10, 0, 0, ctypes.byref(p), None, fake, 1 << 20, None) == enec.E_ARG
    for dt, bad in ((1, (10, 6, 2, 16)), (1, (40, 4, 2, 16)), (2, (122, 9, 3, 16)), (0, (122, 6, 3, 12)), (0, (122, 6, 3, 64))):
        q = enec.Params(*bad)
        assert L.enec_compress(fake, 10, dt, 0, ctypes.byref(q), fake, 1 << 20, None, fake, 1 << 20, None) == enec.E_PARAMS
    assert L.enec_compress(fake, 10, 3, 0, ctypes.byref(p), fake, 1 << 20, None, fake, 1 << 20, None) == enec.E_DTYPE
    assert L.enec_stream_info(None, None, None, None, None, None, None) == enec.E_ARG


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2604_03298_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                for needle in ("import oracle", "from oracle", "enec_oracle", "enec_ref", "orc_"):
                    assert needle not in src, (f, needle)


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: `bench.py --gpus N` with N > 1 exits with a message, before anything touches a GPU."""
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr or "one GPU" in res.stderr.lower()


def test_stream_info_reads_oracle_headers(oracle):
    """The library's header parser against headers the oracle wrote: one tuple per tensor, one per data block, a bad byte 40."""
    import numpy as np
    from paper_2604_03298_amd import enec, workloads as W
    w = W.gaussian(5000, 0.02, 3)
    prm = oracle.tune(w)
    one = oracle.compress(w, prm, 2048)[1]
    info = enec.stream_info(one[:64])
    assert info["rc"] == 0 and info["params"] == prm and not info["per_block"]
    assert info["n_elems"] == 5000 and info["block_size"] == 2048 and info["total_bytes"] == one.size and info["status"] == 0
    per = oracle.compress_per_block(w, 2048, 0, 8)[1]
    info = enec.stream_info(per[:64])
    assert info["rc"] == 0 and info["per_block"] and info["params"] == (0, 0, 0, 8) and info["total_bytes"] == per.size
    bad = per[:64].copy()
    bad[40] = 2
    assert enec.stream_info(bad)["rc"] == enec.E_FORMAT
