"""Pins of the oracle's sampled tuner and its fall-back (CPU only).

Sec. V-E tunes on the exponent histogram; a sample makes phase 1 cheap, and an exponent the sample
misses can fall outside the window of Sec. V-C, for which the full exponent width (a bijection) is
the remedy.  Checked without the oracle's own vectorised selection: the index rule by a plain loop,
every = 1 against the unsampled tuner, the fall-back against a hand-built case and a round trip.
"""
import numpy as np

from paper_2604_03298_amd import workloads as W

BF16, FP16, FP32 = 0, 1, 2


def test_sample_is_every_kth_chunk_of_4096(oracle):
    w = (np.arange(4096 * 7 + 123) % 65521).astype(np.uint16)
    for every in (1, 2, 3, 7, 8, 100):
        want = [int(w[e]) for e in range(w.size) if (e // 4096) % every == 0]
        assert [int(v) for v in oracle.sample(w, every)] == want
    assert oracle.sample(w[:0], 3).size == 0
    # every = 1: nothing is left out, so the tuple is the unsampled tuner's
    g = W.gaussian(50000, 0.02, 3)
    assert oracle.tune(oracle.sample(g, 1)) == oracle.tune(g)


def test_fall_back_widens_n_and_round_trips(oracle):
    w = W.gaussian(4096 * 6, 0.02, 11)
    prm = oracle.tune(oracle.sample(w, 2))
    assert prm[1] < 8
    used, rc, s = oracle.compress_sampled(w, 2, 2048)
    assert rc == oracle.OK and used == prm                      # the sample was representative
    # plant one huge value in a chunk the sample skips (chunk 1): exponent 0xFE is far outside
    w2 = w.copy()
    w2[4096 + 17] = 0x7F00
    assert oracle.tune(oracle.sample(w2, 2)) == prm
    assert oracle.compress(w2, prm, 2048)[0] == oracle.E_RANGE
    used, rc, s = oracle.compress_sampled(w2, 2, 2048)
    assert rc == oracle.OK and used == (prm[0], 8, prm[2], prm[3])
    assert oracle.stream_info(s)["params"] == used
    rc, d = oracle.decompress(s, w2.size)
    assert rc == oracle.OK and (d == w2).all()
    # the same for fp16, whose exponent field has 5 bits
    h = W.gaussian_fp16(4096 * 4, 0.02, 5)
    prm = oracle.tune(oracle.sample(h, 4, FP16), FP16)
    h[4096 * 2 + 1] = 0x7BFF
    used, rc, s = oracle.compress_sampled(h, 4, 2048, FP16)
    if prm[1] < 5:
        assert used == (prm[0], 5, prm[2], prm[3])
    rc2, d = oracle.decompress(s, h.size)
    assert rc == oracle.OK and rc2 == oracle.OK and (d == h).all()
