"""Pins of the oracle for fp16 and fp32 tensors (CPU only).

The paper codes exponents only and keeps sign and mantissa raw (Sec. IV-B, Alg. 1 input line "BF16/FP16/FP32";
Sec. VI-B), Table VI lists fp16 tuples with n <= 5 and fp32 tuples of the bf16 family.  What is checked here
does not come from the C oracle itself: hand-worked blocks, the reduction of fp32 to the (already pinned) bf16
codec on the upper halves, the size accounting, exhaustive round trips, the pure-Python twin.
"""
import struct

import numpy as np
import pytest

from conftest import golden_lines

BF16, FP16, FP32 = 0, 1, 2


def _pairs(text):
    return {int(i): int(v, 16) for i, v in (t.split(":") for t in text.split())}


def test_fp16_block_worked_by_hand(oracle, ref):
    g = dict(ln.split(None, 1) for ln in golden_lines("block128_fp16_handworked.txt"))
    w = np.full(128, 0x2800, np.uint16)
    w[5], w[70], w[100] = 0x2805, 0xA7FF, 0x3408
    prm = (10, 4, 2, 16)
    rc, s = oracle.compress(w, prm, 128, dtype=FP16)
    assert rc == oracle.OK and s.size == int(g["stream_bytes"])
    base = int(g["payload_base"])
    assert oracle.payload_base(128, 128, FP16) == base
    assert [int(s[6]), int(s[27])] == [int(v) for v in g["header_dtype_expbits"].split()]
    assert list(struct.unpack_from("<2Q", s.tobytes(), 64)) == [int(v) for v in g["offset_table"].split()]
    sm, mask = s[base:base + 128], int(s[base + 128])
    low, high = s[base + 129:base + 129 + 80], s[base + 209:base + 213]
    exp = np.zeros(128, np.uint8)
    for i, v in _pairs(g["sm_nonzero"]).items():
        exp[i] = v
    assert (sm == exp).all()
    assert mask == int(g["mask_byte"], 16)
    exp = np.zeros(80, np.uint8)
    for i, v in _pairs(g["low_plane_nonzero"]).items():
        exp[i] = v
    assert (low == exp).all()
    assert high.tobytes() == bytes(int(h, 16) for h in g["high_record"].split())
    assert (s[base + 213:] == 0).all()
    ok, s2 = ref.compress(w, prm, 128, FP16)
    assert ok and s2 == s.tobytes()
    rc, d = oracle.decompress(s, 128)
    assert rc == oracle.OK and d.dtype == np.uint16 and (d == w).all()
    assert ref.decompress(s.tobytes(), 128) == [int(x) for x in w]


def test_fp32_block_worked_by_hand(oracle, ref):
    g = dict(ln.split(None, 1) for ln in golden_lines("block128_fp32_handworked.txt"))
    hi = np.full(128, 0x3D00, np.uint16)
    hi[17], hi[40] = 0x3D80, 0xBD05
    w = hi.astype(np.uint32) << 16
    w[17] |= 0x1234
    w[40] |= 0xFFFF
    w[127] |= 0xABCD
    prm = (122, 6, 3, 16)
    rc, s = oracle.compress(w, prm, 128, dtype=FP32)
    assert rc == oracle.OK and s.size == int(g["stream_bytes"])
    tail_at, base = int(g["tail_at"]), int(g["payload_base"])
    assert oracle.table_end(128, 128) == tail_at and oracle.payload_base(128, 128, FP32) == base
    assert [int(s[6]), int(s[27])] == [int(v) for v in g["header_dtype_expbits"].split()]
    assert list(struct.unpack_from("<2Q", s.tobytes(), 64)) == [int(v) for v in g["offset_table"].split()]
    exp = np.zeros(256, np.uint8)
    for i, v in _pairs(g["tail_nonzero"]).items():
        exp[i] = v
    assert (s[tail_at:base] == exp).all()
    # the payload is the hand-worked bf16 payload of the upper halves
    rc16, s16 = oracle.compress(hi, prm, 128)
    assert rc16 == oracle.OK and (s[base:] == s16[80:]).all()
    ok, s2 = ref.compress(w, prm, 128, FP32)
    assert ok and s2 == s.tobytes()
    rc, d = oracle.decompress(s, 128)
    assert rc == oracle.OK and d.dtype == np.uint32 and (d == w).all()
    assert ref.decompress(s.tobytes(), 128) == [int(x) for x in w]


@pytest.mark.parametrize("n_elems,B", [(5000, 2048), (16384 * 2 + 77, 16384), (1, 2048)])
def test_fp32_is_the_bf16_codec_on_the_upper_halves(oracle, n_elems, B):
    """Only the 8 exponent bits are coded (Sec. VI-B): the fp32 stream is the bf16 stream of the upper halves
    with the lower halves inserted after the table."""
    rng = np.random.default_rng(5)
    w = (0.02 * rng.standard_normal(n_elems)).astype(np.float32).view(np.uint32)
    hi = (w >> 16).astype(np.uint16)
    prm = oracle.tune(hi)
    assert oracle.tune(w, FP32) == prm
    rc, s = oracle.compress(w, prm, B, dtype=FP32)
    rc16, s16 = oracle.compress(hi, prm, B)
    assert rc == rc16 == oracle.OK
    te = oracle.table_end(n_elems, B)
    tail = (2 * n_elems + 15) & ~15
    assert s.size == s16.size + tail
    assert (s[64:te] == s16[64:te]).all()                                   # same offsets
    assert (s[te:te + 2 * n_elems].view("<u2") == (w & 0xFFFF)).all()       # lower halves, element order
    assert (s[te + 2 * n_elems:te + tail] == 0).all()
    assert (s[te + tail:] == s16[te:]).all()                                # same payloads
    h, h16 = s[:64].copy(), s16[:64].copy()
    assert h[6] == FP32 and h16[6] == BF16
    assert struct.unpack_from("<Q", h.tobytes(), 32)[0] == s.size
    h[6] = 0
    h[32:40] = h16[32:40]
    assert (h == h16).all()
    rc, d = oracle.decompress(s, n_elems)
    assert rc == oracle.OK and (d == w).all()


def test_fp16_every_bit_pattern_survives(oracle):
    """All 65536 fp16 patterns (NaN payloads, infinities, subnormals, both zeros) with the bijective n = 5."""
    w = np.arange(65536, dtype=np.uint16)
    np.random.default_rng(1).shuffle(w)
    for prm in [(15, 5, 3, 16), (0, 5, 0, 16), (31, 5, 5, 16), (7, 5, 1, 16)]:
        rc, s = oracle.compress(w, prm, 4096, dtype=FP16)
        assert rc == oracle.OK
        rc, d = oracle.decompress(s, w.size)
        assert rc == oracle.OK and (d == w).all()


def test_fp32_special_values_survive(oracle):
    vals = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-45, -1e-45, 3.4e38, 1.17549435e-38], np.float32)
    w = np.concatenate([vals.view(np.uint32), np.array([0x7FC12345, 0xFFFFFFFF, 0x00000001, 0x807FFFFF], np.uint32)])
    w = np.tile(w, 200)
    rc, s = oracle.compress(w, oracle.tune(w, FP32), 2048, dtype=FP32)
    assert rc == oracle.OK
    rc, d = oracle.decompress(s, w.size)
    assert rc == oracle.OK and (d == w).all()


def test_fp16_window_and_range_error(oracle, ref):
    """n < 5: exponents outside [b - 2^(n-1) + 1, b + 2^(n-1)] are a range error; the transform is Eq. 2 mod 2^n."""
    b, n = 12, 3
    for x in range(32):
        ok = -(1 << (n - 1)) <= b - x <= (1 << (n - 1)) - 1
        assert oracle.in_range_e(x, b, n, 5) == ok == ref.in_range(x, b, n, 5)
        if ok:
            y = oracle.transform(x, b, n)
            assert y == (b - x) % 8 and oracle.inverse_transform_e(y, b, n, 5) == x == ref.inverse_transform(y, b, n, 5)
    for b in range(32):                     # n = 5 is a bijection of the 32 exponents whatever b
        ys = {oracle.transform(x, b, 5) for x in range(32)}
        assert len(ys) == 32
        assert all(oracle.inverse_transform_e(oracle.transform(x, b, 5), b, 5, 5) == x for x in range(32))
    w = np.full(2048, 12 << 10, np.uint16)
    w[100] = 17 << 10                      # b - x = -5 is outside [-4, 3]
    rc, s = oracle.compress(w, (12, 3, 1, 16), 2048, dtype=FP16)
    assert rc == oracle.E_RANGE and struct.unpack_from("<IQ", s.tobytes(), 28) == (oracle.E_RANGE, 0)
    w[100] = 16 << 10                      # -4 is the edge
    rc, s = oracle.compress(w, (12, 3, 1, 16), 2048, dtype=FP16)
    assert rc == oracle.OK
    assert oracle.compress(w, (12, 6, 1, 16), 2048, dtype=FP16)[0] == oracle.E_PARAMS     # n > 5 exponent bits


def test_fp16_tuner_family_and_ratio(oracle, ref):
    """Gaussian fp16 weights land in Table VI's fp16 family (n of 4 or 5, m = 3) and near its ratios
    (Table III / the per-model table: 1.09 - 1.12); Eq. 1's width is capped at the 5 exponent bits."""
    rng = np.random.default_rng(11)
    w = (0.02 * rng.standard_normal(1 << 20)).astype(np.float16).view(np.uint16)
    prm = oracle.tune(w, FP16)
    assert prm[1] in (4, 5) and prm[2] in (2, 3) and prm[3] == 16 and 7 <= prm[0] <= 11
    assert ref.tune(w[:20000], FP16) == oracle.tune(w[:20000], FP16)
    rc, s = oracle.compress(w, prm, 16384, dtype=FP16)
    assert rc == oracle.OK
    ratio = 2 * w.size / s.size
    assert 1.07 < ratio < 1.16
    for l in range(32):
        for h in range(l, 32):
            for b in range(l, h + 1):
                assert oracle.width_for_e(b, l, h, 5) == min(5, oracle.width_for(b, l, h)) == ref.width_for(b, l, h, 5)


@pytest.mark.parametrize("dtype", [FP16, FP32])
def test_size_accounting(oracle, dtype):
    """bits per element = raw bits + 1/16 + m + (n - m) f, f = fraction of anomalous groups (the accounting of
    the paper's appendix example), block by block: S_k = pad16(B + B/128 + low*B/8 + 2(n-m) cnt_k)."""
    rng = np.random.default_rng(21)
    n_elems, B = 16384 * 3 + 1000, 16384
    if dtype == FP32:
        w = (0.02 * rng.standard_normal(n_elems)).astype(np.float32).view(np.uint32)
    else:
        w = (0.02 * rng.standard_normal(n_elems)).astype(np.float16).view(np.uint16)
    b, n, m, L = oracle.tune(w, dtype)
    rc, s = oracle.compress(w, (b, n, m, L), B, dtype=dtype)
    assert rc == oracle.OK
    nb = 4
    te = oracle.table_end(n_elems, B)
    base = oracle.payload_base(n_elems, B, dtype)
    assert base == te + (((2 * n_elems + 15) & ~15) if dtype == FP32 else 0)
    offs = np.frombuffer(s[64:64 + 8 * (nb + 1)].tobytes(), dtype="<u8")
    low = m + (3 if dtype == FP16 else 0)
    for k in range(nb):
        p = base + int(offs[k]) + B
        cnt = int(np.unpackbits(s[p:p + B // 128]).sum())
        S = (B + B // 128 + low * B // 8 + 2 * (n - m) * cnt + 15) & ~15
        assert int(offs[k + 1] - offs[k]) == S
    assert s.size == base + int(offs[nb])


@pytest.mark.parametrize("dtype", [FP16, FP32])
def test_twin_agrees_on_random_small_blocks(oracle, ref, dtype):
    rng = np.random.default_rng(31 + dtype)
    E = 5 if dtype == FP16 else 8
    for trial in range(12):
        n_elems = int(rng.integers(1, 700))
        B = int(rng.choice([128, 256]))
        n = int(rng.integers(1, E + 1))
        m = int(rng.integers(0, n + 1))
        b = int(rng.integers(0, 1 << E))
        lo, hi = max(0, b - (1 << (n - 1)) + 1), min((1 << E) - 1, b + (1 << (n - 1)))
        if n == E:
            lo, hi = 0, (1 << E) - 1
        x = rng.integers(lo, hi + 1, n_elems)
        if dtype == FP16:
            w = ((rng.integers(0, 2, n_elems) << 15) | (x << 10) | rng.integers(0, 1024, n_elems)).astype(np.uint16)
        else:
            w = ((rng.integers(0, 2, n_elems) << 31) | (x << 23) | rng.integers(0, 1 << 23, n_elems)).astype(np.uint32)
        rc, s = oracle.compress(w, (b, n, m, 16), B, dtype=dtype)
        assert rc == oracle.OK, (b, n, m)
        ok, s2 = ref.compress(w, (b, n, m, 16), B, dtype)
        assert ok and s2 == s.tobytes()
        rc, d = oracle.decompress(s, n_elems)
        assert rc == oracle.OK and (d == w).all()
        assert ref.decompress(s.tobytes(), n_elems) == [int(v) for v in w]


def test_empty_tensors(oracle):
    for dtype, dt in ((FP16, np.uint16), (FP32, np.uint32)):
        rc, s = oracle.compress(np.zeros(0, dt), (0, 1, 0, 16), 2048, dtype=dtype)
        assert rc == oracle.OK and s.size == 80 and s[6] == dtype
        rc, d = oracle.decompress(s, 0)
        assert rc == oracle.OK and d.size == 0
