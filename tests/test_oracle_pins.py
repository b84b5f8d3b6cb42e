"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each pin is chosen so that a plausible
mistake in the oracle (dropped term, wrong sign or index, transposed operand, wrong
byte order) fails at least one of them.
"""
import math
import struct

import numpy as np
import pytest

from conftest import golden_lines
from paper_2604_03298_amd import workloads as W


# --------------------------------------------------------------------------
# transform (Sec. V-C, Eq. 2)
# --------------------------------------------------------------------------
def test_transform_paper_example(oracle, ref):
    for ln in golden_lines("transform_example.txt"):
        b, n, x, y = map(int, ln.split())
        assert oracle.transform(x, b, n) == y
        assert ref.transform(x, b, n) == y
        assert oracle.inverse_transform(y, b, n) == x
        assert ref.inverse_transform(y, b, n) == x


def test_width_matches_printed_eq1_where_defined(oracle, ref):
    # Eq. 1 as printed needs b - l >= 1 and h - b >= 1.
    for dl in range(1, 130):
        for dh in range(1, 130):
            n_eq1 = max(math.floor(math.log2(dl)) + 1, math.ceil(math.log2(dh))) + 1
            b = dl
            got = oracle.width_for(b, 0, b + dh) if b + dh <= 255 else None
            if got is not None:
                assert got == min(8, n_eq1)
                assert ref.width_for(b, 0, b + dh) == got


def test_width_is_minimal_and_sufficient_exhaustive(ref):
    # For every (b - l, h - b): both ends of [l, h] are representable with n(b) bits and,
    # unless n is 1 or capped, not with n - 1 bits.
    for dl in range(0, 256):
        for dh in range(0, 256 - dl):
            l, b, h = 0, dl, dl + dh
            n = ref.width_for(b, l, h)
            assert ref.in_range(l, b, n) and ref.in_range(h, b, n)
            if 1 < n < 8 or (n == 8 and not (ref.in_range(l, b, 7) and ref.in_range(h, b, 7))):
                if n > 1:
                    assert not (ref.in_range(l, b, n - 1) and ref.in_range(h, b, n - 1))


def test_transform_injective_and_invertible_on_window(oracle, ref):
    rng = np.random.default_rng(7)
    cases = [(0, 0, 0), (0, 0, 255), (0, 255, 255), (101, 122, 123), (96, 121, 127), (0, 127, 255)]
    for _ in range(300):
        l = int(rng.integers(0, 256)); h = int(rng.integers(l, 256)); b = int(rng.integers(l, h + 1))
        cases.append((l, b, h))
    for l, b, h in cases:
        n = oracle.width_for(b, l, h)
        assert n == ref.width_for(b, l, h)
        ys = [oracle.transform(x, b, n) for x in range(l, h + 1)]
        assert ys == [ref.transform(x, b, n) for x in range(l, h + 1)]
        assert len(set(ys)) == len(ys) and all(0 <= y < (1 << n) for y in ys)
        assert [oracle.inverse_transform(y, b, n) for y in ys] == list(range(l, h + 1))
        assert all(oracle.in_range(x, b, n) for x in range(l, h + 1))


def test_transform_exhaustive_against_twin(oracle, ref):
    for n in range(1, 9):
        for b in range(0, 256, 5):
            for x in range(256):
                assert oracle.transform(x, b, n) == ref.transform(x, b, n)
                assert oracle.in_range(x, b, n) == ref.in_range(x, b, n)
    # n = 8 is a bijection of all exponents whatever b is
    for b in (0, 1, 127, 128, 255):
        ys = [oracle.transform(x, b, 8) for x in range(256)]
        assert sorted(ys) == list(range(256))
        assert [oracle.inverse_transform(y, b, 8) for y in ys] == list(range(256))


def test_high_frequency_values_map_to_small_codes(oracle):
    # Sec. V-C: values just below b map to small positive codes, values above b wrap to the top.
    assert [oracle.transform(x, 122, 6) for x in (122, 121, 120, 119)] == [0, 1, 2, 3]
    assert [oracle.transform(x, 122, 6) for x in (123, 124)] == [63, 62]


# --------------------------------------------------------------------------
# Alg. 2
# --------------------------------------------------------------------------
def test_hh_handworked_vectors(oracle, ref):
    for ln in golden_lines("hh_handworked.txt"):
        a, vals, expect = [p.strip() for p in ln.split("|")]
        a = int(a)
        vals = [int(v) for v in vals.split()]
        expect = bytes(int(h, 16) for h in expect.split())
        assert oracle.hh_pack(vals, a).tobytes() == expect
        assert ref.hh_pack(vals, a) == expect
        assert list(oracle.hh_unpack(np.frombuffer(expect, np.uint8), len(vals), a)) == vals
        assert ref.hh_unpack(expect, len(vals), a) == vals


@pytest.mark.parametrize("a", range(1, 9))
@pytest.mark.parametrize("N", [16, 128, 2048])
def test_hh_is_a_bit_permutation_of_length_aN_over_8(oracle, a, N):
    # every one-hot input gives a one-hot output; all a*N positions are distinct; length a*N/8
    seen = set()
    elems = range(N) if N <= 128 else list(range(0, N, 37)) + [N - 1, N // 2, N // 2 - 1]
    for e in elems:
        for bit in range(a):
            v = np.zeros(N, np.uint16)
            v[e] = 1 << bit
            s = oracle.hh_pack(v, a)
            assert s.size == a * N // 8
            bits = np.unpackbits(s, bitorder="little")
            assert bits.sum() == 1
            pos = int(np.argmax(bits))
            assert pos not in seen
            seen.add(pos)


@pytest.mark.parametrize("a", range(1, 9))
def test_hh_roundtrip_and_twin(oracle, ref, a):
    rng = np.random.default_rng(100 + a)
    for N in (16, 32, 128, 1024, 16384):
        v = rng.integers(0, 1 << a, size=N, dtype=np.uint16)
        s = oracle.hh_pack(v, a)
        assert s.size == a * N // 8
        assert (oracle.hh_unpack(s, N, a) == v).all()
        if N <= 1024:
            assert ref.hh_pack([int(x) for x in v], a) == s.tobytes()
        if N <= 128:
            assert ref.hh_unpack(s.tobytes(), N, a) == [int(x) for x in v]


def test_hh_closed_forms_for_simple_widths(oracle):
    # a = 8: no folding; the stream is the join of the two halves.
    # a = 4: one fold pairs element i with element i + N/2 in one byte.
    # a = 1, N = 16: three folds give two bytes whose bit k holds element 2*k (+1).
    rng = np.random.default_rng(5)
    N = 64
    v = rng.integers(0, 256, size=N, dtype=np.uint16)
    s = oracle.hh_pack(v, 8)
    assert (s[0::2] == v[:N // 2]).all() and (s[1::2] == v[N // 2:]).all()
    v = rng.integers(0, 16, size=N, dtype=np.uint16)
    s = oracle.hh_pack(v, 4)
    nb = (v[:N // 2] | (v[N // 2:] << 4)).astype(np.uint8)
    assert (s[0::2] == nb[:N // 4]).all() and (s[1::2] == nb[N // 4:]).all()
    v = rng.integers(0, 2, size=16, dtype=np.uint16)
    s = oracle.hh_pack(v, 1)
    # folds: lane i gets v[i] | v[i+8]<<1 | v[i+4]<<2 | v[i+12]<<3 | v[i+2]<<4 | ... (i < 2)
    order = [0, 8, 4, 12, 2, 10, 6, 14]
    for lane in range(2):
        byte = sum(int(v[lane + o]) << k for k, o in enumerate(order))
        assert s[lane] == byte


# --------------------------------------------------------------------------
# group test
# --------------------------------------------------------------------------
def test_or_test_equals_max_bit_width(oracle, ref):
    # C oracle uses the bitwise OR (Sec. V-B), the twin the definition (max width > m).
    rng = np.random.default_rng(11)
    for (b, n, m) in [(122, 6, 3), (123, 8, 4), (120, 5, 0), (125, 7, 7), (127, 2, 1)]:
        lo, hi = b - (1 << (n - 1)) + 1, b + (1 << (n - 1))
        x = rng.integers(max(lo, 0), min(hi, 255) + 1, size=256).astype(np.uint16)
        # make most groups quiet so that both mask values occur
        quiet = rng.random(256 // 16) < 0.6
        for g in np.nonzero(quiet)[0]:
            x[g * 16:(g + 1) * 16] = b - rng.integers(0, min(1 << m, 1 << (n - 1)), size=16)
        w = ((x << 7) | rng.integers(0, 128, size=256).astype(np.uint16)).astype(np.uint16)
        rc, s = oracle.compress(w, (b, n, m, 16), 128)
        assert rc == oracle.OK
        ok, s2 = ref.compress(w, (b, n, m, 16), 128)
        assert ok and s.tobytes() == s2


# --------------------------------------------------------------------------
# tuner (Sec. V-E)
# --------------------------------------------------------------------------
def test_tuner_lands_in_table6_family_on_gaussian(oracle):
    table = [ln.split() for ln in golden_lines("table6_bf16_params.txt")]
    bs = {int(r[1]) for r in table}
    assert {(int(r[2]), int(r[3]), int(r[4])) for r in table} == {(6, 3, 16)}
    w = W.config1()
    b, n, m, L = oracle.tune(w)
    assert (n, m, L) == (6, 3, 16)
    assert b in bs


def test_tuner_degenerate_tensors(oracle, ref):
    assert oracle.tune(np.zeros(4096, np.uint16)) == (0, 1, 0, 16)
    assert oracle.tune(np.full(4096, 0x3D12, np.uint16)) == (122, 1, 0, 16)
    assert oracle.tune(np.zeros(0, np.uint16)) == (0, 1, 0, 16)
    rng = np.random.default_rng(3)
    w = rng.integers(0, 1 << 16, size=1 << 16, dtype=np.uint16)
    p = oracle.tune(w)
    assert p[1] == 8
    assert ref.tune_hist(oracle.histogram(w))[0] == p


def test_tuner_cost_is_the_true_minimum(oracle, ref):
    # D of the returned b equals the brute-force minimum of sum c[x]*y over all b in [l, h].
    for seed, std in [(1, 0.02), (2, 0.004), (3, 0.3)]:
        w = W.gaussian(1 << 16, std, seed)
        hist = oracle.histogram(w)
        assert int(hist.sum()) == w.size
        x = (w >> 7) & 0xFF
        assert (np.bincount(x, minlength=256) == hist).all()
        params, D, bexp = oracle.tune_hist(hist)
        occ = np.nonzero(hist)[0]
        l, h = int(occ[0]), int(occ[-1])
        best = min(
            (sum(int(hist[v]) * ((b - v) % (1 << oracle.width_for(b, l, h))) for v in range(l, h + 1)),
             oracle.width_for(b, l, h), b) for b in range(l, h + 1))
        assert (D, params[1], params[0]) == best
        assert ref.tune_hist(hist) == (params, D, bexp)


def test_eq4_predicts_the_actual_exponent_width(oracle):
    # On i.i.d. data the expected width of Eq. 4 must agree with the width the codec
    # really spends (mask + low plane + high records), and the chosen m must beat the
    # other thresholds when they are actually tried.
    w = W.gaussian(1 << 20, 0.02, 9)
    params, D, bexp = oracle.tune_hist(oracle.histogram(w))
    b, n, m, L = params
    sizes = {}
    for mm in range(0, n + 1):
        rc, s = oracle.compress(w, (b, n, mm, 16), 16384)
        assert rc == oracle.OK
        sizes[mm] = s.size
    nb = w.size // 16384
    payload = sizes[m] - oracle.payload_base(w.size, 16384)
    exp_bits = (payload - w.size) * 8 / w.size
    assert abs(exp_bits - bexp) < 0.01 * bexp + 16 * 8 * nb / w.size
    assert sizes[m] == min(sizes.values())


# --------------------------------------------------------------------------
# container: hand-worked block, sizes, accounting
# --------------------------------------------------------------------------
def test_handworked_block_of_128(oracle, ref):
    g = dict(ln.split(None, 1) for ln in golden_lines("block128_handworked.txt"))
    w = np.full(128, 0x3D00, np.uint16)
    w[17] = 0x3D80
    w[40] = 0xBD05
    rc, s = oracle.compress(w, (122, 6, 3, 16), 128)
    assert rc == oracle.OK and s.size == int(g["stream_bytes"])
    base = int(g["payload_base"])
    assert oracle.payload_base(128, 128) == base
    assert s[:4].tobytes() == b"ENEC"
    offs = struct.unpack_from("<2Q", s.tobytes(), 64)
    assert list(offs) == [int(v) for v in g["offset_table"].split()]
    sm, mask = s[base:base + 128], s[base + 128]
    low, high = s[base + 129:base + 129 + 48], s[base + 177:base + 183]
    i, v = g["sm_nonzero"].split(":")
    exp = np.zeros(128, np.uint8); exp[int(i)] = int(v, 16)
    assert (sm == exp).all()
    assert mask == int(g["mask_byte"], 16)
    i, v = g["low_plane_nonzero"].split(":")
    exp = np.zeros(48, np.uint8); exp[int(i)] = int(v, 16)
    assert (low == exp).all()
    assert high.tobytes() == bytes(int(h, 16) for h in g["high_record"].split())
    assert (s[base + 183:] == 0).all()
    ok, s2 = ref.compress(w, (122, 6, 3, 16), 128)
    assert ok and s2 == s.tobytes()
    rc, d = oracle.decompress(s, 128)
    assert rc == oracle.OK and (d == w).all()
    assert ref.decompress(s.tobytes(), 128) == [int(x) for x in w]


def _mask_count(stream, n_elems, B, m):
    """Per-block count of anomalous groups, read from the mask planes."""
    nb = (n_elems + B - 1) // B
    base = (64 + 8 * (nb + 1) + 15) & ~15
    offs = np.frombuffer(stream[64:64 + 8 * (nb + 1)].tobytes(), dtype="<u8")
    cnt = []
    for k in range(nb):
        p = base + int(offs[k]) + B
        cnt.append(int(np.unpackbits(stream[p:p + B // 128]).sum()))
    return offs, cnt


@pytest.mark.parametrize("B", [2048, 16384, 32768])
def test_size_identity_and_offset_table(oracle, B):
    w = W.gaussian(5 * B + 777, 0.02, 21)
    b, n, m, L = oracle.tune(w)
    rc, s = oracle.compress(w, (b, n, m, L), B)
    assert rc == oracle.OK
    info = oracle.stream_info(s)
    assert info["rc"] == 0 and info["total_bytes"] == s.size and info["n_elems"] == w.size
    assert info["block_size"] == B and info["params"] == (b, n, m, 16) and info["status"] == 0
    nb = 6
    offs, cnt = _mask_count(s, w.size, B, m)
    a = n - m
    S = [((B + B // 128 + m * B // 8 + 2 * a * c) + 15) & ~15 for c in cnt]
    assert offs[0] == 0
    assert list(offs) == list(np.concatenate([[0], np.cumsum(S)]))      # serial running sum
    assert s.size == ((64 + 8 * (nb + 1) + 15) & ~15) + sum(S)
    assert s.size <= oracle.compress_bound(w.size, B)


def test_closed_form_sizes(oracle):
    B = 16384
    # all-zero tensor with (0, 1, 0): only sign/mantissa bytes and the mask remain
    w = np.zeros(4 * B, np.uint16)
    rc, s = oracle.compress(w, (0, 1, 0, 16), B)
    assert rc == 0 and s.size == oracle.payload_base(w.size, B) + 4 * (B + B // 128)
    assert abs(2 * w.size / (s.size - oracle.payload_base(w.size, B)) - 1.984) < 0.001
    # every group anomalous with n = 8: full bytes for every exponent
    x = np.tile(np.array([0, 255] * 8, np.uint16), 4 * B // 16)
    w = (x << 7).astype(np.uint16)
    for m in (0, 3, 4, 7):
        rc, s = oracle.compress(w, (127, 8, m, 16), B)
        assert rc == 0 and s.size == oracle.payload_base(w.size, B) + 4 * (B + B // 128 + B)
        rc, d = oracle.decompress(s, w.size)
        assert rc == 0 and (d == w).all()
    # the bound holds for every group length Eq. 4 may choose and is met by the shortest one (longest mask)
    assert s.size < oracle.compress_bound(w.size, B)
    rc, s = oracle.compress(w, (127, 8, 3, 8), B)
    assert rc == 0 and s.size == oracle.payload_base(w.size, B) + 4 * (B + B // 64 + B) == oracle.compress_bound(w.size, B)


def test_bits_per_element_accounting_matches_paper(oracle):
    g = dict(ln.split() for ln in golden_lines("size_accounting.txt"))
    # the paper's own printed figures are mutually consistent with
    # "bits per element = 8 raw + coded exponent bits, nothing else"
    n_el = int(g["total_elements"])
    assert abs(n_el * 2 / 2 ** 20 - float(g["original_mb"])) < 0.01
    bits = float(g["model_bits_per_element"])
    assert abs(bits - (8 + float(g["exponent_bits_per_element"]))) < 1e-9
    # 11.8465 is printed to four decimals: +-0.00005 bit is +-0.2 MB on this model
    assert abs(n_el * bits / 8 / 2 ** 20 - float(g["compressed_mb"])) < 0.2
    assert round(16 / bits, 2) == float(g["ratio"])
    # the oracle spends exactly 8 + 1/16 + m + a*f bits per element (+ 16-byte padding,
    # + 8 bytes of offset table per block)
    w = W.config1()
    b, n, m, L = oracle.tune(w)
    rc, s = oracle.compress(w, (b, n, m, L), 16384)
    offs, cnt = _mask_count(s, w.size, 16384, m)
    f = sum(cnt) / (w.size / 16)
    model_bits = 8 + 1 / 16 + m + (n - m) * f
    real_bits = (s.size - oracle.payload_base(w.size, 16384)) * 8 / w.size
    assert 0 <= real_bits - model_bits <= 16 * 8 / 16384
    ratio = 2 * w.size / s.size
    # plausibility only: the ratio on real checkpoints is "parity unpinned"
    assert float(g["ratio_band_low"]) - 0.02 <= ratio <= float(g["ratio_band_high"]) + 0.02


# --------------------------------------------------------------------------
# whole codec
# --------------------------------------------------------------------------
def test_c_oracle_vs_twin_every_width_pair(oracle, ref):
    rng = np.random.default_rng(77)
    for n in range(1, 9):
        for m in range(0, n + 1):
            b = 128
            lo, hi = b - (1 << (n - 1)) + 1, b + (1 << (n - 1))
            x = rng.integers(lo, min(hi, 255) + 1, size=300).astype(np.uint16)
            x[32:96] = b                                        # some quiet groups
            w = ((rng.integers(0, 2, size=300).astype(np.uint16) << 15) | (x << 7)
                 | rng.integers(0, 128, size=300).astype(np.uint16)).astype(np.uint16)
            rc, s = oracle.compress(w, (b, n, m, 16), 128)
            assert rc == oracle.OK
            ok, s2 = ref.compress(w, (b, n, m, 16), 128)
            assert ok and s2 == s.tobytes()
            rc, d = oracle.decompress(s, w.size)
            assert rc == oracle.OK and (d == w).all()
            assert ref.decompress(s2, w.size) == [int(v) for v in w]


def test_one_hot_blocks(oracle, ref):
    # a single deviating element at every power-of-two position (and neighbours)
    B = 128
    for pos in [0, 1, 2, 4, 8, 15, 16, 17, 32, 63, 64, 127]:
        w = np.full(B, 122 << 7, np.uint16)
        w[pos] = (91 << 7) | 0x8001
        rc, s = oracle.compress(w, (122, 6, 3, 16), B)
        ok, s2 = ref.compress(w, (122, 6, 3, 16), B)
        assert rc == 0 and ok and s.tobytes() == s2
        assert oracle.decompress(s, B)[1].tolist() == w.tolist()


@pytest.mark.parametrize("n_elems", [0, 1, 15, 16, 17, 2047, 2048, 2049, 16384, 16385, 50001])
def test_roundtrip_ragged_lengths(oracle, n_elems):
    w = W.gaussian(n_elems, 0.02, 1000 + n_elems) if n_elems else np.zeros(0, np.uint16)
    B = oracle.default_block(n_elems)
    assert B == (16384 if n_elems >= 16384 else max(2048, 1 << max(0, n_elems.bit_length() - 1)))
    p = oracle.tune(w)
    rc, s = oracle.compress(w, p, B)
    assert rc == oracle.OK
    assert oracle.stream_info(s)["total_bytes"] == s.size
    rc, d = oracle.decompress(s, n_elems)
    assert rc == oracle.OK and (d == w).all()


def test_roundtrip_all_configs_small(oracle):
    # config 1
    w = W.config1(rows=64, cols=4096)
    rc, s = oracle.compress(w, oracle.tune(w), 16384)
    assert rc == 0 and (oracle.decompress(s, w.size)[1] == w).all()
    # config 2 at reduced width
    for name, w in W.config2(hidden=512, ffn=1376):
        B = oracle.default_block(w.size)
        rc, s = oracle.compress(w, oracle.tune(w), B)
        assert rc == 0, name
        assert (oracle.decompress(s, w.size)[1] == w).all(), name
    # config 3: the mix as one tensor, and per category (width-0 planes, full-width groups)
    w, cat = W.config3(n_blocks=32)
    p = oracle.tune(w)
    assert p[1] == 8
    rc, s = oracle.compress(w, p, 16384)
    assert rc == 0 and (oracle.decompress(s, w.size)[1] == w).all()
    parts = W.config3_by_category(n_blocks=32)
    tuned = [oracle.tune(t) for t in parts]
    assert tuned[0] == (0, 1, 0, 16)
    assert tuned[1][2] <= tuned[1][1] <= 6
    assert tuned[3][1] == 8
    for t, p in zip(parts, tuned):
        rc, s = oracle.compress(t, p, 16384)
        assert rc == 0 and (oracle.decompress(s, t.size)[1] == t).all()
    # random bits cannot shrink; growth is bounded by the mask and the table
    assert s.size <= oracle.compress_bound(parts[3].size, 16384)
    # config 4 / 5 tensors at reduced size
    w = W.config4_tensor(3, rows=64, cols=4096)
    rc, s = oracle.compress(w, oracle.tune(w), 16384)
    assert rc == 0 and (oracle.decompress(s, w.size)[1] == w).all()


def test_special_bit_patterns_survive(oracle):
    # -0, NaN payloads, Inf, denormals are only bit patterns
    specials = np.array([0x0000, 0x8000, 0x7F80, 0xFF80, 0x7FC0, 0xFFFF, 0x7F81, 0x0001, 0x807F,
                         0x0080, 0x3F80, 0xBF80], np.uint16)
    w = np.tile(specials, 200)
    p = oracle.tune(w)
    assert p[1] == 8
    rc, s = oracle.compress(w, p, 2048)
    assert rc == 0 and (oracle.decompress(s, w.size)[1] == w).all()


def test_error_paths(oracle):
    w = W.gaussian(4096, 0.02, 5)
    assert oracle.compress(w, (122, 6, 3, 16), 3000)[0] == oracle.E_BLOCK
    assert oracle.compress(w, (122, 9, 3, 16), 2048)[0] == oracle.E_PARAMS
    assert oracle.compress(w, (122, 6, 7, 16), 2048)[0] == oracle.E_PARAMS
    assert oracle.compress(w, (122, 6, 3, 12), 2048)[0] == oracle.E_PARAMS      # group lengths are 8, 16, 32
    assert oracle.compress(w, (122, 6, 3, 16), 2048, capacity=1000)[0] == oracle.E_CAPACITY
    # window [b-2^(n-1)+1, b+2^(n-1)] = [119, 126] does not hold these exponents
    rc, s = oracle.compress(w, (122, 3, 1, 16), 2048)
    assert rc == oracle.E_RANGE
    info = oracle.stream_info(s)
    assert info["status"] == oracle.E_RANGE and info["total_bytes"] == 0
    assert oracle.decompress(s, w.size)[0] == oracle.E_FORMAT
    rc, s = oracle.compress(w, oracle.tune(w), 2048)
    assert oracle.decompress(s, w.size + 1)[0] == oracle.E_FORMAT
    bad = s.copy(); bad[0] = ord("X")
    assert oracle.decompress(bad, w.size)[0] == oracle.E_FORMAT
