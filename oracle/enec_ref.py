"""Pure-Python twin of the ENEC oracle, for brute force on tiny inputs.

TEST INFRASTRUCTURE ONLY (see oracle/enec_oracle.c for the scope of the oracle).
It is written separately from the C file and prefers the *definitions* over the
vectorised forms, so that the two can check each other:

  * the packer is the recursive description of Sec. V-B (fold lanes until a byte
    is full, split into a storable byte and an overflow sub-block, recurse);
  * the unpacker does not replay the packer backwards: it learns, from one-hot
    inputs, where every input bit lands (the packer is a bit permutation) and
    gathers the bits back;
  * the group test uses the definition "largest bit width in the group > m"
    instead of the bitwise OR the paper substitutes for it (Sec. V-B);
  * record positions come from a running count of mask bits (Alg. 1,
    decompression part);
  * elements are taken apart by the IEEE field widths (sign, exponent, mantissa)
    with divisions and remainders, not by per-format shift constants.

Everything works on Python integers; use it for blocks of 128-2048 elements.
"""
from __future__ import annotations

import struct
from functools import lru_cache

L = 16              # default group length
HEADER = 64


# --------------------------------------------------------------------------
# Sec. V-B / Alg. 2
# --------------------------------------------------------------------------
def _normalized_bytes(lanes, width):
    """Recursive form: returns the 'normalized bytes' of Alg. 2 (before the final join)."""
    if width <= 0:
        return []
    lanes = list(lanes)
    while len(lanes) > 1 and width < 8:
        half = len(lanes) // 2
        lanes = [lanes[i] | (lanes[i + half] << width) for i in range(half)]
        width *= 2
    storable = [v & 0xFF for v in lanes]
    overflow = [v >> 8 for v in lanes]
    return storable + _normalized_bytes(overflow, width - 8)


def hh_pack(values, a):
    assert 0 < a <= 8 and len(values) & (len(values) - 1) == 0
    assert all(0 <= v < (1 << a) for v in values)
    nb = _normalized_bytes(values, a)
    if len(nb) % 2:
        nb.append(0)
    half = len(nb) // 2
    out = bytearray()
    for i in range(half):
        out += struct.pack("<H", nb[i] | (nb[i + half] << 8))
    return bytes(out)


@lru_cache(maxsize=None)
def _bit_map(N, a):
    """(element, bit) -> output bit position, learnt from one-hot inputs."""
    where = {}
    for e in range(N):
        for bit in range(a):
            v = [0] * N
            v[e] = 1 << bit
            s = hh_pack(v, a)
            ones = [8 * i + k for i, byte in enumerate(s) for k in range(8) if (byte >> k) & 1]
            assert len(ones) == 1, "packer is not a bit permutation"
            where[(e, bit)] = ones[0]
    assert len(set(where.values())) == N * a
    return where


def hh_unpack(stream, N, a):
    where = _bit_map(N, a)
    out = [0] * N
    for (e, bit), pos in where.items():
        if (stream[pos // 8] >> (pos % 8)) & 1:
            out[e] |= 1 << bit
    return out


# --------------------------------------------------------------------------
# Sec. V-C / Sec. V-E
# --------------------------------------------------------------------------
def transform(x, b, n):
    return (b - x) % (1 << n)          # Python's % is already non-negative


def in_range(x, b, n, E=8):
    return n >= E or -(1 << (n - 1)) <= b - x <= (1 << (n - 1)) - 1


def inverse_transform(y, b, n, E=8):
    s = y - (1 << n) if y >= (1 << (n - 1)) else y
    return (b - s) % (1 << E)


def width_for(b, l, h, E=8):
    pos = (b - l).bit_length()
    neg = (h - b - 1).bit_length() if h > b else 0
    return min(E, max(pos, neg) + 1)


# dtype code -> (exponent bits, mantissa bits); the sign is the top bit
FIELDS = {0: (8, 7), 1: (5, 10), 2: (8, 23)}


def take_apart(w, dtype):
    """-> (exponent, raw byte sign*128 + first seven mantissa bits, left-over mantissa bits)"""
    E, M = FIELDS[dtype]
    mant = w % (1 << M)
    expo = (w // (1 << M)) % (1 << E)
    sign = w // (1 << (M + E))
    return expo, sign * 128 + mant // (1 << (M - 7)), mant % (1 << (M - 7))


def put_together(expo, raw, rest, dtype):
    E, M = FIELDS[dtype]
    mant = (raw % 128) * (1 << (M - 7)) + rest
    return ((raw // 128) * (1 << E) + expo) * (1 << M) + mant


def tune_hist(hist, E=8):
    """Phases 2-3 of Sec. V-E on a 256-bin histogram -> ((b, n, m, L), D, B_exp)."""
    occupied = [x for x in range(256) if hist[x]]
    if not occupied:
        return (0, 1, 0, L), 0, 1.0 / 16.0
    l, h = occupied[0], occupied[-1]
    total = sum(int(hist[x]) for x in occupied)
    best = None
    for b in range(l, h + 1):
        n = width_for(b, l, h, E)
        D = sum(int(hist[x]) * transform(x, b, n) for x in occupied)
        key = (D, n, b)
        if best is None or key < best:
            best = key
    D, n, b = best
    best_m = None
    for m in range(0, n + 1):
        cnt = sum(int(hist[x]) for x in occupied if transform(x, b, n) < (1 << m))
        p = cnt / total
        p2 = p * p
        p4 = p2 * p2
        p8 = p4 * p4
        p16 = p8 * p8
        bexp = (1.0 / 16.0 + float(n)) + (float(m) - float(n)) * p16
        if best_m is None or bexp < best_m[0]:
            best_m = (bexp, m)
    return (b, n, best_m[1], L), D, best_m[0]


def tune_hist_groups(hist, E=8, lengths=(8, 16, 32)):
    """Eq. 4 over m and the group length together; ties: smaller m, then smaller length."""
    (b, n, _, _), D, _ = tune_hist(hist, E)
    occupied = [x for x in range(256) if hist[x]]
    total = sum(int(hist[x]) for x in occupied)
    best = None
    for m in range(0, n + 1):
        p = sum(int(hist[x]) for x in occupied if transform(x, b, n) < (1 << m)) / total if total else 1.0
        for Lg in sorted(lengths):
            q = p
            for _ in range(Lg.bit_length() - 1):       # p^Lg by squarings
                q = q * q
            bexp = (1.0 / Lg + float(n)) + (float(m) - float(n)) * q
            if best is None or bexp < best[0]:
                best = (bexp, m, Lg)
    return (b, n, best[1], best[2]), D, best[0]


def tune(words, dtype=0):
    hist = [0] * 256
    for w in words:
        hist[take_apart(int(w), dtype)[0]] += 1
    return tune_hist(hist, FIELDS[dtype][0])[0]


# --------------------------------------------------------------------------
# container
# --------------------------------------------------------------------------
def _align16(v):
    return (v + 15) & ~15


def compress(words, params, B, dtype=0, per_block=False):
    """-> (range_ok, bytes).  fp16: the three left-over mantissa bits sit on top of the low
    m bits in the low plane; fp32: the sixteen left-over bits of all elements follow the table.
    per_block: params = (0, 0, 0, L) and every block is coded with the tuple tuned on its own
    exponents; the tuples follow the offset table, four bytes each."""
    b, n, m, L = params
    E = FIELDS[dtype][0]
    assert L in (8, 16, 32) and B >= 8 * L and (per_block or (1 <= n <= E and 0 <= m <= n))
    words = [int(w) for w in words]
    N = len(words)
    nb = (N + B - 1) // B
    G = B // L
    payloads, offsets, ok, tuples = [], [0], True, b""
    for k in range(nb):
        blk = list(words[k * B:(k + 1) * B])
        real = len(blk)
        parts = [take_apart(w, dtype) for w in blk]
        if per_block:
            hist = [0] * 256
            for part in parts:
                hist[part[0]] += 1
            b, n, m, _ = tune_hist_groups(hist, E, (L,))[0]      # Eq. 4 with the coding group length
            tuples += bytes([b, n, m, 0])
        a = n - m
        rb = a * L // 8                  # a record without the pad byte Alg. 2 adds to an odd count
        sm = [p[1] for p in parts] + [0] * (B - real)
        rest = [p[2] for p in parts] + [0] * (B - real)
        xs = [p[0] for p in parts]
        ok = ok and all(in_range(x, b, n, E) for x in xs)
        y = [transform(x, b, n) for x in xs] + [0] * (B - real)
        anomalous = [max(v.bit_length() for v in y[g * L:(g + 1) * L]) > m for g in range(G)]
        mask = bytearray(G // 8)
        for g, flag in enumerate(anomalous):
            if flag:
                mask[g // 8] |= 1 << (g % 8)
        if dtype == 1:
            low = hh_pack([v % (1 << m) + r * (1 << m) for v, r in zip(y, rest)], m + 3)
        else:
            low = hh_pack([v & ((1 << m) - 1) for v in y], m) if m else b""
        high = b"".join(hh_pack([v >> m for v in y[g * L:(g + 1) * L]], a)[:rb]
                        for g in range(G) if anomalous[g])
        p = bytes(sm) + bytes(mask) + low + high
        p += bytes(_align16(len(p)) - len(p))
        payloads.append(p)
        offsets.append(offsets[-1] + len(p))
    tail = b""
    if dtype == 2:
        tail = b"".join(struct.pack("<H", take_apart(w, dtype)[2]) for w in words)
        tail += bytes(_align16(len(tail)) - len(tail))
    tuples += bytes(_align16(len(tuples)) - len(tuples))
    base = _align16(HEADER + 8 * (nb + 1)) + len(tuples) + len(tail)
    total = base + offsets[-1]
    status = 0 if ok else 6
    if per_block:
        b = n = m = 0
    hdr = struct.pack("<4sHBBQIIBBBBIQB", b"ENEC", 1, dtype, L, N, B, nb, b, n, m, E, status,
                      total if ok else 0, 1 if per_block else 0)
    hdr += bytes(HEADER - len(hdr))
    table = b"".join(struct.pack("<Q", o) for o in offsets)
    head = hdr + table
    head += bytes(_align16(len(head)) - len(head)) + tuples + tail
    return ok, head + b"".join(payloads)


def decompress(stream, N):
    stream = bytes(stream)
    magic, ver, dtype, L, n_elems, B, nb, b, n, m, ebits, status, total = struct.unpack_from(
        "<4sHBBQIIBBBBIQ", stream, 0)
    assert magic == b"ENEC" and ver == 1 and dtype in FIELDS and L in (8, 16, 32) and ebits == FIELDS[dtype][0]
    assert n_elems == N and status == 0
    per_block = stream[40] == 1
    G = B // L
    tuples_at = _align16(HEADER + 8 * (nb + 1))
    tail_at = tuples_at + (_align16(4 * nb) if per_block else 0)
    base = tail_at + (_align16(2 * N) if dtype == 2 else 0)
    out = []
    for k in range(nb):
        if per_block:
            b, n, m = stream[tuples_at + 4 * k:tuples_at + 4 * k + 3]
        a = n - m
        rb = a * L // 8
        lowbits = m + (3 if dtype == 1 else 0)
        off = struct.unpack_from("<Q", stream, HEADER + 8 * k)[0]
        p = stream[base + off:]
        sm = p[:B]
        mask = p[B:B + G // 8]
        lowplane = p[B + G // 8:B + G // 8 + lowbits * B // 8]
        highplane = p[B + G // 8 + lowbits * B // 8:]
        low = hh_unpack(lowplane, B, lowbits) if lowbits else [0] * B
        seen = 0                                   # running count of mask bits
        for g in range(G):
            bit = (mask[g // 8] >> (g % 8)) & 1
            high = hh_unpack(highplane[rb * seen:rb * (seen + 1)] + b"\0", L, a) if bit else [0] * L
            seen += bit
            for i in range(L):
                e = k * B + g * L + i
                if e >= N:
                    break
                y = low[g * L + i] % (1 << m) + (high[i] << m)
                rest = low[g * L + i] >> m if dtype == 1 else 0
                if dtype == 2:
                    rest = struct.unpack_from("<H", stream, tail_at + 2 * e)[0]
                x = inverse_transform(y, b, n, ebits)
                out.append(put_together(x, sm[g * L + i], rest, dtype))
    return out
