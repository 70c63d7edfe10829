"""Pins for the oracle's pack/unpack (Section 3.3: zero-bit-waste packing) and the unit order."""
import numpy as np
import pytest

from oracle import (pack_w3 as _pack, unpack_w3, packed_bytes, code_bytes, unit_index, to_unit_order,
                    from_unit_order)


def _params(N, K, seed=None):
    """fp16 scales / zeros [N, K/64]: zero bit patterns, or random finite values."""
    G = K // 64
    if seed is None:
        return np.zeros((N, G), np.float16), np.zeros((N, G), np.float16)
    rng = np.random.default_rng(seed)
    return (rng.uniform(1e-3, 0.2, (N, G)).astype(np.float16),
            rng.uniform(-9.0, 9.0, (N, G)).astype(np.float16))


def pack_w3(codes, scales=None, zeros=None):
    """pack with all-zero parameter words unless given (most pins look at the code bits only)."""
    if scales is None:
        scales, zeros = _params(*codes.shape)
    return _pack(codes, scales, zeros)


def _bit_decode(blob, N, K):
    """Bit-at-a-time pure-Python decoder written straight from the layout prose."""
    G = K // 64
    nu = N * G
    out = np.zeros((N, K), dtype=np.uint8)

    def word(u, j):
        off = 16 * u + 4 * j if j < 4 else nu * 16 + 12 * u + 4 * (j - 4)
        return int.from_bytes(bytes(blob[off: off + 4].tolist()), "little")

    for n in range(N):
        for g in range(G):
            u = ((n // 16) * G + g) * 16 + n % 16
            d = [word(u, j) for j in range(6)]
            for P in range(32):
                if P < 30:
                    j, c = divmod(P, 5)
                    lo = (d[j] >> (3 * c)) & 7
                    hi = (d[j] >> (16 + 3 * c)) & 7
                else:
                    base = 0 if P == 30 else 3
                    lo = sum(((d[base + i] >> 15) & 1) << i for i in range(3))
                    hi = sum(((d[base + i] >> 31) & 1) << i for i in range(3))
                out[n, 64 * g + 2 * P] = lo
                out[n, 64 * g + 2 * P + 1] = hi
    return out


def test_zero_waste_length():
    # the codes take exactly 3 bits per weight; the two fp16 parameters per group of 64 add
    # 4 bytes per 24: 3.5 bits per weight in all, nothing else
    for N, K in ((16, 64), (32, 128), (1024, 1024), (48, 1408)):
        assert code_bytes(N, K) * 8 == N * K * 3
        assert packed_bytes(N, K) == code_bytes(N, K) + 4 * (N * K // 64)
        assert packed_bytes(N, K) * 16 == N * K * 7
    codes = np.zeros((32, 128), np.uint8)
    assert pack_w3(codes).size == 32 * 128 * 7 // 16


def test_round_trip_random_and_bit_decoder():
    rng = np.random.default_rng(0)
    for N, K in ((16, 64), (32, 192), (48, 128)):
        codes = rng.integers(0, 8, size=(N, K), dtype=np.uint8)
        sc, zp = _params(N, K, seed=N + K)
        blob = pack_w3(codes, sc, zp)
        assert blob.dtype == np.uint8 and blob.size == N * K * 7 // 16
        c2, s2, z2 = unpack_w3(blob, N, K)
        assert np.array_equal(c2, codes)
        assert np.array_equal(s2.view(np.uint16), sc.view(np.uint16))
        assert np.array_equal(z2.view(np.uint16), zp.view(np.uint16))
        assert np.array_equal(_bit_decode(blob, N, K), codes)
        # the parameters do not disturb the code bits and sit where the layout says
        nu = N * (K // 64)
        for n, g in ((0, 0), (N - 1, K // 64 - 1), (17 % N, min(1, K // 64 - 1))):
            u = unit_index(n, g, K)
            p = int.from_bytes(bytes(blob[nu * 16 + 12 * u + 8: nu * 16 + 12 * u + 12].tolist()), "little")
            assert p & 0xFFFF == int(sc[n, g].view(np.uint16))
            assert p >> 16 == int(zp[n, g].view(np.uint16))


def test_every_position_owns_three_private_bits():
    # one unit (row 0, the only group); code position p set to 7 must light exactly three
    # bits, disjoint between positions, and the 64 positions together cover all 192 bits.
    N, K = 16, 64
    seen = np.zeros(packed_bytes(N, K) * 8, dtype=np.int32)
    unit_bits = None
    for p in range(64):
        codes = np.zeros((N, K), np.uint8)
        codes[0, p] = 7
        bits = np.unpackbits(pack_w3(codes), bitorder="little")
        assert bits.sum() == 3
        seen += bits
        # single-bit values light a subset of those bits
        for v in (1, 2, 4):
            c2 = np.zeros((N, K), np.uint8)
            c2[0, p] = v
            b2 = np.unpackbits(pack_w3(c2), bitorder="little")
            assert b2.sum() == 1 and np.all(b2 <= bits)
    assert seen.max() == 1 and seen.sum() == 192
    # constant-code patterns
    for v in range(8):
        codes = np.full((N, K), v, np.uint8)
        bits = np.unpackbits(pack_w3(codes), bitorder="little")
        assert bits.sum() == N * K * bin(v).count("1")
        assert np.array_equal(unpack_w3(pack_w3(codes), N, K)[0], codes)


def test_documented_bit_positions():
    # pair 0 lo -> word 0 bits 0..2 ; pair 0 hi -> word 0 bits 16..18 ; pair 7 lo (code 14) ->
    # word 1 slot 2 bits 6..8 ; pair 30 lo (code 60) -> bit 15 of words 0,1,2 ;
    # pair 31 hi (code 63) -> bit 31 of words 3,4,5 (words 4,5 live in plane B).
    N, K = 16, 64

    def words(codes):
        blob = pack_w3(codes)
        a = blob[: 16 * 16].view("<u4").reshape(16, 4)
        b = blob[16 * 16:].view("<u4").reshape(16, 3)[:, :2]
        return np.concatenate([a, b], 1)

    def one(p, v, row=0):
        c = np.zeros((N, K), np.uint8)
        c[row, p] = v
        return words(c)[row]

    assert one(0, 5).tolist() == [5, 0, 0, 0, 0, 0]
    assert one(1, 5).tolist() == [5 << 16, 0, 0, 0, 0, 0]
    assert one(14, 3).tolist() == [0, 3 << 6, 0, 0, 0, 0]
    assert one(59, 6).tolist() == [0, 0, 0, 0, 0, 6 << 28]
    assert one(60, 5).tolist() == [1 << 15, 0, 1 << 15, 0, 0, 0]
    assert one(63, 6).tolist() == [0, 0, 0, 0, 1 << 31, 1 << 31]
    # row 3 of the block lands in unit 3
    assert one(0, 7, row=3).tolist() == [7, 0, 0, 0, 0, 0]


def test_unit_order():
    N, K = 48, 256
    G = K // 64
    # formula
    assert unit_index(0, 0, K) == 0 and unit_index(1, 0, K) == 1
    assert unit_index(0, 1, K) == 16 and unit_index(16, 0, K) == 16 * G
    assert unit_index(47, 3, K) == N * G - 1
    per_group = np.arange(N * G, dtype=np.float32).reshape(N, G)
    flat = to_unit_order(per_group)
    for n in (0, 5, 16, 33, 47):
        for g in range(G):
            assert flat[unit_index(n, g, K)] == per_group[n, g]
    assert np.array_equal(from_unit_order(flat, N, K), per_group)
    # the packed blob follows the same order: mark one unit and find its words
    codes = np.zeros((N, K), np.uint8)
    codes[33, 64 * 2] = 7
    blob = pack_w3(codes)
    a = blob[: N * G * 16].view("<u4").reshape(N * G, 4)
    (rows,) = np.nonzero(a[:, 0])
    assert rows.tolist() == [unit_index(33, 2, K)]


def test_rejects_bad_input():
    with pytest.raises(ValueError):
        pack_w3(np.zeros((8, 64), np.uint8))
    with pytest.raises(ValueError):
        pack_w3(np.full((16, 64), 8, np.uint8))
    with pytest.raises(ValueError):
        unpack_w3(np.zeros(10, np.uint8), 16, 64)
    with pytest.raises(ValueError):
        _pack(np.zeros((16, 64), np.uint8), np.zeros((16, 1), np.float32), np.zeros((16, 1), np.float16))
    with pytest.raises(ValueError):
        _pack(np.zeros((16, 64), np.uint8), np.zeros((16, 2), np.float16), np.zeros((16, 2), np.float16))
