"""Zero-waste 3-bit packing: exactly 3 bits per weight, no padding bits.

Test infrastructure only (see the package docstring).

The paper (Section 3.3, "Zero bit waste 3-bit weights packing") fixes only the
requirement: 32 codes occupy 3 x 32 bits, nothing is wasted, and the blob is
split into planes so that every load is naturally aligned.  The concrete bit
layout below is this project's own and is written here from its prose
description, independently of the GPU packer:

  * A *unit* is the 64 codes of one quantization group of one row:
    row n, group g  ->  codes q[n, 64 g .. 64 g + 63].
  * Units are ordered by (row block of 16 rows, group, row within block):
        u(n, g) = ((n // 16) * (K // 64) + g) * 16 + n % 16
  * The codes of a unit are six little-endian 32-bit words d0..d5.  Plane A holds
    d0..d3 of unit u at byte offset 16 u; plane B follows plane A (it starts at
    byte N K / 4) and holds, at byte offset 12 u, the three words d4, d5 and
    p = (scale bits) | (zero-point bits) << 16, both parameters being IEEE
    binary16 bit patterns.  28 bytes per unit = 3.5 bits per weight.
  * The 64 codes form 32 pairs, pair P = (q[2P], q[2P+1]) = (lo, hi).
    Pairs 0..29: word j = P // 5, slot c = P % 5; lo sits in bits 3c..3c+2 and
    hi in bits 16+3c..16+3c+2 of word j.  That leaves bits 15 and 31 of every
    word free.  Pair 30 uses those of words 0, 1, 2: bit i of lo is bit 15 of
    word i and bit i of hi is bit 31 of word i.  Pair 31 does the same with
    words 3, 4, 5.
"""
import numpy as np

GROUP = 64


def packed_bytes(N, K):
    """Bytes of the blob: 24 bytes of codes and 4 bytes of parameters per group of 64."""
    return N * K // GROUP * 28


def code_bytes(N, K):
    """Bytes the codes alone occupy: exactly 3 bits per weight."""
    return N * K * 3 // 8


def unit_index(n, g, K):
    return ((n // 16) * (K // GROUP) + g) * 16 + n % 16


def _check(N, K):
    if N % 16 or K % GROUP or N <= 0 or K <= 0:
        raise ValueError("need N % 16 == 0 and K % 64 == 0")


def to_unit_order(per_group):
    """[N, K/64] array -> flat array in unit order."""
    N, G = per_group.shape
    return np.ascontiguousarray(
        per_group.reshape(N // 16, 16, G).transpose(0, 2, 1)).reshape(-1)


def from_unit_order(flat, N, K):
    G = K // GROUP
    return np.ascontiguousarray(
        np.asarray(flat).reshape(N // 16, G, 16).transpose(0, 2, 1)).reshape(N, G)


def pack_w3(codes, scales, zeros):
    """codes uint8 [N, K] in 0..7, scales and zeros fp16 [N, K/64] -> uint8 blob."""
    codes = np.asarray(codes)
    N, K = codes.shape
    _check(N, K)
    scales = np.asarray(scales)
    zeros = np.asarray(zeros)
    if scales.dtype != np.float16 or zeros.dtype != np.float16:
        raise ValueError("scales and zeros must be float16")
    if scales.shape != (N, K // GROUP) or zeros.shape != (N, K // GROUP):
        raise ValueError("scales and zeros must be [N, K/64]")
    if codes.max(initial=0) > 7:
        raise ValueError("codes must lie in 0..7")
    G = K // GROUP
    # unit-ordered codes: [units, 64]
    cu = codes.reshape(N // 16, 16, G, GROUP).transpose(0, 2, 1, 3).reshape(-1, GROUP)
    cu = cu.astype(np.uint32)
    nu = cu.shape[0]
    d = np.zeros((nu, 6), dtype=np.uint32)
    for P in range(30):
        j, c = divmod(P, 5)
        d[:, j] |= cu[:, 2 * P] << np.uint32(3 * c)
        d[:, j] |= cu[:, 2 * P + 1] << np.uint32(16 + 3 * c)
    for P, base in ((30, 0), (31, 3)):
        lo, hi = cu[:, 2 * P], cu[:, 2 * P + 1]
        for i in range(3):
            d[:, base + i] |= ((lo >> np.uint32(i)) & np.uint32(1)) << np.uint32(15)
            d[:, base + i] |= ((hi >> np.uint32(i)) & np.uint32(1)) << np.uint32(31)
    params = to_unit_order(scales).view(np.uint16).astype(np.uint32) | \
        (to_unit_order(zeros).view(np.uint16).astype(np.uint32) << np.uint32(16))
    plane_a = np.ascontiguousarray(d[:, :4]).astype("<u4").view(np.uint8).reshape(-1)
    plane_b = np.ascontiguousarray(np.concatenate([d[:, 4:], params[:, None]], axis=1)).astype("<u4") \
        .view(np.uint8).reshape(-1)
    blob = np.concatenate([plane_a, plane_b])
    assert blob.size == packed_bytes(N, K)
    return blob


def unpack_w3(blob, N, K):
    """Inverse of pack_w3: (codes uint8 [N, K], scales fp16 [N, K/64], zeros fp16 [N, K/64])."""
    _check(N, K)
    blob = np.asarray(blob, dtype=np.uint8).reshape(-1)
    if blob.size != packed_bytes(N, K):
        raise ValueError("blob has the wrong length")
    G = K // GROUP
    nu = N * G
    a = blob[: nu * 16].view("<u4").reshape(nu, 4).astype(np.uint32)
    b3 = blob[nu * 16:].view("<u4").reshape(nu, 3).astype(np.uint32)
    d = np.concatenate([a, b3[:, :2]], axis=1)
    scales = from_unit_order((b3[:, 2] & np.uint32(0xFFFF)).astype(np.uint16).view(np.float16), N, K)
    zeros = from_unit_order((b3[:, 2] >> np.uint32(16)).astype(np.uint16).view(np.float16), N, K)
    cu = np.zeros((nu, GROUP), dtype=np.uint32)
    seven = np.uint32(7)
    for P in range(30):
        j, c = divmod(P, 5)
        cu[:, 2 * P] = (d[:, j] >> np.uint32(3 * c)) & seven
        cu[:, 2 * P + 1] = (d[:, j] >> np.uint32(16 + 3 * c)) & seven
    for P, base in ((30, 0), (31, 3)):
        for i in range(3):
            cu[:, 2 * P] |= ((d[:, base + i] >> np.uint32(15)) & np.uint32(1)) << np.uint32(i)
            cu[:, 2 * P + 1] |= ((d[:, base + i] >> np.uint32(31)) & np.uint32(1)) << np.uint32(i)
    codes = cu.astype(np.uint8).reshape(N // 16, G, 16, GROUP).transpose(0, 2, 1, 3)
    return np.ascontiguousarray(codes).reshape(N, K), scales, zeros
