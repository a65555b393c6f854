"""Pins for the oracle's chunk fingerprint (paper Sec. 4; Alg. 1 steps 2 and 7).

The fingerprint function is FNV-1a-64 over the little-endian bytes of the int32
token ids.  Pinned to the published FNV test vectors (tests/golden), to python
big-integer arithmetic on byte strings built with ``struct``, and to structural
properties (order sensitivity, no length/seed mixed in, prefix chaining).
"""
import os
import struct

import numpy as np

from oracle import irm_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fnv1a64_vectors.txt")


def golden_vectors():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        data, h = line.split()
        out.append((b"" if data == "-" else bytes.fromhex(data), int(h, 16)))
    return out


def test_published_byte_vectors():
    vec = golden_vectors()
    assert len(vec) >= 5
    for data, want in vec:
        assert orc.fnv1a64_bytes(data) == want


def test_token_chunks_equal_the_byte_hash_of_their_little_endian_image():
    rng = np.random.default_rng(0)
    tokens = rng.integers(-2**31, 2**31, size=5000, dtype=np.int64).astype(np.int32)
    tokens[:10] = [0, 1, 2, 3, 102399, -1, 255, 256, 65536, 2**31 - 1]
    start = np.array([0, 1, 0, 4, 10, 4000, 17], np.uint32)
    length = np.array([1, 3, 0, 1, 1024, 1000, 64], np.uint32)
    got = orc.chunk_hash(tokens, start, length)
    for s, l, h in zip(start, length, got):
        image = b"".join(struct.pack("<i", int(t)) for t in tokens[s:s + l])
        assert int(h) == orc.fnv1a64_bytes(image)
        # python big integers, no C involved
        acc = 0xCBF29CE484222325
        for byte in image:
            acc = ((acc ^ byte) * 0x100000001B3) % (1 << 64)
        assert int(h) == acc


def test_token_vectors():
    # worked by hand from the definition (and cross-checked with the byte vectors):
    # [0] -> four zero bytes, [1,2,3] -> 01 00 00 00 02 00 00 00 03 00 00 00
    tokens = np.array([0, 1, 2, 3, 102399], np.int32)
    got = orc.chunk_hash(tokens, np.array([0, 1, 4], np.uint32), np.array([1, 3, 1], np.uint32))
    assert [int(v) for v in got] == [0x4D25767F9DCE13F5, 0xFD1F0F4381EB0395, 0x4D7FF366C600EA22]


def test_order_matters_and_nothing_else_is_mixed_in():
    t = np.array([5, 9, 5, 9, 9, 5], np.int32)
    s = np.array([0, 2, 4, 1], np.uint32)
    l = np.array([2, 2, 2, 2], np.uint32)
    h = orc.chunk_hash(t, s, l)
    assert h[0] == h[1]              # same content at another offset -> same fingerprint
    assert h[0] != h[2]              # (5,9) vs (9,5)
    assert h[2] == h[3]
    assert int(orc.chunk_hash(t, np.array([3], np.uint32), np.array([0], np.uint32))[0]) == 0xCBF29CE484222325
