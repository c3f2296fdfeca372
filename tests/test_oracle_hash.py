"""Pins for the hashing oracle: the standard's published test vectors for SHA-256 itself, and small
trees written out by hand for the two constructions built on it."""
import hashlib

import pytest

from oracle import hash_tree as ht

ABC = "ba7816bf8f01cfea414140de5dae2223b00361a396177a9cb410ff61f20015ad"
EMPTY = "e3b0c44298fc1c149afbf4c8996fb92427ae41e4649b934ca495991b7852b855"
TWO_BLOCK = "248d6a61d20638b8e5c026930c3e6039a33ce45964ff2167f6ecedd419db06c1"


def test_sha256_standard_vectors():
    assert ht.sha256(b"abc").hex() == ABC
    assert ht.sha256(b"").hex() == EMPTY
    assert ht.sha256(b"abcdbcdecdefdefgefghfghighijhijkijkljklmklmnlmnomnopnopq").hex() == TWO_BLOCK


def test_tree_written_out_by_hand():
    h = lambda b: hashlib.sha256(b).digest()
    data = bytes(range(256)) * 3                      # 768 bytes
    assert ht.sha256_tree(data, 0) == h(data)
    assert ht.sha256_tree(data, 1024) == h(data)      # fits one chunk
    assert ht.sha256_tree(data, 768) == h(data)
    # chunk 256: three chunks -> 96 bytes of digests, one chunk -> hashed
    assert ht.sha256_tree(data, 256) == h(h(data[:256]) + h(data[256:512]) + h(data[512:]))
    # chunk 64 with a ragged tail: 13 chunks -> 416 bytes -> 7 chunks -> 224 bytes -> 4 chunks -> 128 -> 2 -> 64
    d = data + b"tail"
    l1 = b"".join(h(d[i:i + 64]) for i in range(0, len(d), 64))
    l2 = b"".join(h(l1[i:i + 64]) for i in range(0, len(l1), 64))
    l3 = b"".join(h(l2[i:i + 64]) for i in range(0, len(l2), 64))
    l4 = b"".join(h(l3[i:i + 64]) for i in range(0, len(l3), 64))
    assert len(l1) == 13 * 32 and len(l4) == 64
    assert ht.sha256_tree(d, 64) == h(l4)
    assert ht.sha256_tree(b"", 64) == h(b"")
    with pytest.raises(ValueError):
        ht.sha256_tree(data, 100)


def test_merkle_root_written_out_by_hand():
    h = lambda b: hashlib.sha256(b).digest()
    l = [h(bytes([i])) for i in range(5)]
    assert ht.merkle_root(l[:1]) == l[0]
    assert ht.merkle_root(l[:2]) == h(l[0] + l[1])
    assert ht.merkle_root(l[:3]) == h(h(l[0] + l[1]) + l[2])
    assert ht.merkle_root(l[:4]) == h(h(l[0] + l[1]) + h(l[2] + l[3]))
    assert ht.merkle_root(l) == h(h(h(l[0] + l[1]) + h(l[2] + l[3])) + l[4])
    with pytest.raises(ValueError):
        ht.merkle_root([])
