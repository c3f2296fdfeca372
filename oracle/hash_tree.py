"""Oracle for the hashing primitives (Method, primitives hash_sha256 and tree).

TEST INFRASTRUCTURE ONLY, like the rest of oracle/.  SHA-256 itself is the standard library's
hashlib (a library routine used as a step); what is written out here is how the build applies it:

  sha256_tree(data, chunk)   chunk = 0: the SHA-256 of the whole byte string -- the paper's
                             hash of the model weights.  chunk > 0: the same weights hashed as a
                             tree so that a GPU can do it in parallel: the data is cut into
                             chunks of `chunk` bytes (the last may be shorter), every chunk is
                             hashed, the 32-byte digests are concatenated in order, and the result
                             is treated the same way until it fits into one chunk, whose SHA-256
                             is the answer.
  merkle_root(leaves)        binary Merkle tree over 32-byte leaves (one per checkpoint): a parent
                             is SHA-256(left || right); a node without a sibling moves up unchanged.
"""
from __future__ import annotations

import hashlib


def sha256(data: bytes) -> bytes:
    return hashlib.sha256(data).digest()


def sha256_tree(data: bytes, chunk: int = 4096) -> bytes:
    if chunk < 0 or (chunk and chunk % 64):
        raise ValueError("chunk must be 0 or a positive multiple of 64")
    level = bytes(data)
    if chunk == 0:
        return sha256(level)
    while len(level) > chunk:
        level = b"".join(sha256(level[i:i + chunk]) for i in range(0, len(level), chunk))
    return sha256(level)


def merkle_root(leaves) -> bytes:
    level = [bytes(l) for l in leaves]
    if not level or any(len(l) != 32 for l in level):
        raise ValueError("need at least one 32-byte leaf")
    while len(level) > 1:
        nxt = [sha256(level[i] + level[i + 1]) for i in range(0, len(level) - 1, 2)]
        if len(level) % 2:
            nxt.append(level[-1])
        level = nxt
    return level[0]
