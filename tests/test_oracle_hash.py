"""Pins for the oracle's partition hashes (the commitments hash(g_i[j]), hash(g^[j]) of
Alg. 2, lines 2 and 6) -- CPU only.  The paper names no hash function; this build fixes
SHA-256 over a tree of 1024-byte chunks with fan-out 32.  SHA-256 itself is the library's
and is pinned by the standard's known answers; the tree is pinned by composing it by hand
and by a second, recursive, way of writing it on small chunk sizes."""
import hashlib
import os

import numpy as np
import pytest

import oracle


def sha(b):
    return hashlib.sha256(b).digest()


def as_floats(b):
    assert len(b) % 4 == 0
    return np.frombuffer(b, dtype="<f4").reshape(1, -1)


def digest(G, off=None, **kw):
    G = np.atleast_2d(G)
    off = [0, G.shape[1]] if off is None else off
    return oracle.partition_hashes(G, off, **kw)


def test_known_answers_of_the_standard(golden_dir):
    seen = 0
    for line in open(os.path.join(golden_dir, "sha256_kat.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        msg, want = line.split()
        msg = b"" if msg == "-" else msg.encode("ascii")
        got = digest(as_floats(msg))[0, 0]
        assert bytes(got).hex() == want
        seen += 1
    assert seen == 3


def test_tree_composed_by_hand():
    rng = np.random.default_rng(1)
    # exactly one chunk: plain SHA-256 of the bytes
    G = rng.standard_normal((1, 256)).astype(np.float32)
    assert bytes(digest(G)[0, 0]) == sha(G.tobytes())
    # one float more: two chunks, hashed together
    G = rng.standard_normal((1, 257)).astype(np.float32)
    b = G.tobytes()
    assert bytes(digest(G)[0, 0]) == sha(sha(b[:1024]) + sha(b[1024:]))
    # 32 chunks: one node above them; 33 chunks: two nodes above them, then one more level
    G = rng.standard_normal((1, 33 * 256)).astype(np.float32)
    b = G.tobytes()
    leaves = [sha(b[k:k + 1024]) for k in range(0, len(b), 1024)]
    assert bytes(digest(G[:, :32 * 256])[0, 0]) == sha(b"".join(leaves[:32]))
    assert bytes(digest(G)[0, 0]) == sha(sha(b"".join(leaves[:32])) + sha(leaves[32]))


def recursive_tree(data, chunk, fanout):
    """The same tree written top-down: a node covering `span` leaves hashes its children."""
    leaves = max(1, -(-len(data) // chunk))
    span = 1
    while span < leaves:
        span *= fanout

    def node(first, span):
        if span == 1:
            return sha(data[first * chunk:(first + 1) * chunk])
        kids = [node(first + k * (span // fanout), span // fanout)
                for k in range(fanout) if first + k * (span // fanout) < leaves]
        return sha(b"".join(kids))

    return node(0, span)


@pytest.mark.parametrize("words", [1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 33, 64, 65, 100, 127, 129])
def test_deep_trees_on_small_chunks_against_the_top_down_form(words):
    """chunk = 8 bytes, fan-out 2: trees up to 7 levels deep.  In the bottom-up rule a lone
    last node of a level is still hashed (as a run of one digest), which the top-down form
    reproduces by hashing every node's children, however few."""
    G = np.random.default_rng(words).standard_normal((1, words)).astype(np.float32)
    got = bytes(digest(G, chunk_bytes=8, fanout=2)[0, 0])
    data = G.tobytes()
    # bottom-up by hand
    nodes = [sha(data[k:k + 8]) for k in range(0, len(data), 8)]
    while len(nodes) > 1:
        nodes = [sha(b"".join(nodes[k:k + 2])) for k in range(0, len(nodes), 2)]
    assert got == nodes[0]
    # top-down: only comparable when the leaf count is a power of the fan-out
    leaves = -(-len(data) // 8)
    if leaves & (leaves - 1) == 0:
        assert got == recursive_tree(data, 8, 2)


def test_partitions_rows_and_bytes():
    rng = np.random.default_rng(3)
    n, d = 3, 5000
    buf = rng.standard_normal((n, d + 7)).astype(np.float32)
    G = buf[:, :d]                                     # row stride > d
    off = [0, 0, 1200, 1200, 3100, 5000]               # empty partitions included
    H = oracle.partition_hashes(G, off)
    assert H.shape == (n, 5, 32) and H.dtype == np.uint8
    for i in range(n):
        for j in range(5):
            alone = oracle.partition_hashes(np.ascontiguousarray(G[i:i + 1, off[j]:off[j + 1]]),
                                            [0, off[j + 1] - off[j]])
            assert np.array_equal(H[i, j], alone[0, 0])
    assert bytes(H[0, 0]) == sha(b"") and np.array_equal(H[0, 0], H[2, 2])
    # one flipped bit anywhere changes that partition's digest and no other
    G2 = G.copy()
    G2.view(np.uint32)[1, 3000] ^= 1
    H2 = oracle.partition_hashes(G2, off)
    assert not np.array_equal(H2[1, 3], H[1, 3])
    H2[1, 3] = H[1, 3]
    assert np.array_equal(H2, H)
    # bytes are hashed, not values: -0.0 and +0.0 differ
    Z = np.zeros((1, 8), dtype=np.float32)
    Zm = Z.copy(); Zm[0, 5] = -0.0
    assert not np.array_equal(digest(Z), digest(Zm))
