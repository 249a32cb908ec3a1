"""The pool layout once more, for tests, as a reshape and a transposition of a
LOGICAL array [slice][kv][g][token][d] (slice = a block of T tokens, or a
sequence's stretch of C tokens).  Written apart from oracle/kv_layout.py and from
the library so that either one's index arithmetic is checked against it.

A pool is a row of tile slabs (16 tokens, all KV heads); in a slab the KV heads
come in groups of Gg (the largest divisor of G with Gg * d <= 1024), each group
as its K rows, then its V rows: [slice][token // 16][g // Gg][kv][g % Gg][token % 16][d]."""
import numpy as np


def _group(G, d):
    return max(c for c in range(1, G + 1) if G % c == 0 and c * d <= 1024)


def to_pool(logical):
    """[S][2][G][cap][d] (cap a multiple of 16) -> the flat pool."""
    S, two, G, cap, d = logical.shape
    assert two == 2 and cap % 16 == 0
    Gg = _group(G, d)
    x = logical.reshape(S, 2, G // Gg, Gg, cap // 16, 16, d)
    return np.ascontiguousarray(x.transpose(0, 4, 2, 1, 3, 5, 6)).reshape(-1)


def from_pool(flat, S, G, cap, d):
    """The flat pool -> a logical [S][2][G][cap][d] COPY."""
    Gg = _group(G, d)
    x = np.asarray(flat).reshape(S, cap // 16, G // Gg, 2, Gg, 16, d)
    return np.ascontiguousarray(x.transpose(0, 3, 2, 4, 1, 5, 6)).reshape(S, 2, G, cap, d)
