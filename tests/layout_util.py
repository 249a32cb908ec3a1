"""The pool layout once more, for tests, as a reshape and a transposition of a
LOGICAL array [slice][kv][g][token][d] (slice = a block of T tokens, or a
sequence's stretch of C tokens).  Written apart from oracle/kv_layout.py and from
the library so that either one's index arithmetic is checked against it.

A pool is a row of slabs (St tiles of 16 tokens, all KV heads); in a slab the KV heads
come in groups of Gg (the largest divisor of G with Gg * d <= 1024), each group as its
K rows, then its V rows, tile after tile:
[slice][token // (16 St)][g // Gg][kv][(token // 16) % St][g % Gg][token % 16][d].
St doubles from 1 for as long as 2 St Gg d <= 1024 and 2 St divides the slice's tiles."""
import numpy as np


def _group(G, d):
    return max(c for c in range(1, G + 1) if G % c == 0 and c * d <= 1024)


def _tiles(G, d, cap):
    Gg, n = _group(G, d), cap // 16
    return max(s for s in (1, 2, 4, 8, 16, 32, 64) if s * Gg * d <= 1024 and n % s == 0)


def to_pool(logical):
    """[S][2][G][cap][d] (cap a multiple of 16) -> the flat pool."""
    S, two, G, cap, d = logical.shape
    assert two == 2 and cap % 16 == 0
    Gg, St = _group(G, d), _tiles(G, d, cap)
    x = logical.reshape(S, 2, G // Gg, Gg, cap // (16 * St), St, 16, d)
    #                   0  1  2       3   4                  5   6   7
    return np.ascontiguousarray(x.transpose(0, 4, 2, 1, 5, 3, 6, 7)).reshape(-1)


def from_pool(flat, S, G, cap, d):
    """The flat pool -> a logical [S][2][G][cap][d] COPY."""
    Gg, St = _group(G, d), _tiles(G, d, cap)
    x = np.asarray(flat).reshape(S, cap // (16 * St), G // Gg, 2, St, Gg, 16, d)
    #                            0  1                 2       3  4   5   6   7
    return np.ascontiguousarray(x.transpose(0, 3, 2, 5, 1, 4, 6, 7)).reshape(S, 2, G, cap, d)
