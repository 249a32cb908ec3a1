"""What a split-K work list has to satisfy (oracle side).

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

Decode attention over a long context is cut along the keys into work items
that are reduced independently and merged afterwards.  The contract with the
library: with split size S (tokens), sequence b with n_b keys is first cut
into c0 = ceil(n_b / S) equal pieces; the piece length ceil(n_b / c0) is then
rounded up to a multiple of 16 (work items start on 16-key boundaries), and
the sequence contributes the items [c*size, min((c+1)*size, n_b)) for
c = 0, 1, ... while they are non-empty.  Items are listed sequence by
sequence, in order, and each item is processed once per KV head.
"""


def piece_size(n, split_tokens):
    """Keys per item of a sequence with n keys (n >= 1)."""
    pieces = -(-n // split_tokens)
    longest = -(-n // pieces)
    while longest % 16:
        longest += 1
    return longest


def expected_items(ctx_lens, split_tokens):
    """The list of (b, tok_begin, tok_end) written out with plain loops."""
    items = []
    for b, n in enumerate(ctx_lens):
        n = int(n)
        if n < 1:
            continue
        size = piece_size(n, split_tokens)
        start = 0
        while start < n:
            stop = start + size
            if stop > n:
                stop = n
            items.append((b, start, stop))
            start = stop
    return items


def check_tiling(items, ctx_lens):
    """True iff the items cover every key of every sequence exactly once.

    Independent of how the items were produced: marks every token.
    """
    seen = [[0] * int(n) for n in ctx_lens]
    for (b, lo, hi) in items:
        if not (0 <= b < len(ctx_lens)) or not (0 <= lo < hi <= int(ctx_lens[b])):
            return False
        for t in range(lo, hi):
            seen[b][t] += 1
    return all(c == 1 for row in seen for c in row)
