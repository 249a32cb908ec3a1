"""What a split-K work list has to satisfy (oracle side).

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

Decode attention over a long context is cut along the keys into work items
that are reduced independently and merged afterwards.  The contract with the
library: with split size S (tokens), sequence b with n_b keys contributes the
items [c*S, min((c+1)*S, n_b)) for c = 0, 1, ...; items are listed sequence
by sequence, in order, and each item is processed once per KV head.
"""


def expected_items(ctx_lens, split_tokens):
    """The list of (b, tok_begin, tok_end) written out with plain loops."""
    items = []
    for b, n in enumerate(ctx_lens):
        n = int(n)
        start = 0
        while start < n:
            stop = start + split_tokens
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
