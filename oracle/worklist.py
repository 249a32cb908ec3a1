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

When no split size is fixed the library shares the keys of a launch out in
equal stretches instead, so that wavefronts that stream at one rate end
together.  The contract: the 16-key tiles of all sequences are laid end to
end in sequence order (a sequence with n keys has ceil(n / 16) tiles, the
last one possibly partial); with T tiles in all, at most `max_groups`
stretches and a shortest stretch of 8 tiles, there are
g = min(max_groups, max(1, T // 8)) stretches of span = ceil(T / g) tiles:
tile number p of the stream belongs to stretch p // span.  An item is a
maximal run of consecutive tiles of ONE sequence inside ONE stretch; items
are listed in stream order; the items that start in stretch j form group j.
expected_items_equal_stretches below walks the stream tile by tile.

Block-granular offload (paper §IV-C: a share C_off of the cache lives in host
memory) adds one more cut.  Block ids below `resident_blocks` are in HBM
(class 0); the others are in the host pool, which is streamed in chunks of
`chunk_blocks` consecutive blocks (host block i belongs to class 1 + i //
chunk_blocks).  Each class is attended by a launch of its own, so an item may
not cross from one class into another: a sequence is first cut into maximal
runs of consecutive positions whose blocks are in one class, and every run is
then cut into equal pieces exactly as a whole sequence is above (the run's
length taking the place of n_b, positions counted from the run's start).
Items are listed class by class; inside a class sequence by sequence, and
inside a sequence by position.
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


def expected_items_equal_stretches(ctx_lens, max_groups, min_span_tiles=8):
    """(items, group_first, span): the stream of tiles walked one tile at a time.

    items        [(b, tok_begin, tok_end)] in stream order
    group_first  index of the first item of every stretch, then len(items)
    span         tiles per stretch
    """
    stream = []                                   # (sequence, tile of the sequence) for every tile, in order
    for b, n in enumerate(ctx_lens):
        n = int(n)
        for t in range(-(-n // 16)):
            stream.append((b, t))
    total = len(stream)
    groups = min(max_groups, max(1, total // min_span_tiles))
    span = max(1, -(-total // groups))
    items, group_first = [], []
    prev = None                                   # (sequence, stretch) of the previous tile
    for p, (b, t) in enumerate(stream):
        stretch = p // span
        n = int(ctx_lens[b])
        if prev != (b, stretch):
            if prev is None or prev[1] != stretch:
                group_first.append(len(items))
            items.append([b, 16 * t, min(n, 16 * t + 16)])
        else:
            items[-1][2] = min(n, 16 * t + 16)
        prev = (b, stretch)
    group_first.append(len(items))
    return [tuple(i) for i in items], group_first, span


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


def block_class(block_id, resident_blocks, chunk_blocks):
    """0 if the block stays in HBM, else 1 + the chunk of the host pool it is in."""
    if block_id < resident_blocks:
        return 0
    return 1 + (block_id - resident_blocks) // chunk_blocks


def expected_items_by_class(ctx_lens, block_table, block_tokens, resident_blocks, chunk_blocks,
                            split_tokens, n_classes):
    """A list with one item list per class, written out with plain loops over
    the positions of every sequence."""
    per_class = [[] for _ in range(n_classes)]
    for b, n in enumerate(ctx_lens):
        n = int(n)
        if n < 1:
            continue
        cls_of = [block_class(int(block_table[b][t // block_tokens]), resident_blocks, chunk_blocks)
                  for t in range(n)]
        run_start = 0
        for t in range(1, n + 1):
            if t < n and cls_of[t] == cls_of[run_start]:
                continue
            length = t - run_start                      # positions run_start .. t-1 form a run
            size = piece_size(length, split_tokens)
            start = run_start
            while start < t:
                stop = min(start + size, t)
                per_class[cls_of[run_start]].append((b, start, stop))
                start = stop
            run_start = t
    return per_class


def check_classes(per_class, block_table, block_tokens, resident_blocks, chunk_blocks):
    """True iff every position of every item lies in a block of the item's class."""
    for cls, items in enumerate(per_class):
        for (b, lo, hi) in items:
            for t in range(lo, hi):
                if block_class(int(block_table[b][t // block_tokens]), resident_blocks, chunk_blocks) != cls:
                    return False
    return True
