"""Where a token's K row and V row live in a layer's KV pool (oracle side).

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

The KV cache holds, per layer, one key row and one value row of `d` fp16
numbers per sequence, per token, per KV head (paper §II-A: keys and values of
every processed token are kept for reuse by the decode stage).  The library
fixes two pool layouts, written here from their description.  Both are made of
SLABS: the K and V rows of 16 * St consecutive tokens (St tiles of 16) for all G
KV heads, row-major as

  slab[group][kv][tile in slab][head in group][slot][d]
      group < G / Gg, tile in slab < St, head in group < Gg, slot < 16

where the KV heads are taken in groups of Gg consecutive heads, Gg being the
largest divisor of G with Gg * d <= 1024, kv = 0 selects keys and kv = 1
values, and St is the largest power of two with St * Gg * d <= 1024 that divides
the number of 16-token tiles of a pool slice (so that the K rows of a group, and
its V rows, are one run of at most 32 KiB, and of exactly 32 KiB wherever the
slice is long enough; St = 1 when a single tile of a group already is).

  contiguous  sequence b owns the C / (16 St) consecutive slabs from
              b * C / (16 St) on (C = capacity in tokens, a multiple of 16);
              token tok is in slab tok // (16 St) of them, tile
              (tok // 16) % St of it, slot tok % 16
  paged       block blk is the T / (16 St) consecutive slabs from
              blk * T / (16 St) on; token i of sequence b lives in block
              block_table[b][i // T], at token (i % T) of that block

Offsets are in ELEMENTS (fp16), not bytes.
"""
import numpy as np


def head_group(G, d):
    """Gg: the largest divisor of G with Gg * d <= 1024."""
    best = 1
    for c in range(1, G + 1):
        if G % c == 0 and c * d <= 1024:
            best = c
    return best


def slab_tiles(G, d, slice_tokens):
    """St: 16-token tiles per slab for a pool slice (block or sequence) of slice_tokens tokens."""
    assert slice_tokens % 16 == 0
    Gg = head_group(G, d)
    St = 1
    while 2 * St * Gg * d <= 1024 and (slice_tokens // 16) % (2 * St) == 0:
        St *= 2
    return St


def slab_row_offset(kv, g, tok, G, d, St):
    """Element offset of row (kv, g, tok) inside one slab (tok < 16 * St counts the slab's tokens)."""
    assert 0 <= kv < 2 and 0 <= g < G and 0 <= tok < 16 * St
    Gg = head_group(G, d)
    group, within = divmod(g, Gg)
    tile, slot = divmod(tok, 16)
    return (((((group * 2 + kv) * St + tile) * Gg + within) * 16) + slot) * d


def slab_elems(G, d, St):
    return 2 * G * 16 * St * d


def contiguous_row_offset(b, kv, g, tok, G, C, d):
    """Element offset of row (b, kv, g, tok) in a contiguous pool."""
    assert C % 16 == 0 and 0 <= tok < C
    St = slab_tiles(G, d, C)
    slab = b * (C // (16 * St)) + tok // (16 * St)
    return slab * slab_elems(G, d, St) + slab_row_offset(kv, g, tok % (16 * St), G, d, St)


def paged_row_offset(blk, kv, g, slot, G, T, d):
    """Element offset of row (blk, kv, g, slot) in a paged pool (slot < T counts
    tokens inside the block)."""
    assert blk >= 0, "token maps to an unallocated block"
    assert T % 16 == 0 and 0 <= slot < T
    St = slab_tiles(G, d, T)
    slab = blk * (T // (16 * St)) + slot // (16 * St)
    return slab * slab_elems(G, d, St) + slab_row_offset(kv, g, slot % (16 * St), G, d, St)


def token_row_offset(layout, b, kv, g, tok):
    """Element offset of token `tok` of sequence `b` under `layout`.

    layout: dict with keys G, d and either
      {"kind": "contiguous", "C": capacity}
      {"kind": "paged", "T": block tokens, "block_table": int array [B][max_blocks]}
    """
    G, d = layout["G"], layout["d"]
    if layout["kind"] == "contiguous":
        return contiguous_row_offset(b, kv, g, tok, G, layout["C"], d)
    T = layout["T"]
    blk = int(layout["block_table"][b][tok // T])
    return paged_row_offset(blk, kv, g, tok % T, G, T, d)


def gather_rows(pool_flat, layout, b, kv, g, n):
    """Rows 0..n-1 of (b, kv, g) as an [n, d] array of the pool's dtype.

    pool_flat is the layer's pool viewed as a flat 1-D array of fp16 (or of
    raw uint16 bit patterns); one row is copied per token, no arithmetic.
    """
    d = layout["d"]
    out = np.empty((n, d), dtype=pool_flat.dtype)
    for i in range(n):
        off = token_row_offset(layout, b, kv, g, i)
        out[i] = pool_flat[off:off + d]
    return out


def append_scatter(pool_flat, layout, ctx_lens_after, k_new, v_new):
    """What one append does to a layer's pool, in place.

    ctx_lens_after[b] is the number of tokens sequence b holds once this
    step's token is stored, so the new rows go to position ctx_lens_after[b]-1.
    k_new, v_new: [B][G][d] arrays of the pool's dtype (bit copy, no rounding).
    """
    G, d = layout["G"], layout["d"]
    B = len(ctx_lens_after)
    for b in range(B):
        pos = int(ctx_lens_after[b]) - 1
        assert pos >= 0
        for g in range(G):
            ok = token_row_offset(layout, b, 0, g, pos)
            ov = token_row_offset(layout, b, 1, g, pos)
            pool_flat[ok:ok + d] = k_new[b, g]
            pool_flat[ov:ov + d] = v_new[b, g]
    return pool_flat


def bulk_append_scatter(pool_flat, layout, ctx_lens_before, n_new, k_rows, v_rows):
    """What storing a whole prompt (or a run of new tokens) does to a layer's pool,
    in place (paper §II-A: the prefill stage produces the keys and values of every
    prompt token; §IV-D: with offloading they are then moved to host memory).

    Sequence b holds ctx_lens_before[b] tokens and receives n_new[b] more, at
    positions ctx_lens_before[b], ctx_lens_before[b] + 1, ...  k_rows, v_rows:
    [sum(n_new)][G][d] arrays of the pool's dtype, the rows of sequence 0 first,
    then those of sequence 1, ... each in position order (bit copy, no rounding).
    """
    G, d = layout["G"], layout["d"]
    row = 0
    for b in range(len(n_new)):
        for i in range(int(n_new[b])):
            pos = int(ctx_lens_before[b]) + i
            for g in range(G):
                ok = token_row_offset(layout, b, 0, g, pos)
                ov = token_row_offset(layout, b, 1, g, pos)
                pool_flat[ok:ok + d] = k_rows[row, g]
                pool_flat[ov:ov + d] = v_rows[row, g]
            row += 1
    assert row == len(k_rows) == len(v_rows)
    return pool_flat
