"""Pins for the oracle's bulk (prompt) store and the prefill transfer formulas.  CPU only."""
from fractions import Fraction

import numpy as np

from oracle import kv_bytes, kv_layout

from layout_util import from_pool, to_pool


def _random_case(rng, paged):
    G, d, T = int(rng.integers(1, 4)), int(rng.choice([4, 8])), 16
    B = int(rng.integers(1, 5))
    before = rng.integers(0, 40, size=B)
    n_new = rng.integers(0, 50, size=B)
    cap = int((before + n_new).max()) + 3
    if paged:
        nb = -(-cap // T)
        n_blocks = B * nb + 2
        table = rng.permutation(n_blocks)[:B * nb].reshape(B, nb)
        layout = {"kind": "paged", "G": G, "d": d, "T": T, "block_table": table}
        n_el = n_blocks * 2 * G * T * d
    else:
        C = -(-cap // 16) * 16
        layout = {"kind": "contiguous", "G": G, "d": d, "C": C}
        n_el = B * 2 * G * C * d
    pool = rng.integers(0, 60000, size=n_el).astype(np.uint16)
    rows = int(n_new.sum())
    k = rng.integers(0, 60000, size=(rows, G, d)).astype(np.uint16)
    v = rng.integers(0, 60000, size=(rows, G, d)).astype(np.uint16)
    return layout, pool, before, n_new, k, v


def test_bulk_store_equals_indexing_the_reshaped_pool():
    # the same store written through numpy's own N-d indexing of the pool, brought into logical order by a
    # reshape and a transposition and back
    rng = np.random.default_rng(3)
    for trial in range(40):
        paged = trial % 2 == 0
        layout, pool, before, n_new, k, v = _random_case(rng, paged)
        G, d = layout["G"], layout["d"]
        if paged:
            T = layout["T"]
            view = from_pool(pool, len(pool) // (2 * G * T * d), G, T, d)
        else:
            view = from_pool(pool, len(n_new), G, layout["C"], d)
        row = 0
        for b in range(len(n_new)):
            for i in range(int(n_new[b])):
                pos = int(before[b]) + i
                if paged:
                    view[layout["block_table"][b][pos // T], 0, :, pos % T, :] = k[row]
                    view[layout["block_table"][b][pos // T], 1, :, pos % T, :] = v[row]
                else:
                    view[b, 0, :, pos, :] = k[row]
                    view[b, 1, :, pos, :] = v[row]
                row += 1
        want = to_pool(view)
        got = kv_layout.bulk_append_scatter(pool.copy(), layout, before, n_new, k, v)
        np.testing.assert_array_equal(got, want)


def test_bulk_store_equals_token_by_token_appends_and_touches_nothing_else():
    rng = np.random.default_rng(4)
    for trial in range(20):
        layout, pool, before, n_new, k, v = _random_case(rng, trial % 2 == 0)
        G, d = layout["G"], layout["d"]
        B = len(n_new)
        got = kv_layout.bulk_append_scatter(pool.copy(), layout, before, n_new, k, v)
        # one token at a time, sequence by sequence, through the single-token store
        step = pool.copy()
        first = np.concatenate([[0], np.cumsum(n_new)])
        for b in range(B):
            for i in range(int(n_new[b])):
                after = np.zeros(B, dtype=np.int64)
                knew = np.zeros((B, G, d), dtype=np.uint16)
                vnew = np.zeros((B, G, d), dtype=np.uint16)
                # only sequence b stores: give the others a position they already hold and its own bits
                for o in range(B):
                    after[o] = 1
                    for g in range(G):
                        off_k = kv_layout.token_row_offset(layout, o, 0, g, 0)
                        off_v = kv_layout.token_row_offset(layout, o, 1, g, 0)
                        knew[o, g] = step[off_k:off_k + d]
                        vnew[o, g] = step[off_v:off_v + d]
                after[b] = before[b] + i + 1
                knew[b], vnew[b] = k[first[b] + i], v[first[b] + i]
                kv_layout.append_scatter(step, layout, after, knew, vnew)
        np.testing.assert_array_equal(got, step)
        # rows outside the new positions keep their bits
        changed = np.flatnonzero(got != pool)
        allowed = set()
        for b in range(B):
            for i in range(int(n_new[b])):
                for kv in (0, 1):
                    for g in range(G):
                        off = kv_layout.token_row_offset(layout, b, kv, g, int(before[b]) + i)
                        allowed.update(range(off, off + d))
        assert set(changed.tolist()) <= allowed


def test_prefill_transfer_time_formula():
    # §IV-D: C_off * 2 (L_in + 1) h1 prec BS / BW per layer; at C_off = 1 it is the bytes of K and V of
    # L_in + 1 tokens per sequence over the link
    bw = 32 * 10 ** 9
    t = kv_bytes.t_trans_prefill(1, 1024, 4096, 64, bw)
    assert t == Fraction(kv_bytes.kv_bytes_written([1025] * 64, 32, 128), bw)
    assert kv_bytes.t_trans_prefill(Fraction(1, 2), 1024, 4096, 64, bw) == t / 2
    assert kv_bytes.t_trans_prefill(0, 1024, 4096, 64, bw) == 0
    # summed over the layers the prompt's share of Table II's cache: L_out = 1 leaves L_in + 1 tokens
    L = 32
    assert t * L * bw == kv_bytes.mem_kvcache(64, 1024, 1, 4096, L)
    # Eq. 5
    assert kv_bytes.t_prefill(3, 5) == 5 and kv_bytes.t_prefill(7, 5) == 7
