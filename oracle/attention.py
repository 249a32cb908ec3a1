"""Decode attention, written out as its definition in fp64 (oracle side).

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

One decode step (paper §II-A): the token just generated attends over every
key/value stored so far for its sequence, including its own, which was
appended before the attention runs.  The paper prints no attention formula
(it cites the Transformer paper); the reading taken is the standard scaled
dot-product attention with no mask beyond the sequence length, no bias and no
positional term:

    s_i  = (q . k_i) / sqrt(d)            i = 0 .. n-1
    w_i  = exp(s_i - max_j s_j)
    out  = sum_i w_i v_i / sum_i w_i

Query head h reads KV head g = h // (H // G) (consecutive grouping; H == G is
plain multi-head attention).  Where the KV physically lives (HBM, host memory,
which block) never changes the value: offloaded data is fetched back to the
GPU before it is used (paper §II-B).

Inputs are fp16 arrays (or their raw uint16 bit patterns); every value is
converted exactly to fp64 first and all arithmetic is fp64.
"""
import math

import numpy as np

from . import kv_layout


def as_f64(a):
    """Exact fp16 -> fp64 conversion; accepts fp16 arrays or uint16 bit patterns."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.float16)
    return a.astype(np.float64)


def attend_one(q_vec, k_rows, v_rows):
    """One query vector against n key rows and n value rows; returns [d] fp64.

    q_vec [d], k_rows [n][d], v_rows [n][d]; n >= 1.
    """
    q_vec = np.asarray(q_vec, dtype=np.float64)
    k_rows = np.asarray(k_rows, dtype=np.float64)
    v_rows = np.asarray(v_rows, dtype=np.float64)
    n, d = k_rows.shape
    if n < 1:
        raise ValueError("a decode step attends over at least its own token")
    s = (k_rows @ q_vec) / math.sqrt(d)
    m = s.max()
    w = np.exp(s - m)
    z = w.sum()
    return (w @ v_rows) / z


def decode_attn(q, pool_flat, layout, ctx_lens, H, sample=None):
    """Attention output of one layer for a batch; returns fp64 [B][H][d].

    q          fp16 [B][H][d]
    pool_flat  the layer's KV pool as a flat fp16/uint16 array (kv_layout)
    layout     see kv_layout.token_row_offset
    ctx_lens   [B] keys attended per sequence (after this step's append)
    sample     optional iterable of (b, h) pairs; only those are computed and
               the rest of the result is NaN
    """
    G, d = layout["G"], layout["d"]
    assert H % G == 0
    group = H // G
    qf = as_f64(q)
    B = len(ctx_lens)
    out = np.full((B, H, d), np.nan, dtype=np.float64)
    pairs = sample if sample is not None else [(b, h) for b in range(B) for h in range(H)]
    cache = {}
    for (b, h) in pairs:
        g = h // group
        n = int(ctx_lens[b])
        if (b, g) not in cache:
            k = as_f64(kv_layout.gather_rows(pool_flat, layout, b, 0, g, n))
            v = as_f64(kv_layout.gather_rows(pool_flat, layout, b, 1, g, n))
            cache = {(b, g): (k, v)}        # keep one (b, g) at a time
        k, v = cache[(b, g)]
        out[b, h] = attend_one(qf[b, h], k, v)
    return out


def merge_partials(ms, ls, os):
    """Combine per-split (max, sum, weighted-sum) triples into one output.

    Split c holds m_c = max of its scores, l_c = sum exp(s - m_c) and
    o_c = sum exp(s - m_c) v.  The combination
        M = max m_c,  L = sum l_c e^{m_c - M},  out = sum o_c e^{m_c - M} / L
    equals attention over the union of the splits; tests check that identity
    against attend_one by brute force.
    """
    ms = np.asarray(ms, dtype=np.float64)
    ls = np.asarray(ls, dtype=np.float64)
    os = np.asarray(os, dtype=np.float64)
    M = ms.max()
    scale = np.exp(ms - M)
    L = (ls * scale).sum()
    return (os * scale[:, None]).sum(axis=0) / L


def split_partial(q_vec, k_rows, v_rows):
    """(m, l, o) of one split, natural-log domain."""
    k_rows = np.asarray(k_rows, dtype=np.float64)
    v_rows = np.asarray(v_rows, dtype=np.float64)
    s = (k_rows @ np.asarray(q_vec, dtype=np.float64)) / math.sqrt(k_rows.shape[1])
    m = s.max()
    w = np.exp(s - m)
    return m, w.sum(), w @ v_rows
