"""Pins for the attention oracle: closed forms, invariants, a library routine
on the special case it covers, brute force on tiny inputs, and mutants that
show each plausible mistake is caught by at least one pin.  CPU only."""
import math

import numpy as np

from layout_util import to_pool
import pytest

from oracle import attention as oa
from oracle import kv_layout
from paper_2504_11816_amd import synth


def _rand(shape, seed):
    return synth.randn_f16_numpy(shape, seed).astype(np.float64)


# --------------------------------------------------------------------------
# The pins, each a function of an `attend(q, K, V) -> out` callable so that
# the same list can be run on deliberately broken variants.
# --------------------------------------------------------------------------

def pin_single_key(attend):
    q, K, V = _rand(16, 1), _rand((1, 16), 2), _rand((1, 16), 3)
    assert np.array_equal(attend(q, K, V), V[0])            # n = 1: exactly v_0


def pin_identical_keys_give_mean(attend):
    q, k, V = _rand(8, 4), _rand(8, 5), _rand((7, 8), 6)
    K = np.tile(k, (7, 1))
    np.testing.assert_allclose(attend(q, K, V), V.mean(axis=0), rtol=1e-14, atol=1e-15)


def pin_constant_values(attend):
    q, K = _rand(8, 7), _rand((9, 8), 8)
    V = np.full((9, 8), 0.625)
    np.testing.assert_allclose(attend(q, K, V), np.full(8, 0.625), rtol=1e-14)


def pin_zero_query_gives_mean(attend):
    K, V = _rand((5, 8), 9), _rand((5, 8), 10)
    np.testing.assert_allclose(attend(np.zeros(8), K, V), V.mean(axis=0), rtol=1e-14, atol=1e-15)


def pin_two_keys_logistic(attend):
    # out = sigma(D) v0 + (1 - sigma(D)) v1 with D = q.(k0 - k1) / sqrt(d)
    for seed in range(5):
        d = 16
        q, K, V = _rand(d, 20 + seed), _rand((2, d), 30 + seed), _rand((2, d), 40 + seed)
        delta = sum(q[j] * (K[0, j] - K[1, j]) for j in range(d)) / math.sqrt(d)
        sig = 1.0 / (1.0 + math.exp(-delta))
        want = sig * V[0] + (1.0 - sig) * V[1]
        np.testing.assert_allclose(attend(q, K, V), want, rtol=1e-12, atol=1e-14)


def pin_two_keys_hand_numbers(attend):
    # d = 4, q = (2,0,0,0), k0 = (1,0,0,0), k1 = 0: scores 2/sqrt(4) = 1 and 0
    # weights e/(e+1), 1/(e+1);  V rows (1,0,..) and (0,1,..)
    q = np.array([2.0, 0, 0, 0])
    K = np.array([[1.0, 0, 0, 0], [0.0, 0, 0, 0]])
    V = np.array([[1.0, 0, 0, 0], [0.0, 1, 0, 0]])
    e = math.e
    want = np.array([e / (e + 1), 1 / (e + 1), 0, 0])
    np.testing.assert_allclose(attend(q, K, V), want, rtol=1e-14, atol=1e-16)


def pin_key_shift_invariance(attend):
    q, K, V, c = _rand(8, 50), _rand((11, 8), 51), _rand((11, 8), 52), _rand(8, 53)
    np.testing.assert_allclose(attend(q, K + c, V), attend(q, K, V), rtol=1e-11, atol=1e-13)


def pin_dominant_key(attend):
    q, K, V = _rand(8, 60), _rand((6, 8), 61), _rand((6, 8), 62)
    K[3] = 200.0 * q
    np.testing.assert_allclose(attend(q, K, V), V[3], rtol=1e-12, atol=1e-12)


def pin_convex_hull(attend):
    q, K, V = _rand(8, 70), _rand((13, 8), 71), _rand((13, 8), 72)
    out = attend(q, K, V)
    assert np.all(out <= V.max(axis=0) + 1e-15) and np.all(out >= V.min(axis=0) - 1e-15)


def pin_linear_in_values(attend):
    q, K, V1, V2 = _rand(8, 80), _rand((9, 8), 81), _rand((9, 8), 82), _rand((9, 8), 83)
    np.testing.assert_allclose(attend(q, K, V1 + 2 * V2), attend(q, K, V1) + 2 * attend(q, K, V2),
                               rtol=1e-12, atol=1e-14)


def pin_large_scores_do_not_overflow(attend):
    q = np.full(4, 60.0)
    K = np.array([[60.0] * 4, [59.0] * 4, [-60.0] * 4])
    V = np.array([[1.0, 2, 3, 4], [5.0, 6, 7, 8], [9.0, 9, 9, 9]])
    out = attend(q, K, V)
    assert np.all(np.isfinite(out))
    # scores 7200, 7080, -7200 -> weight of key 0 is 1 to 52 bits
    np.testing.assert_allclose(out, V[0], rtol=1e-15)


def pin_brute_force_python(attend):
    # Tiny cases against explicit Python loops with exactly rounded sums.
    for seed, (n, d) in enumerate([(1, 1), (2, 3), (5, 4), (3, 2), (4, 1)]):
        q, K, V = _rand(d, 90 + seed), _rand((n, d), 100 + seed), _rand((n, d), 110 + seed)
        scores = [math.fsum(q[j] * K[i, j] for j in range(d)) / math.sqrt(d) for i in range(n)]
        top = max(scores)
        wts = [math.exp(s - top) for s in scores]
        z = math.fsum(wts)
        want = [math.fsum(wts[i] * V[i, j] for i in range(n)) / z for j in range(d)]
        np.testing.assert_allclose(attend(q, K, V), want, rtol=1e-13, atol=1e-15)


def pin_torch_sdpa_fp64(attend):
    # Library routine on the case it covers: one query row, no mask, default scale.
    import torch
    q, K, V = _rand(32, 120), _rand((37, 32), 121), _rand((37, 32), 122)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None, None, None, :], torch.from_numpy(K)[None, None],
        torch.from_numpy(V)[None, None]).numpy()[0, 0, 0]
    np.testing.assert_allclose(attend(q, K, V), want, rtol=1e-12, atol=1e-14)


PINS = [pin_single_key, pin_identical_keys_give_mean, pin_constant_values, pin_zero_query_gives_mean,
        pin_two_keys_logistic, pin_two_keys_hand_numbers, pin_key_shift_invariance, pin_dominant_key,
        pin_convex_hull, pin_linear_in_values, pin_large_scores_do_not_overflow,
        pin_brute_force_python, pin_torch_sdpa_fp64]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_attend_one_pins(pin):
    pin(oa.attend_one)


# ---- mutants: every plausible slip must trip at least one pin -------------

def _mut(scale=lambda d: 1 / math.sqrt(d), sign=1.0, shift=True, norm=True, use_k_for_v=False,
         transpose_bug=False):
    def attend(q, K, V):
        q, K, V = np.asarray(q, float), np.asarray(K, float), np.asarray(V, float)
        n, d = K.shape
        s = sign * (K @ q) * scale(d)
        if transpose_bug:
            s = s[::-1].copy()
        w = np.exp(s - (s.max() if shift else 0.0))
        src = K if use_k_for_v else V
        out = w @ src
        return out / w.sum() if norm else out
    return attend


MUTANTS = {
    "scale_1_over_d": _mut(scale=lambda d: 1.0 / d),
    "no_scale": _mut(scale=lambda d: 1.0),
    "scale_sqrt_d": _mut(scale=lambda d: math.sqrt(d)),
    "negated_scores": _mut(sign=-1.0),
    "no_max_shift": _mut(shift=False),
    "no_normalisation": _mut(norm=False),
    "keys_as_values": _mut(use_k_for_v=True),
    "weights_reversed": _mut(transpose_bug=True),
}


def test_reference_mutant_is_clean():
    for pin in PINS:
        pin(_mut())


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_each_mutant_fails_some_pin(name):
    attend = MUTANTS[name]
    failed = []
    for pin in PINS:
        try:
            with np.errstate(all="ignore"):
                pin(attend)
        except AssertionError:
            failed.append(pin.__name__)
    assert failed, f"mutant {name} passes every pin"


# ---- batch-level oracle: grouping, layouts, sampling ----------------------

def _contig_case(B, H, G, d, n_list, C, seed):
    pool = synth.randn_f16_numpy((B, 2, G, C, d), seed)
    q = synth.randn_f16_numpy((B, H, d), seed + 1)
    layout = {"kind": "contiguous", "G": G, "d": d, "C": C}
    return q, pool, layout, np.asarray(n_list, dtype=np.int32)


def test_batch_oracle_matches_attend_one_by_direct_slicing():
    B, H, G, d, C = 3, 4, 2, 8, 32
    q, pool, layout, n = _contig_case(B, H, G, d, [1, 17, 32], C, 200)
    out = oa.decode_attn(q, to_pool(pool), layout, n, H)
    for b in range(B):
        for h in range(H):
            g = h // (H // G)
            want = oa.attend_one(q[b, h].astype(float), pool[b, 0, g, :n[b]].astype(float),
                                 pool[b, 1, g, :n[b]].astype(float))
            np.testing.assert_array_equal(out[b, h], want)


def test_gqa_equals_mha_on_replicated_kv():
    B, H, G, d, C = 2, 8, 2, 8, 32
    q, pool, layout, n = _contig_case(B, H, G, d, [20, 4], C, 210)
    out_gqa = oa.decode_attn(q, to_pool(pool), layout, n, H)
    rep = np.repeat(pool, H // G, axis=2)                       # KV head g -> heads g*4 .. g*4+3
    layout_mha = {"kind": "contiguous", "G": H, "d": d, "C": C}
    out_mha = oa.decode_attn(q, to_pool(rep), layout_mha, n, H)
    np.testing.assert_array_equal(out_gqa, out_mha)


def test_paged_equals_contiguous_and_is_invariant_to_block_permutation():
    B, H, G, d, T = 3, 4, 2, 8, 16
    n = np.array([5, 64, 33], dtype=np.int32)
    C = 64
    q, pool_c, layout_c, _ = _contig_case(B, H, G, d, n, C, 220)
    want = oa.decode_attn(q, to_pool(pool_c), layout_c, n, H)
    n_blocks = 20
    for seed in (1, 2):
        table = synth.shuffled_block_table([C] * B, T, n_blocks, seed)
        pool_p = synth.randn_f16_numpy((n_blocks, 2, G, T, d), 999)    # junk in unused blocks
        for b in range(B):
            for i in range(C):
                blk = table[b, i // T]
                pool_p[blk, :, :, i % T, :] = pool_c[b, :, :, i, :]
        layout_p = {"kind": "paged", "G": G, "d": d, "T": T, "block_table": table}
        got = oa.decode_attn(q, to_pool(pool_p), layout_p, n, H)
        np.testing.assert_array_equal(got, want)


def test_sampled_pairs_equal_full_run():
    B, H, G, d, C = 3, 4, 4, 8, 16
    q, pool, layout, n = _contig_case(B, H, G, d, [9, 2, 16], C, 230)
    full = oa.decode_attn(q, to_pool(pool), layout, n, H)
    part = oa.decode_attn(q, to_pool(pool), layout, n, H, sample=[(2, 3), (0, 1)])
    np.testing.assert_array_equal(part[2, 3], full[2, 3])
    np.testing.assert_array_equal(part[0, 1], full[0, 1])
    assert np.isnan(part[1, 0]).all()


def test_uint16_bit_patterns_are_read_as_fp16():
    a = synth.randn_f16_numpy((5, 3), 240)
    np.testing.assert_array_equal(oa.as_f64(a.view(np.uint16)), a.astype(np.float64))
    sub = np.array([0x0001, 0x03FF, 0x8001], dtype=np.uint16)            # fp16 subnormals, exact
    np.testing.assert_array_equal(oa.as_f64(sub), [2.0 ** -24, 1023 * 2.0 ** -24, -(2.0 ** -24)])


def test_split_merge_identity_brute_force():
    # (m, l, o) partials of any partition of the keys merge to the full result.
    rng = np.random.default_rng(5)
    q, K, V = _rand(8, 250), _rand((23, 8), 251), _rand((23, 8), 252)
    want = oa.attend_one(q, K, V)
    for cuts in ([23], [1] * 23, [7, 16], [5, 5, 5, 8], [22, 1]):
        ms, ls, os_, at = [], [], [], 0
        for c in cuts:
            m, l, o = oa.split_partial(q, K[at:at + c], V[at:at + c])
            ms.append(m), ls.append(l), os_.append(o)
            at += c
        np.testing.assert_allclose(oa.merge_partials(ms, ls, os_), want, rtol=1e-13, atol=1e-15)
    # and for a random interleaved partition (splits need not be contiguous)
    idx = rng.permutation(23)
    parts = [idx[:9], idx[9:10], idx[10:]]
    trip = [oa.split_partial(q, K[p], V[p]) for p in parts]
    got = oa.merge_partials([t[0] for t in trip], [t[1] for t in trip], [t[2] for t in trip])
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-15)


def test_output_spread_of_the_synthetic_workload():
    # N(0,1) q, K, V: the output's standard deviation is about sqrt(e / n);
    # a sanity check that data and scale are what the workloads intend.
    n, d = 256, 64
    outs = []
    for s in range(24):
        q, K, V = _rand(d, 300 + s), _rand((n, d), 400 + s), _rand((n, d), 500 + s)
        outs.append(oa.attend_one(q, K, V))
    sd = np.std(np.concatenate(outs))
    assert 0.8 * math.sqrt(math.e / n) < sd < 1.25 * math.sqrt(math.e / n)


def test_append_scatter_then_attend_sees_the_new_token():
    B, H, G, d, T = 2, 2, 2, 4, 16
    n_before = np.array([15, 16], dtype=np.int32)               # second one opens a new block
    table = synth.shuffled_block_table([32, 32], T, 6, 3)
    pool = synth.randn_f16_numpy((6, 2, G, T, d), 260)
    layout = {"kind": "paged", "G": G, "d": d, "T": T, "block_table": table}
    k_new, v_new = synth.randn_f16_numpy((B, G, d), 261), synth.randn_f16_numpy((B, G, d), 262)
    flat = pool.reshape(-1).copy()
    before = flat.copy()
    kv_layout.append_scatter(flat, layout, n_before + 1, k_new, v_new)
    changed = np.flatnonzero(flat.view(np.uint16) != before.view(np.uint16))
    assert len(changed) <= B * G * 2 * d
    for b in range(B):
        for g in range(G):
            rows_k = kv_layout.gather_rows(flat, layout, b, 0, g, n_before[b] + 1)
            rows_v = kv_layout.gather_rows(flat, layout, b, 1, g, n_before[b] + 1)
            np.testing.assert_array_equal(rows_k[-1], k_new[b, g])
            np.testing.assert_array_equal(rows_v[-1], v_new[b, g])
            np.testing.assert_array_equal(
                rows_k[:-1], kv_layout.gather_rows(before, layout, b, 0, g, n_before[b]))
    # dominant new key: the step's output is the new value row
    q = np.zeros((B, H, d), dtype=np.float16)
    k_dom = np.zeros((B, G, d), dtype=np.float16)
    q[:, :, 0] = 60.0
    k_dom[:, :, 0] = 60.0
    flat2 = np.zeros_like(flat)
    kv_layout.append_scatter(flat2, layout, n_before + 1, k_dom, v_new)
    out = oa.decode_attn(q, flat2, layout, n_before + 1, H)
    for b in range(B):
        for h in range(H):
            np.testing.assert_allclose(out[b, h], v_new[b, h].astype(float), rtol=1e-12, atol=1e-300)


def test_layout_offsets_address_probe():
    # Every (coordinate) -> offset map is a bijection onto the pool and row
    # major in the stated order: number the elements of a pool shaped as the
    # description reads ([slabs][group][kv][tile in slab][head in group][slot][d])
    # and look every row up.  St (tiles per slab) is written out per case from the rule's
    # wording: the largest power of two with St * Gg * d <= 1024 that divides the slice's tiles.
    for G, d, Gg, T, St_T, C, St_C in ((16, 128, 8, 32, 1, 48, 1), (32, 64, 16, 32, 1, 48, 1), (3, 64, 3, 32, 2, 48, 1),
                                       (12, 128, 6, 32, 1, 48, 1), (4, 128, 4, 32, 2, 64, 2), (2, 128, 2, 64, 4, 96, 2),
                                       (1, 128, 1, 128, 8, 128, 8), (1, 64, 1, 256, 16, 16, 1), (4, 128, 4, 16, 1, 32, 2),
                                       (8, 64, 8, 64, 2, 80, 1)):
        assert kv_layout.head_group(G, d) == Gg
        assert kv_layout.slab_tiles(G, d, T) == St_T and kv_layout.slab_tiles(G, d, C) == St_C
        nblk, St = 3, St_T
        ref = np.arange(nblk * T * 2 * G * d).reshape(nblk, T // (16 * St), G // Gg, 2, St, Gg, 16, d)
        seen = set()
        for blk in range(nblk):
            for kv in range(2):
                for g in range(G):
                    for s in range(T):
                        off = kv_layout.paged_row_offset(blk, kv, g, s, G, T, d)
                        assert off == ref[blk, s // (16 * St), g // Gg, kv, (s // 16) % St, g % Gg, s % 16, 0]
                        seen.add(off)
        assert len(seen) == nblk * 2 * G * T and max(seen) == ref.size - d
        B, St = 3, St_C
        ref = np.arange(B * C * 2 * G * d).reshape(B, C // (16 * St), G // Gg, 2, St, Gg, 16, d)
        for b in range(B):
            for kv in range(2):
                for g in range(G):
                    for t in range(C):
                        assert kv_layout.contiguous_row_offset(b, kv, g, t, G, C, d) == \
                            ref[b, t // (16 * St), g // Gg, kv, (t // 16) % St, g % Gg, t % 16, 0]


def test_slab_tiles_rule_puts_k_and_v_of_a_tile_32_kib_apart_where_the_slice_allows():
    # distance between a head's K rows and its V rows of the same tile = St * Gg * 16 * d * 2 bytes
    for G, d, slice_tokens, apart in ((32, 128, 16, 32768), (8, 128, 16, 32768), (4, 128, 16, 16384), (4, 128, 32, 32768),
                                      (4, 128, 4096, 32768), (2, 128, 64, 32768), (2, 128, 32, 16384), (1, 128, 128, 32768),
                                      (1, 128, 1024, 32768), (1, 128, 48, 4096), (8, 64, 32, 32768), (16, 64, 16, 32768),
                                      (12, 128, 64, 24576), (3, 64, 64, 24576)):
        St, Gg = kv_layout.slab_tiles(G, d, slice_tokens), kv_layout.head_group(G, d)
        assert St * Gg * 16 * d * 2 == apart, (G, d, slice_tokens)
        assert (slice_tokens // 16) % St == 0 and St & (St - 1) == 0
        k0 = kv_layout.paged_row_offset(0, 0, 0, 0, G, slice_tokens, d)
        v0 = kv_layout.paged_row_offset(0, 1, 0, 0, G, slice_tokens, d)
        assert (v0 - k0) * 2 == apart


def test_head_group_rule():
    # the largest divisor of G whose K rows of one 16-token tile fit in 32 KiB (Gg * d <= 1024)
    want = {(32, 128): 8, (8, 128): 8, (4, 128): 4, (1, 128): 1, (32, 64): 16, (16, 64): 16, (12, 128): 6,
            (7, 128): 7, (9, 128): 3, (40, 128): 8, (24, 64): 12, (11, 128): 1}
    for (G, d), Gg in want.items():
        assert kv_layout.head_group(G, d) == Gg, (G, d)
        assert G % Gg == 0 and Gg * 16 * d * 2 <= 32768
