"""Pins for the integer / scalar oracles: offload plan, byte and flop
formulas, work-list tiling, and the pipeline replay.  CPU only."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import kv_bytes, offload_plan, pipeline_sim, worklist

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---- offload plan -----------------------------------------------------------

def test_plan_counts_and_edges():
    assert offload_plan.plan_layers(32, Fraction(1, 2)) == ([0, 1] * 16, 16)
    on, k = offload_plan.plan_layers(32, Fraction(3, 5))
    assert k == 20 and sum(on) == 20                       # ceil(19.2)
    assert offload_plan.plan_layers(32, 0) == ([0] * 32, 0)
    assert offload_plan.plan_layers(32, 1) == ([1] * 32, 32)   # the C_off = 100 % run of Table VI
    assert offload_plan.plan_layers(1, Fraction(1, 1000)) == ([1], 1)
    assert offload_plan.n_offloaded(10, Fraction(3, 10)) == 3   # exact multiple: no round-up
    assert offload_plan.n_offloaded(10, Fraction(31, 100)) == 4
    with pytest.raises(ValueError):
        offload_plan.n_offloaded(4, Fraction(5, 4))


def test_plan_is_smallest_sufficient_and_evenly_spread():
    for L in range(1, 41):
        for den in range(1, 17):
            for num in range(0, den + 1):
                c = Fraction(num, den)
                on, k = offload_plan.plan_layers(L, c)
                assert len(on) == L and set(on) <= {0, 1} and sum(on) == k
                assert Fraction(k, L) >= c                        # enough leaves the GPU
                assert k == 0 or Fraction(k - 1, L) < c           # and not one layer more
                pos = [i for i, v in enumerate(on) if v]
                if k >= 2:
                    gaps = [b - a for a, b in zip(pos, pos[1:])] + [pos[0] + L - pos[-1]]
                    assert max(gaps) - min(gaps) <= 1             # cyclic gaps differ by <= 1
                if k >= 1:
                    assert on[L - 1] == 1                         # quota completes on the last layer


def test_plan_from_bytes_cases():
    LB = 1000
    # Case 1: everything fits
    assert offload_plan.plan_from_bytes(8, LB, 8 * LB) == ("resident", [0] * 8, 0, 0)
    # Case 2: not one layer fits
    assert offload_plan.plan_from_bytes(8, LB, LB - 1)[0] == "infeasible"
    # Case 3 with room for two staging buffers: 5 layers fit -> 3 resident
    st, on, k, ns = offload_plan.plan_from_bytes(8, LB, 5 * LB + 999)
    assert (st, k, ns, sum(on)) == ("offload", 5, 2, 5)
    # only one layer fits: everything on host, single staging buffer
    st, on, k, ns = offload_plan.plan_from_bytes(8, LB, LB)
    assert (st, k, ns, on) == ("offload", 8, 1, [1] * 8)
    for L in (2, 7, 32):
        for avail in range(LB, L * LB, 137):
            st, on, k, ns = offload_plan.plan_from_bytes(L, LB, avail)
            assert st == "offload"
            assert (L - k + ns) * LB <= avail                     # resident + staging fits
            c_paper = offload_plan.c_off_case3(avail, L * LB)     # the paper's minimum share
            assert Fraction(k, L) >= c_paper


# ---- byte / flop formulas ---------------------------------------------------

def test_kv_bytes_formulas():
    # shapes of the workloads: 32 heads x 128, fp16 -> 16 KiB per token per layer
    assert kv_bytes.kv_bytes_per_token_per_layer(32, 128) == 16384
    assert kv_bytes.kv_bytes_per_token_per_layer(8, 128) == 4096
    assert kv_bytes.mem_kvcache(64, 2048, 0, 4096, 32) == 64 * 2 ** 30
    assert kv_bytes.mem_kvcache_per_layer(64, 2048, 0, 4096, 32) == 2 * 2 ** 30
    assert kv_bytes.kv_bytes_step([2048] * 64, 32, 128) == 2 * 2 ** 30
    # MHA: the step formula and the table formula agree when G*d = h1
    assert kv_bytes.kv_bytes_step([100, 28], 4, 16) == kv_bytes.mem_kvcache(1, 128, 0, 64, 1)
    # flops: paper's average-context form equals the mean of the per-step counts
    BS, L_in, L_out, H, d = 3, 10, 8, 4, 16
    per_step = [kv_bytes.decode_attention_flops_step([L_in + s] * BS, H, d) for s in range(1, L_out)]
    # steps attend L_in+1 .. L_in+L_out-1 keys: mean context L_in + L_out/2
    assert Fraction(sum(per_step), len(per_step)) == kv_bytes.decode_attention_flops_per_layer(
        BS, L_in, L_out, H * d)
    # one flop per fp16 KV byte for MHA
    assert kv_bytes.decode_attention_flops_step([77], 32, 128) == kv_bytes.kv_bytes_step([77], 32, 128)


def test_paper_offline_runs_are_transfer_bound_as_the_formulas_say():
    """The printed decode transfer time x layers x (L_out - 1) steps lands within
    20 % of the run time implied by the measured TPS of the two offloaded runs."""
    with open(os.path.join(GOLDEN, "paper_offline_runs.json")) as f:
        g = json.load(f)
    m, w = g["model"], g["workload"]
    for run in g["runs"]:
        c_off = Fraction(*run["c_off"])
        t_dec = kv_bytes.t_trans_decode(c_off, w["L_in"], w["L_out"], m["h1"], w["BS"],
                                        run["pcie_GBps"] * 10 ** 9, m["prec_bytes"])
        t_model = kv_bytes.t_task(0, t_dec, m["layers"], w["L_out"])
        t_meas = w["BS"] * (w["L_in"] + w["L_out"]) / run["tps_measured"]
        assert abs(float(t_model) / t_meas - 1) < 0.20, (run["instance"], float(t_model), t_meas)
        assert abs(float(kv_bytes.tps(w["BS"], w["L_in"], w["L_out"], Fraction(t_meas))) /
                   run["tps_measured"] - 1) < 1e-12
    ex = g["kv_size_example"]            # the printed example scales linearly with batch
    assert abs(ex["GB_at_BS32"] / ex["GB_at_BS2"] - 16) < 1e-9
    assert kv_bytes.mem_kvcache(32, 1024, 0, 2560, 32) == 16 * kv_bytes.mem_kvcache(2, 1024, 0, 2560, 32)


# ---- work list ----------------------------------------------------------------

def test_worklist_expected_items_tile_exactly():
    rng = np.random.default_rng(3)
    for _ in range(200):
        B = int(rng.integers(1, 6))
        ctx = rng.integers(0, 700, size=B)
        S = int(rng.integers(1, 400))
        items = worklist.expected_items(ctx, S)
        assert worklist.check_tiling(items, ctx)
        for b, n in enumerate(ctx):
            mine = [(lo, hi) for bb, lo, hi in items if bb == b]
            if n == 0:
                assert not mine
                continue
            assert all(lo % 16 == 0 for lo, _ in mine)                 # items start on tile boundaries
            sizes = [hi - lo for lo, hi in mine]
            assert max(sizes) <= max(S, 16) + 15                        # at most S, up to the rounding
            assert len(set(sizes[:-1])) <= 1                            # equal pieces, last one shorter
            assert len(mine) <= -(-int(n) // S)                         # never more items than ceil(n / S)
    # hand cases: 1100 keys, S = 1024 -> two pieces of 560 (not 1024 + 76)
    assert worklist.expected_items([1100], 1024) == [(0, 0, 560), (0, 560, 1100)]
    assert worklist.expected_items([17], 8) == [(0, 0, 16), (0, 16, 17)]
    assert worklist.expected_items([1024, 513], 1024) == [(0, 0, 1024), (1, 0, 513)]
    assert worklist.expected_items([5, 0, 3], 2) == [(0, 0, 5), (2, 0, 3)]


def test_worklist_checker_rejects_bad_tilings():
    ctx = [40, 20]
    good = worklist.expected_items(ctx, 16)
    assert worklist.check_tiling(good, ctx) and len(good) == 5
    assert not worklist.check_tiling(good[:-1], ctx)                  # a gap
    assert not worklist.check_tiling(good + [(1, 0, 1)], ctx)         # an overlap
    assert not worklist.check_tiling(good[:-1] + [(1, 16, 24)], ctx)  # beyond the context
    assert not worklist.check_tiling([(2, 0, 1)] + good, ctx)         # unknown sequence


# ---- pipeline replay ------------------------------------------------------------

def _hand_trace(host_chunks, n_steps, depth, clamp=True, has_resident=None):
    """A correct trace written independently of the library: copies run
    `depth` ahead, each released buffer is refilled at once.  host_chunks[l] is
    the number of streamed chunks of layer l."""
    C, A, T, R, M = (pipeline_sim.COPY, pipeline_sim.APPEND, pipeline_sim.ATTN, pipeline_sim.RELEASE,
                     pipeline_sim.MERGE)
    L = len(host_chunks)
    if has_resident is None:
        has_resident = [1 if host_chunks[l] == 0 else 0 for l in range(L)]
    units = [(l, c) for l in range(L) for c in range(host_chunks[l])]
    k = len(units)
    tr = []
    if k and clamp:
        depth = min(depth, k)
    if k:
        for j in range(depth):
            tr.append((C, j // k, units[j % k][0], units[j % k][1], j % depth, j, -1))
    j = 0
    for s in range(n_steps):
        for l in range(L):
            tr.append((A, s, l, -1, -1, -1, -1))
            if has_resident[l]:
                tr.append((T, s, l, -1, -1, -1, -1))
            for c in range(host_chunks[l]):
                buf = j % depth
                tr += [(T, s, l, c, buf, j, j), (R, s, l, c, buf, j, -1)]
                nj = j + depth
                tr.append((C, nj // k, units[nj % k][0], units[nj % k][1], buf, nj, j))
                j += 1
            tr.append((M, s, l, -1, -1, -1, -1))
    return tr


@pytest.mark.parametrize("on_host", [[0, 1, 0, 1], [1, 1, 1], [0, 0, 1], [1], [0, 0], [1, 0, 1, 1, 0, 1]])
@pytest.mark.parametrize("depth", [1, 2, 3])
def test_replay_accepts_a_correct_trace(on_host, depth):
    tr = _hand_trace(on_host, 4, depth)
    for seed in range(10):
        for cs, ks in ((1.0, 1.0), (20.0, 0.05), (0.05, 20.0)):
            pipeline_sim.replay(tr, on_host, seed=seed, copy_scale=cs, compute_scale=ks)


@pytest.mark.parametrize("chunks,resident", [([3, 3, 3], [1, 1, 1]), ([2, 2], [0, 0]), ([1, 4, 0, 2], [1, 0, 1, 1]),
                                             ([5], [1])])
@pytest.mark.parametrize("depth", [1, 2, 4])
def test_replay_accepts_a_correct_chunked_trace(chunks, resident, depth):
    tr = _hand_trace(chunks, 4, depth, has_resident=resident)
    for seed in range(6):
        for cs, ks in ((1.0, 1.0), (20.0, 0.05), (0.05, 20.0)):
            pipeline_sim.replay(tr, chunks, resident, seed=seed, copy_scale=cs, compute_scale=ks)


def _fails(trace, chunks, resident=None):
    hit = 0
    for seed in range(20):
        for cs, ks in ((1.0, 1.0), (20.0, 0.05), (0.05, 20.0)):
            try:
                pipeline_sim.replay(trace, chunks, resident, seed=seed, copy_scale=cs, compute_scale=ks)
            except pipeline_sim.Hazard:
                hit += 1
    return hit > 0


def test_replay_catches_planted_mistakes():
    C, T = pipeline_sim.COPY, pipeline_sim.ATTN
    on_host = [0, 1, 0, 1, 1]
    good = _hand_trace(on_host, 4, 2)
    assert not _fails(good, on_host)
    # 1. a copy that does not wait for its buffer to be released
    bad = [(k, s, l, ch, b, c, -1) if (k == C and c == 5) else (k, s, l, ch, b, c, w)
           for (k, s, l, ch, b, c, w) in good]
    assert _fails(bad, on_host)
    # 2. an attention that does not wait for its copy
    first = next(i for i, op in enumerate(good) if op[0] == T and op[6] >= 0)
    bad = list(good)
    k, s, l, ch, b, c, w = bad[first]
    bad[first] = (k, s, l, ch, b, c, -1)
    assert _fails(bad, on_host)
    # 2b. ... or waits for the copy before the one it reads
    later = [i for i, op in enumerate(good) if op[0] == T and op[6] >= 2][0]
    bad = list(good)
    k, s, l, ch, b, c, w = bad[later]
    bad[later] = (k, s, l, ch, b, c, w - 2)
    assert _fails(bad, on_host)
    # 3. the copy goes to the other buffer
    bad = [(k, s, l, ch, 1 - b, c, w) if (k == C and c == 3) else (k, s, l, ch, b, c, w)
           for (k, s, l, ch, b, c, w) in good]
    assert _fails(bad, on_host)
    # 4. the copy fetches the wrong layer
    bad = [(k, s, 1 if l == 3 else 3, ch, b, c, w) if (k == C and c == 4) else (k, s, l, ch, b, c, w)
           for (k, s, l, ch, b, c, w) in good]
    assert _fails(bad, on_host)
    # 5. a copy issued before the release it waits on
    idx = next(i for i, op in enumerate(good) if op[0] == C and op[6] >= 0)
    bad = list(good)
    op = bad.pop(idx)
    bad.insert(idx - 2, op)
    assert _fails(bad, on_host)
    # 6. with a single host layer, running two copies ahead reads the host
    #    pool before the previous step's rows have landed
    one = [0, 1, 0]
    for seed in range(5):
        pipeline_sim.replay(_hand_trace(one, 4, 2), one, seed=seed, copy_scale=0.05, compute_scale=20.0)
    with pytest.raises(pipeline_sim.Hazard):
        pipeline_sim.replay(_hand_trace(one, 4, 2, clamp=False), one, seed=0,
                            copy_scale=0.05, compute_scale=20.0)


def test_replay_catches_planted_mistakes_in_chunked_traces():
    C, T, M = pipeline_sim.COPY, pipeline_sim.ATTN, pipeline_sim.MERGE
    chunks, resident = [3, 3], [1, 1]
    good = _hand_trace(chunks, 3, 2, has_resident=resident)
    assert not _fails(good, chunks, resident)
    # the copy fetches the wrong chunk of the right layer
    bad = [(k, s, l, (ch + 1) % 3, b, c, w) if (k == C and c == 4) else (k, s, l, ch, b, c, w)
           for (k, s, l, ch, b, c, w) in good]
    assert _fails(bad, chunks, resident)
    # a chunk is never attended
    victim = next(i for i, op in enumerate(good) if op[0] == T and op[3] == 1)
    assert _fails(good[:victim] + good[victim + 1:], chunks, resident)
    # the keys that stay in HBM are never attended
    victim = next(i for i, op in enumerate(good) if op[0] == T and op[3] == -1)
    assert _fails(good[:victim] + good[victim + 1:], chunks, resident)
    # the merge runs before the layer's last chunk
    m = next(i for i, op in enumerate(good) if op[0] == M)
    bad = list(good)
    op = bad.pop(m)
    bad.insert(m - 4, op)
    assert _fails(bad, chunks, resident)
    # a chunk is attended twice in one step
    t = next(i for i, op in enumerate(good) if op[0] == T and op[3] == 2)
    assert _fails(good[:t + 1] + [good[t]] + good[t + 1:], chunks, resident)
    # one layer with two chunks and three copies in flight: the third copy re-reads chunk 0
    # of the host pool before the rows of the step before have landed
    one = [2]
    assert not _fails(_hand_trace(one, 4, 2, has_resident=[1]), one, [1])
    with pytest.raises(pipeline_sim.Hazard):
        pipeline_sim.replay(_hand_trace(one, 4, 3, clamp=False, has_resident=[1]), one, [1], seed=0,
                            copy_scale=0.05, compute_scale=20.0)


def test_overlap_keeps_the_copy_stream_busy():
    # When copies dominate, a depth-2 pipeline leaves (almost) no gap on the copy engine.
    on_host = [0, 1] * 4
    tr = _hand_trace(on_host, 6, 2)
    r = pipeline_sim.replay(tr, on_host, seed=0, copy_scale=50.0, compute_scale=0.05)
    assert r["copy_busy"] / r["copy_span"] > 0.98
    tr1 = _hand_trace(on_host, 6, 1)
    r1 = pipeline_sim.replay(tr1, on_host, seed=0, copy_scale=50.0, compute_scale=0.05)
    assert r1["copy_busy"] / r1["copy_span"] <= r["copy_busy"] / r["copy_span"]


# ---- block-granular split of the cache and its work list -------------------------

def test_block_split_counts():
    assert offload_plan.block_split(100, Fraction(0)) == (100, 0)
    assert offload_plan.block_split(100, Fraction(1)) == (0, 100)
    assert offload_plan.block_split(100, Fraction(1, 3)) == (66, 34)      # 33.3 -> 34 leave
    assert offload_plan.block_split(7, Fraction(1, 7)) == (6, 1)
    for n in (1, 5, 64, 1000):
        for num in range(0, 11):
            c = Fraction(num, 10)
            res, host = offload_plan.block_split(n, c)
            assert res + host == n and host >= c * n and (host == 0 or host - 1 < c * n)


def test_host_blocks_per_sequence_shares():
    rng = np.random.default_rng(5)
    for _ in range(50):
        nb = [int(x) for x in rng.integers(0, 40, size=int(rng.integers(1, 12)))]
        total = sum(nb)
        for n_host in {0, total, total // 2, total // 3}:
            h = offload_plan.host_blocks_per_sequence(nb, n_host)
            assert sum(h) == n_host
            for hb, n in zip(h, nb):
                assert 0 <= hb <= n
                if total:                                   # each share within one block of its quota
                    assert abs(hb - Fraction(n * n_host, total)) < 1 + 1e-9 or hb in (0, n)
    assert offload_plan.host_blocks_per_sequence([4, 4, 4, 4], 8) == [2, 2, 2, 2]
    assert offload_plan.host_blocks_per_sequence([10, 0, 10], 20) == [10, 0, 10]


def _random_table(rng, ctx_lens, T, n_total):
    ids = rng.permutation(n_total)
    table, at = [], 0
    width = max(-(-int(n) // T) for n in ctx_lens) + 1
    for n in ctx_lens:
        nb = -(-int(n) // T)
        row = [int(x) for x in ids[at:at + nb]] + [-1] * (width - nb)
        at += nb
        table.append(row)
    return table


def test_items_by_class_hand_case():
    # T = 16, blocks 0..1 in HBM, host chunks of 2 blocks: ids 2,3 -> class 1, ids 4,5 -> class 2
    table = [[4, 5, 0, 2], [1, 3, -1, -1]]
    lens = [55, 20]
    got = worklist.expected_items_by_class(lens, table, 16, 2, 2, 1 << 20, 3)
    assert got[0] == [(0, 32, 48), (1, 0, 16)]
    assert got[1] == [(0, 48, 55), (1, 16, 20)]
    assert got[2] == [(0, 0, 32)]
    # a split size of 16 cuts the two-block run in two
    got = worklist.expected_items_by_class(lens, table, 16, 2, 2, 16, 3)
    assert got[2] == [(0, 0, 16), (0, 16, 32)]


def test_items_by_class_tile_and_stay_in_class():
    rng = np.random.default_rng(11)
    for trial in range(30):
        T = int(rng.choice([16, 32, 64]))
        B = int(rng.integers(1, 6))
        lens = [int(x) for x in rng.integers(0, 400, size=B)]
        if max(lens) == 0:
            lens[0] = 7
        need = sum(-(-n // T) for n in lens)
        n_total = need + int(rng.integers(0, 5))
        R = int(rng.integers(0, n_total + 1))
        CB = int(rng.integers(1, 6))
        n_cls = 1 + -(-(n_total - R) // CB) if n_total > R else 1
        table = _random_table(rng, lens, T, n_total)
        S = int(rng.choice([16, 48, 128, 4096]))
        per = worklist.expected_items_by_class(lens, table, T, R, CB, S, n_cls)
        flat = [it for items in per for it in items]
        assert worklist.check_tiling(flat, lens)
        assert worklist.check_classes(per, table, T, R, CB)
        for items in per:
            assert items == sorted(items)                      # by sequence, then position
            for (b, lo, hi) in items:
                assert lo % 16 == 0 and hi - lo <= max(16, -(-S // 16) * 16)
        # planted: an item moved to a neighbouring class is noticed
        donor = next((c for c, items in enumerate(per) if items), None)
        if donor is not None and n_cls > 1:
            wrong = [list(items) for items in per]
            it = wrong[donor].pop()
            wrong[(donor + 1) % n_cls].append(it)
            assert not worklist.check_classes(wrong, table, T, R, CB)


def test_items_by_class_reduces_to_the_plain_list():
    # everything in HBM (or everything in one chunk): one run per sequence = the unsplit-cache list
    lens = [1, 16, 17, 300, 0, 1025]
    T = 16
    table = _random_table(np.random.default_rng(2), lens, T, 200)
    for S in (16, 100, 256, 4096):
        plain = worklist.expected_items(lens, S)
        assert worklist.expected_items_by_class(lens, table, T, 200, 8, S, 1)[0] == plain
        assert worklist.expected_items_by_class(lens, table, T, 0, 200, S, 2) == [[], plain]


# ---- equal stretches (the work list when no split size is fixed) ---------------------------------

def test_equal_stretches_hand_cases():
    # one sequence of 40 tiles, 4 wavefronts per KV head: four stretches of 10 tiles = 160 keys
    items, first, span = worklist.expected_items_equal_stretches([640], 4)
    assert span == 10 and first == [0, 1, 2, 3, 4]
    assert items == [(0, 0, 160), (0, 160, 320), (0, 320, 480), (0, 480, 640)]
    # two sequences of 24 and 8 tiles, 2 stretches of 16 tiles: the first sequence is cut, the second shares a stretch
    items, first, span = worklist.expected_items_equal_stretches([384, 120], 2)
    assert span == 16 and items == [(0, 0, 256), (0, 256, 384), (1, 0, 120)] and first == [0, 1, 3]
    # a short batch is not cut below 8 tiles a stretch: 20 tiles -> 2 stretches although 64 are allowed
    items, first, span = worklist.expected_items_equal_stretches([100, 100, 100], 64)
    assert span == 11 and len(first) == 3
    assert items == [(0, 0, 100), (1, 0, 64), (1, 64, 100), (2, 0, 100)]
    # empty sequences contribute nothing; fewer than 8 tiles in all: one stretch
    items, first, span = worklist.expected_items_equal_stretches([0, 5, 0, 33], 8)
    assert items == [(1, 0, 5), (3, 0, 33)] and first == [0, 2] and span == 4


def test_equal_stretches_tile_exactly_and_evenly():
    rng = np.random.default_rng(7)
    for case in range(60):
        B = int(rng.integers(1, 40))
        lens = rng.integers(0, 3000, size=B)
        if case % 7 == 0:
            lens[:] = int(rng.integers(1, 2000))             # a batch of equal sequences
        G = int(rng.choice([1, 2, 8, 32]))
        max_groups = max(1, 1024 // G)
        items, first, span = worklist.expected_items_equal_stretches(lens, max_groups)
        assert worklist.check_tiling(items, lens)
        assert len(first) - 1 <= max_groups and first[0] == 0 and first[-1] == len(items)
        assert all(a < b for a, b in zip(first, first[1:]))   # every stretch in use opens with an item
        assert all(lo % 16 == 0 for (_, lo, _) in items)
        tiles = [sum(-(-(hi - lo) // 16) for (_, lo, hi) in items[a:b]) for a, b in zip(first, first[1:])]
        if tiles:
            assert all(t == span for t in tiles[:-1]) and 1 <= tiles[-1] <= span
        total = sum(-(-int(n) // 16) for n in lens)
        assert sum(tiles) == total
        if total >= 16:
            assert span >= 8                                   # no stretch shorter than 8 tiles unless the batch is
        # a sequence is cut only where a stretch ends: at most one item per sequence and stretch
        assert len(items) <= int((lens > 0).sum()) + len(first) - 2 + 1
