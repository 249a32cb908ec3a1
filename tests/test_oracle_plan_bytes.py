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

def _hand_trace(on_host, n_steps, depth, clamp=True):
    """A correct trace written independently of the library: copies run
    `depth` ahead, each released buffer is refilled at once."""
    C, A, T, R = pipeline_sim.COPY, pipeline_sim.APPEND, pipeline_sim.ATTN, pipeline_sim.RELEASE
    hl = [l for l, v in enumerate(on_host) if v]
    k = len(hl)
    tr = []
    if k == 0:
        for s in range(n_steps):
            for l in range(len(on_host)):
                tr += [(A, s, l, -1, -1, -1), (T, s, l, -1, -1, -1)]
        return tr
    if clamp:
        depth = min(depth, k)
    for j in range(depth):
        tr.append((C, j // k, hl[j % k], j % depth, j, -1))
    j = 0
    for s in range(n_steps):
        for l in range(len(on_host)):
            if not on_host[l]:
                tr += [(A, s, l, -1, -1, -1), (T, s, l, -1, -1, -1)]
                continue
            buf = j % depth
            tr += [(A, s, l, buf, -1, j), (T, s, l, buf, -1, -1), (R, s, l, buf, j, -1)]
            nj = j + depth
            tr.append((C, nj // k, hl[nj % k], buf, nj, j))
            j += 1
    return tr


@pytest.mark.parametrize("on_host", [[0, 1, 0, 1], [1, 1, 1], [0, 0, 1], [1], [0, 0], [1, 0, 1, 1, 0, 1]])
@pytest.mark.parametrize("depth", [1, 2])
def test_replay_accepts_a_correct_trace(on_host, depth):
    tr = _hand_trace(on_host, 4, depth)
    for seed in range(10):
        for cs, ks in ((1.0, 1.0), (20.0, 0.05), (0.05, 20.0)):
            pipeline_sim.replay(tr, on_host, seed=seed, copy_scale=cs, compute_scale=ks)


def test_replay_catches_planted_mistakes():
    C, A = pipeline_sim.COPY, pipeline_sim.APPEND
    on_host = [0, 1, 0, 1, 1]
    good = _hand_trace(on_host, 4, 2)

    def fails(trace):
        hit = 0
        for seed in range(20):
            for cs, ks in ((1.0, 1.0), (20.0, 0.05), (0.05, 20.0)):
                try:
                    pipeline_sim.replay(trace, on_host, seed=seed, copy_scale=cs, compute_scale=ks)
                except pipeline_sim.Hazard:
                    hit += 1
        return hit > 0

    assert not fails(good)
    # 1. a copy that does not wait for its buffer to be released
    bad = [(k, s, l, b, c, -1) if (k == C and c == 5) else (k, s, l, b, c, w) for (k, s, l, b, c, w) in good]
    assert fails(bad)
    # 2. an append that does not wait for its copy
    first = next(i for i, op in enumerate(good) if op[0] == A and op[5] >= 0)
    bad = list(good)
    k, s, l, b, c, w = bad[first]
    bad[first] = (k, s, l, b, c, -1)
    assert fails(bad)
    # 3. the copy goes to the other buffer
    bad = [(k, s, l, 1 - b, c, w) if (k == C and c == 3) else (k, s, l, b, c, w) for (k, s, l, b, c, w) in good]
    assert fails(bad)
    # 4. the copy fetches the wrong layer
    bad = [(k, s, 1 if l == 3 else 3, b, c, w) if (k == C and c == 4) else (k, s, l, b, c, w)
           for (k, s, l, b, c, w) in good]
    assert fails(bad)
    # 5. a copy issued before the release it waits on
    idx = next(i for i, op in enumerate(good) if op[0] == C and op[5] >= 0)
    bad = list(good)
    op = bad.pop(idx)
    bad.insert(idx - 3, op)
    assert fails(bad)
    # 6. with a single host layer, running two copies ahead reads the host
    #    pool before the previous step's append has landed
    one = [0, 1, 0]
    for seed in range(5):
        pipeline_sim.replay(_hand_trace(one, 4, 2), one, seed=seed, copy_scale=0.05, compute_scale=20.0)
    with pytest.raises(pipeline_sim.Hazard):
        pipeline_sim.replay(_hand_trace(one, 4, 2, clamp=False), one, seed=0,
                            copy_scale=0.05, compute_scale=20.0)


def test_overlap_keeps_the_copy_stream_busy():
    # When copies dominate, a depth-2 pipeline leaves (almost) no gap on the copy stream.
    on_host = [0, 1] * 4
    tr = _hand_trace(on_host, 6, 2)
    r = pipeline_sim.replay(tr, on_host, seed=0, copy_scale=50.0, compute_scale=0.05)
    assert r["copy_busy"] / r["copy_span"] > 0.98
    tr1 = _hand_trace(on_host, 6, 1)
    r1 = pipeline_sim.replay(tr1, on_host, seed=0, copy_scale=50.0, compute_scale=0.05)
    assert r1["copy_busy"] / r1["copy_span"] <= r["copy_busy"] / r["copy_span"]
