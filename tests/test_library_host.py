"""The C-ABI library without a GPU: it loads, exports what the header declares,
and its pure host functions (offload plan, pipeline schedule) agree with the
oracle.  No compute call is made here."""
import os
import re
from fractions import Fraction

import numpy as np
import pytest

from oracle import offload_plan, pipeline_sim
from paper_2504_11816_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "okv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*\(", text)
    return sorted({n for n in names if n.startswith("okv_") or n in ("kv_append", "kv_append_bulk", "decode_attn", "kv_offload_plan")})


def test_library_loads_and_exports_every_declared_symbol():
    lib = binding.lib()
    decl = declared_functions()
    assert len(decl) >= 20
    for name in decl:
        assert hasattr(lib, name), f"{name} is declared in okv.h but not exported"
    assert sorted(binding.EXPORTS) == decl


def test_layer_header_symbols_are_exported():
    text = open(os.path.join(ROOT, "include", "okv_layer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    decl = sorted(set(re.findall(r"\b(okv_[a-z_0-9]+)\s*\(", text)))
    lib = binding.lib()
    for name in decl:
        assert hasattr(lib, name), name
    assert decl == sorted(binding.LAYER_EXPORTS)
    # argument checks need no GPU
    for bad in (dict(m=0), dict(m=4097), dict(n_out=24), dict(n_in=48), dict(n_seg=4), dict(n_seg=3, n_out=64)):
        kw = dict(m=4, n_out=96, n_in=64, n_seg=1)
        kw.update(bad)
        with pytest.raises(binding.OkvError) as e:
            binding.okv_linear(16, 16, None, None, [16] * kw["n_seg"], kw["m"], kw["n_out"], kw["n_in"])
        if "n_seg" not in bad:
            with pytest.raises(binding.OkvError):
                binding.okv_linear_workspace_bytes(kw["m"], kw["n_out"], kw["n_in"])
        assert e.value.code == binding.OKV_EINVAL
    with pytest.raises(binding.OkvError):
        binding.okv_layernorm(16, 16, 16, 16, 4, 100)           # h not a multiple of 8
    with pytest.raises(binding.OkvError):
        binding.okv_pack_linear_weight(16, 32, 100, 64)         # n_out not a multiple of 16


def test_cuts_of_the_product_kernels_follow_the_launch_model():
    # okv_linear_workspace_bytes = cuts * m * n_out * 4 (0: the kernel for few rows or odd input sizes); without a
    # GPU the library assumes the 256 compute units of the GPU it is written for
    def cuts(m, n_out, n_in):
        nbytes = binding.okv_linear_workspace_bytes(m, n_out, n_in)
        assert nbytes % (m * n_out * 4) == 0
        return nbytes // (m * n_out * 4)
    assert cuts(32, 12288, 4096) == 1          # 256 workgroups of three 16-feature tiles: no second kernel
    assert cuts(32, 16384, 4096) == 1          # 256 workgroups of four
    assert cuts(32, 4096, 4096) == 4           # 64 groups of four tiles, four cuts: 256 workgroups
    assert cuts(32, 4096, 16384) == 4
    assert cuts(32, 6144, 4096) == 2           # 128 groups of three tiles, two cuts
    assert cuts(128, 6144, 4096) == 2
    assert cuts(8, 4096, 4096) == 0            # up to 8 rows: the kernel that needs no workspace
    assert cuts(32, 4096, 4000) == 0           # inputs not a multiple of 256
    assert cuts(128, 4096, 4096 + 128) == 0    # from 112 rows on the kernel takes two 128-input chunks at a time
    for m in (9, 33, 65, 97, 128):
        for n_out, n_in in ((16, 256), (48, 512), (2560, 2560), (5120, 13824), (28672, 8192)):
            c = cuts(m, n_out, n_in)
            chunk = 256 if m <= 96 else 128
            assert c >= 1 and (n_in // chunk) % c == 0 and (c == 1 or n_in // chunk // c >= 2)


def test_plan_matches_oracle_brute_force():
    for L in range(1, 65):
        for den in range(1, 33):
            for num in range(0, den + 1):
                on, k = binding.kv_offload_plan(L, num, den)
                want, wk = offload_plan.plan_layers(L, Fraction(num, den))
                assert k == wk and on.tolist() == want, (L, num, den)
    for L in (1, 7, 32, 64):
        for den in (33, 47, 64):
            for num in range(0, den + 1):
                on, k = binding.kv_offload_plan(L, num, den)
                want, wk = offload_plan.plan_layers(L, Fraction(num, den))
                assert k == wk and on.tolist() == want, (L, num, den)


def test_plan_with_byte_sized_ratio_and_errors():
    # C_off given as bytes: 1 - avail / total for a 64 GiB cache with 37 GiB available
    total, avail = 64 << 30, 37 << 30
    on, k = binding.kv_offload_plan(32, total - avail, total)
    want, wk = offload_plan.plan_layers(32, offload_plan.c_off_case3(avail, total))
    assert (on.tolist(), k) == (want, wk)
    for bad in ((0, 1, 2), (4, -1, 2), (4, 3, 2), (4, 1, 0)):
        with pytest.raises(binding.OkvError) as e:
            binding.kv_offload_plan(*bad)
        assert e.value.code == binding.OKV_EINVAL


def test_plan_from_bytes_matches_oracle():
    LB = 4096
    for L in (1, 2, 5, 32):
        for avail in list(range(0, (L + 2) * LB, 509)) + [LB, 2 * LB, L * LB, L * LB - 1]:
            st, on, k, ns = offload_plan.plan_from_bytes(L, LB, avail)
            if st == "infeasible":
                with pytest.raises(binding.OkvError) as e:
                    binding.okv_plan_from_bytes(L, LB, avail)
                assert e.value.code == binding.OKV_ENOSPC
            else:
                got_on, got_k, got_ns = binding.okv_plan_from_bytes(L, LB, avail)
                assert (got_on.tolist(), got_k, got_ns) == (on, k, ns), (L, avail)


@pytest.mark.parametrize("on_host", [[0, 1, 0, 1], [1, 1, 1], [0, 0, 1], [1], [0, 0], [1, 0, 1, 1, 0, 1],
                                     [0, 1] * 16, [1] * 32])
@pytest.mark.parametrize("n_staging", [1, 2, 4])
def test_schedule_trace_replays_without_hazard(on_host, n_staging):
    trace = binding.okv_schedule_trace(on_host, n_staging, 5)
    for seed in range(6):
        for cs, ks in ((1.0, 1.0), (25.0, 0.04), (0.04, 25.0)):
            pipeline_sim.replay(trace, on_host, seed=seed, copy_scale=cs, compute_scale=ks)
    k = sum(on_host)
    copies = [op for op in trace if op[0] == pipeline_sim.COPY]
    if k:
        depth = min(n_staging, k)
        assert len(copies) == 5 * k + depth            # every consumption refills, `depth` run ahead
        assert [c[5] for c in copies] == list(range(len(copies)))
        hl = [l for l, v in enumerate(on_host) if v]
        assert all(c[2] == hl[c[5] % k] and c[3] == 0 and c[4] == c[5] % depth for c in copies)
    else:
        assert not copies


@pytest.mark.parametrize("chunks,resident", [([3, 3, 3], [1, 1, 1]), ([2, 2], [0, 0]), ([1, 4, 0, 2], [1, 0, 1, 1]),
                                             ([5], [1]), ([8] * 32, [1] * 32), ([1], [1])])
@pytest.mark.parametrize("n_staging", [1, 2, 3, 4])
def test_chunked_schedule_trace_replays_without_hazard(chunks, resident, n_staging):
    n_steps = 4
    trace = binding.okv_schedule_trace(chunks, n_staging, n_steps, has_resident=resident)
    for seed in range(4):
        for cs, ks in ((1.0, 1.0), (25.0, 0.04), (0.04, 25.0)):
            pipeline_sim.replay(trace, chunks, resident, seed=seed, copy_scale=cs, compute_scale=ks)
    k = sum(chunks)
    depth = min(n_staging, k)
    copies = [op for op in trace if op[0] == pipeline_sim.COPY]
    assert len(copies) == n_steps * k + depth
    units = [(l, c) for l in range(len(chunks)) for c in range(chunks[l])]
    assert all((c[2], c[3]) == units[c[5] % k] and c[4] == c[5] % depth for c in copies)
    attn = [op for op in trace if op[0] == pipeline_sim.ATTN]
    assert len(attn) == n_steps * (k + sum(resident))


def test_schedule_keeps_the_link_busy_when_copies_dominate():
    on_host = [0, 1] * 16
    trace = binding.okv_schedule_trace(on_host, 2, 6)
    r = pipeline_sim.replay(trace, on_host, seed=0, copy_scale=60.0, compute_scale=0.05)
    assert r["copy_busy"] / r["copy_span"] > 0.99
    chunks = [6] * 8
    trace = binding.okv_schedule_trace(chunks, 2, 6, has_resident=[1] * 8)
    r = pipeline_sim.replay(trace, chunks, [1] * 8, seed=0, copy_scale=60.0, compute_scale=0.05)
    assert r["copy_busy"] / r["copy_span"] > 0.99


def test_schedule_trace_argument_errors():
    with pytest.raises(binding.OkvError):
        binding.okv_schedule_trace([0, 1], 0, 2)          # host layer but no staging buffer
    assert binding.okv_schedule_trace([0, 0], 0, 2)       # fine without host layers
    with pytest.raises(binding.OkvError):
        binding.okv_schedule_trace([0, -1], 2, 2)
    with pytest.raises(binding.OkvError):
        binding.okv_schedule_trace([0, 2], 2, 2, has_resident=[0, 0])   # layer 0 would hold nothing


def test_block_split_matches_oracle():
    for n in list(range(0, 40)) + [1000, 12288, (1 << 31) - 1]:
        for den in (1, 2, 3, 7, 10, 64):
            for num in range(0, den + 1):
                want = offload_plan.block_split(n, Fraction(num, den))
                assert binding.okv_plan_block_split(n, num, den) == want, (n, num, den)
    for bad in ((-1, 1, 2), (4, -1, 2), (4, 3, 2), (4, 1, 0)):
        with pytest.raises(binding.OkvError):
            binding.okv_plan_block_split(*bad)


def test_size_queries_and_shape_errors():
    cfg = binding.make_config(n_layers=32, n_q_heads=32, n_kv_heads=32, head_dim=128, block_tokens=16,
                              max_batch=64, max_blocks_per_seq=128, blocks_per_layer=8192)
    assert binding.okv_layer_pool_bytes(cfg) == 2 << 30            # 2 GiB per layer (Table II per-layer size)
    cfg = binding.make_config(n_layers=32, n_q_heads=32, n_kv_heads=32, head_dim=128, block_tokens=0,
                              max_batch=32, max_ctx=1024)
    assert binding.okv_layer_pool_bytes(cfg) == 512 << 20
    assert binding.okv_workspace_bytes(cfg) == 32 * (8 + 1) * 32 * 130 * 4   # one item per 128 keys and one more per sequence
    assert binding.okv_block_bytes(cfg) == 2 * 32 * 1024 * 128 * 2      # one sequence's slice
    cfg = binding.make_config(n_layers=2, n_q_heads=8, n_kv_heads=8, head_dim=64, block_tokens=16,
                              max_batch=4, max_blocks_per_seq=16, blocks_per_layer=64,
                              resident_blocks=24, chunk_blocks=8)
    assert binding.okv_block_bytes(cfg) == 2 * 8 * 16 * 64 * 2
    # two block-sized slots per sequence and layer for the newest blocks; none without block-granular offload
    assert binding.okv_tail_bytes(cfg) == 2 * 2 * 4 * (2 * 8 * 16 * 64 * 2)
    assert binding.okv_tail_bytes(binding.make_config(n_layers=2, n_q_heads=8, n_kv_heads=8, head_dim=64, block_tokens=16,
                                                      max_batch=4, max_blocks_per_seq=16, blocks_per_layer=64)) == 0
    # KV heads per group of the pool layout: the library's rule against the oracle's statement of it
    from oracle import kv_layout
    for G in list(range(1, 41)) + [48, 64, 96, 128]:
        for d in (64, 128):
            assert binding.okv_kv_head_group(G, d) == kv_layout.head_group(G, d)
    assert binding.okv_kv_head_group(32, 128) == 8 and binding.okv_kv_head_group(32, 64) == 16
    # 16-token tiles per slab: the same for the oracle's statement of the rule
    for G in (1, 2, 3, 4, 6, 8, 12, 16, 32, 40):
        for d in (64, 128):
            for tokens in (16, 32, 48, 64, 80, 96, 128, 256, 1024, 4096, 4112):
                assert binding.okv_slab_tiles(G, d, tokens) == kv_layout.slab_tiles(G, d, tokens), (G, d, tokens)
    assert binding.okv_slab_tiles(32, 128, 4096) == 1 and binding.okv_slab_tiles(4, 128, 64) == 2 and binding.okv_slab_tiles(1, 128, 16) == 1
    with pytest.raises(binding.OkvError):
        binding.okv_slab_tiles(8, 128, 24)
    with pytest.raises(binding.OkvError):
        binding.okv_kv_head_group(8, 96)
    # 16 blocks of 16 tokens at the default split of 512 -> 1 item, plus one per chunk of the host pool (5)
    assert binding.okv_workspace_bytes(cfg) == 4 * (1 + 5) * 8 * 66 * 4
    for bad in (dict(resident_blocks=65), dict(resident_blocks=-1), dict(chunk_blocks=-2), dict(block_tokens=0, max_ctx=256)):
        kw = dict(n_layers=2, n_q_heads=8, n_kv_heads=8, head_dim=64, block_tokens=16, max_batch=4,
                  max_blocks_per_seq=16, blocks_per_layer=64, resident_blocks=24, chunk_blocks=8)
        kw.update(bad)
        with pytest.raises(binding.OkvError):
            binding.okv_block_bytes(binding.make_config(**kw))
    for bad in (dict(head_dim=96), dict(n_q_heads=12), dict(n_q_heads=136), dict(block_tokens=24), dict(max_ctx=1000),
                dict(n_layers=0), dict(out_dtype=3)):
        kw = dict(n_layers=2, n_q_heads=8, n_kv_heads=8, head_dim=64, block_tokens=0, max_batch=4, max_ctx=256)
        kw.update(bad)
        with pytest.raises(binding.OkvError) as e:
            binding.okv_layer_pool_bytes(binding.make_config(**kw))
        assert e.value.code == binding.OKV_EINVAL


def test_equal_stretches_match_the_oracle_walk():
    # the library's closed-form cutting against the oracle's tile-by-tile walk, bit for bit
    from oracle import worklist
    rng = np.random.default_rng(11)
    for case in range(80):
        B = int(rng.integers(1, 60))
        lens = rng.integers(0, 5000, size=B).astype(np.int32)
        if case % 5 == 0:
            lens[:] = int(rng.integers(1, 4100))
        if case % 9 == 0:
            lens[rng.integers(0, B)] = 0
        max_groups = int(rng.choice([1, 3, 32, 85, 128, 1024]))
        if lens.sum() == 0:
            lens[0] = 1
        items, first, span = binding.okv_equal_stretches(lens, max_groups)
        want_items, want_first, want_span = worklist.expected_items_equal_stretches(lens, max_groups)
        assert span == want_span
        assert [tuple(int(v) for v in r) for r in items] == want_items
        assert first.tolist() == want_first
    with pytest.raises(binding.OkvError) as e:
        binding.okv_equal_stretches(np.array([-1], dtype=np.int32), 4)
    assert e.value.code == binding.OKV_EINVAL


def test_static_entry_point_rejects_bad_arguments_without_a_gpu():
    # shape and size checks come before any GPU call
    base = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, block_tokens=16, max_blocks_per_seq=8, max_ctx=0, out_dtype=0, B=4,
                pool=256, block_table=256, ctx_lens=256, q=256, out=256)
    for bad, code in ((dict(head_dim=96), binding.OKV_EINVAL), (dict(B=0), binding.OKV_EINVAL),
                      (dict(B=binding.OKV_STATIC_MAX_BATCH + 1), binding.OKV_EINVAL), (dict(pool=None), binding.OKV_EINVAL),
                      (dict(q=264), binding.OKV_EINVAL), (dict(k_new=256), binding.OKV_EINVAL),
                      (dict(n_q_heads=12), binding.OKV_EINVAL)):
        kw = dict(base)
        kw.update(bad)
        with pytest.raises(binding.OkvError) as e:
            binding.okv_decode_attn_static(**kw)
        assert e.value.code == code, bad


def test_tail_plan_matches_the_oracle_and_serves_every_chunk_in_the_model():
    # which chunks get rows from the slots and which blocks are written out, per step: the library's host code
    # against the rule as oracle/tail_sim.py states it, then the library's decisions drive the model of the pools
    from oracle import tail_sim
    from paper_2504_11816_amd import synth
    rng = np.random.default_rng(7)
    for seed, policy in enumerate(("prefix", "sequence", "scatter", "scatter", "sequence")):
        T, B, cap, chunk = (16, 32)[seed % 2], 6, 192, 3
        need = B * (cap // T)
        n_host = need * 3 // 5
        resident = need - n_host + 1
        table = synth.classed_block_table([cap] * B, T, resident, n_host + 2, n_host, policy, 40 + seed, max_blocks_per_seq=cap // T)
        n_chunks = -(-(n_host + 2) // chunk)
        ctx = rng.integers(0, cap - 80, size=B).astype(np.int32)

        def lib_plan(n, t0):
            patch, fills = binding.okv_tail_plan(table, T, n, t0, resident, chunk, n_chunks)
            want_patch, want_fills = tail_sim.expected_plan(table, T, n, t0, resident, chunk, n_chunks)
            np.testing.assert_array_equal(patch, want_patch)
            np.testing.assert_array_equal(fills, want_fills)
            return patch, fills

        for lag in (0, 1):
            tail_sim.replay(table, T, ctx, resident, chunk, n_chunks, 75, lib_plan, lag)
    with pytest.raises(binding.OkvError):
        binding.okv_tail_plan(table, 24, ctx + 1, ctx, resident, chunk, n_chunks)
    with pytest.raises(binding.OkvError):
        binding.okv_tail_plan(table, T, ctx * 0, ctx, resident, chunk, n_chunks)
