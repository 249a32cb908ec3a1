"""GPU parity: the HIP path through the C ABI against the fp64 CPU oracle,
element by element, on seeded inputs.  Tolerance: max abs error <= 2e-3 and
per-vector relative L2 error <= 1e-2 (fp16 KV, fp32 accumulation); integer
work (work list, append scatter, lengths) bit-exact."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import kv_layout, worklist
from paper_2504_11816_amd import binding, synth
from paper_2504_11816_amd.harness import Stack

from layout_util import from_pool, to_pool
from gpu_util import assert_close, build_stack, make_inputs, oracle_pairs, run_and_check

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


# ---- the small configuration in full ------------------------------------------------

@pytest.mark.parametrize("T", [0, 16])
@pytest.mark.parametrize("out_dtype", [0, 1])
def test_cfg1_single_layer_all_outputs(T, out_dtype):
    say(f"cfg1 T={T} out_dtype={out_dtype}")
    st = build_stack(L=1, H=8, G=8, d=64, T=T, ctx_before=[255] * 4, cap_tokens=256, out_dtype=out_dtype)
    run_and_check(st, n_steps=1)
    assert st.ctx.okv_get_ctx_lens().tolist() == [256] * 4
    st.close()


# ---- several tiles, ragged tails, every head grouping --------------------------------

@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("H,G", [(4, 4), (4, 2), (8, 2), (8, 1), (16, 1), (32, 2), (12, 12), (40, 20), (9, 3)])
@pytest.mark.parametrize("T", [0, 16, 64])
def test_ragged_contexts_all_groupings(d, H, G, T):
    say(f"ragged d={d} H={H} G={G} T={T}")
    ctx = [0, 14, 15, 16, 31, 130, 299, 700]       # after the append: 1, 15, 16, 17, 32, 131, 300, 701
    st = build_stack(L=2, H=H, G=G, d=d, T=T, ctx_before=ctx, cap_tokens=704, out_dtype=1, seed=3)
    run_and_check(st, n_steps=2, seed=5)
    st.close()


@pytest.mark.parametrize("split", [1, 7, 16, 100, 128, 256, 1024])
def test_result_does_not_depend_on_the_split_size(split):
    say(f"split={split}")
    ctx = [9, 127, 128, 300, 513]
    for T in (0, 16):
        st = build_stack(L=1, H=4, G=2, d=128, T=T, ctx_before=ctx, cap_tokens=544, out_dtype=1, seed=7,
                         split_tokens=1024)
        ref = run_and_check(st, n_steps=1, seed=9)[0][0]
        st.close()
        st = build_stack(L=1, H=4, G=2, d=128, T=T, ctx_before=ctx, cap_tokens=544, out_dtype=1, seed=7,
                         split_tokens=split)
        assert st.ctx.okv_get_split_tokens() == split
        got = run_and_check(st, n_steps=1, seed=9)[0][0]
        st.close()
        # one split versus many: equal up to the fp32 summation order and the fp16 rounding of the
        # softmax weights, which is relative to each item's own running maximum
        rel = np.abs(got - ref).max() / np.abs(ref).max()
        assert rel < 1e-3, rel


@pytest.mark.parametrize("H,G,d", [(8, 4, 64), (16, 16, 128)])
def test_more_work_units_than_wavefronts_all_outputs(H, G, d):
    # Thousands of 16-key items, each a group of its own: every wavefront works through several
    # (item, KV head) pairs in fixed rotation, and every sequence needs the merge.
    say(f"more pairs than wavefronts H={H} G={G} d={d}")
    ctx = synth.ragged_ctx_lens(48, 200, 420, 77)
    st = build_stack(L=1, H=H, G=G, d=d, T=16, ctx_before=ctx, cap_tokens=448, out_dtype=1, seed=79,
                     split_tokens=16)
    n_items = len(st.ctx.okv_worklist(from_device=True))
    assert n_items * G > 3000
    run_and_check(st, n_steps=2, seed=81)
    st.close()


@pytest.mark.parametrize("H,G,d,T", [(8, 4, 64, 16), (16, 16, 128, 0), (16, 2, 128, 16)])
def test_equal_sequences_more_work_units_than_wavefronts(H, G, d, T):
    # a batch of equal sequences cut into thousands of 16-key items, dealt to the wavefronts in fixed rotation;
    # a second batch one key off per sequence takes the same path
    say(f"fixed rotation H={H} G={G} d={d} T={T}")
    for ctx in ([333] * 40, [320 + (b % 2) * 15 for b in range(40)]):
        st = build_stack(L=1, H=H, G=G, d=d, T=T, ctx_before=ctx, cap_tokens=352, out_dtype=1, seed=83,
                         split_tokens=16)
        n_items = len(st.ctx.okv_worklist(from_device=True))
        assert n_items * G > 1600
        run_and_check(st, n_steps=2, seed=85, pairs=[(b, h) for b in range(0, 40, 3) for h in range(0, H, 3)])
        st.close()


def test_paged_equals_contiguous_on_the_same_logical_kv_bit_for_bit():
    say("paged == contiguous")
    B, H, G, d, T, C = 3, 4, 2, 128, 16, 320
    ctx = np.array([16, 250, 303], dtype=np.int32)
    stc = build_stack(L=1, H=H, G=G, d=d, T=0, ctx_before=ctx, cap_tokens=C, out_dtype=1, seed=11)
    pool_c = from_pool(stc.read_pool(0), B, G, C, d)
    stp = build_stack(L=1, H=H, G=G, d=d, T=T, ctx_before=ctx, cap_tokens=C, out_dtype=1, seed=12,
                      shuffle_seed=5)
    # write the contiguous run's logical KV into the paged pool through the table
    pool_p = from_pool(stp.read_pool(0), stp.blocks_per_layer, G, T, d)
    for b in range(B):
        for i in range(C):
            blk = stp.block_table[b, i // T]
            pool_p[blk, :, :, i % T, :] = pool_c[b, :, :, i, :]
    stp.pools[0].copy_(torch.from_numpy(to_pool(pool_p)))
    torch.cuda.synchronize()
    outs = []
    for st in (stc, stp):
        st.ctx.okv_set_split_tokens(128)
        q, k, v, out = make_inputs(st, 21, 0, st.device)
        st.step(q, k, v, out)
        st.synchronize()
        outs.append(out[0].cpu().numpy())
    np.testing.assert_array_equal(outs[0], outs[1])
    # and a second shuffle of the physical blocks changes nothing either
    stp2 = build_stack(L=1, H=H, G=G, d=d, T=T, ctx_before=ctx, cap_tokens=C, out_dtype=1, seed=13,
                       shuffle_seed=99)
    pool_p2 = from_pool(stp2.read_pool(0), stp2.blocks_per_layer, G, T, d)
    for b in range(B):
        for i in range(C):
            pool_p2[stp2.block_table[b, i // T], :, :, i % T, :] = pool_c[b, :, :, i, :]
    stp2.pools[0].copy_(torch.from_numpy(to_pool(pool_p2)))
    torch.cuda.synchronize()
    stp2.ctx.okv_set_split_tokens(128)
    q, k, v, out = make_inputs(stp2, 21, 0, stp2.device)
    stp2.step(q, k, v, out)
    stp2.synchronize()
    np.testing.assert_array_equal(out[0].cpu().numpy(), outs[0])
    for st in (stc, stp, stp2):
        st.close()


# ---- closed forms on the GPU ------------------------------------------------------------

def test_closed_forms_on_gpu():
    say("closed forms")
    B, H, G, d = 2, 4, 4, 128
    # context 1: the output is the appended value row, exactly
    st = build_stack(L=1, H=H, G=G, d=d, T=16, ctx_before=[0, 0], cap_tokens=64, out_dtype=0, seed=31)
    q, k, v, out = make_inputs(st, 33, 0, st.device)
    st.step(q, k, v, out)
    st.synchronize()
    np.testing.assert_array_equal(out[0].cpu().numpy(), v[0].cpu().numpy())
    st.close()
    # identical keys: the mean of the value rows; constant values: that constant
    n = 77
    st = build_stack(L=1, H=H, G=G, d=d, T=0, ctx_before=[n - 1, n - 1], cap_tokens=80, out_dtype=1, seed=35)
    pool = from_pool(st.read_pool(0), B, G, st.max_ctx, d)
    key = synth.randn_f16_numpy((B, G, d), 36)
    pool[:, 0, :, :, :] = key[:, :, None, :]
    pool[1, 1] = np.float16(0.625)
    st.pools[0].copy_(torch.from_numpy(to_pool(pool)))
    q, k, v, out = make_inputs(st, 37, 0, st.device)
    k[0].copy_(torch.from_numpy(key))
    v[0][1] = 0.625
    torch.cuda.synchronize()
    st.step(q, k, v, out)
    st.synchronize()
    got = out[0].cpu().numpy()
    vals = from_pool(st.read_pool(0), B, G, st.max_ctx, d)[:, 1, :, :n, :].astype(np.float64)
    np.testing.assert_allclose(got[0], vals[0].mean(axis=1), rtol=2e-6, atol=2e-6)
    np.testing.assert_allclose(got[1], np.full((H, d), 0.625), rtol=1e-6)
    st.close()


def test_unused_slots_full_of_nan_do_not_leak():
    say("NaN in unused slots")
    ctx = [4, 21, 40]
    for T in (0, 16):
        st = build_stack(L=1, H=4, G=2, d=128, T=T, ctx_before=ctx, cap_tokens=64, out_dtype=1, seed=41)
        good = run_and_check(st, n_steps=1, seed=43)[0][0]
        st.close()
        st = build_stack(L=1, H=4, G=2, d=128, T=T, ctx_before=ctx, cap_tokens=64, out_dtype=1, seed=41)
        pool = st.read_pool(0)
        lay = st.layout()
        keep = np.zeros(pool.shape, dtype=bool)
        for b, n in enumerate(ctx):
            for kv in range(2):
                for g in range(2):
                    for i in range(n):
                        off = kv_layout.token_row_offset(lay, b, kv, g, i)
                        keep[off:off + 128] = True
        pool.view(np.uint16)[~keep] = 0x7E00          # fp16 quiet NaN everywhere that holds no token
        st.pools[0].copy_(torch.from_numpy(pool))
        torch.cuda.synchronize()
        got = run_and_check(st, n_steps=1, seed=43)[0][0]
        st.close()
        np.testing.assert_array_equal(got, good)


# ---- integer work: bit-exact --------------------------------------------------------------

def wavefronts_per_kv_head(G):
    """What a context shares a launch out over: 4 wavefronts per compute unit, divided by the KV heads."""
    return max(1, 4 * torch.cuda.get_device_properties(0).multi_processor_count // G)


def test_worklist_on_device_matches_host_and_oracle():
    say("work list")
    ctx = synth.ragged_ctx_lens(37, 1, 900, 51)
    st = build_stack(L=1, H=2, G=2, d=64, T=16, ctx_before=ctx, cap_tokens=1024, seed=53, split_tokens=1)
    for split in (0, 1, 5, 16, 128, 333, 1024):
        st.ctx.okv_set_split_tokens(split)
        S = st.ctx.okv_get_split_tokens()
        host = st.ctx.okv_worklist(from_device=False)
        dev = st.ctx.okv_worklist(from_device=True)
        assert S == (split or 1)                         # 0 = back to the size the context was created with
        want = np.array(worklist.expected_items(ctx, S), dtype=np.int32)
        np.testing.assert_array_equal(host, want)
        np.testing.assert_array_equal(dev, want)
        assert worklist.check_tiling([tuple(r) for r in dev], ctx)
    # after a step every sequence is one token longer, on both sides
    st.ctx.okv_set_split_tokens(100)
    q, k, v, out = make_inputs(st, 55, 0, st.device)
    st.step(q, k, v, out)
    np.testing.assert_array_equal(st.ctx.okv_get_ctx_lens(), ctx + 1)
    dev = st.ctx.okv_worklist(from_device=True)
    np.testing.assert_array_equal(dev, np.array(worklist.expected_items(ctx + 1, 100), dtype=np.int32))
    with pytest.raises(binding.OkvError) as e:            # a fixed split size has no stretches, hence no such table
        st.ctx.okv_pair_heads()
    assert e.value.code == binding.OKV_ESTATE
    st.close()


@pytest.mark.parametrize("H,G,d,T,B,lo,hi", [(32, 8, 128, 16, 40, 300, 2500), (12, 12, 64, 16, 30, 1, 1500),
                                               (4, 1, 128, 0, 3, 2000, 6000), (16, 16, 128, 32, 70, 16, 900)])
def test_equal_stretches_on_the_device_and_every_output(H, G, d, T, B, lo, hi):
    # no split size fixed: the batch's keys are shared out in equal stretches; wavefronts run several items one
    # after the other (the next item's first tile is asked for before this one's results are written), stretches
    # begin and end in the middle of sequences, some sequences are cut several times, and with 12 or 1 KV heads
    # the wavefronts do not divide evenly.  Work list against the oracle's walk, every output against the oracle.
    say(f"equal stretches H={H} G={G} d={d} T={T} B={B}")
    ctx = synth.ragged_ctx_lens(B, lo, hi, 401 + B)
    st = build_stack(L=1, H=H, G=G, d=d, T=T, ctx_before=ctx, cap_tokens=hi + 24, out_dtype=1, seed=403)
    want, first, span = worklist.expected_items_equal_stretches(ctx, wavefronts_per_kv_head(G))
    np.testing.assert_array_equal(st.ctx.okv_worklist(from_device=True), np.array(want, dtype=np.int32))
    np.testing.assert_array_equal(st.ctx.okv_worklist(from_device=False), np.array(want, dtype=np.int32))
    assert worklist.check_tiling(want, ctx)
    # what every wavefront starts from: the first item of its stretch, and where the oracle's layout puts the
    # K rows of that item's first two tiles for the wavefront's KV head
    heads = st.ctx.okv_pair_heads()
    assert heads.shape == ((len(first) - 1) * G, 8)
    layout = st.layout()
    for p, rec in enumerate(heads):
        stretch, g = divmod(p, G)
        it = first[stretch]
        b, lo, hi = want[it]
        assert (rec[0], rec[1], rec[2], rec[3], rec[4]) == (it, first[stretch + 1] - it, b, lo, hi), (p, rec)
        ends_sequence, whole = hi == ctx[b], (lo == 0 and hi == ctx[b])
        assert rec[5] == (1 if ends_sequence else 0) | (2 if whole else 0) | (g << 8), (p, rec)
        last_tile_tok = (hi - 1) // 16 * 16
        for i in (0, 1):
            tok = min(lo + 16 * i, last_tile_tok)
            assert rec[6 + i] * 16 * d == kv_layout.token_row_offset(layout, b, 0, g, tok), (p, i, rec)
    pairs = [(b, h) for b in range(B) for h in range(0, H, max(1, H // 4))]
    run_and_check(st, n_steps=2, seed=405, pairs=pairs)
    want2, _, _ = worklist.expected_items_equal_stretches(ctx + 2, wavefronts_per_kv_head(G))
    np.testing.assert_array_equal(st.ctx.okv_worklist(from_device=True), np.array(want2, dtype=np.int32))
    st.close()


@pytest.mark.parametrize("T", [0, 16, 32])
@pytest.mark.parametrize("on_host", [[0, 0], [1, 0], [1, 1]])
def test_append_scatter_is_bit_exact(T, on_host):
    say(f"append T={T} on_host={on_host}")
    ctx = np.array([0, 15, 16, 31, 47], dtype=np.int32)
    st = build_stack(L=2, H=4, G=2, d=64, T=T, ctx_before=ctx, cap_tokens=64, on_host=on_host, seed=61)
    want = [st.read_pool(l) for l in range(2)]
    n = ctx.copy()
    for step in range(4):
        q, k, v, out = make_inputs(st, 63, step, st.device)
        st.step(q, k, v, out)
        st.synchronize()
        n += 1
        for l in range(2):
            kv_layout.append_scatter(want[l], st.layout(), n, k[l].cpu().numpy(), v[l].cpu().numpy())
    for l in range(2):
        got = st.read_pool(l)
        np.testing.assert_array_equal(got.view(np.uint16), want[l].view(np.uint16))
    st.close()


# ---- offloaded layers: residency never changes the result -------------------------------------

def test_streaming_is_bit_identical_to_resident_and_matches_oracle():
    say("streaming")
    L = 6
    ctx = [100, 257, 31, 480]
    plans = {
        "resident": [0] * L,
        "half": binding.kv_offload_plan(L, 1, 2)[0].tolist(),
        "all": [1] * L,
        "one": [0, 0, 1, 0, 0, 0],
        "sixty": binding.kv_offload_plan(L, 3, 5)[0].tolist(),
    }
    ref = None
    for name, on_host in plans.items():
        for n_staging in ((2, 1) if name in ("half", "all") else (2,)):
            say(f"  plan {name} {on_host} staging {n_staging}")
            st = build_stack(L=L, H=4, G=2, d=128, T=16, ctx_before=ctx, cap_tokens=512, on_host=on_host,
                             out_dtype=0, seed=71, n_staging=n_staging)
            for s in st.staging:
                if s is not None:
                    s.fill_(float("nan"))             # a stale or missing copy poisons the output
            torch.cuda.synchronize()
            outs = run_and_check(st, n_steps=3, seed=73, pairs=[(0, 0), (1, 3), (2, 1), (3, 2)])
            st.close()
            if ref is None:
                ref = outs
            else:
                for step in range(3):
                    for l in range(L):
                        np.testing.assert_array_equal(outs[step][l], ref[step][l])


# ---- failure handling, forced from the host ------------------------------------------------------

def test_error_paths():
    say("error paths")
    st = build_stack(L=2, H=4, G=2, d=64, T=16, ctx_before=[10, 20], cap_tokens=32, seed=81)
    c = st.ctx
    q, k, v, out = make_inputs(st, 83, 0, st.device)

    def code(fn, *a):
        with pytest.raises(binding.OkvError) as e:
            fn(*a)
        return e.value.code

    assert code(c.kv_append, 0, k[0], v[0]) == binding.OKV_ESTATE            # outside a step
    c.okv_step_begin()
    assert code(c.okv_step_begin) == binding.OKV_ESTATE
    assert code(c.decode_attn, 0, q[0], out[0]) == binding.OKV_ESTATE         # attention before append
    assert code(c.kv_append, 1, k[1], v[1]) == binding.OKV_ESTATE             # layer out of order
    assert code(c.kv_append, 5, k[0], v[0]) == binding.OKV_EINVAL
    assert code(c.kv_append, 0, None, v[0]) == binding.OKV_EINVAL
    assert code(c.okv_step_end) == binding.OKV_ESTATE                         # layers missing
    for l in range(2):
        c.kv_append(l, k[l], v[l])
        c.decode_attn(l, q[l], out[l])
    c.okv_step_end()
    # a step given up half way: the batch has to be described again before anything else
    assert code(c.okv_step_abort) == binding.OKV_ESTATE                       # no step open
    c.okv_step_begin()
    c.kv_append(0, k[0], v[0])
    assert code(c.kv_append, 0, k[0], v[0]) == binding.OKV_ESTATE             # the failure a caller gives up after
    assert code(st.set_batch, [10, 20], st.block_table) == binding.OKV_ESTATE # still inside the step
    c.okv_step_abort()
    assert code(c.okv_step_begin) == binding.OKV_ESTATE                       # no batch
    st.set_batch([10, 20], st.block_table)
    run_and_check(st, n_steps=1, seed=87)                                     # and the context works as before
    # capacity: 32 tokens; 20 + 1 stored, 11 more fit
    st.set_batch([10, 32], st.block_table)
    assert code(c.okv_step_begin) == binding.OKV_ENOSPC
    np.testing.assert_array_equal(c.okv_get_ctx_lens(), [10, 32])            # nothing changed
    tbl = st.block_table.copy()
    tbl[0, 1] = -1
    st.set_batch([16, 5], tbl)
    assert code(c.okv_step_begin) == binding.OKV_ENOSPC                       # next block not allocated
    tbl[0, 1] = tbl[1, 0]
    assert code(st.set_batch, [3, 5], tbl) == binding.OKV_EINVAL              # block shared
    tbl[0, 1] = 10 ** 6
    assert code(st.set_batch, [3, 5], tbl) == binding.OKV_EINVAL              # block id out of range
    assert code(st.set_batch, [3, 33], st.block_table) == binding.OKV_EINVAL  # beyond capacity
    assert code(c.okv_set_split_tokens, -1) == binding.OKV_EINVAL
    st.close()
    # creation: staging smaller than a layer, both / neither pool given
    with pytest.raises(binding.OkvError) as e:
        ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
        pool = torch.empty(1 << 16, dtype=torch.float16, device="cuda")
        binding.Context(n_layers=1, n_q_heads=4, n_kv_heads=2, head_dim=64, block_tokens=0, max_batch=2,
                        max_ctx=64, dev_pool=[pool], host_pool=[pool], workspace=ws, workspace_bytes=1 << 20)
    assert e.value.code == binding.OKV_EINVAL
    # more KV heads than a launch has wavefronts (4 per compute unit): a stretch of keys could not have one each
    with pytest.raises(binding.OkvError) as e:
        heads = 4 * torch.cuda.get_device_properties(0).multi_processor_count + 64
        ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
        pool = torch.empty(2 * 2 * heads * 16 * 64, dtype=torch.float16, device="cuda")
        binding.Context(n_layers=1, n_q_heads=heads, n_kv_heads=heads, head_dim=64, block_tokens=0, max_batch=2,
                        max_ctx=16, dev_pool=[pool], host_pool=[None], workspace=ws, workspace_bytes=64 << 20)
    assert e.value.code == binding.OKV_EINVAL and "KV heads" in str(e.value)


def test_probe_kernels_and_link_measurement():
    say("probe kernels")
    n = 1 << 24
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    binding.okv_probe_copy(dst, src, n, s.cuda_stream)
    binding.okv_probe_read(src, n, sink, s.cuda_stream)
    s.synchronize()
    assert torch.equal(dst, src)
    with pytest.raises(binding.OkvError):
        binding.okv_probe_copy(dst, src, n - 3, s.cuda_stream)          # not a multiple of 16
    host = torch.empty(n, dtype=torch.uint8, pin_memory=True)
    host.copy_(src)
    dst.zero_()
    torch.cuda.synchronize()
    gbps = binding.okv_measure_h2d(dst, host, n, 3, s.cuda_stream)
    assert gbps > 1.0
    assert torch.equal(dst, src)


def test_kernel_timing_modes_count_every_launch():
    say("profile modes")
    st = build_stack(L=3, H=4, G=4, d=64, T=16, ctx_before=[40, 100], cap_tokens=128, seed=301)
    for mode in (1, 2):
        st.ctx.okv_profile_enable(mode)
        for step in range(4):
            q, k, v, out = make_inputs(st, 303, step, st.device)
            st.step(q, k, v, out)
        ms, n = st.ctx.okv_profile_read()
        assert n == 3 * 4 and 0 < ms < 100
        st.ctx.okv_profile_enable(0)
        assert st.ctx.okv_profile_read() == (0.0, 0)
    with pytest.raises(binding.OkvError) as e:
        st.ctx.okv_profile_enable(3)
    assert e.value.code == binding.OKV_EINVAL
    st.close()


def test_random_configurations_against_the_oracle():
    # 48 seeded draws over head counts (KV heads that are not powers of two, 1..16 query heads each), head
    # dimension, layout, block size, batch, ragged contexts (from empty), split size and output type
    say("random configurations")
    rng = np.random.default_rng(20250411)
    for case in range(48):
        G = int(rng.choice([1, 2, 3, 4, 6, 8, 12]))
        R = int(rng.integers(1, 17))
        while G * R > 48:
            R = int(rng.integers(1, 17))
        d = int(rng.choice([64, 128]))
        T = int(rng.choice([0, 16, 32, 64]))
        B = int(rng.integers(1, 6))
        ctx = [int(x) for x in rng.integers(0, 400, size=B)]
        split = int(rng.choice([0, 16, 48, 256, 1024]))
        out_dtype = int(rng.integers(0, 2))
        say(f"  case {case}: H={G * R} G={G} d={d} T={T} ctx={ctx} split={split} out={out_dtype}")
        st = build_stack(L=1, H=G * R, G=G, d=d, T=T, ctx_before=ctx, cap_tokens=416, out_dtype=out_dtype,
                         seed=1000 + case, split_tokens=split, shuffle_seed=case)
        pairs = [(b, h) for b in range(B) for h in range(0, G * R, max(1, (G * R) // 6))]
        run_and_check(st, n_steps=2, seed=2000 + case, pairs=pairs)
        st.close()


def test_whole_step_in_one_call_is_the_same_step():
    # okv_decode_step = okv_step_begin + (kv_append, decode_attn) per layer + okv_step_end: same outputs bit for
    # bit, same pools, same lengths; and its error paths
    say("okv_decode_step")
    ctx = [5, 120, 300]
    sts = [build_stack(L=3, H=8, G=4, d=64, T=16, ctx_before=ctx, cap_tokens=320, on_host=[0, 1, 0], seed=311)
           for _ in range(2)]
    for step in range(3):
        q, k, v, out_a = make_inputs(sts[0], 313, step, sts[0].device)
        sts[0].step(q, k, v, out_a)
        _, _, _, out_b = make_inputs(sts[1], 313, step, sts[1].device)
        sts[1].step_bound(sts[1].bind_step(q, k, v, out_b))
        for st in sts:
            st.synchronize()
        for l in range(3):
            np.testing.assert_array_equal(out_a[l].cpu().numpy().view(np.uint16), out_b[l].cpu().numpy().view(np.uint16))
    for l in range(3):
        np.testing.assert_array_equal(sts[0].read_pool(l).view(np.uint16), sts[1].read_pool(l).view(np.uint16))
    assert sts[1].ctx.okv_get_ctx_lens().tolist() == [c + 3 for c in ctx]
    arrays = sts[1].bind_step(q, k, v, out_b)[0]
    with pytest.raises(ValueError):
        sts[1].ctx.okv_decode_step(tuple(a if i else (type(a)._type_ * 2)() for i, a in enumerate(arrays)))
    sts[1].ctx.okv_step_begin()
    with pytest.raises(binding.OkvError) as e:                  # inside a step already
        sts[1].ctx.okv_decode_step(arrays)
    assert e.value.code == binding.OKV_ESTATE
    for st in sts:
        st.close()


def test_two_contexts_side_by_side_do_not_disturb_each_other():
    # two contexts of different shapes, each on streams of its own, issue their steps alternately without waiting
    # for one another: every output equals what the same context gives alone, bit for bit, and the oracle's
    say("two contexts side by side")
    shapes = [dict(L=2, H=8, G=2, d=64, T=16, ctx_before=[30, 200, 77, 5], seed=601, on_host=[0, 1]),
              dict(L=3, H=4, G=4, d=128, T=0, ctx_before=[100, 101, 99], seed=602, on_host=None)]
    n_steps = 3

    def run(which, interleaved):
        stacks = [build_stack(cap_tokens=256, **shapes[i]) for i in which]
        outs = [[] for _ in stacks]
        ins = [[make_inputs(st, 610 + i, step, st.device) for step in range(n_steps)] for i, st in zip(which, stacks)]
        for step in range(n_steps):
            for j, st in enumerate(stacks):
                q, k, v, out = ins[j][step]
                st.step(q, k, v, out)                        # no synchronisation between the two contexts
                if not interleaved:
                    st.synchronize()
        for j, st in enumerate(stacks):
            st.synchronize()
            outs[j] = [[o.cpu().numpy().view(np.uint16).copy() for o in ins[j][step][3]] for step in range(n_steps)]
        last = [(st, ins[j][n_steps - 1]) for j, st in enumerate(stacks)]
        return stacks, outs, last

    stacks, both, last = run([0, 1], interleaved=True)
    for st, (q, k, v, out) in last:                           # the last step against the oracle
        pairs = [(b, h) for b in range(st.B) for h in range(st.H)]
        for l in range(st.L):
            ref = oracle_pairs(st, l, q[l].cpu().numpy(), st.ctx_lens.copy(), pairs)
            got = np.stack([out[l].float().cpu().numpy()[b, h] for (b, h) in pairs])
            assert_close(got, np.stack([ref[p] for p in pairs]), f"layer {l}")
    for st in stacks:
        st.close()
    for i in (0, 1):
        stacks, alone, _ = run([i], interleaved=False)
        for step in range(n_steps):
            for a, b in zip(alone[0][step], both[i][step]):
                np.testing.assert_array_equal(a, b)
        stacks[0].close()
