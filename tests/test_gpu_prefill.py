"""GPU parity for the prefill-side store: whole prompts written into the pools (HBM
and pinned host memory) bit for bit as the oracle's scatter does, and decode steps on
top of them against the fp64 attention oracle."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import kv_layout
from paper_2504_11816_amd import binding, synth
from paper_2504_11816_amd.harness import Stack

from gpu_util import build_stack, make_inputs, run_and_check
from test_gpu_block_classes import classed_stack

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def prompt_rows(st, n_new, seed, step=0):
    """Per-layer K/V rows [sum(n_new)][G][d] on the device, each from its own stream."""
    rows = int(np.sum(n_new))
    k = [synth.randn_f16_torch((rows, st.G, st.d), synth.stream_seed(seed, synth.TENSOR_KNEW, l, step), st.device)
         for l in range(st.L)]
    v = [synth.randn_f16_torch((rows, st.G, st.d), synth.stream_seed(seed, synth.TENSOR_VNEW, l, step), st.device)
         for l in range(st.L)]
    torch.cuda.synchronize()
    return k, v


def unused_slots(st, n_after):
    """Boolean mask over a layer's pool: rows at positions a sequence does not hold yet (in blocks
    it owns).  Their contents are unspecified: a block that is written from its first slot may be
    assembled elsewhere and copied over whole."""
    layout = st.layout()
    mask = np.zeros(st.pool_bytes // 2, dtype=bool)
    for b in range(st.B):
        if st.paged:
            owned = int((st.block_table[b] >= 0).sum()) * st.T
        else:
            owned = st.max_ctx
        for pos in range(int(n_after[b]), owned):
            for kv in (0, 1):
                for g in range(st.G):
                    off = kv_layout.token_row_offset(layout, b, kv, g, pos)
                    mask[off:off + st.d] = True
    return mask


def check_prefill(st, chunks, seed):
    """Runs the given prefills one after the other; after each, every layer's pool must equal the
    oracle's scatter applied to the pool as it was, bit for bit, in every row a sequence holds and
    in everything that belongs to no sequence of the batch."""
    want = [st.read_pool(l) for l in range(st.L)]
    n = st.ctx_lens.copy()
    for i, n_new in enumerate(chunks):
        n_new = np.asarray(n_new, dtype=np.int32)
        k, v = prompt_rows(st, n_new, seed, i)
        st.prefill(n_new, k, v)
        st.synchronize()
        care = ~unused_slots(st, n + n_new)
        for l in range(st.L):
            kv_layout.bulk_append_scatter(want[l], st.layout(), n, n_new, k[l].cpu().numpy(), v[l].cpu().numpy())
            got = st.read_pool(l)
            np.testing.assert_array_equal(got.view(np.uint16)[care], want[l].view(np.uint16)[care])
            want[l] = got                                  # unspecified slots: carry on from what is there
        n = n + n_new
        np.testing.assert_array_equal(st.ctx.okv_get_ctx_lens(), n)


@pytest.mark.parametrize("T", [0, 16, 64])
@pytest.mark.parametrize("on_host", [[0, 0], [1, 0], [1, 1]])
@pytest.mark.parametrize("d,G", [(64, 2), (128, 3)])
def test_prompt_store_is_bit_exact(T, on_host, d, G):
    say(f"prefill T={T} on_host={on_host} d={d} G={G}")
    ctx = np.array([0, 0, 5, 16, 31], dtype=np.int32)
    st = build_stack(L=2, H=2 * G if G == 2 else G, G=G, d=d, T=T, ctx_before=ctx, cap_tokens=256, on_host=on_host, seed=201)
    # a ragged prompt, then a chunk that starts in the middle of a tile, then one with empty sequences
    check_prefill(st, [[100, 1, 43, 16, 0], [17, 64, 0, 33, 7], [0, 0, 0, 0, 3]], seed=203)
    assert st.ctx.okv_prefill_plan()["staged_groups"] == 0          # shuffled single blocks: written directly
    # and the cache is usable: decode steps on top agree with the oracle
    run_and_check(st, n_steps=2, seed=205)
    st.close()


@pytest.mark.parametrize("policy", ["prefix", "sequence", "scatter"])
def test_prompt_store_with_blocks_on_the_host(policy):
    say(f"prefill classes {policy}")
    ctx = np.array([0, 3, 40, 0], dtype=np.int32)
    st = classed_stack(L=2, H=4, G=2, d=64, T=16, ctx_before=ctx, cap_tokens=320, c_off=Fraction(1, 2), chunk_blocks=7,
                       policy=policy, seed=211, workspace_items=4 * 24, split_tokens=64)
    check_prefill(st, [[200, 77, 1, 0], [30, 16, 100, 250]], seed=213)
    run_and_check(st, n_steps=2, seed=215)
    st.close()


@pytest.mark.parametrize("n_staging", [1, 2, 3])
@pytest.mark.parametrize("T", [16, 64])
def test_prompt_store_through_staging_when_blocks_are_adjacent(n_staging, T):
    # blocks handed out in order: a sequence's blocks are neighbours in the host pool, so they are
    # gathered in a staging buffer and moved by hipMemcpyAsync; a second prefill that continues in
    # the middle of a block takes the direct path for that block
    say(f"prefill staged T={T} staging={n_staging}")
    B, cap = 6, 2048
    st = Stack(L=3, H=8, G=8, d=128, B=B, T=T, cap_tokens=cap, on_host=[1, 0, 1], n_staging=n_staging)
    for l in range(3):
        st.fill_pool(l, synth.stream_seed(251, synth.TENSOR_POOL, l))
    st.set_batch([0] * B, synth.identity_block_table([st.cap_tokens] * B, T, max_blocks_per_seq=st.max_blocks))
    check_prefill(st, [[1500, 640, 1, 0, 2000, 333]], seed=253)
    plan = st.ctx.okv_prefill_plan()
    assert plan["staged_groups"] == 1 and plan["copies"] in (4, 5) and plan["direct_tiles"] == 0, plan
    check_prefill(st, [[400, 1000, 1500, 16, 40, 0]], seed=254)
    plan = st.ctx.okv_prefill_plan()
    # sequences 0, 2, 5 continue in the middle of a block: those blocks are written directly
    assert plan["direct_tiles"] > 0 and plan["staged_tiles"] > 0, plan
    run_and_check(st, n_steps=2, seed=255, pairs=[(0, 0), (2, 5), (4, 7), (5, 3)])
    st.close()


def test_prompt_store_through_staging_with_blocks_on_the_host():
    # "prefix" placement hands out host ids in order: staged path with chunk-sized staging buffers,
    # several groups per layer
    say("prefill staged classes")
    ctx = np.array([0, 0, 0, 0], dtype=np.int32)
    st = classed_stack(L=2, H=8, G=8, d=128, T=16, ctx_before=ctx, cap_tokens=1024, c_off=Fraction(1, 2), chunk_blocks=40,
                       policy="prefix", seed=261)
    check_prefill(st, [[1000, 513, 64, 700]], seed=263)
    plan = st.ctx.okv_prefill_plan()
    assert plan["staged_groups"] >= 2 and plan["direct_tiles"] == 0, plan
    check_prefill(st, [[10, 100, 900, 0]], seed=264)
    run_and_check(st, n_steps=2, seed=265, pairs=[(0, 0), (1, 5), (2, 7), (3, 3)])
    st.close()


def test_decode_then_prefill_then_decode():
    # a prefill after decode steps restarts the copy pipeline: staged copies made before it are stale
    say("prefill between decode steps")
    st = build_stack(L=3, H=4, G=2, d=128, T=16, ctx_before=[50, 9], cap_tokens=256, on_host=[1, 0, 1], seed=221)
    run_and_check(st, n_steps=2, seed=223)
    check_prefill(st, [[60, 100]], seed=225)
    run_and_check(st, n_steps=2, seed=227)
    st.close()


def test_decode_then_prefill_then_decode_with_the_newest_blocks_in_hbm():
    # block-granular offload with the slots that keep appended rows in HBM: a prefill must first write out what
    # the decode steps left there (the prompt continues in the middle of those blocks), and the steps after it
    # start the slots afresh.  Nothing is read back on the way: the oracle keeps its own pools.
    say("prefill between decode steps, newest blocks in HBM")
    from gpu_util import assert_close, make_inputs
    from test_gpu_block_classes import oracle_outputs
    ctx = np.array([50, 9, 31], dtype=np.int32)
    st = classed_stack(L=2, H=4, G=2, d=64, T=16, ctx_before=ctx, cap_tokens=320, c_off=Fraction(3, 5), chunk_blocks=5,
                       policy="scatter", seed=231, workspace_items=3 * 24)
    assert st.hot_tails
    layout = st.layout()
    want = [st.read_pool(l) for l in range(2)]
    n = ctx.copy()

    def decode(steps, seed):
        for step in range(steps):
            q, k, v, out = make_inputs(st, seed, step, st.device)
            st.step(q, k, v, out)
            st.synchronize()
            n[:] = n + 1
            for l in range(2):
                kv_layout.append_scatter(want[l], layout, n, k[l].cpu().numpy(), v[l].cpu().numpy())
                ref = oracle_outputs(want[l], layout, q[l].cpu().numpy(), n, 4, 2)
                assert_close(out[l].float().cpu().numpy().reshape(-1, 64), ref.reshape(-1, 64), f"seed {seed} step {step} layer {l}")

    decode(5, 233)
    n_new = np.array([40, 70, 20], dtype=np.int32)
    k, v = prompt_rows(st, n_new, 235)
    st.prefill(n_new, k, v)
    for l in range(2):
        kv_layout.bulk_append_scatter(want[l], layout, n, n_new, k[l].cpu().numpy(), v[l].cpu().numpy())
    n[:] = n + n_new
    decode(20, 237)
    care = ~unused_slots(st, n)
    for l in range(2):
        np.testing.assert_array_equal(st.read_pool(l).view(np.uint16)[care], want[l].view(np.uint16)[care])
    st.close()


def test_prefill_error_paths():
    say("prefill errors")
    st = build_stack(L=2, H=4, G=2, d=64, T=16, ctx_before=[10, 20], cap_tokens=64, seed=231)
    c = st.ctx
    k, v = prompt_rows(st, [4, 4], 233)

    def code(fn, *a):
        with pytest.raises(binding.OkvError) as e:
            fn(*a)
        return e.value.code

    assert code(c.kv_append_bulk, 0, k[0], v[0]) == binding.OKV_ESTATE          # no prefill open
    assert code(c.okv_prefill_end) == binding.OKV_ESTATE
    assert code(c.okv_prefill_begin, [-1, 2]) == binding.OKV_EINVAL
    assert code(c.okv_prefill_begin, [55, 2]) == binding.OKV_ENOSPC             # 10 + 55 > 64
    c.okv_prefill_begin([4, 4])
    assert code(c.okv_prefill_begin, [1, 1]) == binding.OKV_ESTATE
    assert code(c.okv_step_begin) == binding.OKV_ESTATE
    assert code(c.kv_append_bulk, 1, k[1], v[1]) == binding.OKV_ESTATE          # layer out of order
    assert code(c.kv_append_bulk, 0, None, v[0]) == binding.OKV_EINVAL
    assert code(c.okv_prefill_release, 0) == binding.OKV_EINVAL                 # not stored yet
    assert code(c.okv_prefill_end) == binding.OKV_ESTATE                        # layers missing
    for l in range(2):
        c.kv_append_bulk(l, k[l], v[l])
        c.okv_prefill_release(l)
    c.okv_prefill_end()
    np.testing.assert_array_equal(c.okv_get_ctx_lens(), [14, 24])
    tbl = st.block_table.copy()
    tbl[0, 2] = -1
    st.set_batch([14, 24], tbl)
    assert code(c.okv_prefill_begin, [30, 0]) == binding.OKV_ENOSPC             # would reach an unallocated block
    st.close()


def test_full_size_prompt_2048_half_of_the_layers_on_the_host_sampled():
    # batch 64 x prompt 2048, 32 KV heads x 128: 2 GiB of K/V per layer; one resident and one host layer.
    # Sampled check: rows of a few (sequence, position, head) against the input, then a decode step.
    say("prefill full size")
    B, P = 64, 2048
    st = Stack(L=2, H=32, G=32, d=128, B=B, T=16, cap_tokens=P + 16, on_host=[0, 1], out_dtype=0)
    for l in range(2):
        st.fill_pool(l, synth.stream_seed(241, synth.TENSOR_POOL, l))
    table = synth.shuffled_block_table([st.cap_tokens] * B, 16, st.blocks_per_layer, 243, max_blocks_per_seq=st.max_blocks)
    st.set_batch([0] * B, table)
    k, v = prompt_rows(st, [P] * B, 245)
    st.prefill([P] * B, k, v)
    st.synchronize()
    layout = st.layout()
    rng = np.random.default_rng(247)
    for l in range(2):
        picks = [(int(rng.integers(B)), int(rng.integers(P)), int(rng.integers(32))) for _ in range(64)]
        picks += [(0, 0, 0), (B - 1, P - 1, 31)]
        for kv, rows in ((0, k[l]), (1, v[l])):
            offs = [kv_layout.token_row_offset(layout, b, kv, g, pos) for (b, pos, g) in picks]
            got = st.read_rows(l, offs)
            want = np.stack([rows[b * P + pos, g].cpu().numpy() for (b, pos, g) in picks])
            np.testing.assert_array_equal(got.view(np.uint16), want.view(np.uint16))
    del k, v
    run_and_check(st, n_steps=1, seed=249, pairs=[(0, 0), (63, 31), (20, 11)])
    st.close()
