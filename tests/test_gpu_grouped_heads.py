"""GPU parity for grouped query heads (up to 16 per KV head, any count in between) on the
matrix cores (scores and weighted sums as 16 x 16 tiles, softmax weights rounded to fp16
for the second product).  Same bar as the other parity tests: outputs against the fp64
oracle within 2e-3 max abs / 1e-2 relative L2, appended rows bit-exact."""
import numpy as np
import pytest
import torch

from oracle import kv_layout
from paper_2504_11816_amd import binding, synth

from layout_util import from_pool, to_pool
from gpu_util import assert_close, build_stack, make_inputs, oracle_pairs, run_and_check

pytestmark = pytest.mark.gpu

GROUPINGS = [(16, 2, 128), (16, 1, 128), (8, 1, 64), (32, 2, 64), (6, 2, 128), (12, 1, 64)]
# (H, G, d): 8, 16, 8, 16, 3 and 12 query heads per KV head


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("H,G,d", GROUPINGS)
@pytest.mark.parametrize("split", [16, 48, 100, 4096])
def test_split_sizes_ragged_contexts_several_steps(H, G, d, split):
    # items that start and end in the middle of blocks, single-tile items, one item per sequence
    say(f"grouped heads H={H} G={G} d={d} split={split}")
    ctx = [0, 1, 15, 16, 17, 33, 250, 511]
    for T in (0, 16):
        st = build_stack(L=2, H=H, G=G, d=d, T=T, ctx_before=ctx, cap_tokens=528, out_dtype=1, seed=201,
                         split_tokens=split)
        run_and_check(st, n_steps=3, seed=203)
        st.close()


@pytest.mark.parametrize("H,G,d", GROUPINGS[:2])
def test_one_split_versus_many(H, G, d):
    # the weights pass through fp16 on their way into the second product, relative to a running maximum
    # that depends on where the items are cut: results agree to the rounding of those weights, not to
    # the last fp32 bit
    say(f"grouped heads: split independence H={H} G={G}")
    ctx = [9, 127, 128, 300, 513]
    outs = []
    for split in (1024, 16, 112):
        st = build_stack(L=1, H=H, G=G, d=d, T=16, ctx_before=ctx, cap_tokens=544, out_dtype=1, seed=207,
                         split_tokens=split)
        outs.append(run_and_check(st, n_steps=1, seed=209)[0][0])
        st.close()
    for o in outs[1:]:
        assert np.abs(o - outs[0]).max() / np.abs(outs[0]).max() < 1e-3


@pytest.mark.parametrize("H,G,d", GROUPINGS[:3])
def test_closed_forms(H, G, d):
    say(f"grouped heads: closed forms H={H} G={G} d={d}")
    B = 2
    # context 1: the output is the appended value row, exactly, for every head of the group
    st = build_stack(L=1, H=H, G=G, d=d, T=16, ctx_before=[0, 0], cap_tokens=64, out_dtype=0, seed=211)
    q, k, v, out = make_inputs(st, 213, 0, st.device)
    st.step(q, k, v, out)
    st.synchronize()
    got = out[0].cpu().numpy().reshape(B, G, H // G, d)
    np.testing.assert_array_equal(got, np.broadcast_to(v[0].cpu().numpy()[:, :, None, :], got.shape))
    st.close()
    # identical keys: the mean of the value rows (all weights are exactly 1); constant values: that constant
    n = 77
    st = build_stack(L=1, H=H, G=G, d=d, T=0, ctx_before=[n - 1, n - 1], cap_tokens=80, out_dtype=1, seed=215)
    pool = from_pool(st.read_pool(0), B, G, st.max_ctx, d)
    key = synth.randn_f16_numpy((B, G, d), 216)
    pool[:, 0, :, :, :] = key[:, :, None, :]
    pool[1, 1] = np.float16(0.625)
    st.pools[0].copy_(torch.from_numpy(to_pool(pool)))
    q, k, v, out = make_inputs(st, 217, 0, st.device)
    k[0].copy_(torch.from_numpy(key))
    v[0][1] = 0.625
    torch.cuda.synchronize()
    st.step(q, k, v, out)
    st.synchronize()
    got = out[0].cpu().numpy().reshape(B, G, H // G, d)
    vals = from_pool(st.read_pool(0), B, G, st.max_ctx, d)[:, 1, :, :n, :].astype(np.float64)
    want = np.broadcast_to(vals[0].mean(axis=1)[:, None, :], got[0].shape)
    np.testing.assert_allclose(got[0], want, rtol=3e-6, atol=3e-6)
    np.testing.assert_allclose(got[1], np.full(got[1].shape, 0.625), rtol=1e-6)
    st.close()


@pytest.mark.parametrize("H,G,d", GROUPINGS[:2])
def test_peaked_and_flat_softmax(H, G, d):
    # queries 6 times larger give scores of standard deviation 6: nearly all the weight sits on a few keys
    # and most of the other weights fall below the fp16 range; a query of zeros gives the plain mean
    say(f"grouped heads: peaked softmax H={H} G={G}")
    ctx = [200, 1000]
    st = build_stack(L=1, H=H, G=G, d=d, T=16, ctx_before=ctx, cap_tokens=1008, out_dtype=1, seed=221)
    q, k, v, out = make_inputs(st, 223, 0, st.device)
    q[0].mul_(6.0)
    q[0][0, 1].zero_()
    torch.cuda.synchronize()
    st.step(q, k, v, out)
    st.synchronize()
    pairs = [(b, h) for b in range(2) for h in range(H)]
    ref = oracle_pairs(st, 0, q[0].cpu().numpy(), st.ctx_lens.copy(), pairs)
    got = out[0].cpu().numpy()
    assert_close(np.stack([got[b, h] for (b, h) in pairs]), np.stack([ref[p] for p in pairs]), "peaked")
    st.close()


def test_unused_slots_full_of_nan_do_not_leak():
    say("grouped heads: NaN in unused slots")
    H, G, d = 16, 2, 128
    ctx = [4, 21, 40]
    for T in (0, 16):
        st = build_stack(L=1, H=H, G=G, d=d, T=T, ctx_before=ctx, cap_tokens=64, out_dtype=1, seed=231)
        good = run_and_check(st, n_steps=1, seed=233)[0][0]
        st.close()
        st = build_stack(L=1, H=H, G=G, d=d, T=T, ctx_before=ctx, cap_tokens=64, out_dtype=1, seed=231)
        pool = st.read_pool(0)
        lay = st.layout()
        keep = np.zeros(pool.shape, dtype=bool)
        for b, n in enumerate(ctx):
            for kv in range(2):
                for g in range(G):
                    for i in range(n):
                        off = kv_layout.token_row_offset(lay, b, kv, g, i)
                        keep[off:off + d] = True
        pool.view(np.uint16)[~keep] = 0x7E00          # fp16 quiet NaN everywhere that holds no token
        st.pools[0].copy_(torch.from_numpy(pool))
        torch.cuda.synchronize()
        got = run_and_check(st, n_steps=1, seed=233)[0][0]
        st.close()
        np.testing.assert_array_equal(got, good)


@pytest.mark.parametrize("T", [0, 16, 32])
@pytest.mark.parametrize("on_host", [[0, 0], [1, 0]])
def test_append_scatter_is_bit_exact(T, on_host):
    say(f"grouped heads: append T={T} on_host={on_host}")
    ctx = np.array([0, 15, 16, 31, 47], dtype=np.int32)
    st = build_stack(L=2, H=32, G=2, d=64, T=T, ctx_before=ctx, cap_tokens=64, on_host=on_host, seed=241)
    want = [st.read_pool(l) for l in range(2)]
    n = ctx.copy()
    for step in range(4):
        q, k, v, out = make_inputs(st, 243, step, st.device)
        st.step(q, k, v, out)
        st.synchronize()
        n += 1
        for l in range(2):
            kv_layout.append_scatter(want[l], st.layout(), n, k[l].cpu().numpy(), v[l].cpu().numpy())
    for l in range(2):
        np.testing.assert_array_equal(st.read_pool(l).view(np.uint16), want[l].view(np.uint16))
    st.close()


def test_streamed_layers_are_bit_identical_to_resident_ones():
    say("grouped heads: streaming")
    L = 4
    ctx = [100, 257, 31, 480]
    outs = {}
    for name, on_host in (("resident", [0] * L), ("half", binding.kv_offload_plan(L, 1, 2)[0].tolist()), ("all", [1] * L)):
        st = build_stack(L=L, H=16, G=2, d=128, T=16, ctx_before=ctx, cap_tokens=512, on_host=on_host, seed=251)
        for s in st.staging:
            if s is not None:
                s.fill_(float("nan"))
        torch.cuda.synchronize()
        outs[name] = run_and_check(st, n_steps=2, seed=253, pairs=[(0, 0), (1, 9), (2, 15), (3, 7)])
        st.close()
    for name in ("half", "all"):
        for step in range(2):
            for l in range(L):
                np.testing.assert_array_equal(outs[name][step][l], outs["resident"][step][l])


def test_more_work_units_than_wavefronts_all_outputs():
    say("grouped heads: more pairs than wavefronts")
    ctx = synth.ragged_ctx_lens(48, 200, 420, 261)
    st = build_stack(L=1, H=64, G=8, d=128, T=16, ctx_before=ctx, cap_tokens=448, out_dtype=1, seed=263,
                     split_tokens=16)
    n_items = len(st.ctx.okv_worklist(from_device=True))
    assert n_items * 8 > 3000
    run_and_check(st, n_steps=2, seed=265, pairs=[(b, h) for b in range(0, 48, 5) for h in range(0, 64, 7)])
    st.close()


def test_full_size_64_query_heads_8_kv_heads_sampled():
    # 64 x 128 query heads over 8 KV heads, batch 128, context about 2048, 16-token blocks: 1 GiB of KV per layer
    say("grouped heads: full size")
    B = 128
    ctx = synth.ragged_ctx_lens(B, 1900, 2100, 271)
    st = build_stack(L=2, H=64, G=8, d=128, T=16, ctx_before=ctx, cap_tokens=2112, seed=273)
    shortest, longest = int(np.argmin(ctx)), int(np.argmax(ctx))
    run_and_check(st, n_steps=2, seed=275, pairs=[(0, 0), (shortest, 63), (longest, 8), (77, 33)])
    st.close()
