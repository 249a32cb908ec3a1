"""The entry point that allocates nothing (okv_decode_attn_static) against the entry points it is a variant of
(kv_append + decode_attn on a context): same kernels, same cutting of the batch, so the outputs and the pools
must agree bit for bit; and against the fp64 oracle at the usual tolerance.  Two calls in a row share the one
work area inside the library, the second on a smaller batch."""
import numpy as np
import pytest
import torch

from paper_2504_11816_amd import binding, synth

from gpu_util import assert_close, build_stack, make_inputs, oracle_pairs

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[no-alloc] {msg}", flush=True)


def _reference_step(shape, ctx_before, seed):
    """One decode step through a context: (outputs, pool after the step, inputs, stack)."""
    st = build_stack(L=1, ctx_before=ctx_before, seed=seed, **shape)
    q, k, v, out = make_inputs(st, seed + 1, 0, st.device)
    st.step(q, k, v, out)
    st.synchronize()
    return out[0], st.read_pool(0), (q[0], k[0], v[0]), st


def _static_step(shape, ctx_before, seed, inputs):
    """The same step through okv_decode_attn_static on a second, identically filled pool."""
    st = build_stack(L=1, ctx_before=ctx_before, seed=seed, **shape)          # only its pool and table are used
    q, k, v = inputs
    B = len(ctx_before)
    lens = torch.tensor(np.asarray(ctx_before, dtype=np.int32) + 1, dtype=torch.int32, device=st.device)
    table = None if st.block_table is None else torch.tensor(st.block_table, dtype=torch.int32, device=st.device)
    out = torch.full((B, st.H, st.d), float("nan"), dtype=st.out_torch_dtype, device=st.device)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    binding.okv_decode_attn_static(n_q_heads=st.H, n_kv_heads=st.G, head_dim=st.d, block_tokens=st.T,
                                   max_blocks_per_seq=st.max_blocks, max_ctx=st.max_ctx, out_dtype=shape.get("out_dtype", 0),
                                   B=B, pool=st.dev_part[0], block_table=table, ctx_lens=lens, q=q, out=out, k_new=k, v_new=v,
                                   stream=stream.cuda_stream)
    stream.synchronize()
    pool = st.read_pool(0)
    st.close()
    return out, pool


@pytest.mark.parametrize("shape", [dict(H=8, G=2, d=128, T=16, cap_tokens=3000, out_dtype=0),
                                   dict(H=4, G=4, d=64, T=0, cap_tokens=3000, out_dtype=1)])
def test_static_entry_point_equals_the_context_path_twice_in_a_row(shape):
    say(f"shape {shape}")
    # first call: a ragged batch long enough to be cut into several items per sequence; second: a smaller one
    # whose sequences are not cut at all, so nothing of the first call's work list may be read
    for ctx_before in ([2500, 17, 1200, 333, 2047, 1], [40, 300]):
        seed = 900 + len(ctx_before)
        ref_out, ref_pool, inputs, st = _reference_step(shape, ctx_before, seed)
        got_out, got_pool = _static_step(shape, ctx_before, seed, inputs)
        say(f"  batch {ctx_before}: split {st.ctx.okv_get_split_tokens()}, {len(st.ctx.okv_worklist(from_device=False))} items")
        assert torch.equal(ref_out.view(torch.int16 if ref_out.dtype == torch.float16 else torch.int32),
                           got_out.view(torch.int16 if got_out.dtype == torch.float16 else torch.int32))
        np.testing.assert_array_equal(ref_pool.view(np.uint16), got_pool.view(np.uint16))
        pairs = [(b, h) for b in range(len(ctx_before)) for h in range(0, st.H, 3)]
        ref = oracle_pairs(st, 0, inputs[0].cpu().numpy(), st.ctx_lens.copy(), pairs)
        got = got_out.float().cpu().numpy()
        assert_close(np.stack([got[b, h] for (b, h) in pairs]), np.stack([ref[p] for p in pairs]), "static entry")
        st.close()


def test_static_entry_point_refuses_what_does_not_fit():
    say("limits")
    dev = torch.device("cuda:0")
    dummy = torch.zeros(4096, dtype=torch.float16, device=dev)
    lens = torch.ones(4096, dtype=torch.int32, device=dev)
    kw = dict(n_q_heads=128, n_kv_heads=8, head_dim=128, block_tokens=16, max_blocks_per_seq=4, max_ctx=0, out_dtype=0,
              pool=dummy, block_table=lens, ctx_lens=lens, q=dummy, out=dummy)
    with pytest.raises(binding.OkvError) as e:                 # 128 query heads x 130 floats x (4000 + 128) items > 32 MiB
        binding.okv_decode_attn_static(B=4000, **kw)
    assert e.value.code == binding.OKV_ENOSPC and "work space" in str(e.value)
    with pytest.raises(binding.OkvError) as e:
        binding.okv_decode_attn_static(B=binding.OKV_STATIC_MAX_BATCH + 1, **kw)
    assert e.value.code == binding.OKV_EINVAL


def test_static_entry_point_in_a_captured_graph_replays_like_the_eager_calls():
    # what the entry point is for: a caller that captures a decode step into a HIP graph.  The graph holds a
    # length bump and the call; it is replayed several times with eager work and synchronisations in between,
    # and every replay is compared with the same steps made by eager calls on a second, identically filled pool.
    say("graph capture")
    from paper_2504_11816_amd.harness import new_stream
    shape = dict(H=8, G=2, d=128, T=16, cap_tokens=600, out_dtype=0)
    ctx_before = [300, 17, 129, 511]
    stacks, pools = [], []
    for _ in range(2):
        st = build_stack(L=1, ctx_before=ctx_before, seed=930, **shape)
        stacks.append(st)
    st = stacks[0]
    dev, B = st.device, len(ctx_before)
    q, k, v, _ = make_inputs(st, 931, 0, dev)
    q, k, v = q[0], k[0], v[0]
    table = torch.tensor(st.block_table, dtype=torch.int32, device=dev)
    raw, stream = new_stream(dev)

    def call(pool, lens, out):
        binding.okv_decode_attn_static(n_q_heads=st.H, n_kv_heads=st.G, head_dim=st.d, block_tokens=st.T,
                                       max_blocks_per_seq=st.max_blocks, max_ctx=st.max_ctx, out_dtype=0, B=B, pool=pool,
                                       block_table=table, ctx_lens=lens, q=q, out=out, k_new=k, v_new=v, stream=stream.cuda_stream)

    lens_g = torch.tensor(ctx_before, dtype=torch.int32, device=dev)
    lens_e = lens_g.clone()
    out_g = torch.zeros((B, st.H, st.d), dtype=torch.float16, device=dev)
    out_e = torch.zeros_like(out_g)
    warm = torch.zeros_like(out_g)
    call(stacks[1].dev_part[0], lens_e + 0, warm)               # first call on the device, outside any capture
    stream.synchronize()
    torch.cuda.synchronize()
    # (that warm call stored rows at positions ctx_before - 1 of the second pool: positions below every length,
    # overwritten identically in both pools below, since both get the same k / v at the same positions)
    call(stacks[0].dev_part[0], lens_g + 0, warm)
    stream.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        lens_g.add_(1)
        call(stacks[0].dev_part[0], lens_g, out_g)
    torch.cuda.synchronize()
    lens_g.copy_(torch.tensor(ctx_before, dtype=torch.int32))   # the capture ran nothing, but start from a known state
    for step in range(6):
        g.replay()
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            lens_e.add_(1)
        call(stacks[1].dev_part[0], lens_e, out_e)
        stream.synchronize()
        junk = torch.randn(1 << 16, device=dev).sum().item()   # eager work of the program's own between replays
        assert np.isfinite(junk)
        assert torch.equal(lens_g, lens_e), step
        assert torch.equal(out_g.view(torch.int16), out_e.view(torch.int16)), step
        out_g.zero_()
    np.testing.assert_array_equal(stacks[0].read_pool(0).view(np.uint16), stacks[1].read_pool(0).view(np.uint16))
    for s in stacks:
        s.close()
