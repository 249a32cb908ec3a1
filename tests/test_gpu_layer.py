"""GPU parity for the linear layers around the attention: weight rearrangement bit-exact,
okv_linear and okv_layernorm against the fp64 oracle on the same fp16 inputs, and whole decoder
layers (with the attention and the KV cache in between) against the oracle rounding to fp16
where the GPU stores fp16.

Tolerance of one product or layer norm: |gpu - oracle| <= 2e-3 + 2e-3 |oracle| per element
(fp16 inputs are exact in fp32, sums of up to 16384 terms in fp32, one rounding to fp16 of
results of size O(1..8)).  Whole layers: 1.5e-2 + 1.5e-2 |oracle| (a different rounding decision at one
fp16 store moves a value by 2^-11 relative, and four products and two norms follow one another)."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import decode_layer as dl
from oracle import kv_layout
from paper_2504_11816_amd import binding, synth
from paper_2504_11816_amd.harness import BoundLayers, LayerScratch, LayerWeights, decode_step_with_layers

from gpu_util import build_stack

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def close(got, want, atol=2e-3, rtol=2e-3, what=""):
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape and np.all(np.isfinite(got)), what
    err = np.abs(got - want) - rtol * np.abs(want)
    assert err.max() <= atol, f"{what}: worst excess {err.max():.3e} over {atol}"


def packed_layout(w):
    """The rearrangement okv_pack_linear_weight is specified to produce, written with plain loops."""
    n_out, n_in = w.shape
    out = np.empty(n_out * n_in, dtype=w.dtype)
    at = 0
    for nt in range(n_out // 16):
        for kb in range(n_in // 32):
            for lane in range(64):
                n, k = 16 * nt + lane % 16, 32 * kb + 8 * (lane // 16)
                out[at:at + 8] = w[n, k:k + 8]
                at += 8
    return out


@pytest.mark.parametrize("n_out,n_in", [(16, 32), (48, 96), (256, 1024)])
def test_weight_rearrangement_is_bit_exact(n_out, n_in):
    say(f"pack {n_out}x{n_in}")
    w = synth.randn_f16_torch((n_out, n_in), synth.stream_seed(301, 1), DEV)
    dst = torch.zeros_like(w)
    binding.okv_pack_linear_weight(dst, w, n_out, n_in)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(dst.cpu().numpy().reshape(-1).view(np.uint16), packed_layout(w.cpu().numpy()).view(np.uint16))


_WS = {}


def workspace(nbytes):
    """A workspace of at least nbytes, shared by the tests (calls follow one another)."""
    if "t" not in _WS or _WS["t"].numel() < nbytes:
        _WS["t"] = torch.empty(max(nbytes, 1 << 22), dtype=torch.uint8, device=DEV)
    return _WS["t"]


def run_linear(m, n_out, n_in, seed, bias=True, relu=False, residual=False, n_seg=1, fast=True):
    x = synth.randn_f16_torch((m, n_in), synth.stream_seed(seed, 1), DEV)
    w = (synth.randn_f16_torch((n_out, n_in), synth.stream_seed(seed, 2), DEV).float() / n_in ** 0.5).to(torch.float16)
    b = synth.randn_f16_torch((n_out,), synth.stream_seed(seed, 3), DEV) if bias else None
    r = synth.randn_f16_torch((m, n_out), synth.stream_seed(seed, 4), DEV) if residual else None
    wp = torch.empty_like(w)
    binding.okv_pack_linear_weight(wp, w, n_out, n_in)
    outs = [torch.full((m, n_out // n_seg), float("nan"), dtype=torch.float16, device=DEV) for _ in range(n_seg)]
    if fast:
        nb = binding.okv_linear_workspace_bytes(m, n_out, n_in)
        ws = workspace(nb)
        ws.fill_(0xFF)                                           # what the workspace held before means nothing (NaN bits)
        binding.okv_linear(x, wp, b, r, outs, m, n_out, n_in, relu, 0, ws, ws.numel())
        torch.cuda.synchronize()
    else:
        binding.okv_linear(x, wp, b, r, outs, m, n_out, n_in, relu)
        torch.cuda.synchronize()
    want = dl.linear(x.double().cpu().numpy(), w.double().cpu().numpy(), None if b is None else b.double().cpu().numpy())
    if relu:
        want = dl.relu(want)
    if residual:
        want = want + r.double().cpu().numpy()
    got = np.concatenate([o.float().cpu().numpy() for o in outs], axis=1)
    close(got, want, what=f"linear m={m} {n_out}x{n_in}")


@pytest.mark.parametrize("m", [1, 5, 16, 17, 32, 33, 64, 100, 128])
def test_linear_every_row_count(m):
    say(f"linear m={m}")
    run_linear(m, 96, 320, 311 + m)                      # 10 blocks of 32 inputs: uneven shares for the 8 wavefronts
    run_linear(m, 64, 2048, 411 + m, relu=True)


@pytest.mark.parametrize("n_out,n_in", [(16, 32), (32, 64), (48, 4096), (4096, 256), (144, 992), (128, 256), (272, 512),
                                        (2560, 2560), (16, 8192)])
def test_linear_shapes(n_out, n_in):
    say(f"linear {n_out}x{n_in}")
    run_linear(32, n_out, n_in, 321)
    run_linear(7, n_out, n_in, 322, bias=False)
    run_linear(32, n_out, n_in, 323, fast=False)              # the kernel that needs no workspace


@pytest.mark.parametrize("m,n_out,n_in,relu", [(32, 4096, 4096, False), (20, 256, 512, True), (64, 2560, 2560, False),
                                               (8, 256, 512, False), (32, 192, 320, False), (33, 16384, 256, False),
                                               (192, 1024, 2048, True), (150, 4096, 1024, False)])
def test_linear_followed_by_layernorm_in_one_call(m, n_out, n_in, relu):
    # fast path (the norm rides on the share reduction), few rows and odd input sizes (two kernels): same contract
    say(f"linear+layernorm m={m} {n_out}x{n_in}")
    x = synth.randn_f16_torch((m, n_in), synth.stream_seed(381, 1), DEV)
    w = (synth.randn_f16_torch((n_out, n_in), synth.stream_seed(381, 2), DEV).float() / n_in ** 0.5).to(torch.float16)
    b = synth.randn_f16_torch((n_out,), synth.stream_seed(381, 3), DEV)
    r = synth.randn_f16_torch((m, n_out), synth.stream_seed(381, 4), DEV)
    g = (1.0 + 0.2 * synth.randn_f16_torch((n_out,), synth.stream_seed(381, 5), DEV).float()).to(torch.float16)
    be = (0.3 * synth.randn_f16_torch((n_out,), synth.stream_seed(381, 6), DEV).float()).to(torch.float16)
    wp = torch.empty_like(w)
    binding.okv_pack_linear_weight(wp, w, n_out, n_in)
    y = torch.full((m, n_out), float("nan"), dtype=torch.float16, device=DEV)
    z = torch.full((m, n_out), float("nan"), dtype=torch.float16, device=DEV)
    ws = workspace(binding.okv_linear_workspace_bytes(m, n_out, n_in))
    ws.fill_(0xFF)
    binding.okv_linear_layernorm(x, wp, b, r, y, g, be, z, m, n_out, n_in, 1e-5, relu, 0, ws, ws.numel())
    torch.cuda.synchronize()
    want_y = dl.linear(x.double().cpu().numpy(), w.double().cpu().numpy(), b.double().cpu().numpy())
    if relu:
        want_y = dl.relu(want_y)
    want_y = want_y + r.double().cpu().numpy()
    close(y.float().cpu().numpy(), want_y, what="product")
    # the norm is defined on the stored (fp16) result
    want_z = dl.layernorm(y.double().cpu().numpy(), g.double().cpu().numpy(), be.double().cpu().numpy(), 1e-5)
    close(z.float().cpu().numpy(), want_z, what="norm of the product")
    # the two separate calls give the same product bit for bit and the same norm up to its fp32 rounding
    y2, z2 = torch.empty_like(y), torch.empty_like(z)
    binding.okv_linear(x, wp, b, r, y2, m, n_out, n_in, relu, 0, ws, ws.numel())
    binding.okv_layernorm(y2, g, be, z2, m, n_out, 1e-5)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    assert (z.float() - z2.float()).abs().max().item() <= 2e-3
    with pytest.raises(binding.OkvError):
        binding.okv_linear_layernorm(x, wp, b, r, y, g, be, y, m, n_out, n_in)        # out and out_norm must differ


def test_linear_results_do_not_depend_on_arrival_order():
    say("linear determinism")
    m, n_out, n_in = 32, 4096, 4096
    x = synth.randn_f16_torch((m, n_in), synth.stream_seed(371, 1), DEV)
    w = (synth.randn_f16_torch((n_out, n_in), synth.stream_seed(371, 2), DEV).float() / 64).to(torch.float16)
    wp = torch.empty_like(w)
    binding.okv_pack_linear_weight(wp, w, n_out, n_in)
    ws = workspace(binding.okv_linear_workspace_bytes(m, n_out, n_in))
    first = None
    for _ in range(20):
        out = torch.empty((m, n_out), dtype=torch.float16, device=DEV)
        binding.okv_linear(x, wp, None, None, out, m, n_out, n_in, False, 0, ws, ws.numel())
        torch.cuda.synchronize()
        if first is None:
            first = out
        assert torch.equal(out, first)


def test_linear_epilogue_variants():
    say("linear epilogue")
    run_linear(32, 192, 512, 331, bias=True, relu=True, residual=True)
    run_linear(32, 192, 512, 332, bias=False, relu=False, residual=True)
    run_linear(20, 192, 512, 333, n_seg=3)
    run_linear(20, 192, 512, 334, n_seg=2, relu=True)
    # residual aliasing the output: y = y + x W^T
    m, n = 24, 128
    x = synth.randn_f16_torch((m, 256), synth.stream_seed(335, 1), DEV)
    w = (synth.randn_f16_torch((n, 256), synth.stream_seed(335, 2), DEV).float() / 16).to(torch.float16)
    y = synth.randn_f16_torch((m, n), synth.stream_seed(335, 3), DEV)
    y0 = y.double().cpu().numpy()
    wp = torch.empty_like(w)
    binding.okv_pack_linear_weight(wp, w, n, 256)
    binding.okv_linear(x, wp, None, y, y, m, n, 256)
    torch.cuda.synchronize()
    close(y.float().cpu().numpy(), y0 + dl.linear(x.double().cpu().numpy(), w.double().cpu().numpy()), what="aliased residual")


@pytest.mark.parametrize("n_out", [12288, 12272, 11520])
def test_linear_workgroups_of_three_streaming_wavefronts(n_out):
    # feature counts for which three 16-feature tiles per workgroup fill the 256 compute units without a cut of the
    # inputs; 12272 = 767 tiles leaves the last workgroup one tile short
    say(f"linear three-wavefront form {n_out}")
    assert binding.okv_linear_workspace_bytes(32, n_out, 1024) == 32 * n_out * 4       # one share (for a layer norm to follow): no cut
    run_linear(32, n_out, 1024, 341, relu=True, residual=True)
    run_linear(40, n_out, 1024, 342)


def test_linear_full_size_projection_and_feed_forward():
    say("linear full size")
    run_linear(32, 4096, 4096, 341)
    run_linear(64, 12288, 4096, 342, n_seg=3)
    run_linear(32, 16384, 4096, 343, relu=True)
    run_linear(32, 4096, 16384, 344, residual=True)
    run_linear(128, 4096, 4096, 345)


@pytest.mark.parametrize("m,h", [(1, 8), (3, 64), (32, 2560), (64, 4096), (5, 16384), (128, 768)])
def test_layernorm(m, h):
    say(f"layernorm {m}x{h}")
    x = (3.0 * synth.randn_f16_torch((m, h), synth.stream_seed(351, 1), DEV).float() + 1.5).to(torch.float16)
    g = (1.0 + 0.2 * synth.randn_f16_torch((h,), synth.stream_seed(351, 2), DEV).float()).to(torch.float16)
    b = (0.3 * synth.randn_f16_torch((h,), synth.stream_seed(351, 3), DEV).float()).to(torch.float16)
    out = torch.full((m, h), float("nan"), dtype=torch.float16, device=DEV)
    binding.okv_layernorm(x, g, b, out, m, h, 1e-5)
    torch.cuda.synchronize()
    want = dl.layernorm(x.double().cpu().numpy(), g.double().cpu().numpy(), b.double().cpu().numpy(), 1e-5)
    close(out.float().cpu().numpy(), want, what=f"layernorm {m}x{h}")
    # in place
    binding.okv_layernorm(x, g, b, x, m, h, 1e-5)
    torch.cuda.synchronize()
    assert torch.equal(x, out)


@pytest.mark.parametrize("T,on_host,G", [(0, None, 4), (16, [0, 1], 4), (16, None, 2), (0, None, 1)])
def test_whole_decoder_layers_against_the_oracle(T, on_host, G):
    say(f"decoder layers T={T} on_host={on_host} G={G}")
    L, H, d, B = 2, 4, 64, 5
    h1, h2 = H * d, 4 * H * d
    ctx = [3, 40, 100, 17, 64]
    st = build_stack(L=L, H=H, G=G, d=d, T=T, ctx_before=ctx, cap_tokens=128, on_host=on_host, seed=361)
    weights = [LayerWeights(h1, h2, 363, l, st.device, kv_cols=G * d) for l in range(L)]
    scratch = LayerScratch(B, h1, h2, G, d, st.device)
    layout = st.layout()
    pools = [st.read_pool(l).copy() for l in range(L)]
    n = np.array(ctx, dtype=np.int32)
    for step in range(2):
        x = synth.randn_f16_torch((B, h1), synth.stream_seed(365, 1, 0, step), st.device)
        x_ref = x.double().cpu().numpy()
        decode_step_with_layers(st, weights, scratch, x)
        st.synchronize()
        n = n + 1
        for l in range(L):
            p = weights[l].numpy()
            q, k, v = dl.qkv(x_ref, p, fp16_between=True)
            kv_layout.append_scatter(pools[l], layout, n, k.astype(np.float16).reshape(B, G, d), v.astype(np.float16).reshape(B, G, d))
            t = oa.decode_attn(q.reshape(B, H, d), pools[l], layout, n, H)
            t = dl.round16(np.asarray(t).reshape(B, h1))
            x_ref = dl.after_attention(x_ref, t, p, fp16_between=True)
        close(x.float().cpu().numpy(), x_ref, atol=1.5e-2, rtol=1.5e-2, what=f"step {step}")
        # the cache holds the keys and values the oracle's projections produce (fp16 rounding decisions may differ by an ulp)
        for l in range(L):
            got = st.read_pool(l).astype(np.float64)
            assert np.abs(got - pools[l].astype(np.float64)).max() < 2e-2
    st.close()


@pytest.mark.parametrize("T,G", [(0, 4), (16, 4), (16, 2)])
def test_decoder_step_in_one_call_equals_the_calls_one_by_one(T, G):
    # okv_decoder_step issues the same launches as the six calls per layer: same bits in x and in the cache
    say(f"decoder step in one call T={T} G={G}")
    L, H, d, B = 3, 4, 64, 6
    h1, h2 = H * d, 4 * H * d
    ctx = [3, 40, 100, 17, 64, 1]
    results = []
    for one_call in (False, True):
        st = build_stack(L=L, H=H, G=G, d=d, T=T, ctx_before=ctx, cap_tokens=128, seed=371)
        weights = [LayerWeights(h1, h2, 373, l, st.device, kv_cols=G * d) for l in range(L)]
        scratch = LayerScratch(B, h1, h2, G, d, st.device)
        bound = BoundLayers(st, weights, scratch) if one_call else None
        xs = []
        for step in range(3):
            x = synth.randn_f16_torch((B, h1), synth.stream_seed(375, 1, 0, step), st.device)
            if one_call:
                bound.step(x)
            else:
                decode_step_with_layers(st, weights, scratch, x)
            st.synchronize()
            xs.append(x.cpu().numpy().view(np.uint16).copy())
        results.append((xs, [st.read_pool(l).view(np.uint16).copy() for l in range(L)], st.ctx_lens.copy()))
        st.close()
    for a, b in zip(results[0][0], results[1][0]):
        np.testing.assert_array_equal(a, b)
    for a, b in zip(results[0][1], results[1][1]):
        np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(results[0][2], results[1][2])


def test_decoder_step_rejects_what_it_cannot_run():
    say("decoder step errors")
    L, H, d, B = 2, 4, 64, 2
    h1, h2 = H * d, 4 * H * d
    st = build_stack(L=L, H=H, G=H, d=d, T=0, ctx_before=[5, 9], cap_tokens=64, seed=381)
    weights = [LayerWeights(h1, h2, 383, l, st.device) for l in range(L)]
    scratch = LayerScratch(B, h1, h2, H, d, st.device)
    bound = BoundLayers(st, weights, scratch)
    x = synth.randn_f16_torch((B, h1), synth.stream_seed(385, 1), st.device)
    with pytest.raises(binding.OkvError):                     # scratch too small
        st.ctx.okv_decoder_step(bound.layers, h2, x, bound.scratch, bound.scratch_bytes - 256, scratch.ws, scratch.ws_bytes)
    short = binding.Context.decoder_layers([{}])               # one layer of NULL pointers for a two-layer context
    with pytest.raises(binding.OkvError):
        st.ctx.okv_decoder_step(short, h2, x, bound.scratch, bound.scratch_bytes, scratch.ws, scratch.ws_bytes)
    bound.step(x)                                              # and the context is still usable afterwards
    st.synchronize()
    assert torch.isfinite(x.float()).all()
    st.close()
    # a context that writes fp32 attention outputs cannot feed the output projection
    st = build_stack(L=1, H=4, G=4, d=64, T=0, ctx_before=[5, 9], cap_tokens=64, seed=387, out_dtype=1)
    with pytest.raises(binding.OkvError):
        BoundLayers(st, weights[:1], scratch).step(x)
    st.close()


def test_linear_qkv_widths():
    # the stacked projection with narrower keys and values, against three separate products
    say("linear qkv")
    m, h1, kv, n_in = 24, 512, 128, 512
    x = synth.randn_f16_torch((m, n_in), synth.stream_seed(391, 1), DEV)
    w = (synth.randn_f16_torch((h1 + 2 * kv, n_in), synth.stream_seed(391, 2), DEV).float() / n_in ** 0.5).to(torch.float16)
    b = synth.randn_f16_torch((h1 + 2 * kv,), synth.stream_seed(391, 3), DEV)
    wp = torch.empty_like(w)
    binding.okv_pack_linear_weight(wp, w, h1 + 2 * kv, n_in)
    q = torch.full((m, h1), float("nan"), dtype=torch.float16, device=DEV)
    k = torch.full((m, kv), float("nan"), dtype=torch.float16, device=DEV)
    v = torch.full((m, kv), float("nan"), dtype=torch.float16, device=DEV)
    for mm in (m, 5):                                          # the staged kernel and the one for few rows
        ws = workspace(binding.okv_linear_workspace_bytes(mm, h1 + 2 * kv, n_in))
        binding.okv_linear_qkv(x, wp, b, q, k, v, mm, h1, kv, n_in, 0, ws, ws.numel())
        torch.cuda.synchronize()
        want = dl.linear(x[:mm].double().cpu().numpy(), w.double().cpu().numpy(), b.double().cpu().numpy())
        close(q[:mm].float().cpu().numpy(), want[:, :h1], what="q")
        close(k[:mm].float().cpu().numpy(), want[:, h1:h1 + kv], what="k")
        close(v[:mm].float().cpu().numpy(), want[:, h1 + kv:], what="v")
    with pytest.raises(binding.OkvError):
        binding.okv_linear_qkv(x, wp, b, q, k, v, m, h1, 24, n_in)          # widths are multiples of 16


def test_linear_random_shapes_against_the_oracle():
    # every row-fragment count (1..8 fragments of 16 rows), both workgroup forms, cuts or none, the kernel for few
    # rows and for input sizes the staged kernel does not take, with a random epilogue
    say("linear random shapes")
    rng = np.random.Generator(np.random.PCG64(20250427))
    cases = []
    for m in (9, 16, 17, 32, 33, 48, 49, 64, 65, 80, 81, 96, 97, 112, 113, 128):      # each fragment count at both ends
        n_in = int(rng.choice([256, 512, 768, 1024, 2048, 2560]))
        n_out = 16 * int(rng.integers(1, 129))
        cases.append((m, n_out, n_in))
    for m in (24, 72, 128):                                   # wide products: three streaming wavefronts per workgroup
        cases.append((m, 16 * int(rng.integers(700, 769)), 512 * int(rng.integers(2, 5))))
        cases.append((m, 6144, 1024))
    for _ in range(8):                                        # anything else
        cases.append((int(rng.integers(1, 129)), 16 * int(rng.integers(1, 200)), 32 * int(rng.integers(1, 100))))
    for i, (m, n_out, n_in) in enumerate(cases):
        say(f"  m={m} {n_out}x{n_in}")
        run_linear(m, n_out, n_in, 500 + i, bias=bool(rng.integers(0, 2)), relu=bool(rng.integers(0, 2)),
                   residual=bool(rng.integers(0, 2)))


@pytest.mark.parametrize("m", [129, 144, 145, 160, 161, 176, 177, 192])
def test_linear_129_to_192_rows_in_one_launch(m):
    # 9 to 12 fragments of 16 rows: one launch of the staged kernel when the input width is a multiple of 256,
    # both workgroup forms, with cuts (and the norm on the share reduction) or without
    say(f"linear one launch m={m}")
    run_linear(m, 12288 // 8, 512, 800 + m, n_seg=3)                       # three streaming wavefronts, no cut
    run_linear(m, 1024, 1024, 810 + m, bias=True, relu=True, residual=True)
    run_linear(m, 256, 2048, 820 + m, residual=True)
    run_linear(m, 2048, 256, 830 + m, relu=True)


@pytest.mark.parametrize("m", [129, 192, 193, 300, 400])
def test_linear_more_rows_than_one_launch_takes(m):
    # beyond what one launch takes (192 rows for the staged kernel, 128 otherwise) a call issues several launches
    # of nearly equal size; same contract
    say(f"linear m={m}")
    run_linear(m, 320, 512, 700 + m, relu=True, residual=True)
    run_linear(m, 96, 1024, 710 + m, n_seg=3)
    run_linear(m, 64, 96, 720 + m)                            # the kernel for odd input sizes


def test_decoder_step_with_a_batch_of_more_than_128():
    say("decoder step batch 160")
    L, H, G, d, B = 2, 4, 2, 64, 160
    h1, h2 = H * d, 4 * H * d
    ctx = list(np.random.Generator(np.random.PCG64(5)).integers(1, 60, size=B))
    results = []
    for one_call in (False, True):
        st = build_stack(L=L, H=H, G=G, d=d, T=16, ctx_before=ctx, cap_tokens=64, seed=731)
        weights = [LayerWeights(h1, h2, 733, l, st.device, kv_cols=G * d) for l in range(L)]
        scratch = LayerScratch(B, h1, h2, G, d, st.device)
        x = synth.randn_f16_torch((B, h1), synth.stream_seed(735, 1), st.device)
        x_ref = x.double().cpu().numpy()
        if one_call:
            BoundLayers(st, weights, scratch).step(x)
        else:
            decode_step_with_layers(st, weights, scratch, x)
        st.synchronize()
        results.append(x.cpu().numpy().view(np.uint16).copy())
        if not one_call:                                      # against the oracle once
            layout = st.layout()
            n = np.array(ctx, dtype=np.int32) + 1
            pools = None
            st2 = build_stack(L=L, H=H, G=G, d=d, T=16, ctx_before=ctx, cap_tokens=64, seed=731)
            pools = [st2.read_pool(l).copy() for l in range(L)]
            st2.close()
            for l in range(L):
                p = weights[l].numpy()
                q, k, v = dl.qkv(x_ref, p, fp16_between=True)
                kv_layout.append_scatter(pools[l], layout, n, k.astype(np.float16).reshape(B, G, d), v.astype(np.float16).reshape(B, G, d))
                t = oa.decode_attn(q.reshape(B, H, d), pools[l], layout, n, H)
                x_ref = dl.after_attention(x_ref, dl.round16(np.asarray(t).reshape(B, h1)), p, fp16_between=True)
            close(x.float().cpu().numpy(), x_ref, atol=1.5e-2, rtol=1.5e-2, what="batch 160")
        st.close()
    np.testing.assert_array_equal(results[0], results[1])
