"""Helpers for the GPU parity tests: build a Stack, feed it seeded inputs, and
evaluate the CPU oracle on the very bytes the GPU read."""
import numpy as np
import torch

from oracle import attention as oa
from oracle import kv_layout
from paper_2504_11816_amd import synth
from paper_2504_11816_amd.harness import Stack

ATOL = 2e-3      # max abs error (fp16 KV, fp32 accumulation)
RTOL_L2 = 1e-2   # per output vector, ||gpu - oracle||_2 / ||oracle||_2


def assert_close(gpu, ref, what=""):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape
    assert np.all(np.isfinite(gpu)), f"{what}: non-finite GPU output"
    err = np.abs(gpu - ref).max()
    assert err <= ATOL, f"{what}: max abs error {err:.3e} > {ATOL}"
    num = np.linalg.norm((gpu - ref).reshape(-1, ref.shape[-1]), axis=1)
    den = np.linalg.norm(ref.reshape(-1, ref.shape[-1]), axis=1)
    rel = (num / np.maximum(den, 1e-30)).max()
    assert rel <= RTOL_L2, f"{what}: relative L2 error {rel:.3e} > {RTOL_L2}"
    return err, rel


def oracle_pairs(stack, layer, q_np, ctx_lens, pairs):
    """Oracle outputs for the sampled (b, h) pairs; rows are fetched from the
    stack's pool at the offsets the oracle's own indexing computes."""
    layout = stack.layout()
    group = stack.H // stack.G
    out = {}
    for (b, h) in pairs:
        g = h // group
        n = int(ctx_lens[b])
        ok = [kv_layout.token_row_offset(layout, b, 0, g, i) for i in range(n)]
        ov = [kv_layout.token_row_offset(layout, b, 1, g, i) for i in range(n)]
        K = oa.as_f64(stack.read_rows(layer, ok))
        V = oa.as_f64(stack.read_rows(layer, ov))
        out[(b, h)] = oa.attend_one(oa.as_f64(q_np[b, h]), K, V)
    return out


def make_inputs(stack, seed, step, device):
    """Per-layer q / k_new / v_new for one step, each from its own stream."""
    L, B, H, G, d = stack.L, stack.B, stack.H, stack.G, stack.d
    q = [synth.randn_f16_torch((B, H, d), synth.stream_seed(seed, synth.TENSOR_Q, l, step), device) for l in range(L)]
    k = [synth.randn_f16_torch((B, G, d), synth.stream_seed(seed, synth.TENSOR_KNEW, l, step), device) for l in range(L)]
    v = [synth.randn_f16_torch((B, G, d), synth.stream_seed(seed, synth.TENSOR_VNEW, l, step), device) for l in range(L)]
    out = [torch.full((B, H, d), float("nan"), dtype=stack.out_torch_dtype, device=device) for _ in range(L)]
    torch.cuda.synchronize()
    return q, k, v, out


def build_stack(*, L, H, G, d, T, ctx_before, cap_tokens=None, on_host=None, out_dtype=0, split_tokens=0,
                seed=0, shuffle_seed=1, n_staging=2, extra_blocks=3):
    """A Stack whose pools hold N(0,1) everywhere (distinct per layer) and whose
    batch holds ctx_before[b] tokens per sequence."""
    ctx_before = np.asarray(ctx_before, dtype=np.int32)
    B = len(ctx_before)
    cap = cap_tokens or int(ctx_before.max()) + 8
    blocks = None
    if T:
        per = synth.blocks_needed(cap, T)
        blocks = B * per + extra_blocks
    st = Stack(L=L, H=H, G=G, d=d, B=B, T=T, cap_tokens=cap, on_host=on_host, out_dtype=out_dtype,
               split_tokens=split_tokens, blocks_per_layer=blocks, n_staging=n_staging)
    for l in range(L):
        st.fill_pool(l, synth.stream_seed(seed, synth.TENSOR_POOL, l))
    table = None
    if T:
        table = synth.shuffled_block_table([st.cap_tokens] * B, T, st.blocks_per_layer, shuffle_seed,
                                           max_blocks_per_seq=st.max_blocks)
    st.set_batch(ctx_before, table)
    return st


def run_and_check(st, n_steps=1, seed=0, pairs=None, check_layers=None):
    """Run n_steps decode steps; after each, compare every (or the sampled)
    output with the oracle.  Returns the list of GPU outputs per step."""
    dev = st.device
    results = []
    for step in range(n_steps):
        q, k, v, out = make_inputs(st, seed, step, dev)
        st.step(q, k, v, out)
        st.synchronize()
        outs = [o.float().cpu().numpy() for o in out]
        results.append(outs)
        n_now = st.ctx_lens.copy()
        todo = pairs or [(b, h) for b in range(st.B) for h in range(st.H)]
        for l in (check_layers if check_layers is not None else range(st.L)):
            ref = oracle_pairs(st, l, q[l].cpu().numpy(), n_now, todo)
            got = np.stack([outs[l][b, h] for (b, h) in todo])
            want = np.stack([ref[p] for p in todo])
            assert_close(got, want, f"step {step} layer {l}")
    return results
