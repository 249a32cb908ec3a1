"""The benchmark workloads at their full size and full depth, sampled: every one of the 32 layers, a few
(sequence, head) pairs per layer, at the steps the measurement plan names, element by element against the fp64
oracle (max abs error 2e-3 and relative L2 error 1e-2 per output vector: gpu_util.assert_close).  The launch
configuration is the one bench.py times: split size left to the library, outputs in fp16."""
import numpy as np
import pytest
import torch

from paper_2504_11816_amd import binding, synth
from paper_2504_11816_amd.harness import Stack

from gpu_util import run_and_check

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[full size] {msg}", flush=True)


def _stack(name, *, B, H, G, T, cap, on_host=None, L=32, seed=500):
    say(f"{name}: building {L} layers")
    st = Stack(L=L, H=H, G=G, d=128, B=B, T=T, cap_tokens=cap, on_host=on_host, out_dtype=0)
    for l in range(L):
        st.fill_pool(l, synth.stream_seed(seed, synth.TENSOR_POOL, l))
    table = None
    if T:
        table = synth.shuffled_block_table([st.cap_tokens] * B, T, st.blocks_per_layer, seed + 2,
                                           max_blocks_per_seq=st.max_blocks)
    return st, table


def test_cfg2_all_layers_first_middle_and_last_step():
    # 32 layers MHA 32 x 128, batch 32, contiguous pools of 1024 tokens; the steps that attend 513, 768 and 1024 keys
    st, _ = _stack("cfg2", B=32, H=32, G=32, T=0, cap=1024)
    pairs = [(0, 0), (13, 7), (31, 31), (5, 18)]
    for ctx_before in (512, 767, 1023):
        st.set_batch([ctx_before] * 32, None)
        say(f"  step to context {ctx_before + 1}, split {st.ctx.okv_get_split_tokens()}")
        run_and_check(st, n_steps=1, seed=510 + ctx_before, pairs=pairs)
    st.close()
    torch.cuda.empty_cache()


def test_cfg3_all_layers_half_on_the_host_two_steps():
    # batch 64, context 2048, 16-token blocks, 16 of the 32 layers in pinned host memory (32 GiB), streamed
    # through two staging buffers; an odd and an even step, so every staging buffer serves every host layer's parity
    on_host, n_off = binding.kv_offload_plan(32, 1, 2)
    assert n_off == 16
    st, table = _stack("cfg3", B=64, H=32, G=32, T=16, cap=2064, on_host=on_host, seed=520)
    st.set_batch([2046] * 64, table)
    run_and_check(st, n_steps=2, seed=522, pairs=[(0, 0), (63, 31), (20, 11)])
    st.close()
    torch.cuda.empty_cache()


def test_cfg4_all_layers_ragged_grouped_heads():
    # 32 query / 8 KV heads, batch 128, contexts uniform in [512, 4096], paged, all resident
    ctx = synth.ragged_ctx_lens(128, 512, 4096, 97) - 1
    shortest, longest = int(np.argmin(ctx)), int(np.argmax(ctx))
    st, table = _stack("cfg4", B=128, H=32, G=8, T=16, cap=4112, seed=530)
    st.set_batch(ctx, table)
    say(f"  contexts {int(ctx.min()) + 1}..{int(ctx.max()) + 1}, stretches of {st.ctx.okv_get_split_tokens()} keys, "
        f"{len(st.ctx.okv_worklist(from_device=False))} items")
    run_and_check(st, n_steps=2, seed=532, pairs=[(shortest, 0), (longest, 31), (64, 13), (1, 20)])
    st.close()
    torch.cuda.empty_cache()


def test_cfg5_shape_all_layers_reduced_batch():
    # context 4096, 20 of the 32 layers on the host (60 %), batch 16 of the 192 (the host share of the full batch
    # is 240 GiB of pinned memory; the per-sequence shape, the plan and the depth are the workload's own)
    on_host, n_off = binding.kv_offload_plan(32, 3, 5)
    assert n_off == 20
    st, table = _stack("cfg5 shape", B=16, H=32, G=32, T=16, cap=4112, on_host=on_host, seed=540)
    st.set_batch([4094] * 16, table)
    run_and_check(st, n_steps=2, seed=542, pairs=[(0, 0), (15, 31)])
    st.close()
    torch.cuda.empty_cache()


def test_cfg3_share_of_every_layer_on_the_host_newest_blocks_in_hbm_across_a_block_boundary():
    # batch 64, 16-token blocks, half of every layer's blocks in pinned host memory, whole sequences at a time
    # ("sequence" placement: the newest block of half of the sequences is a host block), streamed in 256 MiB
    # chunks.  18 steps from context 2041 to 2058 cross the block boundary at 2048: the rows appended on the way
    # live in HBM slots, the block is written to the host pool after step 8.  The oracle keeps the keys and values
    # of the sampled (layer, sequence, KV head) triples itself, so nothing is read back (and nothing flushed) on
    # the way; sampled outputs at four steps, the host pool's filled block bit for bit at the end.
    from fractions import Fraction
    from oracle import attention as oa, kv_layout
    from gpu_util import assert_close, make_inputs
    L, B, H, G, d, T = 32, 64, 32, 32, 128, 16
    cap = 2064
    need = B * synth.blocks_needed(cap, T)
    n_res, n_host = binding.okv_plan_block_split(need, 1, 2)
    shape = binding.make_config(n_layers=L, n_q_heads=H, n_kv_heads=G, head_dim=d, block_tokens=T, max_batch=B,
                                max_blocks_per_seq=synth.blocks_needed(cap, T), blocks_per_layer=need)
    chunk_blocks = (256 << 20) // binding.okv_block_bytes(shape)
    say(f"cfg3 blocks: building {L} layers, {n_host} of {need} blocks per layer on the host")
    st = Stack(L=L, H=H, G=G, d=d, B=B, T=T, cap_tokens=cap, out_dtype=0, blocks_per_layer=need,
               resident_blocks=n_res, chunk_blocks=chunk_blocks)
    assert st.hot_tails
    for l in range(L):
        st.fill_pool(l, synth.stream_seed(550, synth.TENSOR_POOL, l))
    table = synth.classed_block_table([st.cap_tokens] * B, T, n_res, n_host, n_host, "sequence", 551,
                                      max_blocks_per_seq=st.max_blocks)
    on_host = [b for b in range(B) if table[b, 2040 // T] >= n_res]
    in_hbm = [b for b in range(B) if table[b, 2040 // T] < n_res]
    assert on_host and in_hbm
    st.set_batch([2040] * B, table)
    layout = st.layout()
    pairs = [(on_host[0], 0), (on_host[-1], 31), (in_hbm[0], 17)]
    kept = {}                                              # (layer, b, g) -> [K rows, V rows] as the oracle holds them
    for l in range(L):
        for (b, h) in pairs:
            rows = [[kv_layout.token_row_offset(layout, b, kv, h, i) for i in range(2040)] for kv in (0, 1)]
            kept[(l, b, h)] = [st.read_rows(l, rows[0]), st.read_rows(l, rows[1])]
    for step in range(18):
        q, k, v, out = make_inputs(st, 553, step, st.device)
        st.step(q, k, v, out)
        for l in range(L):
            kl, vl = k[l].cpu().numpy(), v[l].cpu().numpy()
            for (b, h) in pairs:
                kept[(l, b, h)][0] = np.concatenate([kept[(l, b, h)][0], kl[b, h][None]])
                kept[(l, b, h)][1] = np.concatenate([kept[(l, b, h)][1], vl[b, h][None]])
        if step in (0, 7, 8, 17):
            st.synchronize()
            say(f"  step {step + 1}: context {2041 + step}")
            for l in range(L):
                got = out[l].float().cpu().numpy()
                ql = q[l].cpu().numpy()
                for (b, h) in pairs:
                    K, V = kept[(l, b, h)]
                    ref = oa.attend_one(oa.as_f64(ql[b, h]), oa.as_f64(K), oa.as_f64(V))
                    assert_close(got[b, h][None], ref[None], f"step {step} layer {l} pair {(b, h)}")
    # the block that step 8 filled is in the host pool although nothing asked for a flush
    st.synchronize()
    for l in (0, 31):
        host = st.host_part[l].numpy()
        for (b, h) in pairs[:2]:
            for kv in (0, 1):
                for i in (2040, 2047):
                    at = kv_layout.token_row_offset(layout, b, kv, h, i) - st.split_at
                    np.testing.assert_array_equal(host[at:at + d].view(np.uint16), kept[(l, b, h)][kv][i].view(np.uint16))
    st.close()
    torch.cuda.empty_cache()
