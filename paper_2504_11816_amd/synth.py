"""Seeded synthetic inputs: shapes and value distributions of the workloads.

This module holds none of the method's arithmetic.  It only draws numbers:
fp16 N(0,1) tensors for q / K / V, a shuffled block table, ragged context
lengths, and the table of workload shapes.  Both the tests' CPU oracle and
the GPU path are fed from here, so they see the same bytes.

The paper's workloads are fixed token-length patterns (online: 128 prompt /
512 generated; offline: 1024 prompt / 128 generated, §VI-A) run on OPT
models; the shapes below keep the OPT-6.7B-like stack (32 layers, 32 heads of
128) and scale batch and context to a 288 GB GPU.
"""
import numpy as np

_MASK64 = (1 << 64) - 1


def stream_seed(seed, tensor_id, layer=0, step=0):
    """A distinct 63-bit seed per (run seed, tensor, layer, step).

    splitmix64-style mixing of the four integers; any fixed bijective mixing
    would do, the point is that no two tensors share a random stream.
    """
    x = (seed * 0x9E3779B97F4A7C15 + tensor_id * 0xBF58476D1CE4E5B9
         + layer * 0x94D049BB133111EB + step * 0xD6E8FEB86659FD93 + 0x2545F4914F6CDD1D) & _MASK64
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & _MASK64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & _MASK64
    x ^= x >> 31
    return x & ((1 << 63) - 1)


TENSOR_K, TENSOR_V, TENSOR_Q, TENSOR_KNEW, TENSOR_VNEW, TENSOR_POOL = 1, 2, 3, 4, 5, 6


def randn_f16_numpy(shape, seed):
    """N(0,1) rounded to fp16, on the host (numpy Generator, PCG64)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.standard_normal(size=shape, dtype=np.float32).astype(np.float16)


def randn_f16_torch(shape, seed, device):
    """N(0,1) rounded to fp16 as a torch tensor on `device` (its own generator)."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(torch.float16)


def fill_randn_f16_(tensor, seed, chunk_elems=1 << 28):
    """Fill an existing fp16 torch tensor (device or pinned host) with N(0,1),
    chunk by chunk so that no fp32 copy of the whole tensor is ever alive."""
    import torch
    flat = tensor.view(-1)
    dev = flat.device
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    n = flat.numel()
    for lo in range(0, n, chunk_elems):
        hi = min(n, lo + chunk_elems)
        flat[lo:hi] = torch.randn(hi - lo, generator=gen, device=dev, dtype=torch.float32).to(torch.float16)
    return tensor


def ragged_ctx_lens(B, lo, hi, seed):
    """B integers uniform in [lo, hi], both ends included."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(lo, hi + 1, size=B, dtype=np.int64).astype(np.int32)


def blocks_needed(ctx_cap, T):
    return (int(ctx_cap) + T - 1) // T


def shuffled_block_table(ctx_caps, T, blocks_per_layer, seed, max_blocks_per_seq=None):
    """A seeded random permutation of [0, blocks_per_layer) dealt to the
    sequences in order (sequence 0 first), enough blocks for each sequence's
    capacity ctx_caps[b]; unused entries are -1.  Returns int32 [B][max_blocks].
    """
    need = [blocks_needed(c, T) for c in ctx_caps]
    if max_blocks_per_seq is None:
        max_blocks_per_seq = max(need)
    if sum(need) > blocks_per_layer:
        raise ValueError("pool too small for the requested capacities")
    rng = np.random.Generator(np.random.PCG64(seed))
    perm = rng.permutation(blocks_per_layer).astype(np.int32)
    table = np.full((len(ctx_caps), max_blocks_per_seq), -1, dtype=np.int32)
    at = 0
    for b, k in enumerate(need):
        table[b, :k] = perm[at:at + k]
        at += k
    return table


def identity_block_table(ctx_caps, T, max_blocks_per_seq=None):
    """Blocks handed out in order, no shuffle (block b*k+i for sequence b)."""
    need = [blocks_needed(c, T) for c in ctx_caps]
    if max_blocks_per_seq is None:
        max_blocks_per_seq = max(need)
    table = np.full((len(ctx_caps), max_blocks_per_seq), -1, dtype=np.int32)
    at = 0
    for b, k in enumerate(need):
        table[b, :k] = np.arange(at, at + k, dtype=np.int32)
        at += k
    return table


def classed_block_table(ctx_caps, T, resident_blocks, host_blocks, n_host_used, policy, seed,
                        max_blocks_per_seq=None):
    """A block table for a pool whose ids below resident_blocks are in HBM and whose
    other ids (host_blocks of them) are in host memory.  n_host_used of the blocks the
    sequences need are taken from the host part, the rest from the HBM part:
      "prefix"    every sequence keeps its oldest blocks on the host, an even share of
                  n_host_used each (by a running quota), handed out in id order; its
                  newest blocks are in HBM, shuffled;
      "sequence"  whole sequences go to the host, in order, while n_host_used lasts
                  (the sequence at the boundary is cut like "prefix");
      "scatter"   a random choice of n_host_used block positions over all sequences,
                  ids shuffled in both parts (worst case: many short stretches).
    Returns int32 [B][max_blocks]; unused entries are -1."""
    need = [blocks_needed(c, T) for c in ctx_caps]
    total = sum(need)
    if max_blocks_per_seq is None:
        max_blocks_per_seq = max(need)
    if not (0 <= n_host_used <= min(total, host_blocks)) or total - n_host_used > resident_blocks:
        raise ValueError("the requested split does not fit the two parts of the pool")
    rng = np.random.Generator(np.random.PCG64(seed))
    on_host = [np.zeros(k, dtype=bool) for k in need]
    if policy == "prefix":
        cum = 0
        for b, k in enumerate(need):
            share = ((cum + k) * n_host_used) // total - (cum * n_host_used) // total if total else 0
            on_host[b][:share] = True
            cum += k
    elif policy == "sequence":
        left = n_host_used
        for b, k in enumerate(need):
            take = min(k, left)
            on_host[b][:take] = True
            left -= take
    elif policy == "scatter":
        flat = np.zeros(total, dtype=bool)
        flat[rng.choice(total, size=n_host_used, replace=False)] = True
        at = 0
        for b, k in enumerate(need):
            on_host[b] = flat[at:at + k]
            at += k
    else:
        raise ValueError(f"unknown policy {policy}")
    res_ids = rng.permutation(resident_blocks).astype(np.int64)
    host_ids = np.arange(host_blocks, dtype=np.int64)
    if policy == "scatter":
        host_ids = rng.permutation(host_blocks).astype(np.int64)
    table = np.full((len(ctx_caps), max_blocks_per_seq), -1, dtype=np.int32)
    r_at = h_at = 0
    for b, k in enumerate(need):
        for i in range(k):
            if on_host[b][i]:
                table[b, i] = resident_blocks + host_ids[h_at]
                h_at += 1
            else:
                table[b, i] = res_ids[r_at]
                r_at += 1
    return table


# The five workload shapes.  "ctx" is the number of keys attended at the
# first timed step (after that step's append); "steps" how many decode steps
# the full workload runs; c_off as an exact fraction (numerator, denominator).
WORKLOADS = {
    "cfg1": dict(L=1, H=8, G=8, d=64, B=4, ctx=256, steps=1, T=0, c_off=(0, 1), ragged=None,
                 note="single layer, all resident, latency only"),
    "cfg2": dict(L=32, H=32, G=32, d=128, B=32, ctx=513, steps=512, T=0, c_off=(0, 1), ragged=None,
                 note="6.7B-shaped MHA, prompt 512 + 512 generated, contiguous, resident"),
    "cfg3": dict(L=32, H=32, G=32, d=128, B=64, ctx=2048, steps=8, T=16, c_off=(1, 2), ragged=None,
                 note="paged, shuffled table, 50% of layers on host"),
    "cfg4": dict(L=32, H=32, G=8, d=128, B=128, ctx=None, steps=20, T=16, c_off=(0, 1),
                 ragged=(512, 4096), note="GQA 32/8, ragged contexts, paged, resident"),
    "cfg5": dict(L=32, H=32, G=32, d=128, B=192, ctx=4096, steps=3, T=16, c_off=(3, 5), ragged=None,
                 note="offline large batch, 60% of layers on host"),
    "cfg3_resident": dict(L=32, H=32, G=32, d=128, B=64, ctx=2048, steps=8, T=16, c_off=(0, 1), ragged=None,
                          note="the cfg3 stack with every layer in HBM: what the attention alone costs there"),
    # beyond the paper's models (all of them one query head per KV head): larger query groups at the same
    # 1 GiB of KV per layer, the shapes that take the matrix-core kernel
    "gqa8": dict(L=32, H=64, G=8, d=128, B=128, ctx=2048, steps=20, T=16, c_off=(0, 1), ragged=None,
                 note="GQA 64/8, context 2048, paged, resident"),
    "gqa16": dict(L=32, H=128, G=8, d=128, B=128, ctx=2048, steps=20, T=16, c_off=(0, 1), ragged=None,
                  note="GQA 128/8, context 2048, paged, resident"),
    # fewer than 8 KV heads (a model's KV heads divided over several GPUs), again 1 GiB of KV per layer; blocks
    # of 64 tokens, which the pool layout needs to keep a head's K and V tiles 32 KiB apart
    "kv8": dict(L=8, H=32, G=8, d=128, B=128, ctx=2048, steps=8, T=64, c_off=(0, 1), ragged=None,
                note="32 query / 8 KV heads, context 2048, 64-token blocks, resident"),
    "kv4": dict(L=8, H=32, G=4, d=128, B=256, ctx=2048, steps=8, T=64, c_off=(0, 1), ragged=None,
                note="32 query / 4 KV heads, context 2048, 64-token blocks, resident"),
    "kv2": dict(L=8, H=32, G=2, d=128, B=512, ctx=2048, steps=8, T=64, c_off=(0, 1), ragged=None,
                note="32 query / 2 KV heads, context 2048, 64-token blocks, resident"),
}
