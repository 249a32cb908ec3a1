"""Which layers' KV leaves the GPU for an offload ratio C_off (oracle side).

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.  Everything is
exact rational / integer arithmetic (fractions.Fraction), written for
clarity, not speed.

Paper §IV-C: when the KV cache does not fit beside the model, the share that
must leave the GPU is  C_off = 1 - Mem_avail / Mem_KVcache  (Case 3), and an
instance is usable only if one layer's KV fits in what is available (Case 2,
and the layer-level check of Algorithm 1), because attention runs on the GPU.

Readings taken where the paper is silent:
  * offloading is by whole layers; the number of layers moved is the smallest
    integer that is at least C_off * L (C_off is a minimum share: rounding
    down would leave more KV on the GPU than fits);
  * the moved layers are spread evenly through the stack: walking the layers
    in order with a quota that grows by n_off / L per layer, a layer goes to
    the host whenever the whole part of the quota goes up.
"""
from fractions import Fraction


def n_offloaded(n_layers, c_off):
    """Smallest integer >= c_off * n_layers; c_off is a Fraction in [0, 1]."""
    c_off = Fraction(c_off)
    if not (0 <= c_off <= 1):
        raise ValueError("C_off must lie in [0, 1]")
    x = c_off * n_layers
    k = x.numerator // x.denominator
    if Fraction(k) < x:
        k += 1
    return k


def plan_layers(n_layers, c_off):
    """List of 0/1 per layer (1 = on host) and the count of host layers."""
    k = n_offloaded(n_layers, c_off)
    on_host = []
    quota = Fraction(0)
    whole_before = 0
    for _ in range(n_layers):
        quota += Fraction(k, n_layers)
        whole_now = quota.numerator // quota.denominator
        on_host.append(1 if whole_now > whole_before else 0)
        whole_before = whole_now
    return on_host, k


def plan_from_bytes(n_layers, layer_bytes, mem_avail_bytes):
    """Plan from the memory the GPU has left for KV (paper §IV-C, Algorithm 1).

    Returns (status, on_host, n_off, n_staging) with status one of
      "resident"    Case 1: everything fits, nothing is moved
      "infeasible"  Case 2: not even one layer's KV fits
      "offload"     Case 3
    In Case 3 the host layers are streamed through staging buffers that come
    out of the same available memory: two when two layers fit beside the
    resident ones, otherwise one.  Resident layers = what fits after the
    staging buffers; the plan moves the rest.  The share moved is therefore
    never below the paper's C_off.
    """
    total = n_layers * layer_bytes
    if mem_avail_bytes >= total:
        return "resident", [0] * n_layers, 0, 0
    if layer_bytes > mem_avail_bytes:
        return "infeasible", None, None, None
    fit = mem_avail_bytes // layer_bytes          # whole layers that fit, 1 <= fit < L
    n_staging = 2 if fit >= 2 else 1
    resident = fit - n_staging
    n_off = n_layers - resident
    on_host, k = plan_layers(n_layers, Fraction(n_off, n_layers))
    assert k == n_off
    return "offload", on_host, n_off, n_staging


def c_off_case3(mem_avail_bytes, mem_kv_bytes):
    """C_off of Case 3 as an exact fraction."""
    return 1 - Fraction(mem_avail_bytes, mem_kv_bytes)


def block_split(n_blocks, c_off):
    """(blocks that stay in HBM, blocks on the host) of n_blocks blocks for an
    offload ratio c_off: the host gets the smallest integer >= c_off * n_blocks."""
    n_host = n_offloaded(n_blocks, c_off)
    return n_blocks - n_host, n_host


def host_blocks_per_sequence(blocks_per_seq, n_host):
    """How many of each sequence's blocks go to the host when n_host blocks in
    total do: walking the sequences with a quota that grows by
    n_host / total per block, a sequence gives the whole part gained while its
    blocks are walked."""
    total = sum(blocks_per_seq)
    if not (0 <= n_host <= total):
        raise ValueError("n_host outside [0, total]")
    out, quota, whole_before = [], Fraction(0), 0
    for nb in blocks_per_seq:
        quota += Fraction(nb * n_host, total) if total else 0
        whole_now = quota.numerator // quota.denominator
        out.append(whole_now - whole_before)
        whole_before = whole_now
    return out
