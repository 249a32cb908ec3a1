"""The paper's size, flop and transfer-time formulas (oracle side).

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.  These are the
scalar expressions the benchmark's byte and flop accounting is checked
against.  Symbols follow the paper's Table II: BS batch size, L_in / L_out
prompt and output lengths, h1 hidden size (= heads x head dim), L layers,
prec bytes per number (2 for fp16).
"""
from fractions import Fraction


def mem_kvcache(BS, L_in, L_out, h1, L, prec=2):
    """KV cache bytes, Table II.

    The table prints `nh` (head count) where the transfer formulas of §IV-D
    use h1; with `nh` the head dimension would be missing, so h1 is the
    reading taken: 2 (K and V) * BS * (L_in + L_out) * h1 * prec * L.
    """
    return 2 * BS * (L_in + L_out) * h1 * prec * L


def mem_kvcache_per_layer(BS, L_in, L_out, h1, L, prec=2):
    """Table II: the per-layer share is the total divided by L."""
    return Fraction(mem_kvcache(BS, L_in, L_out, h1, L, prec), L)


def kv_bytes_per_token_per_layer(G, d, prec=2):
    """Generalisation to grouped query heads: K and V rows of G KV heads."""
    return 2 * G * d * prec


def kv_bytes_step(ctx_lens, G, d, prec=2):
    """Bytes of KV one layer's decode attention has to read in one step."""
    return sum(int(n) for n in ctx_lens) * kv_bytes_per_token_per_layer(G, d, prec)


def decode_attention_flops_per_layer(BS, L_in, L_out, h1):
    """§IV-D, decode compute time, self-attention term (numerator):
    4 * BS * (L_in + L_out / 2) * h1 -- two multiply-adds per cached K and V
    element at the average context length."""
    return Fraction(4 * BS * h1) * (Fraction(L_in) + Fraction(L_out, 2))


def decode_attention_flops_step(ctx_lens, H, d):
    """Same count for one concrete step: 4 * sum_b n_b * H * d."""
    return 4 * sum(int(n) for n in ctx_lens) * H * d


def t_trans_decode(c_off, L_in, L_out, h1, BS, bw_cpu_to_gpu, prec=2):
    """§IV-D, decode-stage KV transfer time per layer, exactly as printed:
    (C_off * 2 * (L_in + 1) + L_out) * h1 * prec * BS / BW.
    Kept as context only (its L_out term carries neither C_off nor the factor
    2): the byte accounting of the benchmark uses kv_bytes_step."""
    return (Fraction(c_off) * 2 * (L_in + 1) + L_out) * h1 * prec * BS / Fraction(bw_cpu_to_gpu)


def t_trans_prefill(c_off, L_in, h1, BS, bw_gpu_to_cpu, prec=2):
    """§IV-D, prefill-stage KV transfer time per layer, as printed:
    C_off * 2 * (L_in + 1) * h1 * prec * BS / BW  -- the offloaded share of the
    keys and values of the prompt and of the first generated token."""
    return Fraction(c_off) * 2 * (L_in + 1) * h1 * prec * BS / Fraction(bw_gpu_to_cpu)


def t_prefill(t_compute, t_trans):
    """Eq. 5: in the prefill stage a layer's write-out overlaps the computation, so the
    layer takes the longer of the two."""
    return max(t_compute, t_trans)


def kv_bytes_written(n_new, G, d, prec=2):
    """Bytes of K and V that storing n_new[b] tokens per sequence adds to one layer."""
    return sum(int(n) for n in n_new) * kv_bytes_per_token_per_layer(G, d, prec)


def t_task(t_pre, t_dec, n_layers, L_out):
    """Eq. 4: prefill once per layer, decode per layer for L_out - 1 tokens
    (the first output token comes out of the prefill)."""
    return t_pre * n_layers + t_dec * n_layers * (L_out - 1)


def tps(BS, L_in, L_out, t_e2e):
    """Eq. 1: tokens per second counts prompt and generated tokens."""
    return Fraction(BS * (L_in + L_out)) / Fraction(t_e2e)
