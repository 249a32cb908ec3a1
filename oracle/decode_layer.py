"""One decoder layer of the decode stage around the attention (oracle side).

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

The paper counts, per generated token and layer, 8 h1^2 + 4 h1 h2 flops of linear
layers next to the attention (§IV-D): four h1 x h1 projections (query, key, value,
output: 2 h1^2 flops each) and the two matrices of the feed-forward block (h1 -> h2 -> h1,
2 h1 h2 each).  It names no further detail; the models it runs are OPT, whose decoder
layer is taken as the reading:

    a   = LayerNorm(x)                      (learned scale and shift, eps = 1e-5)
    q, k, v = a Wq^T + bq, a Wk^T + bk, a Wv^T + bv
    (k, v join the KV cache; attention of q over the cache gives t)
    y   = x + t Wo^T + bo
    z   = LayerNorm(y)
    out = y + relu(z W1^T + b1) W2^T + b2

Weights are [out features][in features].  Everything is fp64 here.  The GPU path keeps
activations in fp16 between kernels; `round16` marks those points so that a test can ask
the oracle to round where the GPU stores (each op is also compared on its own, without
any rounding inside).
"""
import numpy as np


def round16(x, on=True):
    """Round to fp16 and back (round-to-nearest-even), or leave as is."""
    return np.asarray(x, dtype=np.float64).astype(np.float16).astype(np.float64) if on else np.asarray(x, dtype=np.float64)


def layernorm(x, gamma, beta, eps=1e-5):
    """Per row: (x - mean) / sqrt(var + eps) * gamma + beta, population variance."""
    x = np.asarray(x, dtype=np.float64)
    out = np.empty_like(x)
    for i in range(x.shape[0]):
        row = x[i]
        mean = row.sum() / row.size
        var = ((row - mean) ** 2).sum() / row.size
        out[i] = (row - mean) / np.sqrt(var + eps) * np.asarray(gamma, dtype=np.float64) + np.asarray(beta, dtype=np.float64)
    return out


def linear(x, weight, bias=None):
    """x [M][K], weight [N][K] -> [M][N]: out[m][n] = sum_k x[m][k] weight[n][k] (+ bias[n])."""
    out = np.asarray(x, dtype=np.float64) @ np.asarray(weight, dtype=np.float64).T
    if bias is not None:
        out = out + np.asarray(bias, dtype=np.float64)
    return out


def relu(x):
    return np.maximum(np.asarray(x, dtype=np.float64), 0.0)


def qkv(x, p, fp16_between=False):
    """Steps up to the attention: returns q [M][h1], k, v [M][h1]."""
    a = round16(layernorm(x, p["ln1_g"], p["ln1_b"]), fp16_between)
    q = round16(linear(a, p["wq"], p["bq"]), fp16_between)
    k = round16(linear(a, p["wk"], p["bk"]), fp16_between)
    v = round16(linear(a, p["wv"], p["bv"]), fp16_between)
    return q, k, v


def after_attention(x, t, p, fp16_between=False):
    """Steps after the attention output t [M][h1]: returns the layer's output [M][h1]."""
    y = round16(np.asarray(x, dtype=np.float64) + linear(t, p["wo"], p["bo"]), fp16_between)
    z = round16(layernorm(y, p["ln2_g"], p["ln2_b"]), fp16_between)
    u = round16(relu(linear(z, p["w1"], p["b1"])), fp16_between)
    return round16(y + linear(u, p["w2"], p["b2"]), fp16_between)


def linear_flops_per_token(h1, h2):
    """§IV-D: 8 h1^2 + 4 h1 h2."""
    return 8 * h1 * h1 + 4 * h1 * h2


def linear_weight_bytes(h1, h2, prec=2):
    """Bytes of the six matrices, each read once per decode step: (4 h1^2 + 2 h1 h2) prec."""
    return (4 * h1 * h1 + 2 * h1 * h2) * prec
