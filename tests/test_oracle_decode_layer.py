"""Pins for the oracle of the decoder layer around the attention.  CPU only."""
import numpy as np
import torch

from oracle import decode_layer as dl
from oracle import kv_bytes


def _params(rng, h1, h2):
    def w(n, k):
        return rng.standard_normal((n, k)) / np.sqrt(k)
    return dict(ln1_g=rng.uniform(0.5, 1.5, h1), ln1_b=rng.normal(0, 0.1, h1), ln2_g=rng.uniform(0.5, 1.5, h1),
                ln2_b=rng.normal(0, 0.1, h1), wq=w(h1, h1), wk=w(h1, h1), wv=w(h1, h1), wo=w(h1, h1), w1=w(h2, h1),
                w2=w(h1, h2), bq=rng.normal(0, 0.1, h1), bk=rng.normal(0, 0.1, h1), bv=rng.normal(0, 0.1, h1),
                bo=rng.normal(0, 0.1, h1), b1=rng.normal(0, 0.1, h2), b2=rng.normal(0, 0.1, h1))


def test_layernorm_closed_forms():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 64)) * 3 + 7
    one, zero = np.ones(64), np.zeros(64)
    y = dl.layernorm(x, one, zero, eps=0.0)
    assert np.allclose(y.mean(axis=1), 0, atol=1e-12) and np.allclose((y ** 2).mean(axis=1), 1, atol=1e-12)
    # invariant to a shift and a positive rescale of the row (eps = 0), equivariant to gamma / beta
    assert np.allclose(dl.layernorm(5 * x - 3, one, zero, eps=0.0), y, atol=1e-12)
    g, b = rng.uniform(0.5, 2, 64), rng.normal(0, 1, 64)
    assert np.allclose(dl.layernorm(x, g, b, eps=0.0), y * g + b, atol=1e-12)
    # a row of two values goes to -1, +1; a constant row goes to beta (eps keeps it finite)
    assert np.allclose(dl.layernorm(np.array([[2.0, 6.0]]), np.ones(2), np.zeros(2), eps=0.0), [[-1, 1]])
    assert np.allclose(dl.layernorm(np.full((1, 8), 3.0), np.ones(8), b[:8]), b[:8])
    # eps enters under the root: var = 4, eps = 5 -> divide by 3
    assert np.allclose(dl.layernorm(np.array([[0.0, 4.0]]), np.ones(2), np.zeros(2), eps=5.0), [[-2 / 3, 2 / 3]])
    # torch's layer_norm in fp64
    want = torch.nn.functional.layer_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), torch.from_numpy(b), 1e-5).numpy()
    assert np.allclose(dl.layernorm(x, g, b), want, atol=1e-12)


def test_linear_and_relu_hand_cases():
    x = np.array([[1.0, 2.0, 3.0]])
    w = np.array([[1.0, 0.0, 0.0], [0.0, 1.0, 1.0]])            # [N = 2][K = 3]
    assert dl.linear(x, w).tolist() == [[1.0, 5.0]]
    assert dl.linear(x, w, np.array([10.0, -5.0])).tolist() == [[11.0, 0.0]]
    # the weight is [out][in]: swapping the roles fails on a non-square case
    rng = np.random.default_rng(1)
    x, w, b = rng.standard_normal((4, 6)), rng.standard_normal((3, 6)), rng.standard_normal(3)
    brute = np.array([[sum(x[m, k] * w[n, k] for k in range(6)) + b[n] for n in range(3)] for m in range(4)])
    assert np.allclose(dl.linear(x, w, b), brute, atol=1e-13)
    assert np.allclose(dl.linear(x, w, b), torch.nn.functional.linear(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b)).numpy())
    assert dl.relu(np.array([-1.0, 0.0, 2.5])).tolist() == [0.0, 0.0, 2.5]


def test_layer_against_torch_modules_in_fp64():
    rng = np.random.default_rng(2)
    h1, h2, M = 32, 128, 5
    p = _params(rng, h1, h2)
    x = rng.standard_normal((M, h1))
    t = rng.standard_normal((M, h1))                                  # stands for the attention output
    tp = {k: torch.from_numpy(np.asarray(v)) for k, v in p.items()}
    F = torch.nn.functional
    xt, tt = torch.from_numpy(x), torch.from_numpy(t)
    a = F.layer_norm(xt, (h1,), tp["ln1_g"], tp["ln1_b"], 1e-5)
    q, k, v = dl.qkv(x, p)
    assert np.allclose(q, F.linear(a, tp["wq"], tp["bq"]).numpy(), atol=1e-12)
    assert np.allclose(k, F.linear(a, tp["wk"], tp["bk"]).numpy(), atol=1e-12)
    assert np.allclose(v, F.linear(a, tp["wv"], tp["bv"]).numpy(), atol=1e-12)
    y = xt + F.linear(tt, tp["wo"], tp["bo"])
    z = F.layer_norm(y, (h1,), tp["ln2_g"], tp["ln2_b"], 1e-5)
    want = y + F.linear(F.relu(F.linear(z, tp["w1"], tp["b1"])), tp["w2"], tp["b2"])
    assert np.allclose(dl.after_attention(x, t, p), want.numpy(), atol=1e-11)
    # planted mistakes are seen: residual dropped, activation dropped, second norm fed with x instead of y
    no_res = F.linear(F.relu(F.linear(z, tp["w1"], tp["b1"])), tp["w2"], tp["b2"]).numpy()
    assert not np.allclose(dl.after_attention(x, t, p), no_res, atol=1e-3)
    no_act = (y + F.linear(F.linear(z, tp["w1"], tp["b1"]), tp["w2"], tp["b2"])).numpy()
    assert not np.allclose(dl.after_attention(x, t, p), no_act, atol=1e-3)
    # rounding between the ops changes little and only at fp16 scale
    r = dl.after_attention(x, t, p, fp16_between=True)
    assert 0 < np.abs(r - want.numpy()).max() < 2e-2


def test_flop_and_byte_counts_match_the_paper():
    # §IV-D: decode linear flops per token 8 h1^2 + 4 h1 h2 = twice the number of weights in the six matrices
    for h1, h2 in ((2560, 10240), (4096, 16384), (64, 256)):
        assert dl.linear_flops_per_token(h1, h2) == 2 * (4 * h1 * h1 + 2 * h1 * h2)
        assert dl.linear_weight_bytes(h1, h2) == dl.linear_flops_per_token(h1, h2)          # fp16: one flop per byte and token
    # the whole decode compute term is these plus the attention term
    BS, L_in, L_out, h1, h2 = 32, 512, 128, 2560, 10240
    total = BS * dl.linear_flops_per_token(h1, h2) + kv_bytes.decode_attention_flops_per_layer(BS, L_in, L_out, h1)
    from oracle import infersave_model as m
    assert m.t_compute_decode(BS, L_in, L_out, h1, h2, 1) == total
