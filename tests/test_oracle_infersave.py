"""Pins for the oracle of the paper's selection model (Algorithm 1, Eq. 1-7).  CPU only.

What the paper prints and is self-consistent is pinned: the instance table of §VI-A, the
online selection at the 400 TPS SLO (Table V) with its cost ratios, Eq. 2/3 on hand
numbers.  Table VI's C_off percentages and total prices do not follow from the printed
formulas (FlexGen's own policy and an unstated task size are behind them) and Table III's
alpha / beta need the authors' measurements: those are not pinned ("parity unpinned" for
the fitted constants; the fit itself is pinned against numpy's least squares)."""
from fractions import Fraction as F

import numpy as np
import pytest

from oracle import infersave_model as m

# §VI-A, instance table: price $/h, memory GB, FP16 TFLOPS, PCIe GB/s
AWS = {
    "g6e.xlarge": dict(price=F("2.699"), gpu_mem=48 * 10 ** 9, flops=F("91.61") * 10 ** 12, bw=12 * 10 ** 9),
    "g6.xlarge": dict(price=F("1.167"), gpu_mem=24 * 10 ** 9, flops=F("30.29") * 10 ** 12, bw=12 * 10 ** 9),
    "g5.xlarge": dict(price=F("1.466"), gpu_mem=24 * 10 ** 9, flops=F("31.52") * 10 ** 12, bw=12 * 10 ** 9),
    "g4dn.xlarge": dict(price=F("0.71"), gpu_mem=16 * 10 ** 9, flops=F("8.24") * 10 ** 12, bw=6 * 10 ** 9),
}
ONLINE_TPS = {"g4dn.xlarge": F("620.17"), "g6.xlarge": F("802.19"), "g5.xlarge": F("1206.12"), "g6e.xlarge": F("1506.54")}


def test_table_v_selection_at_400_tps_and_cost_ratios():
    names = list(AWS)
    tps = [ONLINE_TPS[n] for n in names]
    prices = [AWS[n]["price"] for n in names]
    ranked = m.select(tps, prices, 400, 3000, 128, 512)
    assert [names[i] for i in ranked[:2]] == ["g4dn.xlarge", "g6.xlarge"]        # Table V, SLO 400
    # every instance exceeds the SLO, so all are capped at 400 TPS, finish in the same billed hour(s),
    # and cost efficiency is inversely proportional to price
    ce = [m.cost_efficiency(t, 400, 3000, 128, 512, p) for t, p in zip(tps, prices)]
    assert len({c[1] for c in ce}) == 1
    assert ce[0][0] * prices[0] == ce[3][0] * prices[3]
    # "about 280 % more expensive", "56.75 % lower cost" (§VI-C)
    assert round(float(AWS["g6e.xlarge"]["price"] / AWS["g4dn.xlarge"]["price"] - 1) * 100) == 280
    assert abs(float(1 - AWS["g6.xlarge"]["price"] / AWS["g6e.xlarge"]["price"]) * 100 - 56.75) < 0.02
    # an instance below the SLO is dropped
    assert names.index("g4dn.xlarge") not in m.select(tps, prices, 700, 3000, 128, 512)
    # ties in cost efficiency go to the higher TPS
    assert m.select([500, 900], [1, 1], 400, 100, 128, 512) == [1, 0]


def test_cost_efficiency_hand_numbers():
    # 1000 queries of 1152 tokens at 100 TPS: 3.2 h, billed 4 h; CE = 100 * 3600 / (4 * price)
    ce, hours, cost = m.cost_efficiency(169, 100, 1000, 1024, 128, F("0.71"))
    assert hours == F(1152000, 360000) and cost == 4 * F("0.71") and ce == F(360000) / (4 * F("0.71"))
    # below the SLO the actual rate counts
    ce2, hours2, _ = m.cost_efficiency(50, 100, 1000, 1024, 128, 1)
    assert hours2 == F(1152000, 180000) and ce2 == F(50 * 3600, 7)
    # exactly one hour is billed as one hour
    assert m.cost_efficiency(320, 1000, 1000, 1024, 128, 2)[2] == 2


def test_memory_and_algorithm_1_cases():
    mem = m.memory_requirements(2_700_000_000, 2560, 32, 32, 1024, 128)
    assert mem["kvcache"] == 2 * 32 * 1152 * 2560 * 2 * 32 and mem["kvcache_per_layer"] * 32 == mem["kvcache"]
    assert mem["model"] == 5_400_000_000 and mem["activation"] == 2 * 1152 * 32 * 2560
    assert mem["total"] == mem["base"] + mem["kvcache"]
    inst = [dict(price=1, gpu_mem=mem["total"]),                              # fits exactly: Case 1
            dict(price=F(1, 2), gpu_mem=mem["total"] - 1),                     # one byte short: Case 3
            dict(price=2, gpu_mem=mem["model"] - 1),                           # weights do not fit: Case 2
            dict(price=3, gpu_mem=mem["base"] + mem["kvcache_per_layer"]),     # exactly one layer of KV fits: Case 3
            dict(price=4, gpu_mem=mem["base"] + mem["kvcache_per_layer"] - 1), # not even one layer: Case 2
            dict(price=9, gpu_mem=mem["total"] * 2)]                           # too expensive
    got = m.assess(inst, mem, 5)
    assert [i for i, _ in got] == [1, 0, 3]                                     # by price
    c = dict(got)
    assert c[0] == 0
    assert c[1] == F(1) / mem["kvcache"]                                        # one byte of the cache must leave
    assert c[3] == 1 - F(1, 32)                                                 # one of 32 layers stays
    for i, coff in got:
        assert 0 <= coff < 1
    # C_off is exactly the share that does not fit: avail + C_off * KV = KV
    avail = F(inst[1]["gpu_mem"]) - mem["base"]
    assert avail + c[1] * mem["kvcache"] == mem["kvcache"]


def test_times_closed_forms_and_limits():
    model = dict(h1=2560, h2=4 * 2560, n_layers=32)
    work = dict(BS=32, L_in=512, L_out=128)
    inst = dict(flops=AWS["g4dn.xlarge"]["flops"], bw_g2c=6 * 10 ** 9, bw_c2g=6 * 10 ** 9,
                alpha_pre=1, beta_pre=0, alpha_dec=1, beta_dec=0)
    r0 = m.predict(model, work, inst, 0)
    # without offloading: no transfer terms, T_task = n (T_pre + (L_out - 1) T_dec), TPS = BS (L_in + L_out) / T_task
    assert r0["t_trans_pre"] == 0 and r0["t_trans_dec"] == 0
    assert r0["t_task"] == 32 * (r0["t_compute_pre"] + 127 * r0["t_compute_dec"])
    assert r0["tps"] * r0["t_task"] == 32 * 640
    # the flop counts: prefill = L_in x the linear part of decode, attention quadratic in L_in
    lin_dec = F(32 * (8 * 2560 ** 2 + 4 * 2560 * 10240)) / inst["flops"]
    assert r0["t_compute_pre"] == 512 * lin_dec + F(4 * 32 * 512 ** 2 * 2560) / inst["flops"]
    assert r0["t_compute_dec"] == lin_dec + F(4 * 32 * (512 + 64) * 2560) / inst["flops"]
    # with everything offloaded the decode transfer is the printed expression, added to compute (Eq. 6) ...
    r1 = m.predict(model, work, inst, 1)
    assert r1["t_trans_dec"] == F((2 * 513 + 128) * 2560 * 2 * 32, 6 * 10 ** 9)
    assert r1["t_dec"] == r1["t_compute_dec"] + r1["t_trans_dec"]
    # ... while prefill takes the longer of the two (Eq. 5)
    assert r1["t_pre"] == max(r1["t_compute_pre"], r1["t_trans_pre"])
    # overlapped decode is never slower than the paper's sum and never faster than either part
    r2 = m.predict(model, work, inst, 1, overlap_decode=True)
    assert max(r1["t_compute_dec"], r1["t_trans_dec"]) == r2["t_dec"] <= r1["t_dec"]
    # CTCF enters linearly
    inst2 = dict(inst, alpha_dec=F(1, 2), beta_dec=F(3, 1000))
    r3 = m.predict(model, work, inst2, 0)
    assert r3["t_dec"] == r0["t_compute_dec"] / 2 + F(3, 1000)
    # TPS falls as C_off grows
    tps = [m.predict(model, work, inst, F(k, 10))["tps"] for k in range(11)]
    assert all(a > b for a, b in zip(tps, tps[1:]))


def test_ctcf_fit_against_numpy_and_exact_lines():
    rng = np.random.default_rng(0)
    for _ in range(20):
        n = int(rng.integers(2, 12))
        x = rng.uniform(0.1, 5.0, n)
        y = rng.uniform(-1.0, 3.0) * x + rng.uniform(-2, 2) + rng.normal(0, 0.05, n)
        a, b = m.ctcf_fit([F(float(v)) for v in x], [F(float(v)) for v in y])
        pa, pb = np.polyfit(x, y, 1)
        assert abs(float(a) - pa) < 1e-8 * max(1, abs(pa)) and abs(float(b) - pb) < 1e-8 * max(1, abs(pb))
    # points on a line are recovered exactly, negative slopes included (Table III prints negative alphas)
    xs = [F(1), F(2), F(5), F(9)]
    a, b = m.ctcf_fit(xs, [F(-185, 1000) * x + F(2435, 100) for x in xs])
    assert (a, b) == (F(-185, 1000), F(2435, 100))
    with pytest.raises(ValueError):
        m.ctcf_fit([1, 1, 1], [1, 2, 3])
