"""The selection-model C library against its oracle: every formula on random and edge inputs
(double against exact rationals, relative 1e-12), every decision (Algorithm 1 case, candidate
order, ranking) exactly.  CPU only."""
import os
import re
from fractions import Fraction as F

import numpy as np
import pytest

from oracle import infersave_model as om
from paper_2504_11816_amd import infersave as isv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def close(got, want, rel=1e-12):
    want = float(want)
    return abs(got - want) <= rel * max(abs(want), 1e-300)


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "infersave.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    decl = sorted(set(re.findall(r"\b(isv_[a-z_0-9]+)\s*\(", text)))
    lib = isv.lib()
    for name in decl:
        assert hasattr(lib, name), name
    assert decl == sorted(isv.EXPORTS)


def _random_setup(rng):
    h1 = int(rng.choice([768, 2048, 2560, 4096, 5120]))
    model = dict(n_params=float(rng.integers(10 ** 8, 10 ** 10)), h1=h1, h2=4 * h1, n_layers=int(rng.integers(1, 64)))
    work = dict(BS=int(rng.integers(1, 129)), L_in=int(rng.integers(1, 4097)), L_out=int(rng.integers(1, 1025)))
    return model, work


def test_memory_and_assess_match_oracle():
    rng = np.random.default_rng(1)
    for _ in range(200):
        model, work = _random_setup(rng)
        cm = isv.IsvModel(model["n_params"], model["h1"], model["h2"], model["n_layers"], 2)
        cw = isv.IsvWorkload(work["BS"], work["L_in"], work["L_out"])
        mem = isv.isv_memory_requirements(cm, cw)
        want = om.memory_requirements(int(model["n_params"]), model["h1"], model["n_layers"], work["BS"], work["L_in"], work["L_out"])
        for k in ("model", "activation", "kvcache", "kvcache_per_layer", "total", "base"):
            assert close(getattr(mem, k), want[k], 1e-14), k
        # instances around every decision boundary of Algorithm 1 (sizes that are exact in double)
        tot, base, per, mod = (int(want[k]) for k in ("total", "base", "kvcache_per_layer", "model"))
        per = int(np.ceil(float(want["kvcache_per_layer"])))
        sizes = [tot, tot - 1, tot + 1, mod - 1, mod, base + per, base + per - 2, base + per + 1,
                 int(rng.integers(mod, tot + 1)), int(rng.integers(1, tot * 2))]
        prices = [float(rng.integers(1, 8)) / 2 for _ in sizes]
        inst = [isv.IsvInstance(float(s), p, 1e12, 1e9, 1e9, 1, 0, 1, 0) for s, p in zip(sizes, prices)]
        verdict, order = isv.isv_assess(inst, mem, 3.0)
        want_c = om.assess([dict(price=F(p), gpu_mem=s) for s, p in zip(sizes, prices)], want, 3)
        assert order == [i for i, _ in want_c]
        for i, coff in want_c:
            assert verdict[i][0] == (isv.ISV_RESIDENT if coff == 0 else isv.ISV_OFFLOAD)
            assert close(verdict[i][1], coff, 1e-9) or abs(verdict[i][1] - float(coff)) < 1e-12
        for i, (status, c, _) in enumerate(verdict):
            if prices[i] > 3.0:
                assert status == isv.ISV_TOO_DEAR
            elif i not in order:
                assert status == isv.ISV_UNSUITABLE and c == 0


def test_predict_matches_oracle():
    rng = np.random.default_rng(2)
    for trial in range(300):
        model, work = _random_setup(rng)
        flops = float(rng.integers(1, 3000)) * 1e12
        bw1, bw2 = float(rng.integers(1, 128)) * 1e9, float(rng.integers(1, 128)) * 1e9
        ab = [float(x) for x in (rng.integers(-8, 40) / 16, rng.integers(0, 100) / 1024, rng.integers(1, 40) / 16, rng.integers(0, 100) / 4096)]
        c_off = [0.0, 1.0, 0.5, float(rng.integers(0, 1025)) / 1024][trial % 4]
        overlap = bool(trial % 2)
        cm = isv.IsvModel(model["n_params"], model["h1"], model["h2"], model["n_layers"], 2)
        cw = isv.IsvWorkload(work["BS"], work["L_in"], work["L_out"])
        ci = isv.IsvInstance(1e11, 1.0, flops, bw1, bw2, *ab)
        got = isv.isv_predict(cm, cw, ci, c_off, overlap)
        want = om.predict(model, work, dict(flops=F(flops), bw_g2c=F(bw1), bw_c2g=F(bw2), alpha_pre=F(ab[0]), beta_pre=F(ab[1]),
                                            alpha_dec=F(ab[2]), beta_dec=F(ab[3])), F(c_off), overlap_decode=overlap)
        if want["t_task"] <= 0:
            continue                                   # a negative calibrated time: nothing to compare
        for k, v in want.items():
            assert close(got[k], v, 1e-11), (k, got[k], float(v))


def test_attention_flops_is_the_attention_term_of_the_decode_time():
    from oracle import kv_bytes
    for BS, L_in, L_out, h1 in ((32, 512, 128, 2560), (1, 1, 1, 64), (64, 2047, 2, 4096)):
        want = kv_bytes.decode_attention_flops_per_layer(BS, L_in, L_out, h1)
        assert close(isv.isv_attention_flops_decode(BS, L_in + L_out / 2, h1), want, 1e-15)
        # and T_compute^d is the linear part plus this term over FLOPS
        cm = isv.IsvModel(1e9, h1, 4 * h1, 4, 2)
        got = isv.isv_predict(cm, isv.IsvWorkload(BS, L_in, L_out), isv.IsvInstance(1e12, 1, 1e12, 1e9, 1e9, 1, 0, 1, 0), 0.0)
        lin = BS * (8 * h1 * h1 + 4 * h1 * 4 * h1)
        assert close(got["t_compute_dec"], (lin + float(want)) / 1e12, 1e-13)
    with pytest.raises(ValueError):
        isv.isv_attention_flops_decode(0, 10.0, 64)


def test_predict_rejects_bad_arguments():
    cm = isv.IsvModel(1e9, 1024, 4096, 12, 2)
    cw = isv.IsvWorkload(8, 128, 16)
    ok = isv.IsvInstance(1e10, 1.0, 1e13, 1e9, 1e9, 1, 0, 1, 0)
    for bad_c in (-0.1, 1.5, float("nan")):
        with pytest.raises(ValueError):
            isv.isv_predict(cm, cw, ok, bad_c)
    with pytest.raises(ValueError):
        isv.isv_predict(cm, cw, isv.IsvInstance(1e10, 1.0, 0.0, 1e9, 1e9, 1, 0, 1, 0), 0.0)
    with pytest.raises(ValueError):
        isv.isv_predict(cm, cw, isv.IsvInstance(1e10, 1.0, 1e13, 0.0, 1e9, 1, 0, 1, 0), 0.5)
    with pytest.raises(ValueError):
        isv.isv_predict(cm, isv.IsvWorkload(0, 128, 16), ok, 0.0)


def test_ctcf_fit_matches_oracle():
    rng = np.random.default_rng(3)
    for _ in range(100):
        n = int(rng.integers(2, 20))
        x = rng.uniform(1e-4, 2.0, n)
        y = rng.uniform(0.2, 3.0) * x + rng.uniform(0.0, 0.5) + rng.normal(0, 0.01, n)
        a, b, err = isv.isv_ctcf_fit(x, y)
        wa, wb = om.ctcf_fit([F(float(v)) for v in x], [F(float(v)) for v in y])
        assert close(a, wa, 1e-9) and abs(b - float(wb)) < 1e-9
        want_err = np.mean(np.abs(float(wa) * x + float(wb) - y) / np.abs(y))
        assert abs(err - want_err) < 1e-9
    with pytest.raises(ValueError):
        isv.isv_ctcf_fit([1.0, 1.0], [2.0, 3.0])
    with pytest.raises(ValueError):
        isv.isv_ctcf_fit([1.0], [2.0])


def test_cost_efficiency_and_selection_match_oracle():
    rng = np.random.default_rng(4)
    cw = isv.IsvWorkload(32, 1024, 128)
    for _ in range(300):
        n = int(rng.integers(1, 7))
        tps = [float(rng.integers(20, 4000)) / 2 for _ in range(n)]
        price = [float(rng.integers(1, 40)) / 8 for _ in range(n)]
        slo = float(rng.integers(10, 2000))
        nq = int(rng.integers(1, 5000))
        for t, p in zip(tps, price):
            ce, hours, cost = isv.isv_cost_efficiency(t, slo, nq, cw, p)
            wce, wh, wc = om.cost_efficiency(F(t), F(slo), nq, 1024, 128, F(p))
            # a task that ends within 1e-12 of a whole hour may be billed differently in double: skip those
            if abs(float(wh) - round(float(wh))) < 1e-9:
                continue
            assert close(ce, wce) and close(hours, wh) and close(cost, wc)
        want = om.select([F(t) for t in tps], [F(p) for p in price], F(slo), nq, 1024, 128)
        hours = [float(om.cost_efficiency(F(t), F(slo), nq, 1024, 128, F(p))[1]) for t, p in zip(tps, price)]
        if any(abs(h - round(h)) < 1e-9 for h in hours):
            continue
        ces = [om.cost_efficiency(F(t), F(slo), nq, 1024, 128, F(p))[0] for t, p in zip(tps, price)]
        near_tie = any(i != j and ces[i] != ces[j] and abs(float(ces[i] / ces[j]) - 1) < 1e-12 for i in range(n) for j in range(n))
        if near_tie:
            continue
        assert isv.isv_select(tps, price, slo, nq, cw) == want
    # the paper's online table at the 400 TPS objective
    names = ["g6e.xlarge", "g6.xlarge", "g5.xlarge", "g4dn.xlarge"]
    tps = [1506.54, 802.19, 1206.12, 620.17]
    price = [2.699, 1.167, 1.466, 0.71]
    ranked = isv.isv_select(tps, price, 400.0, 3000, isv.IsvWorkload(32, 128, 512))
    assert [names[i] for i in ranked[:2]] == ["g4dn.xlarge", "g6.xlarge"]
