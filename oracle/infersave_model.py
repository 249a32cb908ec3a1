"""The paper's instance-selection model written out (oracle side).

TEST INFRASTRUCTURE ONLY; shares no code with the C library.  Exact rational
arithmetic (fractions.Fraction) wherever the formulas are rational; symbols as in
the paper's Table II.  Each function names the passage it follows.

Readings taken where the paper is silent or at odds with itself:
  * Mem_KVcache uses h1 where Table II prints nh (the transfer formulas of
    §IV-D use h1; with nh the head dimension would be missing);
  * Mem_activation is taken as printed, 2 (L_in + L_out) BS h1, in bytes;
  * Eq. 2's "BS" is the number of queries of the whole task (the evaluation
    runs 1000 or 3000 requests in batches), so it is a separate argument here;
  * Step 4's tie-break (higher TPS) is applied to exactly equal cost
    efficiencies; candidates are otherwise ranked by cost efficiency, descending.
"""
from fractions import Fraction
import math


def memory_requirements(n_params, h1, n_layers, BS, L_in, L_out, prec=2):
    """Table II: model, activation and KV-cache bytes, and §IV-C's totals."""
    model = Fraction(n_params) * prec
    activation = Fraction(2 * (L_in + L_out) * BS * h1)
    kv = Fraction(2 * BS * (L_in + L_out) * h1 * prec * n_layers)
    return {"model": model, "activation": activation, "kvcache": kv, "kvcache_per_layer": kv / n_layers,
            "total": model + activation + kv, "base": model + activation}


def assess(instances, mem, p_max):
    """Algorithm 1.  instances: list of dicts with gpu_mem and price.  Returns a list of
    (index, C_off) sorted by price (ascending; equal prices keep their order), after the
    price filter and the three memory cases of §IV-C."""
    out = []
    for i, inst in enumerate(instances):
        if Fraction(inst["price"]) > Fraction(p_max):
            continue
        gpu = Fraction(inst["gpu_mem"])
        avail = gpu - mem["base"]
        if gpu >= mem["total"]:
            out.append((i, Fraction(0)))                       # Case 1
        elif gpu < mem["model"] or mem["kvcache_per_layer"] > avail:
            continue                                           # Case 2
        else:
            out.append((i, 1 - avail / mem["kvcache"]))        # Case 3
    out.sort(key=lambda t: Fraction(instances[t[0]]["price"]))
    return out


def t_compute_prefill(BS, L_in, h1, h2, flops):
    """§IV-D: linear layers BS (8 L_in h1^2 + 4 L_in h1 h2) plus attention 4 BS L_in^2 h1, over FLOPS."""
    return Fraction(BS * (8 * L_in * h1 * h1 + 4 * L_in * h1 * h2) + 4 * BS * L_in * L_in * h1) / Fraction(flops)


def t_compute_decode(BS, L_in, L_out, h1, h2, flops):
    """§IV-D: BS (8 h1^2 + 4 h1 h2) plus 4 BS (L_in + L_out / 2) h1, over FLOPS."""
    return (Fraction(BS * (8 * h1 * h1 + 4 * h1 * h2)) + Fraction(4 * BS * h1) * (Fraction(L_in) + Fraction(L_out, 2))) / Fraction(flops)


def t_trans_prefill(c_off, BS, L_in, h1, bw, prec=2):
    return Fraction(c_off) * 2 * (L_in + 1) * h1 * prec * BS / Fraction(bw)


def t_trans_decode(c_off, BS, L_in, L_out, h1, bw, prec=2):
    return (Fraction(c_off) * 2 * (L_in + 1) + L_out) * h1 * prec * BS / Fraction(bw)


def ctcf(t, alpha, beta):
    """Eq. 7."""
    return Fraction(alpha) * t + Fraction(beta)


def predict(model, work, inst, c_off, overlap_decode=False):
    """Eq. 4-6 and Eq. 1 for one instance.  model: h1, h2, n_layers; work: BS, L_in, L_out;
    inst: flops, bw_g2c, bw_c2g, alpha_pre, beta_pre, alpha_dec, beta_dec.
    overlap_decode replaces Eq. 6's sum by a max (transfers hidden behind compute, as this
    repository's decode pipeline does); the paper's model is overlap_decode=False."""
    BS, L_in, L_out = work["BS"], work["L_in"], work["L_out"]
    h1, h2, n = model["h1"], model["h2"], model["n_layers"]
    tcp = t_compute_prefill(BS, L_in, h1, h2, inst["flops"])
    tcd = t_compute_decode(BS, L_in, L_out, h1, h2, inst["flops"])
    ttp = t_trans_prefill(c_off, BS, L_in, h1, inst["bw_g2c"]) if c_off else Fraction(0)
    ttd = t_trans_decode(c_off, BS, L_in, L_out, h1, inst["bw_c2g"]) if c_off else Fraction(0)
    t_pre = max(ctcf(tcp, inst["alpha_pre"], inst["beta_pre"]), ttp)                    # Eq. 5
    cd = ctcf(tcd, inst["alpha_dec"], inst["beta_dec"])
    t_dec = max(cd, ttd) if overlap_decode else cd + ttd                                 # Eq. 6
    t_task = t_pre * n + t_dec * n * (L_out - 1)                                         # Eq. 4
    return {"t_compute_pre": tcp, "t_trans_pre": ttp, "t_pre": t_pre, "t_compute_dec": tcd, "t_trans_dec": ttd,
            "t_dec": t_dec, "t_task": t_task, "tps": Fraction(BS * (L_in + L_out)) / t_task}   # Eq. 1


def ctcf_fit(xs, ys):
    """Least-squares line y = alpha x + beta through the points (§IV-F), exact."""
    n = len(xs)
    xs = [Fraction(x) for x in xs]
    ys = [Fraction(y) for y in ys]
    mx, my = sum(xs) / n, sum(ys) / n
    sxx = sum((x - mx) ** 2 for x in xs)
    sxy = sum((x - mx) * (y - my) for x, y in zip(xs, ys))
    if sxx == 0:
        raise ValueError("all abscissae equal")
    alpha = sxy / sxx
    return alpha, my - alpha * mx


def cost_efficiency(tps_actual, tps_slo, n_queries, L_in, L_out, price):
    """Eq. 2 and Eq. 3: effective TPS is capped by the SLO, hours are billed whole.
    Returns (CE, task hours, total cost)."""
    eff = min(Fraction(tps_actual), Fraction(tps_slo))
    hours = Fraction(n_queries * (L_in + L_out)) / (eff * 3600)
    billed = math.ceil(hours)
    return eff * 3600 / (billed * Fraction(price)), hours, billed * Fraction(price)


def select(tps, prices, tps_slo, n_queries, L_in, L_out):
    """Step 4: drop instances below the SLO, rank the rest by cost efficiency (descending),
    ties by TPS (descending).  Returns the ranked list of indices."""
    ok = [i for i in range(len(tps)) if Fraction(tps[i]) >= Fraction(tps_slo)]
    return sorted(ok, key=lambda i: (-cost_efficiency(tps[i], tps_slo, n_queries, L_in, L_out, prices[i])[0],
                                     -Fraction(tps[i])))
