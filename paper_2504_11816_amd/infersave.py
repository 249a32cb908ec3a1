"""ctypes binding of libinfersave.so: the names of include/infersave.h, argument
marshalling only.  A missing library raises."""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libinfersave.so")

EXPORTS = ["isv_memory_requirements", "isv_assess", "isv_predict", "isv_attention_flops_decode", "isv_ctcf_fit", "isv_cost_efficiency", "isv_select"]

ISV_RESIDENT, ISV_OFFLOAD, ISV_UNSUITABLE, ISV_TOO_DEAR = 0, 1, -1, -2


class IsvModel(ctypes.Structure):
    _fields_ = [("n_params", ctypes.c_double), ("h1", ctypes.c_int32), ("h2", ctypes.c_int32),
                ("n_layers", ctypes.c_int32), ("precision_bytes", ctypes.c_int32)]


class IsvWorkload(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("l_in", ctypes.c_int32), ("l_out", ctypes.c_int32)]


class IsvInstance(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in ("gpu_mem_bytes", "price_per_hour", "flops", "bw_gpu_to_cpu",
                                               "bw_cpu_to_gpu", "alpha_pre", "beta_pre", "alpha_dec", "beta_dec")]


class IsvMemory(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in ("model", "activation", "kvcache", "kvcache_per_layer", "total", "base")]


class IsvCandidate(ctypes.Structure):
    _fields_ = [("status", ctypes.c_int32), ("c_off", ctypes.c_double), ("mem_avail", ctypes.c_double)]


class IsvTimes(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in ("t_compute_pre", "t_trans_pre", "t_pre", "t_compute_dec",
                                               "t_trans_dec", "t_dec", "t_task", "tps")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2504_11816_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        D, I32, I64, P = ctypes.c_double, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        pd = ctypes.POINTER(D)
        L.isv_memory_requirements.argtypes = [ctypes.POINTER(IsvModel), ctypes.POINTER(IsvWorkload), ctypes.POINTER(IsvMemory)]
        L.isv_assess.argtypes = [P, I32, ctypes.POINTER(IsvMemory), D, P, P, ctypes.POINTER(I32)]
        L.isv_predict.argtypes = [ctypes.POINTER(IsvModel), ctypes.POINTER(IsvWorkload), ctypes.POINTER(IsvInstance), D, I32,
                                  ctypes.POINTER(IsvTimes)]
        L.isv_ctcf_fit.argtypes = [I32, P, P, pd, pd, pd]
        L.isv_attention_flops_decode.argtypes = [I32, D, I32]
        L.isv_attention_flops_decode.restype = D
        L.isv_cost_efficiency.argtypes = [D, D, I64, ctypes.POINTER(IsvWorkload), D, pd, pd]
        L.isv_cost_efficiency.restype = D
        L.isv_select.argtypes = [I32, P, P, D, I64, ctypes.POINTER(IsvWorkload), P, ctypes.POINTER(I32)]
        _lib = L
    return _lib


def _ok(rc, what):
    if rc != 0:
        raise ValueError(f"{what}: bad argument")


def _as_dict(s):
    return {n: getattr(s, n) for n, _ in s._fields_}


def isv_memory_requirements(model, work):
    out = IsvMemory()
    _ok(lib().isv_memory_requirements(ctypes.byref(model), ctypes.byref(work), ctypes.byref(out)), "isv_memory_requirements")
    return out


def isv_assess(instances, mem, p_max):
    """-> (list of (status, c_off, mem_avail) per instance, candidate indices by price)"""
    n = len(instances)
    arr = (IsvInstance * max(n, 1))(*instances)
    verdict = (IsvCandidate * max(n, 1))()
    order = (ctypes.c_int32 * max(n, 1))()
    k = ctypes.c_int32(0)
    _ok(lib().isv_assess(arr, n, ctypes.byref(mem), p_max, verdict, order, ctypes.byref(k)), "isv_assess")
    return [(verdict[i].status, verdict[i].c_off, verdict[i].mem_avail) for i in range(n)], [order[i] for i in range(k.value)]


def isv_predict(model, work, inst, c_off, overlap_decode=False):
    out = IsvTimes()
    _ok(lib().isv_predict(ctypes.byref(model), ctypes.byref(work), ctypes.byref(inst), c_off, 1 if overlap_decode else 0,
                          ctypes.byref(out)), "isv_predict")
    return _as_dict(out)


def isv_attention_flops_decode(batch, context, h1):
    v = lib().isv_attention_flops_decode(batch, context, h1)
    if v < 0:
        raise ValueError("isv_attention_flops_decode: bad argument")
    return v


def isv_ctcf_fit(t_theory, t_measured):
    """-> (alpha, beta, mean relative error)"""
    x = np.ascontiguousarray(t_theory, dtype=np.float64)
    y = np.ascontiguousarray(t_measured, dtype=np.float64)
    a, b, e = ctypes.c_double(0), ctypes.c_double(0), ctypes.c_double(0)
    _ok(lib().isv_ctcf_fit(len(x), x.ctypes.data, y.ctypes.data, ctypes.byref(a), ctypes.byref(b), ctypes.byref(e))
        if len(x) == len(y) else -1, "isv_ctcf_fit")
    return a.value, b.value, e.value


def isv_cost_efficiency(tps_actual, tps_slo, n_queries, work, price):
    """-> (CE, task hours, total cost)"""
    h, c = ctypes.c_double(0), ctypes.c_double(0)
    ce = lib().isv_cost_efficiency(tps_actual, tps_slo, n_queries, ctypes.byref(work), price, ctypes.byref(h), ctypes.byref(c))
    if ce < 0:
        raise ValueError("isv_cost_efficiency: bad argument")
    return ce, h.value, c.value


def isv_select(tps, price, tps_slo, n_queries, work):
    t = np.ascontiguousarray(tps, dtype=np.float64)
    p = np.ascontiguousarray(price, dtype=np.float64)
    ranked = np.zeros(max(len(t), 1), dtype=np.int32)
    k = ctypes.c_int32(0)
    _ok(lib().isv_select(len(t), t.ctypes.data, p.ctypes.data, tps_slo, n_queries, ctypes.byref(work), ranked.ctypes.data,
                         ctypes.byref(k)), "isv_select")
    return ranked[:k.value].tolist()
