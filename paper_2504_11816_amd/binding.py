"""ctypes binding of libokv.so: the same names as include/okv.h, argument
marshalling only.  Every step of the path runs in the library's kernels; there
is no fallback: a missing library raises."""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# OKV_LIBRARY may name another build of the same library (e.g. one compiled with
# different tuning macros); by default the in-tree build is used.
LIB_PATH = os.environ.get("OKV_LIBRARY") or os.path.join(_HERE, "libokv.so")

OKV_OK, OKV_EINVAL, OKV_ENOSPC, OKV_ESTATE, OKV_EHIP = 0, -1, -2, -3, -4
_CODE_NAMES = {0: "OKV_OK", -1: "OKV_EINVAL", -2: "OKV_ENOSPC", -3: "OKV_ESTATE", -4: "OKV_EHIP"}

# every symbol include/okv.h declares
EXPORTS = [
    "okv_layer_pool_bytes", "okv_block_bytes", "okv_kv_head_group", "okv_slab_tiles", "okv_workspace_bytes", "okv_tail_bytes", "okv_tail_plan", "kv_offload_plan", "okv_plan_from_bytes",
    "okv_plan_block_split", "okv_schedule_trace", "okv_create", "okv_destroy", "okv_last_error", "okv_set_batch",
    "okv_step_begin", "okv_step_end", "okv_step_abort", "okv_flush_tails", "kv_append", "decode_attn", "okv_decode_step", "okv_synchronize",
    "okv_set_split_tokens", "okv_get_split_tokens", "okv_get_ctx_lens", "okv_worklist",
    "okv_worklist_classes", "okv_pair_heads", "okv_prefill_begin", "kv_append_bulk", "okv_prefill_release", "okv_prefill_end", "okv_prefill_plan",
    "okv_measure_d2h",
    "okv_profile_enable", "okv_profile_read", "okv_measure_h2d", "okv_time_copies", "okv_probe_copy",
    "okv_probe_read", "okv_equal_stretches", "okv_decode_attn_static",
]


# every symbol include/okv_layer.h declares (same library)
LAYER_EXPORTS = ["okv_pack_linear_weight", "okv_linear", "okv_linear_qkv", "okv_linear_layernorm", "okv_linear_workspace_bytes", "okv_layernorm",
                 "okv_decoder_scratch_bytes", "okv_decoder_step"]


class OkvDecoderLayer(ctypes.Structure):
    """okv_decoder_layer of include/okv_layer.h: twelve device pointers."""
    FIELDS = ("ln1_gamma", "ln1_beta", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_gamma", "ln2_beta", "w_ff1", "b_ff1", "w_ff2", "b_ff2")
    _fields_ = [(name, ctypes.c_void_p) for name in FIELDS]


class OkvError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"{_CODE_NAMES.get(code, code)}: {message}")
        self.code = code


class OkvConfig(ctypes.Structure):
    _fields_ = [
        ("n_layers", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("block_tokens", ctypes.c_int32), ("max_batch", ctypes.c_int32),
        ("max_blocks_per_seq", ctypes.c_int32), ("max_ctx", ctypes.c_int32),
        ("blocks_per_layer", ctypes.c_int64), ("out_dtype", ctypes.c_int32), ("split_tokens", ctypes.c_int32),
        ("dev_pool", ctypes.POINTER(ctypes.c_void_p)), ("host_pool", ctypes.POINTER(ctypes.c_void_p)),
        ("staging", ctypes.c_void_p * 4), ("staging_bytes", ctypes.c_int64),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_int64),
        ("compute_stream", ctypes.c_void_p), ("h2d_stream", ctypes.c_void_p),
        ("resident_blocks", ctypes.c_int64), ("chunk_blocks", ctypes.c_int64),
        ("tail_blocks", ctypes.c_void_p), ("tail_bytes", ctypes.c_int64),
    ]


class OkvStaticAttn(ctypes.Structure):
    """okv_static_attn of include/okv.h."""
    _fields_ = [
        ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("block_tokens", ctypes.c_int32), ("max_blocks_per_seq", ctypes.c_int32), ("max_ctx", ctypes.c_int32),
        ("out_dtype", ctypes.c_int32), ("B", ctypes.c_int32),
        ("pool", ctypes.c_void_p), ("block_table", ctypes.c_void_p), ("ctx_lens", ctypes.c_void_p),
        ("q", ctypes.c_void_p), ("out", ctypes.c_void_p), ("k_new", ctypes.c_void_p), ("v_new", ctypes.c_void_p),
        ("stream", ctypes.c_void_p),
    ]


OKV_STATIC_SCRATCH_BYTES = 32 << 20
OKV_STATIC_MAX_BATCH = 4096

_lib_handle = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib_handle
    if _lib_handle is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2504_11816_amd.build` "
                "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        P, I32, I64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        cfgp = ctypes.POINTER(OkvConfig)
        sig = {
            "okv_layer_pool_bytes": (I64, [cfgp]),
            "okv_block_bytes": (I64, [cfgp]),
            "okv_kv_head_group": (I32, [I32, I32]),
            "okv_slab_tiles": (I32, [I32, I32, I32]),
            "okv_workspace_bytes": (I64, [cfgp]),
            "okv_tail_bytes": (I64, [cfgp]),
            "okv_tail_plan": (ctypes.c_int, [I32, P, I32, I32, P, P, I64, I64, I32, P, P]),
            "okv_plan_block_split": (ctypes.c_int, [I64, I64, I64, ctypes.POINTER(I64), ctypes.POINTER(I64)]),
            "okv_worklist_classes": (ctypes.c_int, [P, I32, P, I32, ctypes.POINTER(I32)]),
            "okv_pair_heads": (ctypes.c_int, [P, P, I64, ctypes.POINTER(I64)]),
            "kv_offload_plan": (ctypes.c_int, [I32, I64, I64, P, ctypes.POINTER(I32)]),
            "okv_plan_from_bytes": (ctypes.c_int, [I32, I64, I64, P, ctypes.POINTER(I32), ctypes.POINTER(I32)]),
            "okv_schedule_trace": (ctypes.c_int, [I32, P, P, I32, I32, P, I64, ctypes.POINTER(I64)]),
            "okv_create": (ctypes.c_int, [cfgp, ctypes.POINTER(P)]),
            "okv_destroy": (ctypes.c_int, [P]),
            "okv_last_error": (ctypes.c_char_p, [P]),
            "okv_set_batch": (ctypes.c_int, [P, I32, P, P]),
            "okv_step_begin": (ctypes.c_int, [P]),
            "okv_step_end": (ctypes.c_int, [P]),
            "okv_step_abort": (ctypes.c_int, [P]),
            "okv_flush_tails": (ctypes.c_int, [P]),
            "kv_append": (ctypes.c_int, [P, I32, P, P]),
            "decode_attn": (ctypes.c_int, [P, I32, P, P]),
            "okv_decode_step": (ctypes.c_int, [P, P, P, P, P]),
            "okv_synchronize": (ctypes.c_int, [P]),
            "okv_set_split_tokens": (ctypes.c_int, [P, I32]),
            "okv_get_split_tokens": (I32, [P]),
            "okv_get_ctx_lens": (ctypes.c_int, [P, P]),
            "okv_worklist": (ctypes.c_int, [P, I32, P, I64, ctypes.POINTER(I64)]),
            "okv_profile_enable": (ctypes.c_int, [P, I32]),
            "okv_profile_read": (ctypes.c_int, [P, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(I64)]),
            "okv_measure_h2d": (ctypes.c_int, [P, P, I64, I32, P, ctypes.POINTER(ctypes.c_double)]),
            "okv_measure_d2h": (ctypes.c_int, [P, P, I64, I32, P, ctypes.POINTER(ctypes.c_double)]),
            "okv_prefill_begin": (ctypes.c_int, [P, P]),
            "kv_append_bulk": (ctypes.c_int, [P, I32, P, P]),
            "okv_prefill_release": (ctypes.c_int, [P, I32]),
            "okv_prefill_end": (ctypes.c_int, [P]),
            "okv_prefill_plan": (ctypes.c_int, [P] + [ctypes.POINTER(I64)] * 4),
            "okv_time_copies": (ctypes.c_int, [P, I32, I32, ctypes.POINTER(ctypes.c_double)]),
            "okv_probe_copy": (ctypes.c_int, [P, P, I64, P]),
            "okv_pack_linear_weight": (ctypes.c_int, [P, P, I32, I32, P]),
            "okv_linear": (ctypes.c_int, [P, P, P, P, ctypes.POINTER(P), I32, I32, I32, I32, I32, P, I64, P]),
            "okv_linear_workspace_bytes": (I64, [I32, I32, I32]),
            "okv_linear_qkv": (ctypes.c_int, [P, P, P, P, P, P, I32, I32, I32, I32, P, I64, P]),
            "okv_linear_layernorm": (ctypes.c_int, [P, P, P, P, P, P, P, ctypes.c_float, P, I32, I32, I32, I32, P, I64, P]),
            "okv_layernorm": (ctypes.c_int, [P, P, P, P, I32, I32, ctypes.c_float, P]),
            "okv_decoder_scratch_bytes": (I64, [P, I32, I32]),
            "okv_decoder_step": (ctypes.c_int, [P, P, I32, I32, P, ctypes.c_float, P, I64, P, I64]),
            "okv_probe_read": (ctypes.c_int, [P, I64, P, P]),
            "okv_equal_stretches": (ctypes.c_int, [P, I32, I32, P, I64, ctypes.POINTER(I64), P, ctypes.POINTER(I32),
                                                   ctypes.POINTER(I64)]),
            "okv_decode_attn_static": (ctypes.c_int, [ctypes.POINTER(OkvStaticAttn)]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib_handle = L
    return _lib_handle


def _ptr(x):
    """Address of a torch tensor / numpy array / int / None as c_void_p."""
    if x is None:
        return ctypes.c_void_p(0)
    if isinstance(x, int):
        return ctypes.c_void_p(x)
    if hasattr(x, "data_ptr"):
        return ctypes.c_void_p(x.data_ptr())
    if isinstance(x, np.ndarray):
        return ctypes.c_void_p(x.ctypes.data)
    raise TypeError(f"cannot take the address of {type(x)}")


def _check(rc, ctx=None):
    if rc != 0:
        msg = lib().okv_last_error(ctx)
        raise OkvError(rc, msg.decode() if msg else "")
    return rc


# ---- pure host functions --------------------------------------------------------

def kv_offload_plan(n_layers, coff_num, coff_den):
    """-> (on_host uint8 [n_layers], n_off)"""
    on_host = np.zeros(max(n_layers, 1), dtype=np.uint8)
    n_off = ctypes.c_int32(0)
    _check(lib().kv_offload_plan(n_layers, coff_num, coff_den, _ptr(on_host), ctypes.byref(n_off)))
    return on_host[:n_layers], n_off.value


def okv_plan_from_bytes(n_layers, layer_bytes, mem_avail_bytes):
    """-> (on_host uint8 [n_layers], n_off, n_staging)"""
    on_host = np.zeros(max(n_layers, 1), dtype=np.uint8)
    n_off, n_st = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().okv_plan_from_bytes(n_layers, layer_bytes, mem_avail_bytes, _ptr(on_host),
                                     ctypes.byref(n_off), ctypes.byref(n_st)))
    return on_host[:n_layers], n_off.value, n_st.value


def okv_plan_block_split(n_blocks, coff_num, coff_den):
    """-> (resident_blocks, host_blocks)"""
    res, host = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(lib().okv_plan_block_split(n_blocks, coff_num, coff_den, ctypes.byref(res), ctypes.byref(host)))
    return res.value, host.value


def okv_schedule_trace(host_chunks, n_staging, n_steps, has_resident=None):
    """-> list of (kind, step, layer, chunk, buf, copy_idx, wait_idx)"""
    host_chunks = np.ascontiguousarray(host_chunks, dtype=np.int32)
    if has_resident is not None:
        has_resident = np.ascontiguousarray(has_resident, dtype=np.uint8)
    L = len(host_chunks)
    max_ops = (3 + 3 * int(host_chunks.sum())) * max(n_steps, 1) + 3 * L * max(n_steps, 1) + 8
    ops = np.zeros((max_ops, 7), dtype=np.int32)
    n = ctypes.c_int64(0)
    _check(lib().okv_schedule_trace(L, _ptr(host_chunks), _ptr(has_resident), n_staging, n_steps, _ptr(ops),
                                    max_ops, ctypes.byref(n)))
    return [tuple(int(v) for v in row) for row in ops[:n.value]]


def okv_equal_stretches(ctx_lens, max_groups):
    """-> (items int32 [n][3], group_first int32 [n_groups + 1], span_tiles)"""
    ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    B = len(ctx_lens)
    max_items = B + max_groups + 1
    items = np.zeros((max_items, 3), dtype=np.int32)
    first = np.zeros(max_groups + 1, dtype=np.int32)
    n, groups, span = ctypes.c_int64(0), ctypes.c_int32(0), ctypes.c_int64(0)
    _check(lib().okv_equal_stretches(_ptr(ctx_lens), B, max_groups, _ptr(items), max_items, ctypes.byref(n), _ptr(first),
                                     ctypes.byref(groups), ctypes.byref(span)))
    return items[:n.value].copy(), first[:groups.value + 1].copy(), span.value


def okv_decode_attn_static(*, n_q_heads, n_kv_heads, head_dim, block_tokens, max_blocks_per_seq, max_ctx, out_dtype, B, pool,
                           block_table, ctx_lens, q, out, k_new=None, v_new=None, stream=0):
    """One layer's decode attention with no context and no allocation (okv_decode_attn_static)."""
    a = OkvStaticAttn(n_q_heads, n_kv_heads, head_dim, block_tokens, max_blocks_per_seq, max_ctx, out_dtype, B,
                      _ptr(pool), _ptr(block_table), _ptr(ctx_lens), _ptr(q), _ptr(out), _ptr(k_new), _ptr(v_new),
                      ctypes.c_void_p(stream))
    _check(lib().okv_decode_attn_static(ctypes.byref(a)))


def make_config(**kw):
    cfg = OkvConfig()
    for k, v in kw.items():
        setattr(cfg, k, v)
    return cfg


def okv_layer_pool_bytes(cfg):
    r = lib().okv_layer_pool_bytes(ctypes.byref(cfg))
    if r < 0:
        _check(int(r))
    return int(r)


def okv_block_bytes(cfg):
    r = lib().okv_block_bytes(ctypes.byref(cfg))
    if r < 0:
        _check(int(r))
    return int(r)


def okv_kv_head_group(n_kv_heads, head_dim):
    r = lib().okv_kv_head_group(n_kv_heads, head_dim)
    if r < 0:
        _check(int(r))
    return int(r)


def okv_slab_tiles(n_kv_heads, head_dim, slice_tokens):
    r = lib().okv_slab_tiles(n_kv_heads, head_dim, slice_tokens)
    if r < 0:
        _check(int(r))
    return int(r)


def okv_workspace_bytes(cfg):
    r = lib().okv_workspace_bytes(ctypes.byref(cfg))
    if r < 0:
        _check(int(r))
    return int(r)


def okv_tail_plan(block_table, block_tokens, ctx_lens_after, tail_from, resident_blocks, chunk_blocks, n_chunks):
    """(patch_chunk [n_chunks], fills_block [B]) as uint8 arrays."""
    table = np.ascontiguousarray(block_table, dtype=np.int32)
    n = np.ascontiguousarray(ctx_lens_after, dtype=np.int32)
    t0 = np.ascontiguousarray(tail_from, dtype=np.int32)
    B = len(n)
    patch = np.zeros(max(n_chunks, 1), dtype=np.uint8)
    fills = np.zeros(B, dtype=np.uint8)
    _check(lib().okv_tail_plan(B, _ptr(table), table.shape[1], block_tokens, _ptr(n), _ptr(t0), resident_blocks, chunk_blocks,
                               n_chunks, _ptr(patch), _ptr(fills)))
    return patch[:n_chunks], fills


def okv_tail_bytes(cfg):
    r = lib().okv_tail_bytes(ctypes.byref(cfg))
    if r < 0:
        _check(int(r))
    return int(r)


def okv_measure_h2d(dst, src, nbytes, reps, stream):
    g = ctypes.c_double(0)
    _check(lib().okv_measure_h2d(_ptr(dst), _ptr(src), nbytes, reps, _ptr(stream), ctypes.byref(g)))
    return g.value


def okv_measure_d2h(dst, src, nbytes, reps, stream):
    g = ctypes.c_double(0)
    _check(lib().okv_measure_d2h(_ptr(dst), _ptr(src), nbytes, reps, _ptr(stream), ctypes.byref(g)))
    return g.value


def okv_probe_copy(dst, src, nbytes, stream):
    _check(lib().okv_probe_copy(_ptr(dst), _ptr(src), nbytes, _ptr(stream)))


def okv_probe_read(src, nbytes, sink, stream):
    _check(lib().okv_probe_read(_ptr(src), nbytes, _ptr(sink), _ptr(stream)))


# ---- linear layers (include/okv_layer.h) ------------------------------------------------

def okv_pack_linear_weight(dst, src, n_out, n_in, stream=0):
    _check(lib().okv_pack_linear_weight(_ptr(dst), _ptr(src), n_out, n_in, _ptr(stream)))


def okv_linear(x, w_packed, bias, residual, out, m, n_out, n_in, relu=False, stream=0, workspace=None,
               workspace_bytes=0):
    """out: one tensor, or a list of 1..3 tensors that share the n_out output features equally."""
    outs = list(out) if isinstance(out, (list, tuple)) else [out]
    arr = (ctypes.c_void_p * len(outs))(*[_ptr(o) for o in outs])
    _check(lib().okv_linear(_ptr(x), _ptr(w_packed), _ptr(bias), _ptr(residual), arr, len(outs), m, n_out, n_in,
                            1 if relu else 0, _ptr(workspace), workspace_bytes, _ptr(stream)))


def okv_linear_qkv(x, w_packed, bias, q, k, v, m, q_cols, kv_cols, n_in, stream=0, workspace=None, workspace_bytes=0):
    _check(lib().okv_linear_qkv(_ptr(x), _ptr(w_packed), _ptr(bias), _ptr(q), _ptr(k), _ptr(v), m, q_cols, kv_cols, n_in,
                                _ptr(workspace), workspace_bytes, _ptr(stream)))


def okv_linear_layernorm(x, w_packed, bias, residual, out, gamma, beta, out_norm, m, n_out, n_in, eps=1e-5, relu=False,
                         stream=0, workspace=None, workspace_bytes=0):
    _check(lib().okv_linear_layernorm(_ptr(x), _ptr(w_packed), _ptr(bias), _ptr(residual), _ptr(out), _ptr(gamma), _ptr(beta),
                                      eps, _ptr(out_norm), m, n_out, n_in, 1 if relu else 0, _ptr(workspace), workspace_bytes,
                                      _ptr(stream)))


def okv_linear_workspace_bytes(m, n_out, n_in):
    r = lib().okv_linear_workspace_bytes(m, n_out, n_in)
    if r < 0:
        _check(int(r))
    return int(r)


def okv_layernorm(x, gamma, beta, out, m, h, eps=1e-5, stream=0):
    _check(lib().okv_layernorm(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(out), m, h, eps, _ptr(stream)))


# ---- context ------------------------------------------------------------------------

class Context:
    """okv_ctx with the header's calls as methods.  Pointers are raw addresses
    (ints) or objects with data_ptr(); the caller keeps the memory alive."""

    def __init__(self, *, n_layers, n_q_heads, n_kv_heads, head_dim, block_tokens, max_batch,
                 max_blocks_per_seq=0, max_ctx=0, blocks_per_layer=0, out_dtype=0, split_tokens=0,
                 dev_pool, host_pool=None, staging=(None, None), staging_bytes=0,
                 workspace, workspace_bytes, compute_stream=0, h2d_stream=0, resident_blocks=0, chunk_blocks=0,
                 tail_blocks=None, tail_bytes=0):
        L = n_layers
        self._dev = (ctypes.c_void_p * L)(*[_ptr(p) for p in dev_pool])
        self._host = (ctypes.c_void_p * L)(*[_ptr(p) for p in (host_pool or [None] * L)])
        cfg = OkvConfig()
        cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim = n_layers, n_q_heads, n_kv_heads, head_dim
        cfg.block_tokens, cfg.max_batch, cfg.max_blocks_per_seq = block_tokens, max_batch, max_blocks_per_seq
        cfg.max_ctx, cfg.blocks_per_layer, cfg.out_dtype, cfg.split_tokens = max_ctx, blocks_per_layer, out_dtype, split_tokens
        cfg.dev_pool = ctypes.cast(self._dev, ctypes.POINTER(ctypes.c_void_p))
        cfg.host_pool = ctypes.cast(self._host, ctypes.POINTER(ctypes.c_void_p))
        for i in range(4):
            cfg.staging[i] = _ptr(staging[i] if i < len(staging) else None)
        cfg.staging_bytes = staging_bytes
        cfg.workspace, cfg.workspace_bytes = _ptr(workspace), workspace_bytes
        cfg.compute_stream, cfg.h2d_stream = _ptr(compute_stream), _ptr(h2d_stream)
        cfg.resident_blocks, cfg.chunk_blocks = resident_blocks, chunk_blocks
        cfg.tail_blocks, cfg.tail_bytes = _ptr(tail_blocks), tail_bytes
        self.cfg = cfg
        self.B = 0
        self._h = ctypes.c_void_p(0)
        _check(lib().okv_create(ctypes.byref(cfg), ctypes.byref(self._h)))

    def close(self):
        if self._h:
            lib().okv_destroy(self._h)
            self._h = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _c(self, rc):
        return _check(rc, self._h)

    def okv_set_batch(self, block_table, ctx_lens):
        ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
        self.B = len(ctx_lens)
        if block_table is not None:
            block_table = np.ascontiguousarray(block_table, dtype=np.int32)
        self._c(lib().okv_set_batch(self._h, self.B, _ptr(block_table), _ptr(ctx_lens)))

    def okv_step_begin(self):
        self._c(lib().okv_step_begin(self._h))

    def okv_step_end(self):
        self._c(lib().okv_step_end(self._h))

    def okv_step_abort(self):
        self._c(lib().okv_step_abort(self._h))

    def okv_flush_tails(self):
        self._c(lib().okv_flush_tails(self._h))

    def kv_append(self, layer, k_new, v_new):
        self._c(lib().kv_append(self._h, layer, _ptr(k_new), _ptr(v_new)))

    def decode_attn(self, layer, q, out):
        self._c(lib().decode_attn(self._h, layer, _ptr(q), _ptr(out)))

    @staticmethod
    def pointer_arrays(q, k_new, v_new, out):
        """The four HOST arrays of DEVICE pointers okv_decode_step takes, from per-layer lists of
        tensors; build them once for buffers that are reused every step."""
        return tuple((ctypes.c_void_p * len(ts))(*[_ptr(t) for t in ts]) for ts in (q, k_new, v_new, out))

    def okv_decode_step(self, arrays):
        """arrays: what pointer_arrays returned (one entry per layer in each)."""
        q, k, v, o = arrays
        if not (len(q) == len(k) == len(v) == len(o) == self.cfg.n_layers):
            raise ValueError("one pointer per layer in each array")
        self._c(lib().okv_decode_step(self._h, q, k, v, o))

    @staticmethod
    def decoder_layers(layers):
        """The HOST array of okv_decoder_layer that okv_decoder_step takes, from one dict per layer
        (keys: OkvDecoderLayer.FIELDS; values: device tensors or addresses, None for an absent bias).
        Build it once; the caller keeps the tensors alive."""
        arr = (OkvDecoderLayer * len(layers))()
        for i, d in enumerate(layers):
            for name in OkvDecoderLayer.FIELDS:
                setattr(arr[i], name, _ptr(d.get(name)).value)
        return arr

    def okv_decoder_scratch_bytes(self, m, h2):
        r = lib().okv_decoder_scratch_bytes(self._h, m, h2)
        if r < 0:
            _check(int(r))
        return int(r)

    def okv_decoder_step(self, layers, h2, x, scratch, scratch_bytes, workspace, workspace_bytes, eps=1e-5):
        """layers: what decoder_layers returned."""
        self._c(lib().okv_decoder_step(self._h, layers, len(layers), h2, _ptr(x), eps, _ptr(scratch), scratch_bytes,
                                       _ptr(workspace), workspace_bytes))

    def okv_prefill_begin(self, n_new):
        n_new = np.ascontiguousarray(n_new, dtype=np.int32)
        if len(n_new) != self.B:
            raise ValueError("n_new needs one entry per sequence")
        self._c(lib().okv_prefill_begin(self._h, _ptr(n_new)))

    def kv_append_bulk(self, layer, k_rows, v_rows):
        self._c(lib().kv_append_bulk(self._h, layer, _ptr(k_rows), _ptr(v_rows)))

    def okv_prefill_release(self, layer):
        self._c(lib().okv_prefill_release(self._h, layer))

    def okv_prefill_plan(self):
        """-> dict(staged_groups, copies, staged_tiles, direct_tiles) of the last okv_prefill_begin"""
        v = [ctypes.c_int64(0) for _ in range(4)]
        self._c(lib().okv_prefill_plan(self._h, *[ctypes.byref(x) for x in v]))
        return dict(zip(("staged_groups", "copies", "staged_tiles", "direct_tiles"), [x.value for x in v]))

    def okv_prefill_end(self):
        self._c(lib().okv_prefill_end(self._h))

    def okv_synchronize(self):
        self._c(lib().okv_synchronize(self._h))

    def okv_set_split_tokens(self, s):
        self._c(lib().okv_set_split_tokens(self._h, s))

    def okv_get_split_tokens(self):
        return int(lib().okv_get_split_tokens(self._h))

    def okv_get_ctx_lens(self):
        out = np.zeros(self.B, dtype=np.int32)
        self._c(lib().okv_get_ctx_lens(self._h, _ptr(out)))
        return out

    def okv_worklist(self, from_device=False, max_items=1 << 20):
        items = np.zeros((max_items, 3), dtype=np.int32)
        n = ctypes.c_int64(0)
        self._c(lib().okv_worklist(self._h, 1 if from_device else 0, _ptr(items), max_items, ctypes.byref(n)))
        return items[:n.value].copy()

    def okv_worklist_classes(self, from_device=False, max_classes=8192):
        first = np.zeros(max_classes, dtype=np.int32)
        n = ctypes.c_int32(0)
        self._c(lib().okv_worklist_classes(self._h, 1 if from_device else 0, _ptr(first), max_classes, ctypes.byref(n)))
        return first[:n.value + 1].copy()

    def okv_pair_heads(self, max_records=1 << 16):
        """int32 [stretches in use * G][8]: what the wavefronts of a launch start from (okv_pair_heads)."""
        rec = np.zeros((max_records, 8), dtype=np.int32)
        n = ctypes.c_int64(0)
        self._c(lib().okv_pair_heads(self._h, _ptr(rec), max_records, ctypes.byref(n)))
        return rec[:n.value].copy()

    def okv_time_copies(self, as_pipelined=False, n_steps=1):
        """ms per step of the copy half alone (back to back, or issued as the pipeline issues it)."""
        ms = ctypes.c_double(0)
        self._c(lib().okv_time_copies(self._h, 1 if as_pipelined else 0, n_steps, ctypes.byref(ms)))
        return ms.value

    def okv_profile_enable(self, on):
        """0 / False: off; 1 / True: a bracket per split-K launch; 2: a bracket per step."""
        self._c(lib().okv_profile_enable(self._h, int(on)))

    def okv_profile_read(self):
        ms, n = ctypes.c_double(0), ctypes.c_int64(0)
        self._c(lib().okv_profile_read(self._h, ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value
