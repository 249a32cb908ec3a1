"""Memory and stream plumbing around the okv library for tests, smoke and bench.

PyTorch is used here only to own device / pinned-host memory and the two HIP
streams; every computation is a call into libokv.so through binding.Context.
"""
import ctypes

import numpy as np
import torch

from . import binding, synth


_hip = None


def _hip_runtime():
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipHostMalloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t, ctypes.c_uint]
        _hip.hipHostMalloc.restype = ctypes.c_int
        _hip.hipHostFree.argtypes = [ctypes.c_void_p]
        _hip.hipHostFree.restype = ctypes.c_int
        _hip.hipGetLastError.argtypes = []
        _hip.hipGetLastError.restype = ctypes.c_int
        _hip.hipExtStreamCreateWithCUMask.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint32,
                                                      ctypes.POINTER(ctypes.c_uint32)]
        _hip.hipExtStreamCreateWithCUMask.restype = ctypes.c_int
        _hip.hipStreamDestroy.argtypes = [ctypes.c_void_p]
        _hip.hipStreamDestroy.restype = ctypes.c_int
    return _hip


def new_stream(device):
    """A HIP stream with a hardware queue of its own (default priority), wrapped for torch.

    The runtime spreads the streams of a process over a handful of hardware queues (4 here) and a queue is
    worked through in order.  When the compute stream shares a queue with a copy stream, its kernels wait
    behind the marker that follows every copy: in the copy trace no attention kernel started before the copy
    stream's current 2 GiB copy had finished, and which streams share depends on how many were created before
    (torch alone makes 32 at its first torch.cuda.Stream()).  A stream created with a compute-unit mask gets a
    queue that no other stream uses; the mask names every compute unit, so nothing is masked.
    """
    hip = _hip_runtime()
    words = (torch.cuda.get_device_properties(device).multi_processor_count + 31) // 32
    mask = (ctypes.c_uint32 * words)(*([0xFFFFFFFF] * words))
    raw = ctypes.c_void_p(0)
    rc = hip.hipExtStreamCreateWithCUMask(ctypes.byref(raw), words, mask)
    if rc != 0 or not raw.value:
        raise RuntimeError(f"hipExtStreamCreateWithCUMask failed with {rc}")
    return raw.value, torch.cuda.ExternalStream(raw.value, device=device)


class PinnedHalfBuffer:
    """n fp16 elements of pinned, device-mapped host memory (hipHostMalloc of
    exactly that size; torch's pinned allocator would round it up to a power of
    two), viewed as a torch CPU tensor."""

    def __init__(self, n_elems):
        self.nbytes = n_elems * 2
        p = ctypes.c_void_p(0)
        rc = _hip_runtime().hipHostMalloc(ctypes.byref(p), self.nbytes, 0)
        if rc != 0 or not p.value:
            # the runtime keeps the refusal as its "last error", and the next library that looks (torch after
            # any call of its own) would report it as its own failure: read it, which clears it
            _hip_runtime().hipGetLastError()
            raise MemoryError(f"hipHostMalloc({self.nbytes}) failed with {rc}")
        self.ptr = p.value
        raw = (ctypes.c_char * self.nbytes).from_address(self.ptr)
        self.tensor = torch.frombuffer(raw, dtype=torch.float16)

    def free(self):
        if self.ptr:
            self.tensor = None
            _hip_runtime().hipHostFree(ctypes.c_void_p(self.ptr))
            self.ptr = 0


class Stack:
    """All buffers of one decode workload plus the okv context that uses them.

    on_host[l] = 1 puts layer l's pool in pinned host memory (streamed through
    two staging buffers), 0 keeps it in HBM.  With chunk_blocks > 0 every layer
    instead keeps the blocks with ids below resident_blocks in HBM and the others
    in pinned host memory, streamed in chunks of chunk_blocks blocks.
    """

    def __init__(self, *, L, H, G, d, B, T, cap_tokens, on_host=None, out_dtype=0, split_tokens=0,
                 blocks_per_layer=None, n_staging=2, device="cuda:0", resident_blocks=0, chunk_blocks=0,
                 workspace_items=None, hot_tails=None):
        if not torch.cuda.is_available():
            raise RuntimeError("the okv library needs a GPU; there is no CPU path")
        self.L, self.H, self.G, self.d, self.B, self.T = L, H, G, d, B, T
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.on_host = np.zeros(L, dtype=np.uint8) if on_host is None else np.asarray(on_host, dtype=np.uint8)
        self.paged = T != 0
        if self.paged:
            self.max_blocks = synth.blocks_needed(cap_tokens, T)
            self.cap_tokens = self.max_blocks * T
            self.blocks_per_layer = blocks_per_layer or B * self.max_blocks
            self.max_ctx = 0
        else:
            self.max_blocks = 0
            # a multiple of the tokens of a full slab (16 with 8 or more KV heads at d = 128), so that the layout
            # can keep a head's K and V tiles 32 KiB apart
            unit = 16 * binding.okv_slab_tiles(G, d, 1 << 20)
            self.max_ctx = (cap_tokens + unit - 1) // unit * unit
            self.cap_tokens = self.max_ctx
            self.blocks_per_layer = 0
        shape = binding.make_config(n_layers=L, n_q_heads=H, n_kv_heads=G, head_dim=d, block_tokens=T,
                                    max_batch=B, max_blocks_per_seq=self.max_blocks, max_ctx=self.max_ctx,
                                    blocks_per_layer=self.blocks_per_layer, out_dtype=out_dtype,
                                    split_tokens=split_tokens, resident_blocks=resident_blocks,
                                    chunk_blocks=chunk_blocks)
        self.pool_bytes = binding.okv_layer_pool_bytes(shape)
        self.workspace_bytes = binding.okv_workspace_bytes(shape)
        if workspace_items:
            self.workspace_bytes = max(self.workspace_bytes, workspace_items * H * (d + 2) * 4)
        n_el = self.pool_bytes // 2
        self.by_class = chunk_blocks > 0
        self.resident_blocks, self.chunk_blocks = resident_blocks, chunk_blocks
        self.pools, self._pinned = [], []
        self.dev_part, self.host_part = [None] * L, [None] * L
        try:
            self._allocate_pools(L, n_el, resident_blocks, chunk_blocks, shape)
        except MemoryError:
            for p in self._pinned:                       # what was pinned before the refusal goes back at once
                p.free()
            self._pinned = []
            raise
        any_host, staging_el = self._any_host, self._staging_el
        self.staging_bytes = staging_el * 2 if any_host else 0
        self.staging = [torch.empty(staging_el, dtype=torch.float16, device=self.device) if any_host and i < n_staging
                        else None for i in range(4)]
        self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=self.device)
        # block-granular offload: rows appended to host blocks stay in HBM slots until their block is full
        # (hot_tails=False: every row is stored through the mapped pointer in its own step)
        self.hot_tails = bool(self.by_class and any_host and (hot_tails is None or hot_tails))
        self.tail_bytes = binding.okv_tail_bytes(shape) if self.hot_tails else 0
        self.tail_blocks = torch.empty(self.tail_bytes, dtype=torch.uint8, device=self.device) if self.hot_tails else None
        self._raw_streams = []
        for name in ("compute_stream", "h2d_stream"):
            raw, wrapped = new_stream(self.device)
            self._raw_streams.append(raw)
            setattr(self, name, wrapped)
        self.out_torch_dtype = torch.float32 if out_dtype else torch.float16
        self.ctx = binding.Context(
            n_layers=L, n_q_heads=H, n_kv_heads=G, head_dim=d, block_tokens=T, max_batch=B,
            max_blocks_per_seq=self.max_blocks, max_ctx=self.max_ctx, blocks_per_layer=self.blocks_per_layer,
            out_dtype=out_dtype, split_tokens=split_tokens,
            dev_pool=self.dev_part, host_pool=self.host_part,
            staging=tuple(self.staging), staging_bytes=self.staging_bytes,
            resident_blocks=resident_blocks, chunk_blocks=chunk_blocks,
            workspace=self.workspace, workspace_bytes=self.workspace_bytes,
            tail_blocks=self.tail_blocks, tail_bytes=self.tail_bytes,
            compute_stream=self.compute_stream.cuda_stream, h2d_stream=self.h2d_stream.cuda_stream)
        self.block_table = None
        self.ctx_lens = None

    def _allocate_pools(self, L, n_el, resident_blocks, chunk_blocks, shape):
        if self.by_class:
            self.block_elems = binding.okv_block_bytes(shape) // 2
            self.split_at = resident_blocks * self.block_elems      # first element of the host part
            host_el = n_el - self.split_at
            for l in range(L):
                if self.split_at:
                    self.dev_part[l] = torch.empty(self.split_at, dtype=torch.float16, device=self.device)
                if host_el:
                    self._pinned.append(PinnedHalfBuffer(host_el))
                    self.host_part[l] = self._pinned[-1].tensor
            self._any_host = host_el > 0
            self._staging_el = min(chunk_blocks, self.blocks_per_layer - resident_blocks) * self.block_elems
        else:
            for l in range(L):
                if self.on_host[l]:
                    self._pinned.append(PinnedHalfBuffer(n_el))
                    self.pools.append(self._pinned[-1].tensor)
                    self.host_part[l] = self.pools[-1]
                else:
                    self.pools.append(torch.empty(n_el, dtype=torch.float16, device=self.device))
                    self.dev_part[l] = self.pools[-1]
            self._any_host = bool(self.on_host.any())
            self._staging_el = n_el

    # ---- batch ------------------------------------------------------------------
    def set_batch(self, ctx_lens, block_table=None):
        self.ctx_lens = np.asarray(ctx_lens, dtype=np.int32).copy()
        self.block_table = None if block_table is None else np.asarray(block_table, dtype=np.int32).copy()
        self.ctx.okv_set_batch(self.block_table, self.ctx_lens)

    def layout(self):
        """The pool layout in the form the CPU oracle's own indexing takes."""
        if self.paged:
            return {"kind": "paged", "G": self.G, "d": self.d, "T": self.T, "block_table": self.block_table}
        return {"kind": "contiguous", "G": self.G, "d": self.d, "C": self.max_ctx}

    # ---- data -------------------------------------------------------------------
    def fill_pool(self, layer, seed, chunk_elems=1 << 27):
        """N(0,1) fp16 into the whole pool of `layer` (generated on the GPU;
        host pools receive it by plain copies)."""
        parts = [p for p in (self.dev_part[layer], self.host_part[layer]) if p is not None]
        for part, sd in zip(parts, (seed, seed ^ 0x5DEECE66D)):     # a layer in one piece gets `seed` wherever it lives
            if part.is_cuda:
                synth.fill_randn_f16_(part, sd, chunk_elems)
                continue
            gen = torch.Generator(device=self.device)
            gen.manual_seed(sd)
            n = part.numel()
            for lo in range(0, n, chunk_elems):
                hi = min(n, lo + chunk_elems)
                tmp = torch.randn(hi - lo, generator=gen, device=self.device, dtype=torch.float32).to(torch.float16)
                part[lo:hi].copy_(tmp)
        torch.cuda.synchronize(self.device)

    def _parts(self, layer):
        """[(first element, tensor)] of the layer's pool in id order."""
        out, at = [], 0
        for part in (self.dev_part[layer], self.host_part[layer]):
            if part is not None:
                out.append((at, part))
                at += part.numel()
        return out

    def read_pool(self, layer, flush=True):
        """A host numpy copy (fp16, flat) of the layer's pool as it is stored
        (HBM part first, then the host part).  Rows still held in HBM slots are written out first
        unless flush is False."""
        if flush and self.hot_tails and self.ctx_lens is not None:
            self.ctx.okv_flush_tails()
        torch.cuda.synchronize(self.device)
        return np.concatenate([p.cpu().numpy() for _, p in self._parts(layer)])

    def read_rows(self, layer, row_offsets):
        """Rows of d fp16 numbers at the given element offsets -> [n][d] numpy."""
        if self.hot_tails and self.ctx_lens is not None:
            self.ctx.okv_flush_tails()
        torch.cuda.synchronize(self.device)
        idx = torch.as_tensor(np.asarray(row_offsets, dtype=np.int64))
        cols = torch.arange(self.d, dtype=torch.int64)
        out = torch.empty((len(row_offsets), self.d), dtype=torch.float16)
        for first, part in self._parts(layer):
            sel = (idx >= first) & (idx < first + part.numel())
            if not bool(sel.any()):
                continue
            flat = ((idx[sel] - first)[:, None] + cols[None, :]).reshape(-1)
            rows = part[flat.to(self.device)].cpu() if part.is_cuda else part[flat]
            out[sel] = rows.reshape(-1, self.d)
        return out.numpy().copy()

    # ---- one decode step ---------------------------------------------------------
    def step(self, q, k_new, v_new, out):
        """One pass of the hot path: for every layer append, then attend.
        q / k_new / v_new / out are per-layer lists of device tensors (or single
        tensors reused for every layer)."""
        def pick(x, l):
            return x[l] if isinstance(x, (list, tuple)) else x
        c = self.ctx
        c.okv_step_begin()
        for l in range(self.L):
            c.kv_append(l, pick(k_new, l), pick(v_new, l))
            c.decode_attn(l, pick(q, l), pick(out, l))
        c.okv_step_end()
        if self.ctx_lens is not None:
            self.ctx_lens += 1

    def bind_step(self, q, k_new, v_new, out):
        """Pointer arrays for step_bound: build once for buffers that every step reuses."""
        def per_layer(x):
            return list(x) if isinstance(x, (list, tuple)) else [x] * self.L
        tensors = tuple(per_layer(x) for x in (q, k_new, v_new, out))
        return self.ctx.pointer_arrays(*tensors), tensors          # the tensors ride along to stay alive

    def step_bound(self, bound):
        """The same pass as step(), all layers issued by one call into the library."""
        self.ctx.okv_decode_step(bound[0])
        if self.ctx_lens is not None:
            self.ctx_lens += 1

    def prefill(self, n_new, k_rows, v_rows, release=True):
        """Stores n_new[b] new tokens per sequence in every layer.  k_rows / v_rows are
        per-layer lists of device tensors [sum(n_new)][G][d] (or single tensors reused)."""
        def pick(x, l):
            return x[l] if isinstance(x, (list, tuple)) else x
        c = self.ctx
        c.okv_prefill_begin(n_new)
        for l in range(self.L):
            c.kv_append_bulk(l, pick(k_rows, l), pick(v_rows, l))
            if release:
                c.okv_prefill_release(l)
        c.okv_prefill_end()
        if self.ctx_lens is not None:
            self.ctx_lens += np.asarray(n_new, dtype=np.int32)

    def ctx_units(self):
        """The chunks of the host pool that hold blocks of the current batch (block-class
        mode): each is copied once per layer and step."""
        host_ids = self.block_table[self.block_table >= self.resident_blocks] - self.resident_blocks
        return sorted(set((host_ids // self.chunk_blocks).tolist()))

    def synchronize(self):
        self.ctx.okv_synchronize()

    def close(self):
        self.ctx.close()
        for raw in self._raw_streams:
            _hip_runtime().hipStreamDestroy(ctypes.c_void_p(raw))
        self._raw_streams = []
        self.pools, self.dev_part, self.host_part = [], [], []
        for p in self._pinned:
            p.free()
        self._pinned = []


class LayerWeights:
    """The matrices and vectors of one decoder layer (fp16 on the device), row-major as a
    framework holds them, plus the rearranged copies okv_linear reads.  The query, key and
    value projections are stacked into one [h1 + 2 kv_cols][h1] matrix so that one product serves
    all three."""

    NAMES = ("ln1_g", "ln1_b", "wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")

    def __init__(self, h1, h2, seed, layer, device, kv_cols=None):
        """kv_cols: width of the key and value projections (n_kv_heads * head_dim); h1 when the heads are not grouped."""
        self.h1, self.h2 = h1, h2
        self.kv_cols = kv = h1 if kv_cols is None else kv_cols
        t = {}
        for i, name in enumerate(self.NAMES):
            sd = synth.stream_seed(seed, 100 + i, layer)
            if name.startswith("w"):
                n_out, n_in = (h2, h1) if name == "w1" else (h1, h2) if name == "w2" else (kv, h1) if name in ("wk", "wv") else (h1, h1)
                t[name] = (synth.randn_f16_torch((n_out, n_in), sd, device).float() / n_in ** 0.5).to(torch.float16)
            elif name.endswith("_g"):
                t[name] = (1.0 + 0.1 * synth.randn_f16_torch((h1,), sd, device).float()).to(torch.float16)
            else:
                n = h2 if name == "b1" else kv if name in ("bk", "bv") else h1
                t[name] = (0.1 * synth.randn_f16_torch((n,), sd, device).float()).to(torch.float16)
        self.t = t
        self.wqkv = torch.cat([t["wq"], t["wk"], t["wv"]], dim=0).contiguous()
        self.bqkv = torch.cat([t["bq"], t["bk"], t["bv"]], dim=0).contiguous()
        self.packed = {}
        for name, w in (("wqkv", self.wqkv), ("wo", t["wo"]), ("w1", t["w1"]), ("w2", t["w2"])):
            dst = torch.empty_like(w)
            binding.okv_pack_linear_weight(dst, w, w.shape[0], w.shape[1])
            self.packed[name] = dst
        torch.cuda.synchronize(device)

    def numpy(self):
        """fp64 copies for the oracle."""
        return {k: v.double().cpu().numpy() for k, v in self.t.items()}

    def bytes_read_per_step(self):
        return sum(w.numel() * 2 for w in self.packed.values())


class LayerScratch:
    """Activation buffers of one decode step (fp16, reused by every layer)."""

    def __init__(self, B, h1, h2, G, d, device):
        def buf(*shape):
            return torch.empty(shape, dtype=torch.float16, device=device)
        self.a, self.q, self.k, self.v = buf(B, h1), buf(B, h1), buf(B, G * d), buf(B, G * d)
        self.t, self.y, self.z, self.u = buf(B, h1), buf(B, h1), buf(B, h1), buf(B, h2)
        # one workspace for the four products of a layer (they follow one another on one stream)
        self.ws_bytes = max(16, max(binding.okv_linear_workspace_bytes(B, n_out, n_in)
                                    for n_out, n_in in ((h1 + 2 * G * d, h1), (h1, h1), (h2, h1), (h1, h2))))
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)


class BoundLayers:
    """The stack's decoder layers handed to the library once: the array of okv_decoder_layer and the
    scratch that okv_decoder_step works in.  step(x) is then one call per decode step."""

    def __init__(self, st, weights, scratch):
        self.st, self.weights, self.ws = st, weights, scratch          # keeps the tensors alive
        self.h2 = weights[0].h2
        self.layers = binding.Context.decoder_layers([
            dict(ln1_gamma=w.t["ln1_g"], ln1_beta=w.t["ln1_b"], w_qkv=w.packed["wqkv"], b_qkv=w.bqkv, w_o=w.packed["wo"], b_o=w.t["bo"],
                 ln2_gamma=w.t["ln2_g"], ln2_beta=w.t["ln2_b"], w_ff1=w.packed["w1"], b_ff1=w.t["b1"], w_ff2=w.packed["w2"],
                 b_ff2=w.t["b2"]) for w in weights])
        self.scratch_bytes = st.ctx.okv_decoder_scratch_bytes(st.B, self.h2)
        self.scratch = torch.empty(self.scratch_bytes, dtype=torch.uint8, device=scratch.ws.device)

    def step(self, x):
        self.st.ctx.okv_decoder_step(self.layers, self.h2, x, self.scratch, self.scratch_bytes, self.ws.ws, self.ws.ws_bytes)
        if self.st.ctx_lens is not None:
            self.st.ctx_lens += 1


def decode_step_with_layers(st, weights, scratch, x):
    """One decode step of whole decoder layers: for every layer, layer norm, the stacked
    query/key/value projection, kv_append + decode_attn, output projection with residual,
    layer norm, feed-forward block with ReLU and residual.  x: fp16 [B][h1] on the device,
    overwritten with the stack's output.  Every operation is a call into the library on the
    stack's compute stream."""
    c, s, B = st.ctx, scratch, st.B
    cs = st.compute_stream.cuda_stream
    h1, h2 = weights[0].h1, weights[0].h2
    c.okv_step_begin()
    binding.okv_layernorm(x, weights[0].t["ln1_g"], weights[0].t["ln1_b"], s.a, B, h1, 1e-5, cs)
    for l, w in enumerate(weights):
        binding.okv_linear_qkv(s.a, w.packed["wqkv"], w.bqkv, s.q, s.k, s.v, B, h1, w.kv_cols, h1, cs, s.ws, s.ws_bytes)
        c.kv_append(l, s.k, s.v)
        c.decode_attn(l, s.q, s.t)
        # output projection + residual, and the second norm of its result in the same pass
        binding.okv_linear_layernorm(s.t, w.packed["wo"], w.t["bo"], x, s.y, w.t["ln2_g"], w.t["ln2_b"], s.z, B, h1, h1, 1e-5,
                                     False, cs, s.ws, s.ws_bytes)
        binding.okv_linear(s.z, w.packed["w1"], w.t["b1"], None, s.u, B, h2, h1, True, cs, s.ws, s.ws_bytes)
        if l + 1 < len(weights):                         # ... and the next layer's first norm rides on the feed-forward block
            nxt = weights[l + 1]
            binding.okv_linear_layernorm(s.u, w.packed["w2"], w.t["b2"], s.y, x, nxt.t["ln1_g"], nxt.t["ln1_b"], s.a, B, h1, h2,
                                         1e-5, False, cs, s.ws, s.ws_bytes)
        else:
            binding.okv_linear(s.u, w.packed["w2"], w.t["b2"], s.y, x, B, h1, h2, False, cs, s.ws, s.ws_bytes)
    c.okv_step_end()
    if st.ctx_lens is not None:
        st.ctx_lens += 1
