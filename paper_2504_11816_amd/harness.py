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
    return _hip


class PinnedHalfBuffer:
    """n fp16 elements of pinned, device-mapped host memory (hipHostMalloc of
    exactly that size; torch's pinned allocator would round it up to a power of
    two), viewed as a torch CPU tensor."""

    def __init__(self, n_elems):
        self.nbytes = n_elems * 2
        p = ctypes.c_void_p(0)
        rc = _hip_runtime().hipHostMalloc(ctypes.byref(p), self.nbytes, 0)
        if rc != 0 or not p.value:
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
    two staging buffers), 0 keeps it in HBM.
    """

    def __init__(self, *, L, H, G, d, B, T, cap_tokens, on_host=None, out_dtype=0, split_tokens=0,
                 blocks_per_layer=None, n_staging=2, device="cuda:0"):
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
            self.max_ctx = (cap_tokens + 15) // 16 * 16
            self.cap_tokens = self.max_ctx
            self.blocks_per_layer = 0
        shape = binding.make_config(n_layers=L, n_q_heads=H, n_kv_heads=G, head_dim=d, block_tokens=T,
                                    max_batch=B, max_blocks_per_seq=self.max_blocks, max_ctx=self.max_ctx,
                                    blocks_per_layer=self.blocks_per_layer, out_dtype=out_dtype,
                                    split_tokens=split_tokens)
        self.pool_bytes = binding.okv_layer_pool_bytes(shape)
        self.workspace_bytes = binding.okv_workspace_bytes(shape)
        n_el = self.pool_bytes // 2
        self.pools, self._pinned = [], []
        for l in range(L):
            if self.on_host[l]:
                self._pinned.append(PinnedHalfBuffer(n_el))
                self.pools.append(self._pinned[-1].tensor)
            else:
                self.pools.append(torch.empty(n_el, dtype=torch.float16, device=self.device))
        any_host = bool(self.on_host.any())
        self.staging = [torch.empty(n_el, dtype=torch.float16, device=self.device) if any_host and i < n_staging
                        else None for i in range(4)]
        self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=self.device)
        self.compute_stream = torch.cuda.Stream(device=self.device)
        self.h2d_stream = torch.cuda.Stream(device=self.device)
        self.out_torch_dtype = torch.float32 if out_dtype else torch.float16
        self.ctx = binding.Context(
            n_layers=L, n_q_heads=H, n_kv_heads=G, head_dim=d, block_tokens=T, max_batch=B,
            max_blocks_per_seq=self.max_blocks, max_ctx=self.max_ctx, blocks_per_layer=self.blocks_per_layer,
            out_dtype=out_dtype, split_tokens=split_tokens,
            dev_pool=[None if self.on_host[l] else self.pools[l] for l in range(L)],
            host_pool=[self.pools[l] if self.on_host[l] else None for l in range(L)],
            staging=tuple(self.staging), staging_bytes=self.pool_bytes if any_host else 0,
            workspace=self.workspace, workspace_bytes=self.workspace_bytes,
            compute_stream=self.compute_stream.cuda_stream, h2d_stream=self.h2d_stream.cuda_stream)
        self.block_table = None
        self.ctx_lens = None

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
        pool = self.pools[layer]
        if pool.is_cuda:
            synth.fill_randn_f16_(pool, seed, chunk_elems)
            return
        gen = torch.Generator(device=self.device)
        gen.manual_seed(seed)
        n = pool.numel()
        for lo in range(0, n, chunk_elems):
            hi = min(n, lo + chunk_elems)
            tmp = torch.randn(hi - lo, generator=gen, device=self.device, dtype=torch.float32).to(torch.float16)
            pool[lo:hi].copy_(tmp)
        torch.cuda.synchronize(self.device)

    def read_pool(self, layer):
        """A host numpy copy (fp16, flat) of the layer's pool as it is stored."""
        torch.cuda.synchronize(self.device)
        return self.pools[layer].cpu().numpy().copy()

    def read_rows(self, layer, row_offsets):
        """Rows of d fp16 numbers at the given element offsets -> [n][d] numpy."""
        torch.cuda.synchronize(self.device)
        pool = self.pools[layer]
        idx = torch.as_tensor(np.asarray(row_offsets, dtype=np.int64))
        cols = torch.arange(self.d, dtype=torch.int64)
        flat = (idx[:, None] + cols[None, :]).reshape(-1)
        if pool.is_cuda:
            rows = pool[flat.to(self.device)].cpu()
        else:
            rows = pool[flat]
        return rows.numpy().reshape(len(row_offsets), self.d).copy()

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

    def synchronize(self):
        self.ctx.okv_synchronize()

    def close(self):
        self.ctx.close()
        self.pools = []
        for p in self._pinned:
            p.free()
        self._pinned = []
