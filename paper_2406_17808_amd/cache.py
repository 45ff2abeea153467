"""Thin convenience layer over the binding for callers that hold torch tensors.

It owns the device workspace (a torch uint8 tensor) and passes data pointers and the current
stream to the C ABI.  No arithmetic of the method happens here.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B
from .workloads import Workload


def config_of(wl: Workload, max_chunk: Optional[int] = None, batch: Optional[int] = None, **overrides) -> B.cascade_config:
    kw = dict(batch=wl.batch if batch is None else batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
              head_dim=wl.head_dim, dtype=B.CASCADE_BF16 if wl.dtype == "bf16" else B.CASCADE_F32,
              n_sink=wl.n_sink, cascade_sizes=list(wl.cascade_sizes), ema_beta=wl.ema_beta,
              rope_base=wl.rope_base, max_chunk=wl.chunk if max_chunk is None else max_chunk)
    kw.update(overrides)
    return B.make_config(**kw)


class CascadeKVCache:
    def __init__(self, cfg: B.cascade_config, device: str = "cuda:0", init_state: Optional[B.cascade_init_state] = None,
                 _layer_of=None, static_workspace: bool = False):
        self.cfg = cfg
        self.device = torch.device(device)
        self.torch_dtype = torch.bfloat16 if cfg.dtype == B.CASCADE_BF16 else torch.float32
        if _layer_of is not None:      # a layer of CascadeKVLayers: the context exists, the workspace is the owner's
            self.workspace, self.ctx, self.workspace_bytes = _layer_of
            return
        if static_workspace:           # the library's own device array: nothing is allocated here
            self.workspace, self.workspace_bytes = None, B.cascade_workspace_bytes(cfg)
            with torch.cuda.device(self.device):
                self.ctx = B.cascade_init_static(cfg, init_state, self._stream())
            return
        nbytes = B.cascade_workspace_bytes(cfg)
        if nbytes == 0:
            # let cascade_init report why
            B.cascade_init(cfg, 256, 0)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        ptr = (self.workspace.data_ptr() + 255) & ~255
        with torch.cuda.device(self.device):
            self.ctx = B.cascade_init(cfg, ptr, nbytes, init_state, self._stream())
        self.workspace_bytes = nbytes

    def _stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def close(self):
        if getattr(self, "ctx", None):
            torch.cuda.synchronize(self.device)
            B.cascade_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, x: torch.Tensor, shape):
        assert x.is_cuda and x.dtype == self.torch_dtype and x.is_contiguous() and tuple(x.shape) == tuple(shape), \
            (x.dtype, tuple(x.shape), tuple(shape))

    def prefill_chunk(self, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, out: Optional[torch.Tensor] = None):
        c = self.cfg
        n = q.shape[1]
        self._check(q, (c.batch, n, c.n_q_heads, c.head_dim))
        self._check(k, (c.batch, n, c.n_kv_heads, c.head_dim))
        self._check(v, (c.batch, n, c.n_kv_heads, c.head_dim))
        if out is None:
            out = torch.empty_like(q)
        self._check(out, q.shape)
        B.cascade_prefill_chunk(self.ctx, q.data_ptr(), k.data_ptr(), v.data_ptr(), n, out.data_ptr(), self._stream())
        return out

    def decode_step(self, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, out: Optional[torch.Tensor] = None):
        c = self.cfg
        self._check(q, (c.batch, c.n_q_heads, c.head_dim))
        self._check(k, (c.batch, c.n_kv_heads, c.head_dim))
        self._check(v, (c.batch, c.n_kv_heads, c.head_dim))
        if out is None:
            out = torch.empty_like(q)
        self._check(out, q.shape)
        B.cascade_decode_step(self.ctx, q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), self._stream())
        return out

    def read_state(self, with_kv: bool = False, kv_pairs=None) -> B.StateArrays:
        return B.cascade_read_state(self.ctx, self.cfg, with_kv, self._stream(), kv_pairs)


class CascadeKVLayers:
    """The caches of several attention layers over one workspace (the layer loop of Alg. 1): every
    layer is a CascadeKVCache of its own, the per-call scratch exists once.  Calls on the layers
    must be ordered with each other; issuing them on one stream, as here, does that."""

    def __init__(self, cfg: B.cascade_config, n_layers: int, device: str = "cuda:0", init_states=None):
        self.cfg = cfg
        self.device = torch.device(device)
        nbytes = B.cascade_layers_workspace_bytes(cfg, n_layers)
        if nbytes == 0:
            B.cascade_init_layers(cfg, n_layers, 256, 0)      # reports why
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        self.workspace_bytes = nbytes
        ptr = (self.workspace.data_ptr() + 255) & ~255
        with torch.cuda.device(self.device):
            ctxs = B.cascade_init_layers(cfg, n_layers, ptr, nbytes, init_states,
                                         torch.cuda.current_stream(self.device).cuda_stream)
        self.layers = [CascadeKVCache(cfg, device, _layer_of=(self.workspace, c, nbytes)) for c in ctxs]

    def __len__(self):
        return len(self.layers)

    def __getitem__(self, i) -> CascadeKVCache:
        return self.layers[i]

    def close(self):
        for layer in self.layers:
            layer.close()
