"""GPU-side plumbing shared by the tests, the smoke check and the benchmark:
torch allocates device memory and hands out streams, everything else is a call
into libzz.so.  Holds no reference arithmetic and never imports the oracle."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as zb


def to_dev_bf16(x: np.ndarray) -> torch.Tensor:
    """bf16-exact float32 numpy array -> contiguous bf16 CUDA tensor (exact)."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device="cuda", dtype=torch.bfloat16).contiguous()


def from_dev(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(dtype=torch.float32, device="cpu").numpy()


class Stack:
    """A context plus the device memory it lives in."""

    def __init__(self, n_layers, n_q_heads, n_kv_heads, head_dim, batch, max_ctx, sink, window, max_chunk=0,
                 layout=zb.ZZ_ZIGZAG, layer_is_streaming=None, kvhead_is_streaming=None, softmax_scale=0.0,
                 poison_arena=False):
        self.cfg, keep = zb.make_config(n_layers, n_q_heads, n_kv_heads, head_dim, batch, max_ctx, sink, window,
                                        max_chunk, layout, softmax_scale, layer_is_streaming, kvhead_is_streaming)
        self.arena_nbytes = zb.arena_bytes(self.cfg)
        self.ws_nbytes = zb.workspace_bytes(self.cfg)
        if self.arena_nbytes == 0:
            raise ValueError("invalid configuration")
        self.arena = torch.empty(self.arena_nbytes, dtype=torch.uint8, device="cuda")
        if poison_arena:
            # 0xFF bytes are bf16 NaN patterns: an unwritten slot that leaks into a result shows up
            self.arena.fill_(0xFF)
        self.workspace = torch.empty(self.ws_nbytes, dtype=torch.uint8, device="cuda")
        self.ctx = zb.Context(self.cfg, self.arena, self.workspace, keep=keep)
        self.shape = dict(L=n_layers, Hq=n_q_heads, Hkv=n_kv_heads, D=head_dim, B=batch)

    def stream_ptr(self):
        return torch.cuda.current_stream().cuda_stream

    def append(self, layer, k_new, v_new):
        n_new = k_new.shape[1]
        self.ctx.kv_append(layer, k_new, v_new, n_new, self.stream_ptr())

    def prefill(self, layer, q, k_new, v_new):
        out = torch.empty_like(q)
        self.ctx.attn_prefill(layer, q, k_new, v_new, q.shape[1], out, self.stream_ptr())
        return out

    def decode(self, layer, q, out=None):
        if out is None:
            out = torch.empty_like(q)
        self.ctx.attn_decode(layer, q, out, self.stream_ptr())
        return out

    def decode_step(self, layer, q, k_new, v_new, out=None):
        if out is None:
            out = torch.empty_like(q)
        self.ctx.decode_step(layer, q, k_new, v_new, out, self.stream_ptr())
        return out

    def arena_host(self) -> np.ndarray:
        torch.cuda.synchronize()
        return self.arena.cpu().numpy()

    def read_cache_rows(self, arena_host, layer, which, b, kv_head, slots) -> np.ndarray:
        """uint16 [len(slots), D] bit patterns of the given slots, every element
        located through zz_kv_elem_offset (offsets are looked up once and kept)."""
        D = self.shape["D"]
        key = (layer, which, b, kv_head)
        cache = self.__dict__.setdefault("_off", {})
        if key not in cache:
            cap = 0
            while self.ctx.kv_elem_offset(layer, which, b, kv_head, cap, 0) >= 0:
                cap += 1
            off = np.empty((cap, D), dtype=np.int64)
            for s in range(cap):
                for d in range(D):
                    off[s, d] = self.ctx.kv_elem_offset(layer, which, b, kv_head, s, d)
            assert (off >= 0).all() and (off % 2 == 0).all()
            cache[key] = off // 2
        a16 = arena_host.view(np.uint16)
        return a16[cache[key][np.asarray(slots, dtype=np.int64)]]
