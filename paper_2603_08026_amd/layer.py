"""Device-side holder of one layer's weights, caches and index buffers.

Convenience over the raw binding for tests and the bench: it allocates torch
tensors, uploads numpy inputs and calls the library.  No step of the method is
computed here.
"""
from __future__ import annotations

from typing import Dict, Optional, Tuple

import numpy as np
import torch

from . import binding as B_


def torch_dtype(dtype: str):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def to_device(a: np.ndarray, dtype: str) -> torch.Tensor:
    """fp32 numpy values (already representable in dtype) -> device tensor of the storage type."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t if dtype == "f32" else t.to(torch.bfloat16)


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


MATRICES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


class Layer:
    def __init__(self, hidden, n_heads, n_kv_heads, head_dim, ffn, dtype: str, batch: int, seq: int,
                 max_rows: int = 0, rms_eps: float = 1e-5, rope_theta: float = 10000.0, ctx=None,
                 keep_lse: bool = False):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the dyllm library only runs on a HIP device")
        self.dtype = dtype
        self.B, self.L = batch, seq
        self.hidden, self.H, self.Hkv, self.dh, self.F = hidden, n_heads, n_kv_heads, head_dim, ffn
        self.dq, self.dkv = n_heads * head_dim, n_kv_heads * head_dim
        self.cfg = B_.LayerCfg(hidden, n_heads, n_kv_heads, head_dim, ffn, batch, seq, max_rows,
                               B_.F32 if dtype == "f32" else B_.BF16, rms_eps, rope_theta)
        self.ctx = B_.Context(self.cfg) if ctx is None else ctx  # layers of a stack share one
        td = torch_dtype(dtype)
        T = batch * seq
        self.k = torch.zeros(batch, seq, n_kv_heads, head_dim, dtype=td, device="cuda")
        self.v = torch.zeros_like(self.k)
        self.c = torch.zeros(batch, seq, self.dq, dtype=td, device="cuda")
        self.out = torch.zeros(batch, seq, hidden, dtype=td, device="cuda")
        # optional fifth cache: log-normalisers of every token's last exact attention row (needed by the
        # reused-normaliser variant of the approximate update; the dense step then runs its merge kernel)
        self.lse = torch.zeros(batch, seq, n_heads, dtype=torch.float32, device="cuda") if keep_lse else None
        self.cache = B_.make_cache(self.k, self.v, self.c, self.out, self.lse)
        self.rows_cap = max_rows if max_rows > 0 else T
        self.idx_out = B_.IndexList.empty(self.rows_cap, batch)
        self.cos = torch.zeros(self.rows_cap, dtype=torch.float32, device="cuda")
        self.wt: Dict[str, torch.Tensor] = {}
        self.w = None

    @classmethod
    def from_shape(cls, shape, batch, seq, max_rows=0, ctx=None, keep_lse=False):
        return cls(shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.ffn, shape.dtype,
                   batch, seq, max_rows, shape.rms_eps, shape.rope_theta, ctx, keep_lse)

    def pack(self, t: torch.Tensor) -> torch.Tensor:
        """Row-major bf16 matrix -> a new tensor in the panel layout the bf16 kernels read (library call)."""
        out = torch.empty_like(t)
        B_.pack_weight(t, out)
        return out

    def _install(self, wt: Dict[str, torch.Tensor], packed: bool):
        if self.dtype != "f32" and not packed:
            wt = {n: (self.pack(t) if n in MATRICES else t) for n, t in wt.items()}
        self.wt = dict(wt)  # what the library reads (bf16: packed matrices)
        self.w = B_.make_weights(self.wt)

    def set_weights(self, w: Dict[str, np.ndarray]):
        """Row-major host weights [out, in]; bf16 layers re-lay the matrices on the device."""
        self._install({k: to_device(v, self.dtype) for k, v in w.items() if v is not None}, False)

    def set_device_weights(self, wt: Dict[str, torch.Tensor], packed: bool = False):
        """Weights that already live on the device in the storage type (large synthetic stacks);
        packed: the bf16 matrices are already in the panel layout (e.g. another layer's `wt`)."""
        self._install(wt, packed)

    def set_caches(self, caches: Dict[str, np.ndarray]):
        for name in ("k", "v", "c", "out"):
            getattr(self, name).copy_(to_device(caches[name].astype(np.float32), self.dtype))
        if "lse" in caches and self.lse is not None:
            self.lse.copy_(torch.from_numpy(np.ascontiguousarray(caches["lse"], dtype=np.float32)).cuda())

    def get_caches(self) -> Dict[str, np.ndarray]:
        return {n: to_host(getattr(self, n)) for n in ("k", "v", "c", "out")}

    def make_list(self, idx: np.ndarray, offsets: np.ndarray, cap: Optional[int] = None) -> B_.IndexList:
        cap = int(idx.size if cap is None else cap)
        buf = np.zeros(max(cap, 1), dtype=np.int32)
        buf[:idx.size] = idx
        il = B_.IndexList(torch.from_numpy(buf).cuda()[:cap],
                          torch.from_numpy(np.ascontiguousarray(offsets, dtype=np.int32)).cuda())
        return il

    def upload(self, x: np.ndarray) -> torch.Tensor:
        return to_device(x, self.dtype)

    def full_step(self, x_dev: torch.Tensor):
        self.ctx.full_step(self.w, self.cache, x_dev, self.B, self.L)

    def layer_step(self, x_dev: torch.Tensor, idx_in: B_.IndexList, tau: float,
                   idx_out: Optional[B_.IndexList] = None, want_cos: bool = True):
        out = self.idx_out if idx_out is None else idx_out
        self.ctx.layer_step(self.w, self.cache, x_dev, idx_in, self.B, self.L, tau, out,
                            self.cos if want_cos else None)
        return out

    def layer_step_approx(self, x_dev: torch.Tensor, idx_in: B_.IndexList, tau: float,
                          idx_out: Optional[B_.IndexList] = None, cos_out: Optional[torch.Tensor] = None,
                          row_lo: int = 0, cached_norm: bool = False):
        """Sparse step with the approximate update of the other tokens; the context must cover B*L rows.
        cos_out: [B*L] fp32 (by token) or None; row_lo > 0: response-only step; cached_norm: reuse the
        cached softmax normalisers instead of Alg. 4's sum over all keys."""
        out = self.idx_out if idx_out is None else idx_out
        self.ctx.layer_step_approx(self.w, self.cache, x_dev, idx_in, self.B, self.L, tau, out, cos_out, row_lo,
                                   cached_norm)
        return out

    def read_list(self, il: B_.IndexList) -> Tuple[np.ndarray, np.ndarray]:
        off = il.offsets.cpu().numpy()
        n = int(off[-1])
        return il.idx[:n].cpu().numpy(), off

    def close(self):
        self.ctx.close()


class Stack:
    """n_layers layers sharing one library context; layer l reads layer l-1's output cache."""

    def __init__(self, shape, n_layers: int, batch: int, seq: int, max_rows: int = 0, keep_lse: bool = False):
        first = Layer.from_shape(shape, batch, seq, max_rows, keep_lse=keep_lse)
        self.layers = [first] + [Layer.from_shape(shape, batch, seq, max_rows, ctx=first.ctx, keep_lse=keep_lse)
                                 for _ in range(n_layers - 1)]
        self.ctx, self.B, self.L, self.dtype = first.ctx, batch, seq, first.dtype
        cap = first.rows_cap
        self.idx_outs = [l.idx_out for l in self.layers]
        self.cos = torch.zeros(n_layers, cap, dtype=torch.float32, device="cuda")

    def upload(self, x: np.ndarray) -> torch.Tensor:
        return to_device(x, self.dtype)

    def make_list(self, idx, offsets, cap=None):
        return self.layers[0].make_list(idx, offsets, cap)

    def full_step(self, x_dev: torch.Tensor):
        self.ctx.stack_full_step([l.w for l in self.layers], [l.cache for l in self.layers], x_dev,
                                 self.B, self.L)

    def stack_step(self, x_dev: torch.Tensor, idx_in: B_.IndexList, tau: float, want_cos: bool = True):
        """cos rows are strided by idx_in's capacity, as the library writes them."""
        cos = self.cos.view(-1)[:len(self.layers) * idx_in.cap] if want_cos else None
        self.ctx.stack_step([l.w for l in self.layers], [l.cache for l in self.layers], x_dev, idx_in,
                            self.B, self.L, tau, self.idx_outs, cos)
        return self.idx_outs

    def stack_step_approx(self, x_dev: torch.Tensor, idx_in: B_.IndexList, tau: float, row_lo: int = 0,
                          cos_out: Optional[torch.Tensor] = None, cached_norm: bool = False):
        """cos_out: [n_layers, B*L] fp32 (by token) or None."""
        self.ctx.stack_step_approx([l.w for l in self.layers], [l.cache for l in self.layers], x_dev, idx_in,
                                   self.B, self.L, tau, self.idx_outs, cos_out, row_lo, cached_norm)
        return self.idx_outs

    def denoise_step(self, sched: B_.Schedule, t: int, x_dev: torch.Tensor, decoded, carry, cand: B_.IndexList):
        """One iteration of the generation loop; returns (step kind, the list to carry or None)."""
        kind = self.ctx.denoise_step(sched, t, [l.w for l in self.layers], [l.cache for l in self.layers],
                                     x_dev, decoded, carry, self.B, self.L, cand, self.idx_outs)
        return kind, (None if kind == B_.STEP_DENSE else self.idx_outs[-1])

    def close(self):
        self.ctx.close()
