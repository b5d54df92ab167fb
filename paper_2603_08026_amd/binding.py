"""ctypes binding of libdyllm.so: argument marshalling only.

Every function mirrors one entry point of include/dyllm.h and passes raw
device pointers of torch tensors (torch is used for device memory and streams
only).  There is no fallback: if the HIP library is missing or fails, calls
raise.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdyllm.so")

F32, BF16 = 0, 1
OK, ERR_INVALID_ARG, ERR_BAD_SHAPE, ERR_UNSUPPORTED, ERR_NO_MEM, ERR_HIP, ERR_CAPACITY = 0, -1, -2, -3, -4, -5, -6

SYMBOLS = [
    "dyllm_workspace_bytes", "dyllm_create", "dyllm_destroy", "dyllm_strerror", "dyllm_last_error",
    "dyllm_poll_status", "dyllm_saliency", "dyllm_compact", "dyllm_compact_static", "dyllm_qkv_refresh",
    "dyllm_partial_attention", "dyllm_salient_ffn", "dyllm_layer_step", "dyllm_layer_step_approx",
    "dyllm_stack_step_approx", "dyllm_merge_lists", "dyllm_step_kind", "dyllm_denoise_step", "dyllm_full_step",
    "dyllm_stack_step", "dyllm_stack_full_step", "dyllm_pack_weight",
    "dyllm_profile_begin", "dyllm_profile_end", "dyllm_stage_count", "dyllm_stage_name",
]


class DyllmError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("dyllm error %d: %s" % (code, msg))
        self.code = code


class LayerCfg(C.Structure):
    _fields_ = [
        ("hidden", C.c_int32), ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("ffn_dim", C.c_int32), ("max_batch", C.c_int32),
        ("max_seq", C.c_int32), ("max_rows", C.c_int32), ("dtype", C.c_int32),
        ("rms_eps", C.c_float), ("rope_theta", C.c_float),
    ]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in (
        "wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "bq", "bk", "bv", "g_attn", "g_ffn")]


class LayerCache(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("k", "v", "c", "out", "lse")]


class IndexListC(C.Structure):
    _fields_ = [("idx", C.c_void_p), ("offsets", C.c_void_p), ("cap", C.c_int32)]


class Schedule(C.Structure):
    _fields_ = [("t_full", C.c_int32), ("full_period", C.c_int32), ("prompt_len", C.c_int32),
                ("approx", C.c_int32), ("tau", C.c_float)]


STEP_DENSE, STEP_FULL, STEP_RESPONSE = 0, 1, 2


_lib = None


def load_library() -> C.CDLL:
    """Loads the built library; raises if it is not there (build it with build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s not found: build it first (python -m paper_2603_08026_amd.build)" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
    P = C.POINTER
    lib.dyllm_workspace_bytes.argtypes = [P(LayerCfg), P(C.c_size_t)]
    lib.dyllm_create.argtypes = [P(LayerCfg), P(vp)]
    lib.dyllm_destroy.argtypes = [vp]
    lib.dyllm_strerror.argtypes = [C.c_int]
    lib.dyllm_strerror.restype = C.c_char_p
    lib.dyllm_last_error.argtypes = [vp]
    lib.dyllm_last_error.restype = C.c_char_p
    lib.dyllm_poll_status.argtypes = [vp, P(i32), vp]
    lib.dyllm_saliency.argtypes = [vp, vp, vp, P(IndexListC), i32, i32, f32, vp, vp, C.c_int, vp]
    lib.dyllm_compact.argtypes = [vp, vp, P(IndexListC), i32, i32, P(IndexListC), vp]
    lib.dyllm_compact_static.argtypes = [vp, P(IndexListC), i32, i32, P(IndexListC), vp, vp]
    lib.dyllm_qkv_refresh.argtypes = [vp, P(LayerWeights), vp, P(IndexListC), i32, i32, P(LayerCache), vp, vp]
    lib.dyllm_partial_attention.argtypes = [vp, vp, vp, vp, P(IndexListC), i32, i32, vp, vp]
    lib.dyllm_salient_ffn.argtypes = [vp, P(LayerWeights), vp, vp, P(IndexListC), i32, i32, vp, vp]
    lib.dyllm_layer_step.argtypes = [vp, P(LayerWeights), P(LayerCache), vp, P(IndexListC), i32, i32, f32,
                                     P(IndexListC), vp, vp]
    lib.dyllm_layer_step_approx.argtypes = [vp, P(LayerWeights), P(LayerCache), vp, P(IndexListC), i32, i32, i32,
                                            f32, i32, P(IndexListC), vp, vp]
    lib.dyllm_stack_step_approx.argtypes = [vp, i32, P(LayerWeights), P(LayerCache), vp, P(IndexListC), i32, i32,
                                            i32, f32, i32, P(IndexListC), vp, vp]
    lib.dyllm_merge_lists.argtypes = [vp, P(IndexListC), P(IndexListC), i32, i32, i32, P(IndexListC), vp]
    lib.dyllm_step_kind.argtypes = [P(Schedule), i32]
    lib.dyllm_denoise_step.argtypes = [vp, P(Schedule), i32, i32, P(LayerWeights), P(LayerCache), vp,
                                       P(IndexListC), P(IndexListC), i32, i32, P(IndexListC), P(IndexListC), vp]
    lib.dyllm_full_step.argtypes = [vp, P(LayerWeights), P(LayerCache), vp, i32, i32, vp]
    lib.dyllm_stack_step.argtypes = [vp, i32, P(LayerWeights), P(LayerCache), vp, P(IndexListC), i32, i32, f32,
                                     P(IndexListC), vp, vp]
    lib.dyllm_stack_full_step.argtypes = [vp, i32, P(LayerWeights), P(LayerCache), vp, i32, i32, vp]
    lib.dyllm_profile_begin.argtypes = [vp, i32]
    lib.dyllm_profile_end.argtypes = [vp, P(f32), P(i32)]
    lib.dyllm_stage_count.argtypes = []
    lib.dyllm_stage_name.argtypes = [C.c_int]
    lib.dyllm_stage_name.restype = C.c_char_p
    for name in SYMBOLS:
        fn = getattr(lib, name)
        if name not in ("dyllm_strerror", "dyllm_last_error", "dyllm_stage_name"):
            fn.restype = C.c_int
    _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return C.c_void_p(t.data_ptr())


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


@dataclass
class IndexList:
    """Device-resident token list: idx int32 [cap], offsets int32 [B+1]."""
    idx: torch.Tensor
    offsets: torch.Tensor

    @property
    def cap(self) -> int:
        return int(self.idx.numel())

    def c(self) -> IndexListC:
        assert self.idx.dtype == torch.int32 and self.offsets.dtype == torch.int32
        return IndexListC(self.idx.data_ptr(), self.offsets.data_ptr(), self.cap)

    @staticmethod
    def empty(cap: int, B: int, device="cuda") -> "IndexList":
        return IndexList(torch.zeros(max(cap, 1), dtype=torch.int32, device=device)[:cap],
                         torch.zeros(B + 1, dtype=torch.int32, device=device))


def make_weights(tensors: dict) -> LayerWeights:
    w = LayerWeights()
    for name, _ in LayerWeights._fields_:
        t = tensors.get(name)
        setattr(w, name, None if t is None else t.data_ptr())
    return w


def make_cache(k, v, c, out, lse=None) -> LayerCache:
    """lse: fp32 [B, L, H] tensor for the log-normaliser cache, or None."""
    return LayerCache(k.data_ptr(), v.data_ptr(), c.data_ptr(), out.data_ptr(),
                      lse.data_ptr() if lse is not None else None)


def pack_weight(src: torch.Tensor, dst: torch.Tensor) -> None:
    """Row-major bf16 [n_out, n_in] device matrix -> the panel layout bf16 contexts read (dst: same size)."""
    if src.dim() != 2 or src.dtype != torch.bfloat16 or dst.dtype != torch.bfloat16 or dst.numel() != src.numel():
        raise ValueError("pack_weight takes a 2-D bf16 matrix and a bf16 destination of the same size")
    lib = load_library()
    rc = lib.dyllm_pack_weight(_ptr(src), C.c_int32(src.shape[0]), C.c_int32(src.shape[1]), _ptr(dst), _stream())
    if rc:
        raise DyllmError(rc, lib.dyllm_strerror(rc).decode())


COMPACT_STATIC_MAX_ROWS = 1 << 20


def compact_static(flag: torch.Tensor, rows: Optional["IndexList"], B: int, L: int, out: "IndexList",
                   status: Optional[torch.Tensor] = None) -> None:
    """dyllm_compact without a context: no device memory is allocated by the call."""
    lib = load_library()
    r = rows.c() if rows is not None else None
    o = out.c()
    rc = lib.dyllm_compact_static(_ptr(flag), C.byref(r) if r is not None else None, C.c_int32(B), C.c_int32(L),
                                  C.byref(o), _ptr(status), _stream())
    if rc:
        raise DyllmError(rc, lib.dyllm_strerror(rc).decode())


def workspace_bytes(cfg: LayerCfg) -> int:
    n = C.c_size_t(0)
    rc = load_library().dyllm_workspace_bytes(C.byref(cfg), C.byref(n))
    if rc:
        raise DyllmError(rc, load_library().dyllm_strerror(rc).decode())
    return int(n.value)


class Context:
    """Owns a dyllm_ctx (device scratch only)."""

    def __init__(self, cfg: LayerCfg):
        self.lib = load_library()
        self.cfg = cfg
        h = C.c_void_p()
        rc = self.lib.dyllm_create(C.byref(cfg), C.byref(h))
        if rc:
            raise DyllmError(rc, self.lib.dyllm_strerror(rc).decode())
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            torch.cuda.synchronize()
            self.lib.dyllm_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc:
            raise DyllmError(rc, self.lib.dyllm_last_error(self.h).decode())

    def poll_status(self) -> int:
        st = C.c_int32(0)
        self._check(self.lib.dyllm_poll_status(self.h, C.byref(st), _stream()))
        return int(st.value)

    def profile_begin(self, max_calls: int):
        self._check(self.lib.dyllm_profile_begin(self.h, max_calls))

    def profile_end(self):
        """Returns ({stage name: mean ms}, calls)."""
        n = self.lib.dyllm_stage_count()
        ms = (C.c_float * n)()
        calls = C.c_int32(0)
        self._check(self.lib.dyllm_profile_end(self.h, ms, C.byref(calls)))
        return {self.lib.dyllm_stage_name(i).decode(): float(ms[i]) for i in range(n)}, int(calls.value)

    def saliency(self, c_new, c_cache, rows: Optional[IndexList], B, L, tau, cos_out, flag_out, commit=False):
        r = rows.c() if rows is not None else None
        self._check(self.lib.dyllm_saliency(self.h, _ptr(c_new), _ptr(c_cache),
                                            C.byref(r) if r is not None else None, B, L, tau,
                                            _ptr(cos_out), _ptr(flag_out), int(commit), _stream()))

    def compact(self, flag, rows: Optional[IndexList], B, L, out: IndexList):
        r = rows.c() if rows is not None else None
        o = out.c()
        self._check(self.lib.dyllm_compact(self.h, _ptr(flag), C.byref(r) if r is not None else None,
                                           B, L, C.byref(o), _stream()))

    def qkv_refresh(self, w: LayerWeights, x, rows: IndexList, B, L, cache: LayerCache, q_sal_out):
        r = rows.c()
        self._check(self.lib.dyllm_qkv_refresh(self.h, C.byref(w), _ptr(x), C.byref(r), B, L,
                                               C.byref(cache), _ptr(q_sal_out), _stream()))

    def partial_attention(self, q_sal, k_cache, v_cache, rows: IndexList, B, L, c_sal_out):
        r = rows.c()
        self._check(self.lib.dyllm_partial_attention(self.h, _ptr(q_sal), _ptr(k_cache), _ptr(v_cache),
                                                     C.byref(r), B, L, _ptr(c_sal_out), _stream()))

    def salient_ffn(self, w: LayerWeights, x, c, rows_out: IndexList, B, L, out_cache):
        r = rows_out.c()
        self._check(self.lib.dyllm_salient_ffn(self.h, C.byref(w), _ptr(x), _ptr(c), C.byref(r), B, L,
                                               _ptr(out_cache), _stream()))

    def layer_step(self, w: LayerWeights, cache: LayerCache, x, idx_in: IndexList, B, L, tau,
                   idx_out: IndexList, cos_out=None):
        i, o = idx_in.c(), idx_out.c()
        self._check(self.lib.dyllm_layer_step(self.h, C.byref(w), C.byref(cache), _ptr(x), C.byref(i),
                                              B, L, tau, C.byref(o), _ptr(cos_out), _stream()))

    def layer_step_approx(self, w: LayerWeights, cache: LayerCache, x, idx_in: IndexList, B, L, tau,
                          idx_out: IndexList, cos_out=None, row_lo=0, cached_norm=False):
        i, o = idx_in.c(), idx_out.c()
        self._check(self.lib.dyllm_layer_step_approx(self.h, C.byref(w), C.byref(cache), _ptr(x), C.byref(i),
                                                     B, L, row_lo, tau, int(cached_norm), C.byref(o),
                                                     _ptr(cos_out), _stream()))

    def stack_step_approx(self, ws, caches, x, idx_in: IndexList, B, L, tau, idx_outs, cos_out=None, row_lo=0,
                          cached_norm=False):
        n = len(ws)
        wa = (LayerWeights * n)(*ws)
        ca = (LayerCache * n)(*caches)
        oa = (IndexListC * n)(*[o.c() for o in idx_outs])
        i = idx_in.c()
        self._check(self.lib.dyllm_stack_step_approx(self.h, n, wa, ca, _ptr(x), C.byref(i), B, L, row_lo, tau,
                                                     int(cached_norm), oa, _ptr(cos_out), _stream()))

    def merge_lists(self, a, b, B, L, pos_lo, out: IndexList):
        """a, b: IndexList or None."""
        ac, bc, oc = (a.c() if a is not None else None), (b.c() if b is not None else None), out.c()
        self._check(self.lib.dyllm_merge_lists(self.h, C.byref(ac) if ac is not None else None,
                                               C.byref(bc) if bc is not None else None, B, L, pos_lo,
                                               C.byref(oc), _stream()))

    def denoise_step(self, sched: Schedule, t, ws, caches, x, decoded, carry, B, L, cand: IndexList, idx_outs):
        """decoded, carry: IndexList or None.  Returns the step kind (STEP_*)."""
        n = len(ws)
        wa = (LayerWeights * n)(*ws)
        ca = (LayerCache * n)(*caches)
        oa = (IndexListC * n)(*[o.c() for o in idx_outs])
        dc, cc, kc = (decoded.c() if decoded is not None else None), (carry.c() if carry is not None else None), cand.c()
        self._check(self.lib.dyllm_denoise_step(self.h, C.byref(sched), t, n, wa, ca, _ptr(x),
                                                C.byref(dc) if dc is not None else None,
                                                C.byref(cc) if cc is not None else None, B, L, C.byref(kc), oa,
                                                _stream()))
        return int(self.lib.dyllm_step_kind(C.byref(sched), t))

    def full_step(self, w: LayerWeights, cache: LayerCache, x, B, L):
        self._check(self.lib.dyllm_full_step(self.h, C.byref(w), C.byref(cache), _ptr(x), B, L, _stream()))

    def stack_step(self, ws, caches, x, idx_in: IndexList, B, L, tau, idx_outs, cos_out=None):
        """ws / caches / idx_outs: one LayerWeights / LayerCache / IndexList per layer."""
        n = len(ws)
        wa = (LayerWeights * n)(*ws)
        ca = (LayerCache * n)(*caches)
        oa = (IndexListC * n)(*[o.c() for o in idx_outs])
        i = idx_in.c()
        self._check(self.lib.dyllm_stack_step(self.h, n, wa, ca, _ptr(x), C.byref(i), B, L, tau, oa,
                                              _ptr(cos_out), _stream()))

    def stack_full_step(self, ws, caches, x, B, L):
        n = len(ws)
        wa = (LayerWeights * n)(*ws)
        ca = (LayerCache * n)(*caches)
        self._check(self.lib.dyllm_stack_full_step(self.h, n, wa, ca, _ptr(x), B, L, _stream()))
