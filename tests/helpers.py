"""Shared helpers of the GPU parity tests (no method arithmetic: conversions and error metrics)."""
from __future__ import annotations

import numpy as np

from oracle import dyllm_oracle as O
from synth import workload as W

TOL = {"f32": 1e-4, "bf16": 2e-2}  # max|gpu - ref| / max|ref| on a tensor
BAND = 1e-3  # tokens whose oracle cosine lies within BAND of tau may fall either way


def oracle_cfg(s: W.LayerShape) -> O.LayerCfg:
    return O.LayerCfg(s.hidden, s.n_heads, s.n_kv_heads, s.head_dim, s.ffn, s.rms_eps, s.rope_theta)


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    denom = np.max(np.abs(ref)) if ref.size else 1.0
    if denom == 0:
        denom = 1.0
    return float(np.max(np.abs(got - ref)) / denom) if ref.size else 0.0


def assert_close(got, ref, tol, what=""):
    e = rel_err(got, ref)
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), "%s: non-finite values" % what
    assert e <= tol, "%s: max relative error %.3e > %.1e" % (what, e, tol)
    return e


def assert_index_sets_match(idx_gpu, idx_ref, rows_in, cos_ref, tau, what=""):
    """Exact agreement for every candidate whose oracle cosine is further than BAND from tau."""
    rows_in = np.asarray(rows_in)
    firm = np.abs(np.asarray(cos_ref) - tau) > BAND
    g, r = set(np.asarray(idx_gpu).tolist()), set(np.asarray(idx_ref).tolist())
    firm_rows = set(rows_in[firm].tolist())
    assert (g & firm_rows) == (r & firm_rows), "%s: salient sets differ outside the tolerance band" % what
    assert g <= set(rows_in.tolist()), "%s: selected a token that was not a candidate" % what
    lst = np.asarray(idx_gpu)
    assert np.all(np.diff(lst) > 0), "%s: index list not ascending/unique" % what


def small_shape(dtype: str, gqa: bool = False, dh: int = 64) -> W.LayerShape:
    if dtype == "f32":
        return W.LayerShape(hidden=128, n_heads=4 if not gqa else 4, n_kv_heads=4 if not gqa else 2,
                            head_dim=dh, ffn=192, dtype="f32", rope_theta=10000.0)
    return W.LayerShape(hidden=256, n_heads=4, n_kv_heads=4 if not gqa else 1, head_dim=dh, ffn=384,
                        dtype="bf16", rope_theta=10000.0)


def rand_weights(shape: W.LayerShape, seed: int, bias: bool = False, std: float = 0.05):
    w = W.make_weights(shape, layer=seed, std=std)
    if bias:
        for name, n in (("bq", shape.dq), ("bk", shape.dkv), ("bv", shape.dkv)):
            b = W.philox(seed, "bias", name).standard_normal(n, dtype=np.float32) * np.float32(0.1)
            w[name] = W.round_bf16(b) if shape.dtype == "bf16" else b
    return w


def rand_rows(seed: int, B: int, L: int, counts) -> tuple:
    """Ascending unique token ids with the given per-sequence counts."""
    idx, off = [], np.zeros(B + 1, dtype=np.int32)
    for b in range(B):
        r = np.sort(W.philox(seed, "rows", b).choice(L, size=int(counts[b]), replace=False))
        idx.append(r + b * L)
        off[b + 1] = off[b] + r.size
    return (np.concatenate(idx).astype(np.int32) if idx else np.zeros(0, np.int32)), off
