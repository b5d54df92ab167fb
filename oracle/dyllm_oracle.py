"""CPU oracle for DyLLM's per-denoising-step sparse layer update.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow numpy implementation in
float64 of what the GPU library computes.  It is written from the paper alone
and shares no code with the HIP path; only tests, the smoke check and the
bench's CPU-baseline leg may import it.  Library matmuls serve as steps; there
is no blocking, fusion or reordering beyond what the algorithm states.

What each function follows:
  cosine_rows, salient_mask ....... Sec. 3.1 (temporal cosine similarity) and
                                    Sec. 3.2 (salient set A = {i : s < tau})
  attention_rows .................. Sec. 3.3, salient path: exact attention rows
                                    for salient queries against all keys/values
  layer_step ...................... App. C.3, Alg. 3 (SparseStep), the body of
                                    its layer loop restricted to the salient
                                    (row-sparse) path
  full_step ....................... App. C.2, Alg. 2 (FullStep), one layer
  approx_attention ................ App. C.4, Alg. 4 (approximate attention): the
                                    salient columns of the full softmax times the
                                    value residual of the salient tokens  [Eq. 3]
  approx_attention_cached ......... variant of Alg. 4 with the softmax normalisers reused from each
                                    query's last exact evaluation (Sec. 3.3: cost O(N |A| d),
                                    "attention weights are reused"); not the printed algorithm
  layer_step_approx ............... Alg. 3 layer body with both attention paths
                                    (exact rows for the salient set, approximate
                                    context update for all other rows)
  stack_step, stack_full_step ..... the layer loops of Alg. 3 and Alg. 2: a layer
                                    reads the previous layer's output cache and,
                                    in Alg. 3, the previous layer's salient set
  Schedule, step_kind, merge_lists,
  denoise_step .................... App. C.1, Alg. 1 (the generation loop) without
                                    its token side: dense warm-up steps, then sparse
                                    steps that take the whole sequence every
                                    full_period-th step and the response only
                                    otherwise (Sec. 3.5), the salient set carried
                                    from step to step
  compact ......................... the where(...) of Alg. 3
  rmsnorm ......................... App. E, proof of Prop. 1 (RMSNorm definition)

Readings taken where the paper is silent (also listed in the design notes):
pre-norm residual block (h = x + Wo C, y = h + FFN(RMSNorm(h))); the "FFN
output cache" holds the layer's output hidden state; one cosine per token over
the concatenated per-head context, before Wo; strict '<' against tau; each norm
in the cosine clamped below at 1e-8; rotary embedding on q and k in the
half-split pairing (j, j + dh/2), keys cached after rotation; softmax scale
1/sqrt(dh), no mask; query head h reads KV head h // g; SwiGLU FFN
down(silu(gate) * up).

Parity pins: every function here is pinned by tests/test_oracle_pins.py
(closed forms, brute-force loops on tiny inputs, the paper's propositions and
the dense == all-salient equivalence).  The approximation quality of the method
against the dense model is "parity unpinned": the paper shows it only through
benchmark accuracy with trained weights.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional, Tuple

import numpy as np

F64 = np.float64
COS_NORM_FLOOR = 1e-8


@dataclass(frozen=True)
class LayerCfg:
    hidden: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0


def _f64(a):
    return None if a is None else np.asarray(a, dtype=F64)


# --------------------------------------------------------------------------
# elementary pieces
# --------------------------------------------------------------------------

def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """RMSNorm(y) = y / RMS(y) * g with RMS(y) = sqrt(mean(y^2) (+ eps)).  [App. E, Prop. 1 proof]"""
    x = _f64(x)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * _f64(gain)


def silu(z: np.ndarray) -> np.ndarray:
    z = _f64(z)
    return z / (1.0 + np.exp(-z))


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, half-split pairing.

    x: [n, heads, dh]; pos: [n] positions inside the sequence.  Pair j couples
    elements j and j + dh/2 and is rotated by the angle pos * theta^(-2j/dh).
    """
    x = _f64(x)
    n, _, dh = x.shape
    half = dh // 2
    j = np.arange(half, dtype=F64)
    inv_freq = theta ** (-2.0 * j / dh)
    ang = _f64(pos)[:, None] * inv_freq[None, :]  # [n, half]
    cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    out = np.empty_like(x)
    out[..., :half] = x1 * cos - x2 * sin
    out[..., half:] = x2 * cos + x1 * sin
    return out


def swiglu_ffn(f: np.ndarray, w: Dict[str, np.ndarray]) -> np.ndarray:
    """down( silu(gate f) * (up f) ) for rows f [m, hidden]."""
    gate = f @ _f64(w["w_gate"]).T
    up = f @ _f64(w["w_up"]).T
    return (silu(gate) * up) @ _f64(w["w_down"]).T


def project_qkv(n_rows: np.ndarray, pos: np.ndarray, w: Dict[str, np.ndarray], cfg: LayerCfg):
    """q, k, v for normalised rows n_rows [m, hidden] at sequence positions pos [m]."""
    q = n_rows @ _f64(w["wq"]).T
    k = n_rows @ _f64(w["wk"]).T
    v = n_rows @ _f64(w["wv"]).T
    if w.get("bq") is not None:
        q = q + _f64(w["bq"])
    if w.get("bk") is not None:
        k = k + _f64(w["bk"])
    if w.get("bv") is not None:
        v = v + _f64(w["bv"])
    m = n_rows.shape[0]
    q = rope(q.reshape(m, cfg.n_heads, cfg.head_dim), pos, cfg.rope_theta)
    k = rope(k.reshape(m, cfg.n_kv_heads, cfg.head_dim), pos, cfg.rope_theta)
    v = v.reshape(m, cfg.n_kv_heads, cfg.head_dim)
    return q, k, v


def attention_rows(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """Exact attention rows of one sequence.  [Sec. 3.3 salient path; Alg. 3 C_sal]

    q: [m, H, dh] queries of the selected rows; k, v: [L, Hkv, dh] all keys and
    values of the sequence.  Every query attends to all L keys (no mask).
    Returns [m, H*dh].
    """
    q, k, v = _f64(q), _f64(k), _f64(v)
    m, H, dh = q.shape
    Hkv = k.shape[1]
    g = H // Hkv
    out = np.empty((m, H, dh), dtype=F64)
    for h in range(H):
        kh, vh = k[:, h // g, :], v[:, h // g, :]
        z = (q[:, h, :] @ kh.T) / np.sqrt(dh)  # [m, L]
        z = z - z.max(axis=1, keepdims=True)
        p = np.exp(z)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ vh
    return out.reshape(m, H * dh)


def attention_lse(q: np.ndarray, k: np.ndarray) -> np.ndarray:
    """Log of the softmax normaliser of every (query, head): log sum_j exp(q.k_j / sqrt(dh)) over all
    keys of the sequence.  q: [m, H, dh], k: [L, Hkv, dh]; returns [m, H]."""
    q, k = _f64(q), _f64(k)
    m, H, dh = q.shape
    g = H // k.shape[1]
    out = np.empty((m, H), dtype=F64)
    for h in range(H):
        z = (q[:, h, :] @ k[:, h // g, :].T) / np.sqrt(dh)
        top = z.max(axis=1)
        out[:, h] = top + np.log(np.exp(z - top[:, None]).sum(axis=1))
    return out


def cosine_rows(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """s = <a,b> / (max(|a|, floor) * max(|b|, floor)) per row.  [Sec. 3.1]"""
    a, b = _f64(a), _f64(b)
    dot = np.sum(a * b, axis=-1)
    na = np.maximum(np.sqrt(np.sum(a * a, axis=-1)), COS_NORM_FLOOR)
    nb = np.maximum(np.sqrt(np.sum(b * b, axis=-1)), COS_NORM_FLOOR)
    return dot / (na * nb)


def salient_mask(s: np.ndarray, tau: float) -> np.ndarray:
    """A = {i : s_i < tau}, strict.  [Sec. 3.2]"""
    return np.asarray(s) < tau


def compact(flag: np.ndarray, rows: Optional[np.ndarray], B: int, L: int) -> Tuple[np.ndarray, np.ndarray]:
    """Ascending list of flagged token ids and per-sequence offsets [B+1].

    flag[j] belongs to token rows[j] (rows ascending flat ids b*L+i), or to
    token j when rows is None.
    """
    flag = np.asarray(flag).astype(bool)
    ids = np.arange(flag.size, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    out = ids[flag]
    offsets = np.zeros(B + 1, dtype=np.int32)
    for b in range(B):
        offsets[b + 1] = offsets[b] + int(np.sum((out >= b * L) & (out < (b + 1) * L)))
    return out.astype(np.int32), offsets


# --------------------------------------------------------------------------
# stand-alone forms of the boundary calls
# --------------------------------------------------------------------------

def saliency(c_new: np.ndarray, c_cache: np.ndarray, rows: Optional[np.ndarray], tau: float,
             commit: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """Cosine and salient flag per candidate.  [Sec. 3.1-3.2; Alg. 3 cosine line]

    rows given: c_new is [M, D] (one row per candidate), c_cache is [T, D] and
    candidate j is compared with c_cache[rows[j]].  rows None: both are [T, D].
    With commit the old cache row is read first and then overwritten by the new
    context (cache commit of Alg. 3); c_cache must then be a float64 array.
    """
    cn = _f64(c_new)
    if rows is None:
        old = _f64(c_cache)
    else:
        old = _f64(c_cache)[np.asarray(rows, dtype=np.int64)]
    s = cosine_rows(cn, old)
    flag = salient_mask(s, tau)
    if commit:
        if rows is None:
            c_cache[...] = cn
        else:
            c_cache[np.asarray(rows, dtype=np.int64)] = cn
    return s, flag


def partial_attention(q_sal: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                      rows: np.ndarray, B: int, L: int) -> np.ndarray:
    """C rows for the tokens in rows (flat ids), each against its own sequence's K/V.

    q_sal: [M, H, dh]; k_cache, v_cache: [B, L, Hkv, dh].  Returns [M, H*dh].
    """
    rows = np.asarray(rows, dtype=np.int64)
    M, H, dh = q_sal.shape
    out = np.empty((M, H * dh), dtype=F64)
    for b in range(B):
        sel = np.nonzero((rows >= b * L) & (rows < (b + 1) * L))[0]
        if sel.size:
            out[sel] = attention_rows(q_sal[sel], k_cache[b], v_cache[b])
    return out


def partial_lse(q_sal: np.ndarray, k_cache: np.ndarray, rows: np.ndarray, B: int, L: int) -> np.ndarray:
    """attention_lse for the tokens in rows (flat ids), each against its own sequence's keys: [M, H]."""
    rows = np.asarray(rows, dtype=np.int64)
    out = np.empty((q_sal.shape[0], q_sal.shape[1]), dtype=F64)
    for b in range(B):
        sel = np.nonzero((rows >= b * L) & (rows < (b + 1) * L))[0]
        if sel.size:
            out[sel] = attention_lse(q_sal[sel], k_cache[b])
    return out


def salient_ffn(x: np.ndarray, c: np.ndarray, rows_out: np.ndarray, w: Dict[str, np.ndarray],
                cfg: LayerCfg, out_cache: np.ndarray) -> None:
    """Output projection, residual, norm, FFN, residual for rows_out; commit into out_cache.

    x: [T, hidden] layer input; c: [T, H*dh] merged attention context;
    out_cache: [T, hidden] float64, updated in place at rows_out only.
    [Alg. 3: the out_proj / FFN / cache lines]
    """
    r = np.asarray(rows_out, dtype=np.int64)
    if r.size == 0:
        return
    h = _f64(x)[r] + _f64(c)[r] @ _f64(w["wo"]).T
    f = rmsnorm(h, w["g_ffn"], cfg.rms_eps)
    out_cache[r] = h + swiglu_ffn(f, w)


# --------------------------------------------------------------------------
# the two steps
# --------------------------------------------------------------------------

def new_caches(B: int, L: int, cfg: LayerCfg) -> Dict[str, np.ndarray]:
    """K, V, C and layer-output caches (zero-filled).  [Alg. 1 initialisation]"""
    return {
        "k": np.zeros((B, L, cfg.n_kv_heads, cfg.head_dim), dtype=F64),
        "v": np.zeros((B, L, cfg.n_kv_heads, cfg.head_dim), dtype=F64),
        "c": np.zeros((B, L, cfg.n_heads * cfg.head_dim), dtype=F64),
        "out": np.zeros((B, L, cfg.hidden), dtype=F64),
    }


def full_step(x: np.ndarray, w: Dict[str, np.ndarray], cfg: LayerCfg,
              caches: Dict[str, np.ndarray]) -> None:
    """Dense pass of one layer over all rows; fills all four caches.  [Alg. 2]

    Written on its own (matrix form, rotary embedding through complex
    multiplication) and not through layer_step's helpers, so that the
    "all rows salient == dense" pin compares two separate derivations.
    """
    x = _f64(x)
    B, L, d = x.shape
    H, Hkv, dh = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    g = H // Hkv
    wq, wk, wv, wo = (_f64(w[n]) for n in ("wq", "wk", "wv", "wo"))
    wg, wu, wd = (_f64(w[n]) for n in ("w_gate", "w_up", "w_down"))
    ga, gf = _f64(w["g_attn"]), _f64(w["g_ffn"])
    half = dh // 2
    # rotation factors e^{i * pos * theta^(-2j/dh)}
    phase = np.exp(1j * np.outer(np.arange(L, dtype=F64),
                                 cfg.rope_theta ** (-2.0 * np.arange(half, dtype=F64) / dh)))

    def rot(t):  # t: [L, heads, dh]
        z = (t[..., :half] + 1j * t[..., half:]) * phase[:, None, :]
        return np.concatenate([z.real, z.imag], axis=-1)

    for b in range(B):
        xb = x[b]
        n = xb * (1.0 / np.sqrt((xb ** 2).mean(axis=1, keepdims=True) + cfg.rms_eps)) * ga
        Q, K, V = n @ wq.T, n @ wk.T, n @ wv.T
        if w.get("bq") is not None:
            Q = Q + _f64(w["bq"])
        if w.get("bk") is not None:
            K = K + _f64(w["bk"])
        if w.get("bv") is not None:
            V = V + _f64(w["bv"])
        Q = rot(Q.reshape(L, H, dh))
        K = rot(K.reshape(L, Hkv, dh))
        V = V.reshape(L, Hkv, dh)
        C = np.empty((L, H, dh), dtype=F64)
        for h in range(H):
            S = Q[:, h] @ K[:, h // g].T / np.sqrt(dh)
            E = np.exp(S - S.max(axis=1, keepdims=True))
            C[:, h] = (E / E.sum(axis=1, keepdims=True)) @ V[:, h // g]
        C = C.reshape(L, H * dh)
        hcur = xb + C @ wo.T
        f = hcur / np.sqrt((hcur ** 2).mean(axis=1, keepdims=True) + cfg.rms_eps) * gf
        gate = f @ wg.T
        y = hcur + ((gate / (1.0 + np.exp(-gate))) * (f @ wu.T)) @ wd.T
        caches["k"][b], caches["v"][b], caches["c"][b], caches["out"][b] = K, V, C, y
        if "lse" in caches:  # optional fifth cache: log-normalisers of the exact rows (cached-normaliser variant)
            caches["lse"][b] = attention_lse(Q, K)


def layer_step(x: np.ndarray, idx_in: np.ndarray, w: Dict[str, np.ndarray], cfg: LayerCfg,
               caches: Dict[str, np.ndarray], tau: float):
    """One layer of SparseStep on the salient path.  [Alg. 3 layer body; Sec. 3.2-3.3]

    x: [B, L, hidden] layer input; idx_in: ascending flat token ids b*L+i (the
    salient set handed over by the previous layer / step); caches are updated
    in place.  Returns (idx_out, offsets_out, cos) where cos[j] belongs to
    idx_in[j] and idx_out lists the tokens with cos < tau.

    Order, as in Alg. 3: (1) norm, q/k/v projection and rotation of the
    idx_in rows; (2) their K and V rows replace the cached ones, for all of
    idx_in, before any attention row is evaluated; (3) exact attention rows
    against the merged K/V; (4) cosine against the old cached context, then the
    '<' test; (5) commit the new contexts; (6) out-projection + residual, norm,
    FFN + residual for the newly selected rows only, committed to the output
    cache.  Rows outside idx_in keep all four cache rows; rows of idx_in that
    fail the test keep their cached output row.
    """
    x = _f64(x)
    B, L, d = x.shape
    idx_in = np.asarray(idx_in, dtype=np.int64)
    xf = x.reshape(B * L, d)
    kc = caches["k"].reshape(B * L, cfg.n_kv_heads, cfg.head_dim)
    vc = caches["v"].reshape(B * L, cfg.n_kv_heads, cfg.head_dim)
    cc = caches["c"].reshape(B * L, cfg.n_heads * cfg.head_dim)
    oc = caches["out"].reshape(B * L, d)
    if idx_in.size == 0:
        return np.zeros(0, np.int32), np.zeros(B + 1, np.int32), np.zeros(0, F64)

    # (1) projections of the salient rows
    n_rows = rmsnorm(xf[idx_in], w["g_attn"], cfg.rms_eps)
    q, k, v = project_qkv(n_rows, idx_in % L, w, cfg)
    # (2) K/V merge
    kc[idx_in] = k
    vc[idx_in] = v
    # (3) exact rows
    c_new = partial_attention(q, caches["k"], caches["v"], idx_in, B, L)
    if "lse" in caches:
        caches["lse"].reshape(B * L, -1)[idx_in] = partial_lse(q, caches["k"], idx_in, B, L)
    # (4) cosine against the cached context, selection
    cos = cosine_rows(c_new, cc[idx_in])
    flag = salient_mask(cos, tau)
    # (5) context commit
    cc[idx_in] = c_new
    idx_out, offsets_out = compact(flag, idx_in, B, L)
    # (6) out-projection and FFN for the newly selected rows
    salient_ffn(xf, cc, idx_out, w, cfg, oc)
    return idx_out, offsets_out, cos


def approx_attention(q_all: np.ndarray, k_cache: np.ndarray, dv: np.ndarray, idx_sal: np.ndarray,
                     B: int, L: int) -> np.ndarray:
    """Residual update of the attention context of EVERY token.  [Alg. 4; Eq. 3, first term]

    q_all: [B*L, H, dh] queries of all tokens; k_cache: [B, L, Hkv, dh] (merged keys);
    dv: [M, Hkv, dh] value residual V_new - V_cached of the tokens idx_sal (ascending flat ids).
    Steps of Alg. 4 per sequence and head: scores of all queries against ALL keys, softmax over all
    keys, the columns of the salient tokens, times their value residual.  Returns [B*L, H*dh].
    """
    idx_sal = np.asarray(idx_sal, dtype=np.int64)
    T, H, dh = q_all.shape
    Hkv = k_cache.shape[2]
    g = H // Hkv
    out = np.zeros((T, H * dh), dtype=F64)
    qa, dv = _f64(q_all), _f64(dv)
    for b in range(B):
        sel = np.nonzero((idx_sal >= b * L) & (idx_sal < (b + 1) * L))[0]
        if sel.size == 0:
            continue
        cols = idx_sal[sel] - b * L
        for h in range(H):
            S = qa[b * L:(b + 1) * L, h] @ _f64(k_cache[b, :, h // g]).T / np.sqrt(dh)  # [L, L]
            E = np.exp(S - S.max(axis=1, keepdims=True))
            A = E / E.sum(axis=1, keepdims=True)
            out[b * L:(b + 1) * L, h * dh:(h + 1) * dh] = A[:, cols] @ dv[sel, h // g]
    return out


def approx_attention_cached(q_all: np.ndarray, k_cache: np.ndarray, dv: np.ndarray, idx_sal: np.ndarray,
                            lse: np.ndarray, B: int, L: int) -> np.ndarray:
    """Approximate attention with REUSED normalisers: the weight of salient key j for query i is
    exp(q_i.k_j / sqrt(dh) - lse_i), with lse_i the log-normaliser cached at query i's last exact
    evaluation, so that only the salient columns are ever scored -- the O(N |A| d) cost that
    Sec. 3.3 states and its remark that attention weights are reused.  This is a variant of Alg. 4,
    which renormalises over all keys; the two agree whenever lse is the current log-normaliser.

    q_all: [T, H, dh]; k_cache: [B, L, Hkv, dh] (merged); dv: [M, Hkv, dh]; idx_sal: [M] flat ids;
    lse: [T, H].  Returns dC [T, H*dh].
    """
    q_all, k_cache, dv, lse = _f64(q_all), _f64(k_cache), _f64(dv), _f64(lse)
    idx_sal = np.asarray(idx_sal, dtype=np.int64)
    T, H, dh = q_all.shape
    g = H // k_cache.shape[2]
    out = np.zeros((T, H, dh), dtype=F64)
    for b in range(B):
        sel = np.nonzero((idx_sal >= b * L) & (idx_sal < (b + 1) * L))[0]
        if sel.size == 0:
            continue
        cols = idx_sal[sel] - b * L
        for h in range(H):
            z = (q_all[b * L:(b + 1) * L, h, :] @ k_cache[b, cols, h // g, :].T) / np.sqrt(dh)  # [L, |A_b|]
            wgt = np.exp(z - lse[b * L:(b + 1) * L, h][:, None])
            out[b * L:(b + 1) * L, h, :] = wgt @ dv[sel, h // g, :]
    return out.reshape(T, H * dh)


def layer_step_approx(x: np.ndarray, idx_in: np.ndarray, w: Dict[str, np.ndarray], cfg: LayerCfg,
                      caches: Dict[str, np.ndarray], tau: float, row_lo: int = 0, cached_norm: bool = False):
    """One layer of SparseStep with both attention paths.  [Alg. 3 layer body; Sec. 3.3]

    cached_norm: the residual of the non-salient tokens comes from approx_attention_cached with the
    log-normalisers in caches["lse"] ([B, L, H], kept by full_step and by every exact row) instead of
    Alg. 4's full softmax.

    As layer_step, plus: queries are projected for ALL tokens of the step; the value residual dV of
    the idx_in tokens is taken before their V rows are merged; every other token of the step gets
    C = C_cached + approx_attention(...) (Sec. 3.3, non-salient path); the cosine test then runs over
    ALL tokens of the step, so idx_out may hold tokens that were not in idx_in.

    row_lo > 0 is a response-only step (Sec. 3.5; Alg. 3, comment on its first line): the step's
    tokens are the positions [row_lo, L) of every sequence, the keys and values still cover the whole
    sequence (App. C.4), tokens below row_lo keep every cache row and take no part in the test.
    Returns (idx_out, offsets_out, cos) with cos of length B*L (1 for tokens outside the step).
    """
    x = _f64(x)
    B, L, d = x.shape
    T = B * L
    idx_in = np.asarray(idx_in, dtype=np.int64)
    assert np.all(idx_in % L >= row_lo), "a response-only step takes no prompt token"
    xf = x.reshape(T, d)
    kc = caches["k"].reshape(T, cfg.n_kv_heads, cfg.head_dim)
    vc = caches["v"].reshape(T, cfg.n_kv_heads, cfg.head_dim)
    cc = caches["c"].reshape(T, cfg.n_heads * cfg.head_dim)
    oc = caches["out"].reshape(T, d)
    pos_all = np.arange(T) % L
    step_rows = np.flatnonzero(pos_all >= row_lo)
    # norm and q projection of every token of the step; k, v of the salient tokens only
    n_all = rmsnorm(xf, w["g_attn"], cfg.rms_eps)
    q_all = n_all @ _f64(w["wq"]).T
    if w.get("bq") is not None:
        q_all = q_all + _f64(w["bq"])
    q_all = rope(q_all.reshape(T, cfg.n_heads, cfg.head_dim), pos_all, cfg.rope_theta)
    c_new = cc.copy()
    if idx_in.size:
        _, k, v = project_qkv(n_all[idx_in], idx_in % L, w, cfg)
        dv = v - vc[idx_in]            # before the merge
        kc[idx_in] = k
        vc[idx_in] = v
        c_sal = partial_attention(q_all[idx_in], caches["k"], caches["v"], idx_in, B, L)
        if cached_norm:
            lse = caches["lse"].reshape(T, cfg.n_heads)
            dc = approx_attention_cached(q_all, caches["k"], dv, idx_in, lse, B, L)  # stale lse of the others
            lse[idx_in] = partial_lse(q_all[idx_in], caches["k"], idx_in, B, L)
        else:
            dc = approx_attention(q_all, caches["k"], dv, idx_in, B, L)
            if "lse" in caches:
                caches["lse"].reshape(T, cfg.n_heads)[idx_in] = partial_lse(q_all[idx_in], caches["k"], idx_in, B, L)
        others = np.setdiff1d(step_rows, idx_in)
        c_new[others] = cc[others] + dc[others]
        c_new[idx_in] = c_sal
    cos = np.ones(T, dtype=F64)
    cos[step_rows] = cosine_rows(c_new[step_rows], cc[step_rows])
    flag = np.zeros(T, dtype=bool)
    flag[step_rows] = salient_mask(cos[step_rows], tau)
    cc[:] = c_new
    idx_out, offsets_out = compact(flag, None, B, L)
    salient_ffn(xf, cc, idx_out, w, cfg, oc)
    return idx_out, offsets_out, cos


def stack_step(x: np.ndarray, idx_in: np.ndarray, ws, cfg: LayerCfg, caches, tau: float):
    """SparseStep over a stack of layers.  [Alg. 3, loop over l]

    ws / caches: one weight dict / cache dict per layer.  Layer 1 reads x and
    idx_in; layer l > 1 reads the output cache of layer l-1 (its full [B, L, d]
    content: recomputed rows and reused rows alike) and the salient set that
    layer l-1 selected.  Returns the per-layer (idx_out, offsets_out, cos).
    """
    h, idx = x, idx_in
    per_layer = []
    for w, c in zip(ws, caches):
        idx, off, cos = layer_step(h, idx, w, cfg, c, tau)
        per_layer.append((idx, off, cos))
        h = c["out"]
    return per_layer


def stack_full_step(x: np.ndarray, ws, cfg: LayerCfg, caches) -> None:
    """FullStep over a stack of layers.  [Alg. 2, loop over l]"""
    h = x
    for w, c in zip(ws, caches):
        full_step(h, w, cfg, c)
        h = c["out"]


def stack_step_approx(x: np.ndarray, idx_in: np.ndarray, ws, cfg: LayerCfg, caches, tau: float,
                      row_lo: int = 0, cached_norm: bool = False):
    """SparseStep over a stack of layers with both attention paths.  [Alg. 3, loop over l]"""
    h, idx = x, idx_in
    per_layer = []
    for w, c in zip(ws, caches):
        idx, off, cos = layer_step_approx(h, idx, w, cfg, c, tau, row_lo, cached_norm)
        per_layer.append((idx, off, cos))
        h = c["out"]
    return per_layer


@dataclass(frozen=True)
class Schedule:
    """The step schedule of the generation loop.  [App. C.1, Alg. 1; Sec. 3.2; Sec. 3.5]"""
    t_full: int        # leading dense steps
    full_period: int   # a sparse step t with t % full_period == 0 takes the whole sequence ...
    prompt_len: int    # ... every other one only the positions [prompt_len, L) of each sequence
    approx: bool       # approximate update of the non-salient tokens (Sec. 3.3) on or off
    tau: float
    cached_norm: bool = False  # with approx: reuse the cached softmax normalisers (approx_attention_cached)


def step_kind(t: int, sched: Schedule) -> str:
    """'dense' for the first t_full steps, then 'full' (whole sequence) or 'response'.  [Alg. 1]"""
    if t < sched.t_full:
        return "dense"
    return "full" if (sched.full_period <= 1 or t % sched.full_period == 0) else "response"


def merge_lists(a: Optional[np.ndarray], b: Optional[np.ndarray], L: int, pos_lo: int) -> np.ndarray:
    """Ascending unique union of two token lists, kept to positions >= pos_lo of their sequence."""
    parts = [np.asarray(v, dtype=np.int64) for v in (a, b) if v is not None]
    u = np.unique(np.concatenate(parts)) if parts else np.zeros(0, dtype=np.int64)
    return u[u % L >= pos_lo]


def denoise_step(t: int, sched: Schedule, x: np.ndarray, decoded: np.ndarray, carry: Optional[np.ndarray],
                 ws, cfg: LayerCfg, caches):
    """One iteration of the generation loop without its token side.  [App. C.1, Alg. 1]

    x: hidden states of the whole sequence [B, L, d] (a response-only step reads the response rows
    only); decoded: tokens unmasked by the previous step; carry: the salient set the previous sparse
    step returned, or None after a dense step.  Dense step: FullStep, returns None.  Sparse step:
    the candidates are the decoded positions when there is no carried set (Alg. 1), else the carried
    set joined with the decoded positions (reading: a token whose input embedding just changed must
    be recomputed), kept to the step's tokens; returns the last layer's salient set.
    """
    kind = step_kind(t, sched)
    if kind == "dense":
        stack_full_step(x, ws, cfg, caches)
        return None
    B, L, _ = np.asarray(x).shape
    row_lo = 0 if kind == "full" else sched.prompt_len
    idx = merge_lists(carry, decoded, L, row_lo)
    if sched.approx:
        per_layer = stack_step_approx(x, idx, ws, cfg, caches, sched.tau, row_lo, sched.cached_norm)
    else:
        per_layer = stack_step(x, idx, ws, cfg, caches, sched.tau)
    return per_layer[-1][0]


def kv_only_bytes_per_token(cfg: LayerCfg, elem: int) -> int:
    return 2 * cfg.n_kv_heads * cfg.head_dim * elem


def cache_bytes_per_token(cfg: LayerCfg, elem: int) -> int:
    """K + V + C + layer output per token.  [Sec. 5 memory discussion]"""
    return (2 * cfg.n_kv_heads * cfg.head_dim + cfg.n_heads * cfg.head_dim + cfg.hidden) * elem
