"""Pins for the CPU oracle: closed forms, brute force on tiny inputs, the paper's
propositions and structural equivalences.  None of these re-uses the oracle's
own formulas: brute-force checks are scalar Python loops written here, library
checks call torch routines the oracle does not use.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import dyllm_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _weights(cfg, rng, std=0.3, bias=False):
    d, dq, dkv, f = cfg.hidden, cfg.n_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim, cfg.ffn
    w = {
        "wq": rng.normal(0, std, (dq, d)), "wk": rng.normal(0, std, (dkv, d)),
        "wv": rng.normal(0, std, (dkv, d)), "wo": rng.normal(0, std, (d, dq)),
        "w_gate": rng.normal(0, std, (f, d)), "w_up": rng.normal(0, std, (f, d)),
        "w_down": rng.normal(0, std, (d, f)),
        "g_attn": 1 + 0.2 * rng.normal(size=d), "g_ffn": 1 + 0.2 * rng.normal(size=d),
    }
    if bias:
        w["bq"], w["bk"], w["bv"] = rng.normal(size=dq), rng.normal(size=dkv), rng.normal(size=dkv)
    return w


# ---------------------------------------------------------------- cosine / selection

def test_cosine_hand_cases_from_fixture():
    with open(os.path.join(GOLD, "cosine_cases.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            a, b, s = line.split(";")
            a = np.array([float(t) for t in a.split()])[None]
            b = np.array([float(t) for t in b.split()])[None]
            assert O.cosine_rows(a, b)[0] == pytest.approx(float(s), abs=1e-15)


def test_cosine_identical_scaled_and_zero_rows():
    r = _rng(0)
    a = r.normal(size=(7, 33))
    assert np.all(O.cosine_rows(a, a) >= 1 - 1e-12)
    assert np.allclose(O.cosine_rows(3.7 * a, a), 1.0, atol=1e-12)
    assert np.allclose(O.cosine_rows(-a, a), -1.0, atol=1e-12)
    z = np.zeros_like(a)
    assert np.all(O.cosine_rows(a, z) == 0.0)  # zero cache row: s = 0, never NaN
    assert np.all(O.cosine_rows(z, z) == 0.0)


def test_cosine_matches_torch_library():
    r = _rng(1)
    a, b = r.normal(size=(11, 64)), r.normal(size=(11, 64))
    ref = torch.nn.functional.cosine_similarity(torch.from_numpy(a), torch.from_numpy(b), dim=-1, eps=1e-8)
    assert np.allclose(O.cosine_rows(a, b), ref.numpy(), atol=1e-14)


def test_selection_rule_is_strict_and_bruteforce():
    s = np.array([0.5, 0.99, 0.98999, 0.99001, 1.0, -1.0])
    assert O.salient_mask(s, 0.99).tolist() == [True, False, True, False, False, True]
    assert O.salient_mask(s, 1.5).all()
    assert not O.salient_mask(s, -1.0).any()
    r = _rng(2)
    s = r.uniform(-1, 1, 64)
    want = [i for i in range(64) if s[i] < 0.3]
    got, off = O.compact(O.salient_mask(s, 0.3), None, 4, 16)
    assert got.tolist() == want
    assert off.tolist() == [sum(1 for i in want if i < 16 * b) for b in range(5)]


def test_compact_with_candidate_rows_and_empty_sequences():
    rows = np.array([3, 9, 17, 18, 40, 47])  # L = 16: seq 0,0,1,1,2,2 ; seq 3 empty
    flag = np.array([1, 0, 0, 1, 1, 1], dtype=np.uint8)
    idx, off = O.compact(flag, rows, 4, 16)
    assert idx.tolist() == [3, 18, 40, 47]
    assert off.tolist() == [0, 1, 2, 4, 4]
    idx, off = O.compact(np.zeros(6, np.uint8), rows, 4, 16)
    assert idx.size == 0 and off.tolist() == [0] * 5


# ---------------------------------------------------------------- rmsnorm / silu / rope

def test_rmsnorm_closed_forms():
    g = np.array([1.0, 2.0, 3.0, 4.0])
    assert np.allclose(O.rmsnorm(np.full((1, 4), 5.0), g, 0.0), g)
    y = O.rmsnorm(np.array([[3.0, -4.0, 0.0, 0.0]]), np.ones(4), 0.0)
    assert np.allclose(y, np.array([[3, -4, 0, 0]]) / math.sqrt(25 / 4))
    # eps sits inside the square root, added to the mean square
    y = O.rmsnorm(np.array([[2.0, 2.0]]), np.ones(2), 5.0)
    assert np.allclose(y, 2.0 / 3.0)
    r = _rng(3)
    x = r.normal(size=(5, 16))
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (16,), torch.from_numpy(np.ones(16)), 1e-5)
    assert np.allclose(O.rmsnorm(x, np.ones(16), 1e-5), ref.numpy(), atol=1e-13)


def test_silu_closed_forms():
    z = np.linspace(-6, 6, 25)
    s = O.silu(z)
    assert s[12] == 0.0
    assert np.allclose(s - O.silu(-z), z, atol=1e-13)  # silu(z) - silu(-z) = z
    assert O.silu(np.array([1.0]))[0] == pytest.approx(1 / (1 + math.exp(-1)), abs=1e-15)
    assert np.allclose(s, torch.nn.functional.silu(torch.from_numpy(z)).numpy(), atol=1e-14)


def test_rope_closed_forms():
    # head_dim 2: one pair, plain rotation by the angle pos (theta^0 = 1)
    x = np.array([[[1.0, 0.0]], [[0.0, 1.0]], [[2.0, 3.0]]])
    y = O.rope(x, np.array([0.5, 0.5, 0.0]), 10000.0)
    assert np.allclose(y[0, 0], [math.cos(0.5), math.sin(0.5)])
    assert np.allclose(y[1, 0], [-math.sin(0.5), math.cos(0.5)])
    assert np.allclose(y[2, 0], [2.0, 3.0])  # position 0 is the identity
    # head_dim 4, theta 100: pair (0,2) turns by pos, pair (1,3) by pos / 10
    x = np.array([[[1.0, 1.0, 0.0, 0.0]]])
    y = O.rope(x, np.array([2.0]), 100.0)
    assert np.allclose(y[0, 0], [math.cos(2.0), math.cos(0.2), math.sin(2.0), math.sin(0.2)])


def test_rope_preserves_norm_and_is_relative():
    r = _rng(4)
    q, k = r.normal(size=(1, 3, 16)), r.normal(size=(1, 3, 16))
    for m, n in [(5, 2), (105, 102), (40, 37)]:
        qm, kn = O.rope(q, np.array([m]), 10000.0), O.rope(k, np.array([n]), 10000.0)
        assert np.allclose(np.linalg.norm(qm, axis=-1), np.linalg.norm(q, axis=-1))
        dots = np.sum(qm * kn, axis=-1)
        if m == 5:
            first = dots
        assert np.allclose(dots, first, atol=1e-10)  # depends on m - n only


# ---------------------------------------------------------------- attention

def _attn_bruteforce(q, k, v):
    m, H, dh = q.shape
    L, Hkv, _ = k.shape
    g = H // Hkv
    out = np.zeros((m, H * dh))
    for i in range(m):
        for h in range(H):
            z = [sum(q[i, h, e] * k[j, h // g, e] for e in range(dh)) / math.sqrt(dh) for j in range(L)]
            zmax = max(z)
            p = [math.exp(t - zmax) for t in z]
            tot = sum(p)
            for e in range(dh):
                out[i, h * dh + e] = sum(p[j] * v[j, h // g, e] for j in range(L)) / tot
    return out


@pytest.mark.parametrize("H,Hkv", [(2, 2), (4, 2), (6, 1)])
def test_attention_rows_vs_bruteforce(H, Hkv):
    r = _rng(5)
    q, k, v = r.normal(size=(3, H, 4)), r.normal(size=(7, Hkv, 4)), r.normal(size=(7, Hkv, 4))
    assert np.allclose(O.attention_rows(q, k, v), _attn_bruteforce(q, k, v), atol=1e-13)


def test_attention_special_cases():
    r = _rng(6)
    q = r.normal(size=(4, 2, 8))
    k1, v1 = r.normal(size=(1, 2, 8)), r.normal(size=(1, 2, 8))
    assert np.allclose(O.attention_rows(q, k1, v1), np.tile(v1.reshape(1, 16), (4, 1)))  # one key
    k = np.tile(r.normal(size=(1, 2, 8)), (9, 1, 1))  # all keys equal -> uniform weights
    v = r.normal(size=(9, 2, 8))
    assert np.allclose(O.attention_rows(q, k, v), np.tile(v.mean(axis=0).reshape(1, 16), (4, 1)))
    # grouped-query layout with repeated KV heads equals multi-head attention
    kk, vv = r.normal(size=(9, 1, 8)), r.normal(size=(9, 1, 8))
    assert np.allclose(O.attention_rows(q, kk, vv),
                       O.attention_rows(q, np.repeat(kk, 2, 1), np.repeat(vv, 2, 1)))


def test_attention_vs_torch_sdpa():
    r = _rng(7)
    H, Hkv, dh, L, m = 4, 2, 16, 33, 5
    q, k, v = r.normal(size=(m, H, dh)), r.normal(size=(L, Hkv, dh)), r.normal(size=(L, Hkv, dh))
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, H // Hkv, 1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, H // Hkv, 1)).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0].permute(1, 0, 2).reshape(m, H * dh)
    assert np.allclose(O.attention_rows(q, k, v), ref.numpy(), atol=1e-12)


def test_partial_attention_uses_each_rows_own_sequence():
    r = _rng(8)
    B, L, H, dh = 3, 6, 2, 4
    kc, vc = r.normal(size=(B, L, H, dh)), r.normal(size=(B, L, H, dh))
    rows = np.array([1, 4, 13, 17])  # seq 0, 0, 2, 2 ; seq 1 empty
    q = r.normal(size=(4, H, dh))
    got = O.partial_attention(q, kc, vc, rows, B, L)
    assert np.allclose(got[:2], _attn_bruteforce(q[:2], kc[0], vc[0]))
    assert np.allclose(got[2:], _attn_bruteforce(q[2:], kc[2], vc[2]))


# ---------------------------------------------------------------- propositions

def test_prop1_scale_invariance():
    r = _rng(9)
    d = 24
    wo, c, g = r.normal(size=(d, d)), r.normal(size=(5, d)), 1 + 0.3 * r.normal(size=d)
    base = O.rmsnorm(c @ wo.T, g, 0.0)
    for alpha in (1e-3, 0.5, 7.0, 1e4):
        assert np.allclose(O.rmsnorm((alpha * c) @ wo.T, g, 0.0), base, rtol=1e-10, atol=1e-12)


def test_prop2_error_bound_unit_normalised_form():
    # the proof normalises to unit vectors: |f(u) - f(v)| <= kappa(Wo) * sqrt(2 (1 - s))
    r = _rng(10)
    d = 16
    for trial in range(20):
        wo = np.eye(d) + 0.2 * r.normal(size=(d, d))
        kappa = np.linalg.cond(wo)
        a = r.normal(size=(1, d))
        b = a + (10.0 ** r.uniform(-4, 0)) * r.normal(size=(1, d))
        s = O.cosine_rows(a, b)[0]
        ya, yb = a @ wo.T, b @ wo.T
        # RMSNorm with unit gain is the unit vector times sqrt(d)
        delta = np.linalg.norm(O.rmsnorm(ya, np.ones(d), 0.0) - O.rmsnorm(yb, np.ones(d), 0.0)) / math.sqrt(d)
        assert delta <= kappa * math.sqrt(max(0.0, 2 * (1 - s))) + 1e-9


def test_memory_factor_matches_paper_formula():
    with open(os.path.join(GOLD, "memory_factor.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            name, d, H, Hkv, dh, factor = line.split()
            cfg = O.LayerCfg(int(d), int(H), int(Hkv), int(dh), 4 * int(d))
            g = int(H) // int(Hkv)
            assert O.cache_bytes_per_token(cfg, 2) / O.kv_only_bytes_per_token(cfg, 2) == int(factor)
            assert (2 * int(d) / g + 2 * int(d)) / (2 * int(d) / g) == int(factor)


# ---------------------------------------------------------------- GEMM-level pieces

def test_ffn_and_projection_vs_scalar_loops():
    r = _rng(11)
    cfg = O.LayerCfg(hidden=6, n_heads=2, n_kv_heads=1, head_dim=4, ffn=5)
    w = _weights(cfg, r, bias=True)
    f = r.normal(size=(2, 6))
    got = O.swiglu_ffn(f, w)
    for i in range(2):
        act = []
        for n in range(5):
            gate = sum(w["w_gate"][n, k] * f[i, k] for k in range(6))
            up = sum(w["w_up"][n, k] * f[i, k] for k in range(6))
            act.append(gate / (1 + math.exp(-gate)) * up)
        for o in range(6):
            assert got[i, o] == pytest.approx(sum(w["w_down"][o, n] * act[n] for n in range(5)), abs=1e-12)
    # projection + bias at position 0 (rotation = identity): [out, in] weights, y = W n + b
    q, k, v = O.project_qkv(f, np.zeros(2), w, cfg)
    for i in range(2):
        for o in range(8):
            want = sum(w["wq"][o, kk] * f[i, kk] for kk in range(6)) + w["bq"][o]
            assert q.reshape(2, 8)[i, o] == pytest.approx(want, abs=1e-12)
        for o in range(4):
            assert k.reshape(2, 4)[i, o] == pytest.approx(
                sum(w["wk"][o, kk] * f[i, kk] for kk in range(6)) + w["bk"][o], abs=1e-12)
            assert v.reshape(2, 4)[i, o] == pytest.approx(
                sum(w["wv"][o, kk] * f[i, kk] for kk in range(6)) + w["bv"][o], abs=1e-12)


def _dense_layer_torch(x, w, cfg):
    """Third opinion for a whole dense layer built from torch library routines."""
    t = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in w.items()}
    X = torch.from_numpy(x)
    B, L, d = X.shape
    H, Hkv, dh = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    n = torch.nn.functional.rms_norm(X, (d,), t["g_attn"], cfg.rms_eps)
    q = torch.nn.functional.linear(n, t["wq"], t.get("bq")).view(B, L, H, dh)
    k = torch.nn.functional.linear(n, t["wk"], t.get("bk")).view(B, L, Hkv, dh)
    v = torch.nn.functional.linear(n, t["wv"], t.get("bv")).view(B, L, Hkv, dh)
    inv = cfg.rope_theta ** (-torch.arange(0, dh, 2, dtype=torch.float64) / dh)
    ang = torch.arange(L, dtype=torch.float64)[:, None] * inv[None]
    cos, sin = torch.cat([ang.cos(), ang.cos()], -1)[None, :, None], torch.cat([ang.sin(), ang.sin()], -1)[None, :, None]

    def rot_half(u):
        return torch.cat([-u[..., dh // 2:], u[..., :dh // 2]], -1)

    q, k = q * cos + rot_half(q) * sin, k * cos + rot_half(k) * sin
    kk, vv = k.repeat_interleave(H // Hkv, 2), v.repeat_interleave(H // Hkv, 2)
    c = torch.nn.functional.scaled_dot_product_attention(
        q.transpose(1, 2), kk.transpose(1, 2), vv.transpose(1, 2)).transpose(1, 2).reshape(B, L, H * dh)
    h = X + torch.nn.functional.linear(c, t["wo"])
    f = torch.nn.functional.rms_norm(h, (d,), t["g_ffn"], cfg.rms_eps)
    y = h + torch.nn.functional.linear(
        torch.nn.functional.silu(torch.nn.functional.linear(f, t["w_gate"])) * torch.nn.functional.linear(f, t["w_up"]),
        t["w_down"])
    return k.numpy(), v.numpy(), c.numpy(), y.numpy()


@pytest.mark.parametrize("H,Hkv,bias", [(4, 4, False), (4, 2, True)])
def test_full_step_vs_torch_library_layer(H, Hkv, bias):
    r = _rng(12)
    cfg = O.LayerCfg(hidden=32, n_heads=H, n_kv_heads=Hkv, head_dim=8, ffn=48, rope_theta=100.0)
    w = _weights(cfg, r, std=0.2, bias=bias)
    x = r.normal(size=(2, 9, 32))
    caches = O.new_caches(2, 9, cfg)
    O.full_step(x, w, cfg, caches)
    k, v, c, y = _dense_layer_torch(x, w, cfg)
    for name, ref in (("k", k), ("v", v), ("c", c), ("out", y)):
        assert np.allclose(caches[name], ref, atol=1e-11), name


# ---------------------------------------------------------------- whole step

def _setup(seed=13, B=2, L=10, H=4, Hkv=2, bias=False):
    r = _rng(seed)
    cfg = O.LayerCfg(hidden=16, n_heads=H, n_kv_heads=Hkv, head_dim=4, ffn=24, rope_theta=50.0)
    w = _weights(cfg, r, std=0.3, bias=bias)
    x0 = r.normal(size=(B, L, 16))
    caches = O.new_caches(B, L, cfg)
    O.full_step(x0, w, cfg, caches)
    return r, cfg, w, x0, caches


def _copy(c):
    return {k: v.copy() for k, v in c.items()}


def test_step_with_empty_input_set_is_a_noop():
    r, cfg, w, x0, caches = _setup()
    before = _copy(caches)
    idx_out, off, cos = O.layer_step(r.normal(size=x0.shape), np.zeros(0, np.int64), w, cfg, caches, 0.99)
    assert idx_out.size == 0 and cos.size == 0 and off.tolist() == [0, 0, 0]
    for k in caches:
        assert np.array_equal(caches[k], before[k])


@pytest.mark.parametrize("bias", [False, True])
def test_all_rows_salient_equals_dense_step(bias):
    r, cfg, w, x0, caches = _setup(bias=bias)
    x1 = r.normal(size=x0.shape)
    dense = O.new_caches(*x0.shape[:2], cfg)
    O.full_step(x1, w, cfg, dense)
    idx_out, off, cos = O.layer_step(x1, np.arange(x0.shape[0] * x0.shape[1]), w, cfg, caches, 1.5)
    assert idx_out.tolist() == list(range(20)) and off.tolist() == [0, 10, 20]
    for k in caches:
        assert np.allclose(caches[k], dense[k], rtol=1e-11, atol=1e-12), k


def test_repeating_a_step_with_unchanged_input_selects_nothing():
    r, cfg, w, x0, caches = _setup()
    x1 = x0.copy()
    idx = np.array([1, 4, 7, 12, 19])
    x1.reshape(20, -1)[idx] = r.normal(size=(5, 16))
    out1, _, cos1 = O.layer_step(x1, idx, w, cfg, caches, 0.99)
    snap = _copy(caches)
    out2, off2, cos2 = O.layer_step(x1, idx, w, cfg, caches, 0.99)
    assert np.all(cos2 >= 1 - 1e-12) and out2.size == 0 and off2.tolist() == [0, 0, 0]
    for k in ("k", "v", "out"):
        assert np.array_equal(caches[k], snap[k])
    assert np.allclose(caches["c"], snap["c"], atol=1e-14)


def test_sparse_step_touches_only_its_rows_and_matches_dense_rows():
    r, cfg, w, x0, caches = _setup()
    B, L = x0.shape[:2]
    before = _copy(caches)
    x1 = x0.copy()
    idx = np.array([0, 3, 8, 11, 15])
    x1.reshape(B * L, -1)[idx] = r.normal(size=(5, 16))
    idx_out, off, cos = O.layer_step(x1, idx, w, cfg, caches, 0.999999)
    others = np.setdiff1d(np.arange(B * L), idx)
    for k in caches:
        flat_new = caches[k].reshape(B * L, -1)
        flat_old = before[k].reshape(B * L, -1)
        assert np.array_equal(flat_new[others], flat_old[others]), k
    # K and V rows of idx equal a dense projection of x1 (dense K/V depend on their own row only)
    dense = O.new_caches(B, L, cfg)
    O.full_step(x1, w, cfg, dense)
    for k in ("k", "v"):
        assert np.allclose(caches[k].reshape(B * L, -1)[idx], dense[k].reshape(B * L, -1)[idx], atol=1e-12)
    # x1 differs from x0 only on idx, so merged K/V == dense K/V and the recomputed rows are exact
    assert np.allclose(caches["c"].reshape(B * L, -1)[idx], dense["c"].reshape(B * L, -1)[idx], atol=1e-12)
    assert np.allclose(caches["out"].reshape(B * L, -1)[idx_out], dense["out"].reshape(B * L, -1)[idx_out], atol=1e-11)
    assert set(idx_out.tolist()) <= set(idx.tolist())
    assert off[-1] == idx_out.size


def test_rows_failing_the_test_keep_their_cached_output():
    r, cfg, w, x0, caches = _setup()
    B, L = x0.shape[:2]
    x1 = x0.copy()
    idx = np.array([2, 5, 13, 17])
    flat = x1.reshape(B * L, -1)
    flat[[2, 13]] += 1e-7 * r.normal(size=(2, 16))  # tiny change: cosine ~ 1
    # rows 5 and 17: input unchanged, but their cached context is stale (negated): cosine = -1
    caches["c"].reshape(B * L, -1)[[5, 17]] *= -1.0
    before = _copy(caches)
    idx_out, off, cos = O.layer_step(x1, idx, w, cfg, caches, 0.9999)
    assert cos[0] > 0.9999 and cos[2] > 0.9999
    assert cos[1] < -0.9999 and cos[3] < -0.9999
    assert idx_out.tolist() == [5, 17] and off.tolist() == [0, 1, 2]
    out_new, out_old = caches["out"].reshape(B * L, -1), before["out"].reshape(B * L, -1)
    assert np.array_equal(out_new[[2, 13]], out_old[[2, 13]])  # output row reused
    assert not np.array_equal(caches["k"].reshape(B * L, -1)[2], before["k"].reshape(B * L, -1)[2])  # K refreshed
    assert not np.array_equal(caches["c"].reshape(B * L, -1)[2], before["c"].reshape(B * L, -1)[2])  # C committed


def test_saliency_reads_old_cache_before_commit():
    r = _rng(14)
    cache = r.normal(size=(6, 8))
    old = cache.copy()
    rows = np.array([1, 4])
    new = r.normal(size=(2, 8))
    s, flag = O.saliency(new, cache, rows, 0.5, commit=True)
    for j, row in enumerate(rows):
        want = float(new[j] @ old[row] / (np.linalg.norm(new[j]) * np.linalg.norm(old[row])))
        assert s[j] == pytest.approx(want, abs=1e-14)
    assert np.array_equal(cache[rows], new)
    assert np.array_equal(cache[[0, 2, 3, 5]], old[[0, 2, 3, 5]])
    s_all, _ = O.saliency(cache, old, None, 0.5)
    assert s_all[0] == pytest.approx(1.0) and s_all[1] == pytest.approx(s[0])


def test_context_delta_decomposition_identity():
    # Eq. 3: dC = S_t dV + dS V_{t-1}; with unchanged scores (dS = 0) the update S dV is exact
    r = _rng(15)
    L, dh = 7, 4
    q, k = r.normal(size=(L, 1, dh)), r.normal(size=(L, 1, dh))
    v0 = r.normal(size=(L, 1, dh))
    v1 = v0.copy()
    v1[[2, 5]] = r.normal(size=(2, 1, dh))
    c0, c1 = O.attention_rows(q, k, v0), O.attention_rows(q, k, v1)
    S = np.exp(q[:, 0] @ k[:, 0].T / math.sqrt(dh))
    S /= S.sum(axis=1, keepdims=True)
    assert np.allclose(c1 - c0, S[:, [2, 5]] @ (v1 - v0)[[2, 5], 0], atol=1e-13)


# ---------------------------------------------------------------- stack of layers

def _stack_setup(n_layers=3, seed=21, B=2, L=10):
    r = _rng(seed)
    cfg = O.LayerCfg(hidden=16, n_heads=4, n_kv_heads=2, head_dim=4, ffn=24, rope_theta=50.0)
    ws = [_weights(cfg, r, std=0.3) for _ in range(n_layers)]
    x0 = r.normal(size=(B, L, 16))
    caches = [O.new_caches(B, L, cfg) for _ in range(n_layers)]
    O.stack_full_step(x0, ws, cfg, caches)
    return r, cfg, ws, x0, caches


def test_dense_stack_is_the_composition_of_library_layers():
    # each layer of the dense stack against the torch-library layer applied to the previous output
    r, cfg, ws, x0, caches = _stack_setup()
    h = x0
    for w, c in zip(ws, caches):
        k, v, ctx, y = _dense_layer_torch(h, w, cfg)
        assert np.allclose(c["k"], k, atol=1e-10) and np.allclose(c["c"], ctx, atol=1e-10)
        assert np.allclose(c["out"], y, atol=1e-9)
        h = y


def test_stack_with_all_rows_salient_equals_dense_stack():
    r, cfg, ws, x0, caches = _stack_setup()
    x1 = r.normal(size=x0.shape)
    dense = [O.new_caches(2, 10, cfg) for _ in ws]
    O.stack_full_step(x1, ws, cfg, dense)
    per_layer = O.stack_step(x1, np.arange(20), ws, cfg, caches, 1.5)
    for (idx, off, cos), c, dn in zip(per_layer, caches, dense):
        assert idx.tolist() == list(range(20)) and off.tolist() == [0, 10, 20]
        for k in c:
            assert np.allclose(c[k], dn[k], rtol=1e-10, atol=1e-11), k


def test_stack_carries_the_salient_set_and_the_output_cache_between_layers():
    r, cfg, ws, x0, caches = _stack_setup(n_layers=4)
    before = [_copy(c) for c in caches]
    x1 = x0.copy()
    idx = np.array([0, 3, 8, 11, 15, 16])
    # three rows change a lot, three hardly at all: the set shrinks on the way down
    x1.reshape(20, -1)[idx[:3]] = r.normal(size=(3, 16))
    x1.reshape(20, -1)[idx[3:]] += 1e-7 * r.normal(size=(3, 16))
    per_layer = O.stack_step(x1, idx, ws, cfg, caches, 0.9999)
    prev = idx
    for l, ((out, off, cos), c, b) in enumerate(zip(per_layer, caches, before)):
        assert cos.size == prev.size                      # candidates = previous layer's selection
        assert set(out.tolist()) <= set(prev.tolist())
        assert off[-1] == out.size
        untouched = np.setdiff1d(np.arange(20), prev)
        for k in c:                                      # rows outside the candidates: all caches kept
            a = c[k].reshape(20, -1)
            assert np.array_equal(a[untouched], b[k].reshape(20, -1)[untouched]), (l, k)
        kept = np.setdiff1d(np.arange(20), out)           # rows not selected keep the cached output
        assert np.array_equal(c["out"].reshape(20, -1)[kept], b["out"].reshape(20, -1)[kept])
        prev = out
    # sequence 1 holds only the barely moved rows: their contexts stay put and they drop out at layer 1
    assert per_layer[0][0].tolist() == [0, 3, 8] and per_layer[-1][0].tolist() == [0, 3, 8]
    assert np.all(per_layer[0][2][3:] > 1 - 1e-9)
    # a one-layer stack is the layer step
    one = [_copy(before[0])]
    (o1, f1, c1), = O.stack_step(x1, idx, ws[:1], cfg, one, 0.9999)
    assert np.array_equal(o1, per_layer[0][0]) and np.array_equal(c1, per_layer[0][2])
    # layer l's recomputed rows equal a dense layer applied to the layer input it actually saw
    h = x1
    for l, ((out, off, cos), c, w) in enumerate(zip(per_layer, caches, ws)):
        if out.size:
            # context of selected rows against a dense evaluation with the merged K/V of this layer
            for t in out[:2]:
                bsel, i = divmod(int(t), 10)
                q = O.project_qkv(O.rmsnorm(h.reshape(20, -1)[[t]], w["g_attn"], cfg.rms_eps), np.array([i]), w, cfg)[0]
                ref = O.attention_rows(q, c["k"][bsel], c["v"][bsel]).reshape(-1)
                assert np.allclose(c["c"][bsel, i], ref, atol=1e-12)
        h = c["out"]


# ---------------------------------------------------------------- approximate attention (Alg. 4)

def _dense_attention(q, k, v):
    """q [L,H,dh], k,v [L,Hkv,dh] -> [L, H*dh], through torch's library attention."""
    H, Hkv = q.shape[1], k.shape[1]
    tq = torch.from_numpy(q).transpose(0, 1)[None]
    tk = torch.from_numpy(k).repeat_interleave(H // Hkv, 1).transpose(0, 1)[None]
    tv = torch.from_numpy(v).repeat_interleave(H // Hkv, 1).transpose(0, 1)[None]
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0].transpose(0, 1)
    return o.reshape(q.shape[0], -1).numpy()


@pytest.mark.parametrize("H,Hkv", [(4, 4), (6, 2)])
def test_approx_attention_is_exact_when_only_values_change(H, Hkv):
    # Eq. 3 with unchanged scores: C_old + A[:, idx] dV == exact attention with the new values
    r = _rng(31)
    B, L, dh = 2, 11, 8
    q = r.normal(size=(B * L, H, dh))
    k = r.normal(size=(B, L, Hkv, dh))
    v_old = r.normal(size=(B, L, Hkv, dh))
    idx = np.array([1, 4, 9, 12, 13, 21])
    v_new = v_old.copy()
    v_new.reshape(B * L, Hkv, dh)[idx] = r.normal(size=(idx.size, Hkv, dh))
    dv = (v_new - v_old).reshape(B * L, Hkv, dh)[idx]
    dc = O.approx_attention(q, k, dv, idx, B, L)
    for b in range(B):
        c_old = _dense_attention(q[b * L:(b + 1) * L], k[b], v_old[b])
        c_new = _dense_attention(q[b * L:(b + 1) * L], k[b], v_new[b])
        assert np.allclose(c_old + dc[b * L:(b + 1) * L], c_new, atol=1e-12)


def test_approx_attention_bruteforce_and_degenerate_cases():
    r = _rng(32)
    B, L, H, Hkv, dh = 2, 5, 4, 2, 4
    q = r.normal(size=(B * L, H, dh))
    k = r.normal(size=(B, L, Hkv, dh))
    idx = np.array([0, 3, 7])
    dv = r.normal(size=(3, Hkv, dh))
    got = O.approx_attention(q, k, dv, idx, B, L)
    ref = np.zeros_like(got)
    for t in range(B * L):           # scalar loops
        b = t // L
        for h in range(H):
            z = [sum(q[t, h, e] * k[b, j, h // 2, e] for e in range(dh)) / math.sqrt(dh) for j in range(L)]
            m = max(z)
            den = sum(math.exp(zj - m) for zj in z)
            for jj, tok in enumerate(idx):
                if tok // L != b:
                    continue
                a = math.exp(z[tok % L] - m) / den
                for e in range(dh):
                    ref[t, h * dh + e] += a * dv[jj, h // 2, e]
    assert np.allclose(got, ref, atol=1e-13)
    # no residual, or no salient token: no update; sequence 1 has one salient token only
    assert np.all(O.approx_attention(q, k, np.zeros_like(dv), idx, B, L) == 0)
    assert np.all(O.approx_attention(q, k, dv[:0], idx[:0], B, L) == 0)
    # every token salient: the full softmax times dV, i.e. library attention with V := dV
    allidx = np.arange(B * L)
    dv_all = r.normal(size=(B * L, Hkv, dh))
    got = O.approx_attention(q, k, dv_all, allidx, B, L)
    for b in range(B):
        assert np.allclose(got[b * L:(b + 1) * L],
                           _dense_attention(q[b * L:(b + 1) * L], k[b], dv_all[b * L:(b + 1) * L]), atol=1e-12)


def test_layer_step_approx_structure():
    r, cfg, w, x0, caches = _setup(seed=33)
    T = 20
    # (i) empty salient set: nothing changes, every cosine is 1
    before = _copy(caches)
    out, off, cos = O.layer_step_approx(r.normal(size=x0.shape), np.zeros(0, np.int64), w, cfg, caches, 0.99)
    assert out.size == 0 and np.all(cos >= 1 - 1e-12)
    for k in caches:
        assert np.allclose(caches[k], before[k], atol=1e-14), k
    # (ii) every token salient: the exact path only, equal to layer_step and to the dense step
    x1 = r.normal(size=x0.shape)
    a, b_ = _copy(caches), _copy(caches)
    o1 = O.layer_step_approx(x1, np.arange(T), w, cfg, a, 1.5)
    o2 = O.layer_step(x1, np.arange(T), w, cfg, b_, 1.5)
    assert np.array_equal(o1[0], o2[0])
    for k in a:
        assert np.allclose(a[k], b_[k], rtol=1e-11, atol=1e-12), k
    # (iii) a few salient tokens: K/V of the others untouched, contexts of the others move by the
    #       approximate update, and tokens outside idx_in can become salient
    idx = np.array([2, 5, 13])
    x2 = x0.copy()
    x2.reshape(T, -1)[idx] = 3.0 * r.normal(size=(3, 16))
    c = _copy(caches)
    v_before = c["v"].copy()
    out, off, cos = O.layer_step_approx(x2, idx, w, cfg, c, 0.999)
    others = np.setdiff1d(np.arange(T), idx)
    assert np.array_equal(c["k"].reshape(T, -1)[others], caches["k"].reshape(T, -1)[others])
    assert np.array_equal(c["v"].reshape(T, -1)[others], v_before.reshape(T, -1)[others])
    assert cos.shape == (T,) and off[-1] == out.size
    assert set(out.tolist()) - set(idx.tolist()), "some non-salient token should cross the threshold"
    # the contexts of the other tokens: cached + (softmax columns of idx) x dV, recomputed here from
    # the exact attention with old and new values (scores of non-salient queries use merged keys)
    n_all = O.rmsnorm(x2.reshape(T, -1), w["g_attn"], cfg.rms_eps)
    q_all = O.rope((n_all @ w["wq"].T).reshape(T, cfg.n_heads, cfg.head_dim), np.arange(T) % 10, cfg.rope_theta)
    for b in range(2):
        qs = q_all[b * 10:(b + 1) * 10]
        exact_new = O.attention_rows(qs, c["k"][b], c["v"][b])
        exact_oldv = O.attention_rows(qs, c["k"][b], v_before[b])
        rows = others[(others >= b * 10) & (others < (b + 1) * 10)]
        want = caches["c"].reshape(T, -1)[rows] + (exact_new - exact_oldv)[rows - b * 10]
        assert np.allclose(c["c"].reshape(T, -1)[rows], want, atol=1e-12)
    # rows not selected keep their cached output
    kept = np.setdiff1d(np.arange(T), out)
    assert np.array_equal(c["out"].reshape(T, -1)[kept], caches["out"].reshape(T, -1)[kept])


# ---- response-only steps and the step schedule  [Sec. 3.5; App. C.1, Alg. 1] -----------------------

def test_merge_lists_vs_python_sets():
    r = _rng(41)
    L = 12
    for _ in range(20):
        a = np.sort(r.choice(3 * L, size=int(r.integers(0, 15)), replace=False))
        b = np.sort(r.choice(3 * L, size=int(r.integers(0, 15)), replace=False))
        lo = int(r.integers(0, L))
        want = sorted(t for t in set(a.tolist()) | set(b.tolist()) if t % L >= lo)
        assert O.merge_lists(a, b, L, lo).tolist() == want
        assert O.merge_lists(None, b, L, lo).tolist() == sorted(t for t in b.tolist() if t % L >= lo)
    assert O.merge_lists(None, None, L, 0).size == 0


def test_step_kinds_follow_the_schedule():
    s = O.Schedule(t_full=4, full_period=4, prompt_len=6, approx=False, tau=0.99)
    kinds = [O.step_kind(t, s) for t in range(16)]
    assert kinds[:4] == ["dense"] * 4
    assert [k for t, k in enumerate(kinds) if t >= 4 and t % 4 == 0] == ["full"] * 3
    assert all(k == "response" for t, k in enumerate(kinds) if t >= 4 and t % 4)
    # three of four sparse steps take the response only (Sec. 3.5 / App. C.1: 75 % of the steps)
    sparse = [O.step_kind(t, s) for t in range(4, 4 + 400)]
    assert sparse.count("response") / len(sparse) == 0.75
    assert O.step_kind(9, O.Schedule(2, 1, 6, False, 0.9)) == "full"


def test_response_only_step_of_the_approximate_path():
    """A response-only step computes, for every response token, exactly what the whole-sequence step
    computes for it (rows are independent given K, V), and leaves the prompt tokens alone."""
    r, cfg, w, x0, caches = _setup(seed=43)
    B, L, T, lo = 2, 10, 20, 4
    idx = np.array([5, 8, 14, 19])  # response tokens only
    x1 = x0.copy()
    x1.reshape(T, -1)[idx] = 2.0 * r.normal(size=(idx.size, 16))
    x1.reshape(T, -1)[[1, 12]] += 5.0  # prompt inputs differ too: a response-only step never reads them
    full, resp = _copy(caches), _copy(caches)
    of, _, cf = O.layer_step_approx(x1, idx, w, cfg, full, 0.999)
    orr, offr, cr = O.layer_step_approx(x1, idx, w, cfg, resp, 0.999, row_lo=lo)
    pos = np.arange(T) % L
    in_resp = pos >= lo
    assert np.array_equal(orr, of[in_resp[of]])
    assert offr[-1] == orr.size and np.all(cr[~in_resp] == 1.0)
    assert np.allclose(cr[in_resp], cf[in_resp], atol=1e-13)
    for k in ("k", "v", "c", "out"):
        a, b_ = resp[k].reshape(T, -1), full[k].reshape(T, -1)
        assert np.allclose(a[in_resp], b_[in_resp], atol=1e-12), k
        assert np.array_equal(a[~in_resp], caches[k].reshape(T, -1)[~in_resp]), k
    # some prompt token does move in the whole-sequence step, so the restriction is not vacuous
    assert not np.allclose(full["c"].reshape(T, -1)[~in_resp], caches["c"].reshape(T, -1)[~in_resp])
    with pytest.raises(AssertionError):
        O.layer_step_approx(x1, np.array([1, 5]), w, cfg, _copy(caches), 0.9, row_lo=lo)


@pytest.mark.parametrize("row_lo", [0, 4])
@pytest.mark.parametrize("cached_norm", [False, True])
def test_stack_step_approx_is_the_hand_composed_layer_loop(row_lo, cached_norm):
    """The layer loop of the approximate path against layer_step_approx applied by hand, layer after
    layer: layer l reads the output cache layer l-1 holds after its update and the list layer l-1
    selected, with the same response window and normaliser choice in every layer.  [Alg. 3, loop over l]
    A wrong hand-through of row_lo / cached_norm, a broken list chain or a layer reading the step's
    input instead of the previous output cache each change a cache or a set here."""
    r, cfg, ws, x0, caches = _stack_setup(n_layers=3, seed=47)
    B, L, T = 2, 10, 20
    if cached_norm:
        for c in caches:
            c["lse"] = np.zeros((B, L, cfg.n_heads))
        O.stack_full_step(x0, ws, cfg, caches)  # fills the normalisers
    idx = np.array([5, 8, 14, 19])
    x1 = x0.copy()
    x1.reshape(T, -1)[idx] += 0.3 * r.normal(size=(idx.size, 16))
    x1.reshape(T, -1)[[1, 12]] += 3.0   # prompt rows move too: only a whole-sequence step may see them
    tau = 0.99
    loop = [_copy(c) for c in caches]
    per_layer = O.stack_step_approx(x1, idx, ws, cfg, loop, tau, row_lo, cached_norm)
    hand = [_copy(c) for c in caches]
    h, cur = x1, idx
    sets = []
    for l, w in enumerate(ws):
        cur, off, cos = O.layer_step_approx(h, cur, w, cfg, hand[l], tau, row_lo=row_lo, cached_norm=cached_norm)
        assert np.array_equal(per_layer[l][0], cur) and np.array_equal(per_layer[l][1], off)
        assert np.array_equal(per_layer[l][2], cos)
        sets.append(cur)
        h = hand[l]["out"]
    for a, b_ in zip(loop, hand):
        assert a.keys() == b_.keys()
        for k in a:
            assert np.array_equal(a[k], b_[k]), k
    # the case is not degenerate: sets differ between layers, tokens outside the candidates get
    # selected, and the switches matter (each alternative gives another result)
    assert len({tuple(s_.tolist()) for s_ in sets}) > 1
    assert any(set(s_.tolist()) - set(idx.tolist()) for s_ in sets)
    pos = np.arange(T) % L
    for l in range(3):
        assert np.all(sets[l] % L >= row_lo)
        for k in ("k", "v", "c", "out"):
            assert np.array_equal(loop[l][k].reshape(T, -1)[pos < row_lo], caches[l][k].reshape(T, -1)[pos < row_lo])
    other = [_copy(c) for c in caches]
    alt = O.stack_step_approx(x1, idx, ws, cfg, other, tau, 4 - row_lo, cached_norm)
    assert not all(np.array_equal(a["c"], b_["c"]) for a, b_ in zip(loop, other))
    if "lse" in caches[0]:
        other = [_copy(c) for c in caches]
        O.stack_step_approx(x1, idx, ws, cfg, other, tau, row_lo, not cached_norm)
        assert not all(np.allclose(a["c"], b_["c"], atol=1e-9) for a, b_ in zip(loop, other))
    # a layer that read the step's input x instead of the output cache above it would differ
    wrong = [_copy(c) for c in caches]
    cur = idx
    for l, w in enumerate(ws):
        cur, _, _ = O.layer_step_approx(x1, cur, w, cfg, wrong[l], tau, row_lo=row_lo, cached_norm=cached_norm)
    assert not np.allclose(wrong[1]["out"], loop[1]["out"], atol=1e-9)


@pytest.mark.parametrize("approx", [False, True])
def test_denoise_step_composes_the_schedule(approx):
    r, cfg, ws, x, caches = _stack_setup(n_layers=2, seed=45)
    B, L, T = 2, 10, 20
    s = O.Schedule(t_full=2, full_period=4, prompt_len=4, approx=approx, tau=0.999)
    # dense steps: FullStep through the stack, no carried set
    a, b_ = [_copy(c) for c in caches], [_copy(c) for c in caches]
    assert O.denoise_step(0, s, x, np.array([3]), None, ws, cfg, a) is None
    O.stack_full_step(x, ws, cfg, b_)
    for ca, cb in zip(a, b_):
        for k in ca:
            assert np.array_equal(ca[k], cb[k])
    # first sparse step (t = 2, response-only): no carried set -> the decoded positions, kept to the response
    decoded = np.array([2, 6, 17])
    x1 = x.copy()
    x1.reshape(T, -1)[decoded] = r.normal(size=(3, x.shape[-1]))
    c1, c2 = [_copy(c) for c in a], [_copy(c) for c in a]
    carry = O.denoise_step(2, s, x1, decoded, None, ws, cfg, c1)
    cand = np.array([6, 17])
    if approx:
        want = O.stack_step_approx(x1, cand, ws, cfg, c2, s.tau, row_lo=4)[-1][0]
    else:
        want = O.stack_step(x1, cand, ws, cfg, c2, s.tau)[-1][0]
    assert np.array_equal(carry, want)
    for ca, cb in zip(c1, c2):
        for k in ca:
            assert np.array_equal(ca[k], cb[k])
    # a whole-sequence step (t = 4): carried set joined with the newly decoded positions, prompt included
    decoded2 = np.array([1, 13])
    c3, c4 = [_copy(c) for c in c1], [_copy(c) for c in c1]
    carry2 = O.denoise_step(4, s, x1, decoded2, carry, ws, cfg, c3)
    cand2 = np.union1d(carry, decoded2)
    if approx:
        want2 = O.stack_step_approx(x1, cand2, ws, cfg, c4, s.tau)[-1][0]
    else:
        want2 = O.stack_step(x1, cand2, ws, cfg, c4, s.tau)[-1][0]
    assert np.array_equal(carry2, want2)
    # with the approximate path off, a response-only step equals the whole-sequence step whenever no
    # prompt token is a candidate
    if not approx:
        c5, c6 = [_copy(c) for c in c1], [_copy(c) for c in c1]
        r5 = O.denoise_step(5, s, x1, np.array([7]), np.array([6, 17]), ws, cfg, c5)   # response-only
        r6 = O.denoise_step(8, s, x1, np.array([7]), np.array([6, 17]), ws, cfg, c6)   # whole sequence
        assert np.array_equal(r5, r6)
        for ca, cb in zip(c5, c6):
            for k in ca:
                assert np.array_equal(ca[k], cb[k])


# ---- approximate attention with reused normalisers (variant of Alg. 4; Sec. 3.3 cost claim) -------

def test_attention_lse_is_the_log_of_the_softmax_normaliser():
    from scipy.special import logsumexp
    r = _rng(51)
    q, k = r.normal(size=(7, 4, 8)), r.normal(size=(13, 2, 8))
    got = O.attention_lse(q, k)
    for i in range(7):
        for h in range(4):
            z = np.array([q[i, h] @ k[j, h // 2] for j in range(13)]) / math.sqrt(8)
            assert abs(got[i, h] - logsumexp(z)) < 1e-12
    # one key: the normaliser is that key's score
    assert np.allclose(O.attention_lse(q, k[:1]), np.einsum("ihd,hd->ih", q, k[0].repeat(2, axis=0)) / math.sqrt(8))


def test_cached_normaliser_variant_equals_alg4_with_fresh_normalisers():
    r = _rng(53)
    B, L, H, Hkv, dh = 2, 9, 4, 2, 8
    T = B * L
    q = r.normal(size=(T, H, dh))
    k = r.normal(size=(B, L, Hkv, dh))
    idx = np.array([1, 4, 8, 10, 16])
    dv = r.normal(size=(idx.size, Hkv, dh))
    lse = np.concatenate([O.attention_lse(q[b * L:(b + 1) * L], k[b]) for b in range(B)])
    a = O.approx_attention(q, k, dv, idx, B, L)
    c = O.approx_attention_cached(q, k, dv, idx, lse, B, L)
    assert np.allclose(a, c, rtol=1e-12, atol=1e-13)
    # scalar-loop definition with an arbitrary (stale) normaliser
    stale = lse + r.normal(size=lse.shape) * 0.3
    c2 = O.approx_attention_cached(q, k, dv, idx, stale, B, L).reshape(T, H, dh)
    for i in (0, 7, 12):
        b = i // L
        for h in range(H):
            want = np.zeros(dh)
            for n, j in enumerate(idx):
                if j // L == b:
                    want += math.exp(q[i, h] @ k[b, j % L, h // 2] / math.sqrt(dh) - stale[i, h]) * dv[n, h // 2]
            assert np.allclose(c2[i, h], want, atol=1e-12)
    # no salient token in a sequence: no residual there
    only0 = O.approx_attention_cached(q, k, dv[:3], idx[:3], lse, B, L).reshape(B, L, -1)
    assert np.all(only0[1] == 0)


def test_layer_step_with_reused_normalisers():
    """The fifth cache is filled by the dense step and refreshed for the exact rows; with unchanged
    keys the variant reproduces the literal step, with changed keys the two differ only in the
    contexts of the non-salient tokens."""
    r, cfg, w, x0, caches = _setup(seed=55)
    B, L, T = 2, 10, 20
    caches["lse"] = np.zeros((B, L, cfg.n_heads))
    O.full_step(x0, w, cfg, caches)
    q_all = O.rope((O.rmsnorm(x0.reshape(T, -1), w["g_attn"], cfg.rms_eps) @ w["wq"].T).reshape(T, cfg.n_heads, cfg.head_dim),
                   np.arange(T) % L, cfg.rope_theta)
    fresh = np.concatenate([O.attention_lse(q_all[b * L:(b + 1) * L], caches["k"][b]) for b in range(B)])
    assert np.allclose(caches["lse"].reshape(T, -1), fresh, atol=1e-12)
    # (i) keys that cannot change (a zero key projection): the reused normalisers are the current ones
    idx = np.array([3, 6, 15])
    w0 = dict(w)
    w0["wk"] = np.zeros_like(w["wk"])
    c0 = O.new_caches(B, L, cfg)
    c0["lse"] = np.zeros((B, L, cfg.n_heads))
    O.full_step(x0, w0, cfg, c0)
    x1 = x0.copy()
    x1.reshape(T, -1)[idx] = r.normal(size=(idx.size, x0.shape[-1]))
    a, b_ = _copy(c0), _copy(c0)
    oa = O.layer_step_approx(x1, idx, w0, cfg, a, 0.999)
    ob = O.layer_step_approx(x1, idx, w0, cfg, b_, 0.999, cached_norm=True)
    assert np.array_equal(oa[0], ob[0])
    for k_ in ("k", "v", "c", "out", "lse"):
        assert np.allclose(a[k_], b_[k_], rtol=1e-10, atol=1e-12), k_
    # (ii) keys change: exact rows, K, V and the refreshed normalisers agree; the other contexts differ
    a, b_ = _copy(caches), _copy(caches)
    O.layer_step_approx(x1, idx, w, cfg, a, -2.0)
    O.layer_step_approx(x1, idx, w, cfg, b_, -2.0, cached_norm=True)
    others = np.setdiff1d(np.arange(T), idx)
    for k_ in ("k", "v"):
        assert np.array_equal(a[k_], b_[k_])
    assert np.allclose(a["c"].reshape(T, -1)[idx], b_["c"].reshape(T, -1)[idx], atol=1e-13)
    assert np.allclose(a["lse"].reshape(T, -1)[idx], b_["lse"].reshape(T, -1)[idx], atol=1e-13)
    assert np.array_equal(b_["lse"].reshape(T, -1)[others], caches["lse"].reshape(T, -1)[others])
    assert not np.allclose(a["c"].reshape(T, -1)[others], b_["c"].reshape(T, -1)[others], atol=1e-9)
    # ... by exactly the ratio of stale to fresh normalisers, head by head
    qn = O.rope((O.rmsnorm(x1.reshape(T, -1), w["g_attn"], cfg.rms_eps) @ w["wq"].T).reshape(T, cfg.n_heads, cfg.head_dim),
                np.arange(T) % L, cfg.rope_theta)
    fresh = np.concatenate([O.attention_lse(qn[b * L:(b + 1) * L], a["k"][b]) for b in range(B)])
    ratio = np.exp(fresh - caches["lse"].reshape(T, -1))  # [T, H]
    da = (a["c"] - caches["c"]).reshape(T, cfg.n_heads, -1)
    db = (b_["c"] - caches["c"]).reshape(T, cfg.n_heads, -1)
    assert np.allclose(db[others], da[others] * ratio[others][:, :, None], rtol=1e-9, atol=1e-12)
