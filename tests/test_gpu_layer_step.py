"""Whole-step parity of dyllm_layer_step / dyllm_full_step against the CPU oracle, through the C ABI:
multi-step runs on the tiny fp32 configuration, a threshold sweep that exercises the filter path,
the structural equivalences, and the 8B-shaped configurations (batch slices where the oracle would
otherwise take minutes)."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import dyllm_oracle as O
from paper_2603_08026_amd import binding as Bd
from paper_2603_08026_amd.layer import Layer, to_host
from synth import workload as W
from tests.helpers import (BAND, TOL, assert_close, assert_index_sets_match, oracle_cfg, rand_rows,
                           rand_weights, small_shape)

pytestmark = pytest.mark.gpu


def _say(*a):
    print("[case]", *a, flush=True)


def _compare_caches(lay, ref, tol, what, rows=None):
    got = lay.get_caches()
    errs = {}
    for name in ("k", "v", "c", "out"):
        g, r = got[name].reshape(lay.B * lay.L, -1), ref[name].reshape(lay.B * lay.L, -1)
        if rows is not None:
            g, r = g[rows], r[rows]
        errs[name] = assert_close(g, r, tol, "%s cache %s" % (what, name))
    return errs


def _run_stream(wl: W.Workload, n_steps: int, teacher_forced: bool, seed_w: int = 0):
    """Runs n_steps of the workload on both sides and compares after every step."""
    s = wl.shape
    cfg = oracle_cfg(s)
    tol = TOL[s.dtype]
    w = W.make_weights(s, layer=seed_w)
    lay = Layer.from_shape(s, wl.batch, wl.seq)
    lay.set_weights(w)
    ref = O.new_caches(wl.batch, wl.seq, cfg)
    worst = 0.0
    for st in W.step_stream(wl, n_steps):
        _say(wl.name, "step", st.t, "dense" if st.dense else "sparse M=%d" % st.idx.size,
             "teacher-forced" if teacher_forced else "free-running")
        xd = lay.upload(st.x)
        if st.dense:
            O.full_step(st.x, w, cfg, ref)
            lay.full_step(xd)
            errs = _compare_caches(lay, ref, tol, "dense step %d" % st.t)
        else:
            if teacher_forced:
                # start the step from the oracle's caches (rounded to the storage type)
                start = {k: (W.round_bf16(v.astype(np.float32)) if s.dtype == "bf16" else v.astype(np.float32))
                         for k, v in ref.items()}
                lay.set_caches(start)
                ref = {k: v.astype(np.float64) for k, v in start.items()}
            before = lay.get_caches()
            idx_ref, off_ref, cos_ref = O.layer_step(st.x, st.idx, w, cfg, ref, wl.tau)
            il = lay.make_list(st.idx, st.offsets)
            out = lay.layer_step(xd, il, wl.tau)
            idx_g, off_g = lay.read_list(out)
            cos_g = lay.cos[:st.idx.size].cpu().numpy()
            assert_index_sets_match(idx_g, idx_ref, st.idx, cos_ref, wl.tau, "step %d" % st.t)
            assert off_g[-1] == idx_g.size
            for b in range(wl.batch):
                seg = idx_g[off_g[b]:off_g[b + 1]]
                assert np.all((seg >= b * wl.seq) & (seg < (b + 1) * wl.seq))
            assert np.max(np.abs(cos_g - cos_ref)) < (5e-5 if s.dtype == "f32" else 2e-2)
            errs = _compare_caches(lay, ref, tol, "sparse step %d" % st.t)
            # rows outside idx_in keep every cache byte
            after = lay.get_caches()
            others = np.setdiff1d(np.arange(wl.tokens), st.idx)
            for name in after:
                a = after[name].reshape(wl.tokens, -1)[others]
                b_ = before[name].reshape(wl.tokens, -1)[others]
                assert np.array_equal(a, b_), name
        worst = max(worst, max(errs.values()))
    lay.close()
    return worst


def test_c1_tiny_fp32_all_steps_free_running():
    wl = W.CONFIGS["c1"]
    worst = _run_stream(wl, wl.steps, teacher_forced=False)
    assert worst <= 1e-4


def test_small_bf16_stream_free_running_and_teacher_forced():
    s = small_shape("bf16", gqa=True, dh=128)
    wl = W.Workload("small-bf16", s, 3, 150, 42, 6, 0.1, ragged=True, t_full=2, tau=0.99)
    _run_stream(wl, 6, teacher_forced=False)
    _run_stream(wl, 5, teacher_forced=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_threshold_sweep_filters_candidates(dtype):
    """Candidates whose input moved by sigma in [1e-4, 1] give cosines on both sides of tau, so that
    idx_out is a proper, non-empty subset of idx_in; rows failing the test keep their output row."""
    _say("threshold sweep", dtype)
    s = small_shape(dtype)
    cfg = oracle_cfg(s)
    B, L = 2, 96
    w = rand_weights(s, 41, std=0.08)
    lay = Layer.from_shape(s, B, L)
    lay.set_weights(w)
    x0 = W.philox(42, "x0").standard_normal((B, L, s.hidden), dtype=np.float32)
    x0 = W.round_bf16(x0) if dtype == "bf16" else x0
    ref = O.new_caches(B, L, cfg)
    O.full_step(x0, w, cfg, ref)
    lay.full_step(lay.upload(x0))
    start = {k: (W.round_bf16(v.astype(np.float32)) if dtype == "bf16" else v.astype(np.float32)) for k, v in ref.items()}
    lay.set_caches(start)
    ref = {k: v.astype(np.float64) for k, v in start.items()}
    idx, off = rand_rows(43, B, L, [20, 11])
    # a few candidates move a lot, most move a little: contexts of the small movers stay near cos = 1
    sig = 10.0 ** W.philox(44, "sig").uniform(-4, -1, idx.size)
    sig[::5] = 1.0
    x1 = x0.copy().reshape(B * L, -1)
    x1[idx] = W.perturbed_rows(x1[idx], sig, 45)
    x1 = (W.round_bf16(x1) if dtype == "bf16" else x1).reshape(B, L, -1)
    cos_probe = O.layer_step(x1, idx, w, cfg, {k: v.copy() for k, v in ref.items()}, 0.5)[2]
    tau = float(np.median(cos_probe))  # half of the candidates on each side
    before_out = ref["out"].copy()
    idx_ref, off_ref, cos_ref = O.layer_step(x1, idx, w, cfg, ref, tau)
    assert 0 < idx_ref.size < idx.size
    out = lay.layer_step(lay.upload(x1), lay.make_list(idx, off), tau)
    idx_g, off_g = lay.read_list(out)
    assert_index_sets_match(idx_g, idx_ref, idx, cos_ref, tau, "sweep")
    firm = np.abs(cos_ref - tau) > BAND
    if np.all(firm):
        assert np.array_equal(idx_g, idx_ref) and np.array_equal(off_g, off_ref)
    got = lay.get_caches()
    kept = np.setdiff1d(idx, idx_g)
    assert kept.size > 0
    assert np.array_equal(got["out"].reshape(B * L, -1)[kept], before_out.reshape(B * L, -1)[kept])
    both = np.intersect1d(idx_g, idx_ref)
    assert_close(got["out"].reshape(B * L, -1)[both], ref["out"].reshape(B * L, -1)[both], TOL[dtype], "out rows")
    assert_close(got["c"], ref["c"], TOL[dtype], "context cache")
    lay.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_structural_equivalences(dtype):
    _say("structural equivalences", dtype)
    s = small_shape(dtype, gqa=True)
    B, L = 2, 80
    T = B * L
    w = rand_weights(s, 51, bias=True)
    lay = Layer.from_shape(s, B, L)
    lay.set_weights(w)
    x0 = W.philox(52, "x").standard_normal((B, L, s.hidden), dtype=np.float32)
    x1 = W.philox(53, "x").standard_normal((B, L, s.hidden), dtype=np.float32)
    if dtype == "bf16":
        x0, x1 = W.round_bf16(x0), W.round_bf16(x1)
    lay.full_step(lay.upload(x0))
    snap = {k: getattr(lay, k).clone() for k in ("k", "v", "c", "out")}
    # (i) empty idx_in: no cache byte changes, idx_out empty
    empty = lay.make_list(np.zeros(0, np.int32), np.zeros(B + 1, np.int32), cap=8)
    out = lay.layer_step(lay.upload(x1), empty, 0.99)
    idx_g, off_g = lay.read_list(out)
    assert idx_g.size == 0 and off_g.tolist() == [0] * (B + 1)
    for k in snap:
        assert torch.equal(getattr(lay, k), snap[k]), k
    # also with capacity 0
    out = lay.layer_step(lay.upload(x1), lay.make_list(np.zeros(0, np.int32), np.zeros(B + 1, np.int32)), 0.99)
    assert lay.read_list(out)[0].size == 0
    # (ii) idx_in = all rows, tau > 1: identical to the dense step, every row selected
    allrows = lay.make_list(np.arange(T, dtype=np.int32), np.arange(B + 1, dtype=np.int32) * L)
    out = lay.layer_step(lay.upload(x1), allrows, 1.5)
    idx_g, off_g = lay.read_list(out)
    assert np.array_equal(idx_g, np.arange(T)) and off_g.tolist() == [0, L, 2 * L]
    sparse = {k: getattr(lay, k).clone() for k in snap}
    lay.full_step(lay.upload(x1))
    for k in snap:
        assert torch.equal(getattr(lay, k), sparse[k]), k
    # (iii) the same step again with unchanged input: every cosine is 1, nothing selected
    some, off = rand_rows(54, B, L, [13, 30])
    il = lay.make_list(some, off)
    lay.layer_step(lay.upload(x1), il, 0.99)
    out = lay.layer_step(lay.upload(x1), il, 0.99)
    idx_g, _ = lay.read_list(out)
    cos = lay.cos[:some.size].cpu().numpy()
    assert idx_g.size == 0 and np.all(cos >= 1 - 1e-5)
    lay.close()


def _slice_batch(wl: W.Workload, nb: int) -> W.Workload:
    return replace(wl, batch=nb, name=wl.name + "-first%d" % nb)


@pytest.mark.parametrize("name,nb,steps", [("c2", 1, 7), ("c3", 2, 6), ("c4", 2, 6), ("c6", 2, 5)])
def test_8b_shapes_teacher_forced(name, nb, steps):
    """1..4 dense warm-up steps then sparse steps at the real layer shape (first nb sequences)."""
    wl = _slice_batch(W.CONFIGS[name], nb)
    wl = replace(wl, t_full=2)
    _run_stream(wl, steps - 2, teacher_forced=True)


def test_c2_free_running():
    wl = replace(W.CONFIGS["c2"], t_full=2)
    _run_stream(wl, 5, teacher_forced=False)


@pytest.mark.parametrize("dtype,dh", [("f32", 64), ("bf16", 64), ("bf16", 128)])
def test_weights_between_poisoned_guard_bands(dtype, dh):
    """Every weight tensor sits between NaN-filled guard bands, so a read past either end of a
    matrix (e.g. a column tile that spans the stacked q/k/v weights) poisons the result."""
    _say("guard bands", dtype, dh)
    s = small_shape(dtype, gqa=True, dh=dh)
    cfg = oracle_cfg(s)
    B, L = 2, 100
    w = rand_weights(s, 97, bias=True)
    lay = Layer.from_shape(s, B, L)
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    held, wt = [], {}
    for name, a in w.items():
        if a is None:
            continue
        guard = 70000
        buf = torch.full((a.size + 2 * guard,), float("nan"), dtype=td, device="cuda")
        view = buf[guard:guard + a.size].view(*a.shape)
        val = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(td)
        # the guarded buffer must hold what the kernels read: for bf16 the re-laid matrix
        view.copy_(lay.pack(val) if dtype == "bf16" and a.ndim == 2 else val)
        held.append(buf)
        wt[name] = view
    lay.set_device_weights(wt, packed=True)
    x0 = W.philox(98, "x").standard_normal((B, L, s.hidden), dtype=np.float32)
    x1 = W.philox(99, "x").standard_normal((B, L, s.hidden), dtype=np.float32)
    if dtype == "bf16":
        x0, x1 = W.round_bf16(x0), W.round_bf16(x1)
    ref = O.new_caches(B, L, cfg)
    O.full_step(x0, w, cfg, ref)
    lay.full_step(lay.upload(x0))
    _compare_caches(lay, ref, TOL[dtype], "guarded dense")
    for counts in ([9, 30], [70, 64]):  # one-tile and several-tile row counts
        idx, off = rand_rows(100 + counts[0], B, L, counts)
        idx_ref, _, cos_ref = O.layer_step(x1, idx, w, cfg, ref, 0.99)
        out = lay.layer_step(lay.upload(x1), lay.make_list(idx, off), 0.99)
        assert_index_sets_match(lay.read_list(out)[0], idx_ref, idx, cos_ref, 0.99, "guarded sparse")
        _compare_caches(lay, ref, TOL[dtype], "guarded sparse")
    lay.close()


@pytest.mark.parametrize("name,frac,seqs", [("c3", 0.10, (5, 15)), ("c4", 0.10, (0, 9)),
                                            ("c3", 0.05, (7,)), ("c3", 0.25, (2,))])
def test_full_batch_at_bench_size_on_sampled_sequences(name, frac, seqs):
    """The launch configurations bench.py times (all 16 sequences; about 1000, 2000 and 5000 salient
    rows at the three salient fractions of the sweep, which take different GEMM tile plans and
    attention splits) checked on sampled sequences: sequences are independent, so the oracle runs
    the same two steps on each sampled one alone."""
    wl = replace(W.with_frac(W.CONFIGS[name], frac), t_full=1)
    s = wl.shape
    cfg = oracle_cfg(s)
    w = W.make_weights(s)
    lay = Layer.from_shape(s, wl.batch, wl.seq)
    lay.set_weights(w)
    steps = list(W.step_stream(wl, 2))
    _say(wl.name, "full batch: dense step, then sparse step with M=%d" % steps[1].idx.size)
    lay.full_step(lay.upload(steps[0].x))
    st = steps[1]
    out = lay.layer_step(lay.upload(st.x), lay.make_list(st.idx, st.offsets), wl.tau)
    idx_g, off_g = lay.read_list(out)
    cos_g = lay.cos[:st.idx.size].cpu().numpy()
    got = lay.get_caches()
    assert lay.ctx.poll_status() == 0
    L = wl.seq
    for b in seqs:
        _say(wl.name, "oracle for sequence", b)
        ref = O.new_caches(1, L, cfg)
        O.full_step(steps[0].x[b:b + 1], w, cfg, ref)
        lo, hi = int(st.offsets[b]), int(st.offsets[b + 1])
        rows_b = st.idx[lo:hi] - b * L
        idx_ref, _, cos_ref = O.layer_step(st.x[b:b + 1], rows_b, w, cfg, ref, wl.tau)
        sel_g = idx_g[off_g[b]:off_g[b + 1]] - b * L
        assert_index_sets_match(sel_g, idx_ref, rows_b, cos_ref, wl.tau, "sequence %d" % b)
        assert np.max(np.abs(cos_g[lo:hi] - cos_ref)) < 2e-2
        for cname in ("k", "v", "c", "out"):
            assert_close(got[cname][b], ref[cname][0], TOL["bf16"], "%s sequence %d cache %s" % (wl.name, b, cname))
    lay.close()


@pytest.mark.parametrize("dh,hkv", [(64, 8), (128, 4)])
def test_wide_batch_with_bias_in_the_large_tile_regime(dh, hkv):
    """8192 rows x 1536 q|k|v columns with q/k/v bias: the 256x256-tile plan of the large regime with
    both head sizes.  Dense step against the oracle, then the sparse step over all rows (index list
    instead of the identity) against the dense step."""
    _say("wide batch with bias", dh, hkv)
    nh = 512 // dh
    s = W.LayerShape(hidden=512, n_heads=nh, n_kv_heads=hkv, head_dim=dh, ffn=384, dtype="bf16")
    cfg = oracle_cfg(s)
    B, L = 16, 512
    T = B * L
    w = rand_weights(s, 131, bias=True, std=0.08)
    lay = Layer.from_shape(s, B, L)
    lay.set_weights(w)
    x0 = W.round_bf16(W.philox(132, "x").standard_normal((B, L, s.hidden), dtype=np.float32))
    x1 = W.round_bf16(W.philox(133, "x").standard_normal((B, L, s.hidden), dtype=np.float32))
    ref = O.new_caches(B, L, cfg)
    O.full_step(x0, w, cfg, ref)
    lay.full_step(lay.upload(x0))
    _compare_caches(lay, ref, TOL["bf16"], "wide dense")
    allrows = lay.make_list(np.arange(T, dtype=np.int32), np.arange(B + 1, dtype=np.int32) * L)
    out = lay.layer_step(lay.upload(x1), allrows, 1.5)
    idx_g, _ = lay.read_list(out)
    assert np.array_equal(idx_g, np.arange(T))
    sparse = {k: getattr(lay, k).clone() for k in ("k", "v", "c", "out")}
    lay.full_step(lay.upload(x1))
    for k in sparse:
        assert torch.equal(getattr(lay, k), sparse[k]), k
    O.full_step(x1, w, cfg, ref)
    _compare_caches(lay, ref, TOL["bf16"], "wide dense, second input")
    lay.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_salient_ablation_variant(dtype):
    """Table 1's 'Salient' variant: every token is a candidate (exact attention and the cosine test
    over all rows), out-projection and FFN only for the tokens the test selects."""
    _say("salient ablation", dtype)
    s = small_shape(dtype, gqa=True)
    cfg = oracle_cfg(s)
    B, L = 2, 96
    T = B * L
    w = rand_weights(s, 151, std=0.08)
    lay = Layer.from_shape(s, B, L)
    lay.set_weights(w)
    x0 = W.philox(152, "x0").standard_normal((B, L, s.hidden), dtype=np.float32)
    x0 = W.round_bf16(x0) if dtype == "bf16" else x0
    ref = O.new_caches(B, L, cfg)
    O.full_step(x0, w, cfg, ref)
    start = {k: (W.round_bf16(v.astype(np.float32)) if dtype == "bf16" else v.astype(np.float32)) for k, v in ref.items()}
    lay.set_caches(start)
    ref = {k: v.astype(np.float64) for k, v in start.items()}
    # every row moves by its own amount, so that the cosines spread and the median threshold splits them
    sig = 10.0 ** W.philox(153, "sig").uniform(-3, 0, T)
    x1 = W.perturbed_rows(x0.reshape(T, -1), sig, 154)
    x1 = (W.round_bf16(x1) if dtype == "bf16" else x1).reshape(B, L, -1)
    allrows = np.arange(T, dtype=np.int32)
    probe = O.layer_step(x1, allrows, w, cfg, {k: v.copy() for k, v in ref.items()}, 0.5)[2]
    tau = float(np.median(probe))
    before_out = ref["out"].copy()
    idx_ref, off_ref, cos_ref = O.layer_step(x1, allrows, w, cfg, ref, tau)
    assert 0 < idx_ref.size < T
    out = lay.layer_step(lay.upload(x1), lay.make_list(allrows, np.arange(B + 1, dtype=np.int32) * L), tau)
    idx_g, off_g = lay.read_list(out)
    assert_index_sets_match(idx_g, idx_ref, allrows, cos_ref, tau, "ablation")
    got = lay.get_caches()
    for name in ("k", "v", "c"):
        assert_close(got[name], ref[name], TOL[dtype], "ablation %s" % name)
    both = np.intersect1d(idx_g, idx_ref)
    assert_close(got["out"].reshape(T, -1)[both], ref["out"].reshape(T, -1)[both], TOL[dtype], "ablation out rows")
    kept = np.setdiff1d(allrows, np.union1d(idx_g, idx_ref))
    assert kept.size > 0
    assert np.array_equal(got["out"].reshape(T, -1)[kept], before_out.reshape(T, -1)[kept])  # cached rows reused
    lay.close()
