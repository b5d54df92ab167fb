"""Parity of dyllm_stack_step / dyllm_stack_full_step (the layer loops of Alg. 3 and Alg. 2) against
the CPU oracle through the C ABI: small stacks in both storage types, the structural equivalences of
the loop, its argument checks, and a slice of the 32-layer configuration at the real layer shape."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import dyllm_oracle as O
from paper_2603_08026_amd import binding as Bd
from paper_2603_08026_amd.layer import Stack, to_device, to_host
from synth import workload as W
from tests.helpers import (BAND, TOL, assert_close, assert_index_sets_match, oracle_cfg, rand_rows,
                           rand_weights, rel_err, small_shape)

pytestmark = pytest.mark.gpu


def _say(*a):
    print("[case]", *a, flush=True)


def _round(a, dtype):
    a = a.astype(np.float32)
    return W.round_bf16(a) if dtype == "bf16" else a


def _drift(stk, refs):
    """Free-running figure (printed, never asserted): the largest relative error of any cache of any
    layer against an oracle that ran the whole stack on its own values."""
    worst = 0.0
    for lay, ref in zip(stk.layers, refs):
        got = lay.get_caches()
        worst = max([worst] + [rel_err(got[n], ref[n]) for n in ("k", "v", "c", "out")])
    return worst


def _slice(caches, b):
    return caches if b is None else {k: v[b:b + 1] for k, v in caches.items()}


def _dense_layers_isolated(stk, x, ws, cfg, tol, what, b=None):
    """FullStep, one layer at a time: layer l of the oracle runs on the output cache the GPU's layer
    l-1 wrote, so every layer is held to the one-layer bound.  [Alg. 2, loop over l]
    b: compare sequence b of the batch only (sequences are independent); x is then that sequence."""
    h = x
    B, L = h.shape[:2]
    for l, lay in enumerate(stk.layers):
        got = _slice(lay.get_caches(), b)
        ref = O.new_caches(B, L, cfg)
        O.full_step(h, ws[l], cfg, ref)
        for name in ("k", "v", "c", "out"):
            assert_close(got[name], ref[name], tol, "%s layer %d cache %s" % (what, l, name))
        h = got["out"]


def _sparse_layers_isolated(stk, x, idx0, ws, cfg, before, outs, il_cap, tau, tol, dtype, what, b=None):
    """SparseStep, one layer at a time.  [Alg. 3, loop over l]

    Layer l of the oracle starts from the cache state the GPU's layer l had before the call, reads the
    output cache the GPU's layer l-1 holds after it and the candidate list the GPU's layer l-1
    selected -- exactly the inputs the GPU's layer l read -- and is then compared with the GPU's layer l
    alone at the one-layer bound.  A candidate whose cosine lies inside the tolerance band may fall
    either way; such a token's output row is then left out of the comparison (and counted), every
    other row of every cache is compared.  Returns the number of tokens left out.
    b: follow sequence b of the batch only; x, idx0 and before are then that sequence's (ids from 0)."""
    L = x.shape[1]
    T = x.shape[0] * L
    h, cand, left_out = x, np.asarray(idx0), 0
    lo = 0  # where this layer's candidates start in the GPU's list (and in its cosine row)
    if b is not None:
        lo = None
    for l, lay in enumerate(stk.layers):
        idx_g, off_g = lay.read_list(outs[l])
        assert off_g[-1] == idx_g.size and np.all(np.diff(off_g) >= 0)
        if b is not None:
            idx_g = idx_g[off_g[b]:off_g[b + 1]] - b * L
        ref = {k: v.copy() for k, v in before[l].items()}
        idx_ref, off_ref, cos_ref = O.layer_step(h, cand, ws[l], cfg, ref, tau)
        assert_index_sets_match(idx_g, idx_ref, cand, cos_ref, tau, "%s layer %d" % (what, l))
        if lo is not None:
            cos_g = stk.cos.view(-1)[l * il_cap + lo: l * il_cap + lo + cand.size].cpu().numpy()
            assert np.max(np.abs(cos_g - cos_ref), initial=0.0) < (5e-5 if dtype == "f32" else 2e-2), (what, l)
        got = _slice(lay.get_caches(), b)
        for name in ("k", "v", "c"):
            assert_close(got[name], ref[name], tol, "%s layer %d cache %s" % (what, l, name))
        swapped = np.setxor1d(idx_g, idx_ref)  # inside the band, by the set check above
        left_out += swapped.size
        keep = np.setdiff1d(np.arange(T), swapped)
        assert_close(got["out"].reshape(T, -1)[keep], ref["out"].reshape(T, -1)[keep], tol,
                     "%s layer %d cache out" % (what, l))
        # rows outside this layer's candidates keep every cache byte
        others = np.setdiff1d(np.arange(T), cand)
        for name in got:
            assert np.array_equal(got[name].reshape(T, -1)[others], before[l][name].reshape(T, -1)[others]), (l, name)
        h, cand = got["out"], idx_g
    return left_out


def _run_stack(wl: W.Workload, ws, n_steps: int, teacher_forced: bool, drift: bool = True):
    """Every step of the stream through the GPU stack; every layer of every step is compared with the
    oracle at the one-layer tolerance with its input isolated (see the two helpers above).  With
    drift=True a second oracle runs the whole stream on its own values and the compounded error of
    the GPU against it is printed as a figure."""
    s = wl.shape
    cfg = oracle_cfg(s)
    tol = TOL[s.dtype]
    n_layers = len(ws)
    stk = Stack(s, n_layers, wl.batch, wl.seq)
    for lay, w in zip(stk.layers, ws):
        lay.set_weights(w)
    refs = [O.new_caches(wl.batch, wl.seq, cfg) for _ in ws]
    compared = 0
    for st in W.step_stream(wl, n_steps):
        _say(wl.name, "%d layers" % n_layers, "step", st.t,
             "dense" if st.dense else "sparse M=%d" % st.idx.size,
             "teacher-forced" if teacher_forced else "free-running")
        xd = stk.upload(st.x)
        x_seen = to_host(xd)
        if st.dense:
            stk.full_step(xd)
            _dense_layers_isolated(stk, x_seen, ws, cfg, tol, "dense step %d" % st.t)
            if drift or teacher_forced:
                O.stack_full_step(st.x, ws, cfg, refs)
        else:
            if teacher_forced:
                for lay, l in zip(stk.layers, range(n_layers)):
                    lay.set_caches({k: _round(v, s.dtype) for k, v in refs[l].items()})
            before = [lay.get_caches() for lay in stk.layers]
            il = stk.make_list(st.idx, st.offsets)
            outs = stk.stack_step(xd, il, wl.tau)
            left = _sparse_layers_isolated(stk, x_seen, st.idx, ws, cfg, before, outs, il.cap, wl.tau, tol,
                                           s.dtype, "sparse step %d" % st.t)
            if left:
                _say("step", st.t, ": %d output rows of in-band tokens left out of the comparison" % left)
            if drift or teacher_forced:
                O.stack_step(st.x, st.idx, ws, cfg, refs, wl.tau)
        compared += 1
        if drift:
            _say("step", st.t, "compounded error against the free-running oracle: %.3e" % _drift(stk, refs))
    assert compared == n_steps
    assert stk.ctx.poll_status() == 0
    stk.close()


def test_small_f32_stack_free_running():
    s = small_shape("f32", gqa=True)
    wl = W.Workload("stack-small-f32", s, 2, 64, 32, 8, 0.12, ragged=True, t_full=1, tau=0.99, n_layers=4)
    ws = [rand_weights(s, 60 + l, std=0.08) for l in range(4)]
    _run_stack(wl, ws, 5, teacher_forced=False)


def test_small_bf16_stack_free_running_and_teacher_forced():
    s = small_shape("bf16", gqa=True, dh=128)
    wl = W.Workload("stack-small-bf16", s, 3, 110, 40, 8, 0.1, ragged=True, t_full=2, tau=0.99, n_layers=3)
    ws = [rand_weights(s, 70 + l) for l in range(3)]
    _run_stack(wl, ws, 5, teacher_forced=False)
    _run_stack(wl, ws, 4, teacher_forced=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stack_structure(dtype):
    """The loop against its own single-layer calls, the dense equivalence, shrinking sets, and the
    empty set, all bit for bit on the GPU."""
    _say("stack structure", dtype)
    s = small_shape(dtype, gqa=True)
    B, L, NL = 2, 80, 3
    T = B * L
    ws = [rand_weights(s, 80 + l, bias=(l == 1), std=0.08) for l in range(NL)]
    stk = Stack(s, NL, B, L)
    for lay, w in zip(stk.layers, ws):
        lay.set_weights(w)
    x0 = _round(W.philox(81, "x").standard_normal((B, L, s.hidden), dtype=np.float32), dtype)
    stk.full_step(stk.upload(x0))
    names = ("k", "v", "c", "out")

    def snap():
        return [{k: getattr(lay, k).clone() for k in names} for lay in stk.layers]

    def restore(sn):
        for lay, d in zip(stk.layers, sn):
            for k in names:
                getattr(lay, k).copy_(d[k])

    base = snap()
    # (i) a dense stack equals dense single-layer calls chained by hand
    h = stk.upload(x0)
    for lay in stk.layers:
        for k in names:
            getattr(lay, k).zero_()
        lay.full_step(h)
        h = lay.out
    for got, want in zip(snap(), base):
        for k in names:
            assert torch.equal(got[k], want[k]), k
    # (ii) candidates with large and tiny moves: the stack equals single-layer calls chained by hand,
    #      and the set only shrinks on the way down
    idx, off = rand_rows(82, B, L, [17, 9])
    sig = np.where(np.arange(idx.size) % 3 == 0, 1.0, 1e-4)
    x1 = x0.copy().reshape(T, -1)
    x1[idx] = W.perturbed_rows(x1[idx], sig, 83)
    x1 = _round(x1, dtype).reshape(B, L, -1)
    xd = stk.upload(x1)
    il = stk.make_list(idx, off)
    tau = 0.9
    outs = stk.stack_step(xd, il, tau)
    got_sets = [stk.layers[l].read_list(o)[0] for l, o in enumerate(outs)]
    got = snap()
    restore(base)
    h, cur = xd, il
    hand_sets = []
    for lay in stk.layers:
        o = Bd.IndexList.empty(il.cap, B)
        lay.layer_step(h, cur, tau, idx_out=o)
        hand_sets.append(lay.read_list(o)[0])
        h, cur = lay.out, o
    for l in range(NL):
        assert np.array_equal(got_sets[l], hand_sets[l])
        for k in names:
            assert torch.equal(getattr(stk.layers[l], k), got[l][k]), (l, k)
    prev = idx
    for sset in got_sets:
        assert set(sset.tolist()) <= set(prev.tolist())
        prev = sset
    assert 0 < got_sets[0].size <= idx.size
    # (iii) all rows, tau > 1: the dense stack, every row selected in every layer
    restore(base)
    allrows = stk.make_list(np.arange(T, dtype=np.int32), np.arange(B + 1, dtype=np.int32) * L)
    outs = stk.stack_step(xd, allrows, 1.5)
    for l, o in enumerate(outs):
        assert np.array_equal(stk.layers[l].read_list(o)[0], np.arange(T))
    sparse = snap()
    stk.full_step(xd)
    for a, b in zip(snap(), sparse):
        for k in names:
            assert torch.equal(a[k], b[k]), k
    # (iv) empty candidate set: nothing changes anywhere, every list empty
    now = snap()
    empty = stk.make_list(np.zeros(0, np.int32), np.zeros(B + 1, np.int32), cap=4)
    outs = stk.stack_step(stk.upload(x0), empty, 0.99)
    for l, o in enumerate(outs):
        assert stk.layers[l].read_list(o)[0].size == 0
    for a, b in zip(snap(), now):
        for k in names:
            assert torch.equal(a[k], b[k]), k
    # (v) two alternating output lists serve any depth
    restore(base)
    ping = [Bd.IndexList.empty(il.cap, B), Bd.IndexList.empty(il.cap, B)]
    stk.ctx.stack_step([l.w for l in stk.layers], [l.cache for l in stk.layers], xd, il, B, L, tau,
                       [ping[l % 2] for l in range(NL)])
    assert np.array_equal(stk.layers[0].read_list(ping[(NL - 1) % 2])[0], got_sets[-1])
    for l in range(NL):
        for k in names:
            assert torch.equal(getattr(stk.layers[l], k), got[l][k]), (l, k)
    assert stk.ctx.poll_status() == 0
    stk.close()


def test_stack_argument_checks():
    s = small_shape("f32")
    B, L = 1, 32
    stk = Stack(s, 2, B, L)
    for lay, l in zip(stk.layers, range(2)):
        lay.set_weights(rand_weights(s, 90 + l))
    x = stk.upload(np.zeros((B, L, s.hidden), np.float32))
    il = stk.make_list(np.array([1, 5], np.int32), np.array([0, 2], np.int32))
    ws, cs = [l.w for l in stk.layers], [l.cache for l in stk.layers]
    one = Bd.IndexList.empty(4, B)
    with pytest.raises(Bd.DyllmError) as e:  # consecutive layers sharing one output list
        stk.ctx.stack_step(ws, cs, x, il, B, L, 0.99, [one, one])
    assert e.value.code == Bd.ERR_INVALID_ARG
    with pytest.raises(Bd.DyllmError) as e:  # layer 1 reading and writing the same output cache
        stk.ctx.stack_step(ws, [cs[0], cs[0]], x, il, B, L, 0.99, stk.idx_outs)
    assert e.value.code == Bd.ERR_INVALID_ARG
    with pytest.raises(Bd.DyllmError) as e:
        stk.ctx.stack_full_step(ws, [cs[0], cs[0]], x, B, L)
    assert e.value.code == Bd.ERR_INVALID_ARG
    with pytest.raises(Bd.DyllmError) as e:  # input aliasing the first layer's output cache
        stk.ctx.stack_full_step(ws, cs, stk.layers[0].out, B, L)
    assert e.value.code == Bd.ERR_INVALID_ARG
    assert stk.ctx.lib.dyllm_stack_step(stk.ctx.h, 0, None, None, None, None, B, L, 0.99, None, None, None) \
        == Bd.ERR_INVALID_ARG
    # nothing was enqueued by the rejected calls: caches still zero
    torch.cuda.synchronize()
    assert float(stk.layers[0].out.abs().max()) == 0.0 and float(stk.layers[1].k.abs().max()) == 0.0
    stk.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", ["steady", "shrinking"])
def test_deep_stack_32_layers(dtype, case):
    """The depth of the 32-layer configuration at a small shape: the output cache and the selected
    list of layer l feed layer l+1 for 32 layers.  'steady': the selection of the first layer
    survives every deeper layer; 'shrinking': weaker weights, so the sets thin out with depth and the
    last layers run on empty lists.  Every layer is compared on its own inputs at the one-layer
    bound, the compounded error against a free-running oracle is printed, and the same call with two
    alternating output lists (all a caller needs at any depth) must give the same bytes."""
    _say("deep stack", dtype, case)
    s = W.LayerShape(hidden=256, n_heads=4, n_kv_heads=2, head_dim=64, ffn=384, dtype=dtype, rope_theta=10000.0)
    cfg = oracle_cfg(s)
    NL, B, L = 32, 2, 100
    T = B * L
    std, tau, lo = (0.08, 0.99, 1e-3) if case == "steady" else (0.04, 0.99, 1e-2)
    ws = [rand_weights(s, 300 + l, std=std) for l in range(NL)]
    stk = Stack(s, NL, B, L)
    for lay, w in zip(stk.layers, ws):
        lay.set_weights(w)
    x0 = _round(W.philox(301, "x").standard_normal((B, L, s.hidden), dtype=np.float32), dtype)
    xd0 = stk.upload(x0)
    stk.full_step(xd0)
    _dense_layers_isolated(stk, to_host(xd0), ws, cfg, TOL[dtype], "dense")
    refs = [O.new_caches(B, L, cfg) for _ in ws]
    O.stack_full_step(x0, ws, cfg, refs)
    _say("dense: compounded error against the free-running oracle after 32 layers: %.3e" % _drift(stk, refs))
    idx, off = rand_rows(302, B, L, [30, 22])
    sig = np.exp(np.linspace(np.log(lo), 0.0, idx.size))[W.philox(303, "perm").permutation(idx.size)]
    x1 = x0.copy().reshape(T, -1)
    x1[idx] = W.perturbed_rows(x1[idx], sig, 304)
    x1 = _round(x1, dtype).reshape(B, L, -1)
    names = ("k", "v", "c", "out")
    base = [{k: getattr(lay, k).clone() for k in names} for lay in stk.layers]
    before = [lay.get_caches() for lay in stk.layers]
    xd = stk.upload(x1)
    il = stk.make_list(idx, off)
    outs = stk.stack_step(xd, il, tau)
    left = _sparse_layers_isolated(stk, to_host(xd), idx, ws, cfg, before, outs, il.cap, tau, TOL[dtype], dtype,
                                   "sparse")
    sizes = [stk.layers[0].read_list(o)[0].size for o in outs]
    per = O.stack_step(x1, idx, ws, cfg, refs, tau)
    _say("set sizes by layer:", sizes, "| oracle, free-running:", [p[0].size for p in per],
         "| in-band output rows left out:", left,
         "| compounded error after 32 layers: %.3e" % _drift(stk, refs))
    assert all(a >= b for a, b in zip(sizes, sizes[1:]))
    if case == "steady":
        assert sizes[-1] == sizes[0] > 0
    else:
        assert sizes[0] > sizes[NL // 4] > 0 and sizes[-1] == 0 and len(set(sizes)) >= 6
    # the same step with two alternating output lists
    got = [{k: getattr(lay, k).clone() for k in names} for lay in stk.layers]
    last = stk.layers[0].read_list(outs[-1])
    for lay, d in zip(stk.layers, base):
        for k in names:
            getattr(lay, k).copy_(d[k])
    ping = [Bd.IndexList.empty(il.cap, B), Bd.IndexList.empty(il.cap, B)]
    stk.ctx.stack_step([l.w for l in stk.layers], [l.cache for l in stk.layers], xd, il, B, L, tau,
                       [ping[l % 2] for l in range(NL)])
    again = stk.layers[0].read_list(ping[(NL - 1) % 2])
    assert np.array_equal(again[0], last[0]) and np.array_equal(again[1], last[1])
    for lay, d in zip(stk.layers, got):
        for k in names:
            assert torch.equal(getattr(lay, k), d[k]), k
    assert stk.ctx.poll_status() == 0
    stk.close()


def test_c5_slice_four_layers():
    """The 32-layer configuration's layer shape and sequence length: first two sequences, four
    layers, one dense and two sparse steps (the oracle needs minutes for more)."""
    wl = replace(W.CONFIGS["c5"], batch=2, t_full=1, n_layers=4, name="c5-first2-4layers")
    ws = [W.make_weights(wl.shape, layer=l) for l in range(4)]
    _run_stack(wl, ws, 3, teacher_forced=False, drift=False)


def test_c5_full_batch_three_layers_on_a_sampled_sequence():
    """All 16 sequences of the stack configuration (about 3300 salient rows per layer, the launch
    configuration bench.py times), three layers deep; the oracle follows one sampled sequence, one
    layer at a time on the inputs the GPU's layer read."""
    wl = replace(W.CONFIGS["c5"], t_full=1, n_layers=3)
    s = wl.shape
    cfg = oracle_cfg(s)
    ws = [W.make_weights(s, layer=l) for l in range(3)]
    stk = Stack(s, 3, wl.batch, wl.seq)
    for lay, w in zip(stk.layers, ws):
        lay.set_weights(w)
    steps = list(W.step_stream(wl, 2))
    st = steps[1]
    _say(wl.name, "full batch, 3 layers: dense step, then sparse step with M=%d" % st.idx.size)
    b, L = 11, wl.seq
    x0 = stk.upload(steps[0].x)
    stk.full_step(x0)
    _dense_layers_isolated(stk, to_host(x0[b:b + 1]), ws, cfg, TOL["bf16"], "dense step", b=b)
    before = [_slice(lay.get_caches(), b) for lay in stk.layers]
    il = stk.make_list(st.idx, st.offsets)
    x1 = stk.upload(st.x)
    outs = stk.stack_step(x1, il, wl.tau)
    assert stk.ctx.poll_status() == 0
    rows_b = st.idx[int(st.offsets[b]):int(st.offsets[b + 1])] - b * L
    left = _sparse_layers_isolated(stk, to_host(x1[b:b + 1]), rows_b, ws, cfg, before, outs, il.cap, wl.tau,
                                   TOL["bf16"], "bf16", "sparse step", b=b)
    _say("in-band output rows left out:", left)
    stk.close()
