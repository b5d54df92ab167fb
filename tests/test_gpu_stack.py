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
                           rand_weights, small_shape)

pytestmark = pytest.mark.gpu


def _say(*a):
    print("[case]", *a, flush=True)


def _round(a, dtype):
    a = a.astype(np.float32)
    return W.round_bf16(a) if dtype == "bf16" else a


def _compare_layers(stk, refs, tol, what):
    """One call runs all layers, so layer l is compared after l layers of the GPU's own rounding went
    into its input: its bound is the one-layer bound times sqrt(l + 1) (independent errors of equal
    size add in quadrature)."""
    worst = 0.0
    for l, (lay, ref) in enumerate(zip(stk.layers, refs)):
        got = lay.get_caches()
        for name in ("k", "v", "c", "out"):
            worst = max(worst, assert_close(got[name], ref[name], tol * np.sqrt(l + 1.0),
                                            "%s layer %d cache %s" % (what, l, name)))
    return worst


def _run_stack(wl: W.Workload, ws, n_steps: int, teacher_forced: bool):
    s = wl.shape
    cfg = oracle_cfg(s)
    tol = TOL[s.dtype]
    n_layers = len(ws)
    stk = Stack(s, n_layers, wl.batch, wl.seq)
    for lay, w in zip(stk.layers, ws):
        lay.set_weights(w)
    refs = [O.new_caches(wl.batch, wl.seq, cfg) for _ in ws]
    for st in W.step_stream(wl, n_steps):
        _say(wl.name, "%d layers" % n_layers, "step", st.t,
             "dense" if st.dense else "sparse M=%d" % st.idx.size,
             "teacher-forced" if teacher_forced else "free-running")
        xd = stk.upload(st.x)
        if st.dense:
            O.stack_full_step(st.x, ws, cfg, refs)
            stk.full_step(xd)
            _compare_layers(stk, refs, tol, "dense step %d" % st.t)
            continue
        if teacher_forced:
            for lay, l in zip(stk.layers, range(n_layers)):
                start = {k: _round(v, s.dtype) for k, v in refs[l].items()}
                lay.set_caches(start)
                refs[l] = {k: v.astype(np.float64) for k, v in start.items()}
        before = [lay.get_caches() for lay in stk.layers]
        per_layer = O.stack_step(st.x, st.idx, ws, cfg, refs, wl.tau)
        il = stk.make_list(st.idx, st.offsets)
        outs = stk.stack_step(xd, il, wl.tau)
        cand, agree = st.idx, True
        for l, ((idx_ref, off_ref, cos_ref), out) in enumerate(zip(per_layer, outs)):
            idx_g, off_g = stk.layers[l].read_list(out)
            assert off_g[-1] == idx_g.size
            if not agree:
                break  # an in-band candidate fell the other way above: deeper candidate sets differ
            assert_index_sets_match(idx_g, idx_ref, cand, cos_ref, wl.tau, "step %d layer %d" % (st.t, l))
            cos_g = stk.cos.view(-1)[l * il.cap: l * il.cap + cand.size].cpu().numpy()
            assert np.max(np.abs(cos_g - cos_ref)) < (5e-5 if s.dtype == "f32" else 2e-2), (st.t, l)
            # rows outside this layer's candidates keep every cache byte
            after = stk.layers[l].get_caches()
            others = np.setdiff1d(np.arange(wl.tokens), cand)
            for name in after:
                assert np.array_equal(after[name].reshape(wl.tokens, -1)[others],
                                      before[l][name].reshape(wl.tokens, -1)[others]), (l, name)
            agree = np.array_equal(idx_g, idx_ref)
            cand = idx_ref
        if agree:
            _compare_layers(stk, refs, tol, "sparse step %d" % st.t)
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


def test_c5_slice_four_layers_teacher_forced():
    """The 32-layer configuration's layer shape and sequence length: first two sequences, four
    layers, one dense and two sparse steps (the oracle needs minutes for more)."""
    wl = replace(W.CONFIGS["c5"], batch=2, t_full=1, n_layers=4, name="c5-first2-4layers")
    ws = [W.make_weights(wl.shape, layer=l) for l in range(4)]
    _run_stack(wl, ws, 3, teacher_forced=True)


def test_c5_full_batch_three_layers_on_a_sampled_sequence():
    """All 16 sequences of the stack configuration (about 3300 salient rows per layer, the launch
    configuration bench.py times), three layers deep; the oracle follows one sampled sequence."""
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
    stk.full_step(stk.upload(steps[0].x))
    il = stk.make_list(st.idx, st.offsets)
    outs = stk.stack_step(stk.upload(st.x), il, wl.tau)
    assert stk.ctx.poll_status() == 0
    b, L = 11, wl.seq
    refs = [O.new_caches(1, L, cfg) for _ in ws]
    O.stack_full_step(steps[0].x[b:b + 1], ws, cfg, refs)
    rows_b = st.idx[int(st.offsets[b]):int(st.offsets[b + 1])] - b * L
    per_layer = O.stack_step(st.x[b:b + 1], rows_b, ws, cfg, refs, wl.tau)
    cand = rows_b
    for l, (idx_ref, _, cos_ref) in enumerate(per_layer):
        idx_g, off_g = stk.layers[l].read_list(outs[l])
        sel_g = idx_g[off_g[b]:off_g[b + 1]] - b * L
        assert_index_sets_match(sel_g, idx_ref, cand, cos_ref, wl.tau, "layer %d" % l)
        assert np.array_equal(sel_g, idx_ref), "a candidate inside the tolerance band: deeper layers not comparable"
        got = stk.layers[l].get_caches()
        for cname in ("k", "v", "c", "out"):
            assert_close(got[cname][b], refs[l][cname][0], TOL["bf16"], "layer %d cache %s" % (l, cname))
        cand = idx_ref
    stk.close()
