"""The step schedule on the GPU against the CPU oracle, through the C ABI: list merge, response-only
steps of the approximate path, the approximate path through a stack, and a run of the generation
loop's steps (dense warm-up, whole-sequence and response-only sparse steps, carried salient set)."""
import numpy as np
import pytest
import torch

from oracle import dyllm_oracle as O
from paper_2603_08026_amd import binding as Bd
from paper_2603_08026_amd.layer import Layer, Stack, to_host
from synth import workload as W
from tests.helpers import BAND, TOL, assert_close, assert_index_sets_match, oracle_cfg, rand_rows, rand_weights, small_shape

pytestmark = pytest.mark.gpu


def _say(*a):
    print("[case]", *a, flush=True)


def _round(v, dtype):
    v = np.asarray(v, dtype=np.float32)
    return W.round_bf16(v) if dtype == "bf16" else v


def _offsets(idx, B, L):
    return np.searchsorted(idx, np.arange(B + 1) * L).astype(np.int32)


def test_merge_lists_against_oracle():
    _say("merge lists")
    s = small_shape("f32")
    B, L = 3, 70
    lay = Layer.from_shape(s, B, L)
    out = Bd.IndexList.empty(B * L, B)
    g = W.philox(81, "merge")
    for case in range(8):
        na, nb = int(g.integers(0, 60)), int(g.integers(0, 60))
        a = np.sort(g.choice(B * L, size=na, replace=False)).astype(np.int32)
        b = np.sort(g.choice(B * L, size=nb, replace=False)).astype(np.int32)
        lo = int(g.integers(0, L)) if case % 2 else 0
        la, lb = lay.make_list(a, _offsets(a, B, L), cap=na + 3), lay.make_list(b, _offsets(b, B, L))
        for pa, pb, ra, rb in ((la, lb, a, b), (None, lb, None, b), (la, None, a, None)):
            lay.ctx.merge_lists(pa, pb, B, L, lo, out)
            idx_g, off_g = lay.read_list(out)
            want = O.merge_lists(ra, rb, L, lo)
            assert np.array_equal(idx_g, want), (case, lo)
            assert np.array_equal(off_g, _offsets(want, B, L))
    assert lay.ctx.poll_status() == 0
    # overflow of the output list is reported, arguments are checked
    a = np.arange(40, dtype=np.int32)
    short = Bd.IndexList.empty(8, B)
    lay.ctx.merge_lists(lay.make_list(a, _offsets(a, B, L)), None, B, L, 0, short)
    torch.cuda.synchronize()
    assert lay.ctx.poll_status() == Bd.ERR_CAPACITY
    with pytest.raises(Bd.DyllmError):
        lay.ctx.merge_lists(out, None, B, L, 0, out)
    with pytest.raises(Bd.DyllmError):
        lay.ctx.merge_lists(None, None, B, L, L, out)
    lay.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_response_only_step_against_oracle(dtype):
    _say("approx response-only", dtype)
    s = small_shape(dtype, gqa=True, dh=128 if dtype == "bf16" else 64)
    cfg = oracle_cfg(s)
    B, L, lo = 2, 200, 72
    T = B * L
    w = rand_weights(s, 91, std=0.08)
    lay = Layer.from_shape(s, B, L)
    lay.set_weights(w)
    x0 = _round(W.philox(92, "x0").standard_normal((B, L, s.hidden), dtype=np.float32), dtype)
    ref = O.new_caches(B, L, cfg)
    O.full_step(x0, w, cfg, ref)
    start = {k: _round(v, dtype) for k, v in ref.items()}
    lay.set_caches(start)
    ref = {k: v.astype(np.float64) for k, v in start.items()}
    # candidates inside the response; prompt inputs change as well and must not be read
    idx = np.concatenate([lo + np.sort(W.philox(93, "r", b).choice(L - lo, size=n, replace=False)) + b * L
                          for b, n in enumerate((30, 11))]).astype(np.int32)
    off = _offsets(idx, B, L)
    x1 = x0.copy().reshape(T, -1)
    x1[idx] = W.perturbed_rows(x1[idx], np.full(idx.size, 1.5), 94)
    x1[[3, L + 10]] += 4.0
    x1 = _round(x1, dtype).reshape(B, L, -1)
    probe = O.layer_step_approx(x1, idx, w, cfg, {k: v.copy() for k, v in ref.items()}, 0.5, row_lo=lo)[2]
    step_rows = np.flatnonzero(np.arange(T) % L >= lo)
    others = np.setdiff1d(step_rows, idx)
    tau = float(np.median(probe[others]))
    before = {k: v.copy() for k, v in start.items()}
    idx_ref, off_ref, cos_ref = O.layer_step_approx(x1, idx, w, cfg, ref, tau, row_lo=lo)
    assert np.setdiff1d(idx_ref, idx).size > 0
    full = Bd.IndexList.empty(T, B)
    cos = torch.ones(T, dtype=torch.float32, device="cuda")
    out = lay.layer_step_approx(lay.upload(x1), lay.make_list(idx, off), tau, full, cos, row_lo=lo)
    assert lay.ctx.poll_status() == 0
    idx_g, off_g = lay.read_list(out)
    cos_g = cos.cpu().numpy()
    assert np.max(np.abs(cos_g - cos_ref)) < (5e-5 if dtype == "f32" else 2e-2)
    assert_index_sets_match(idx_g, idx_ref, step_rows, cos_ref[step_rows], tau, "response-only")
    assert np.all(idx_g % L >= lo) and np.array_equal(off_g, _offsets(idx_g, B, L))
    got = lay.get_caches()
    prompt = np.flatnonzero(np.arange(T) % L < lo)
    for name in ("k", "v", "c", "out"):
        g_, r_ = got[name].reshape(T, -1), ref[name].reshape(T, -1)
        if name != "out":
            assert_close(g_, r_, TOL[dtype], "response-only: %s cache" % name)
        assert np.array_equal(g_[prompt], before[name].reshape(T, -1)[prompt]), name
    both = np.intersect1d(idx_g, idx_ref)
    assert_close(got["out"].reshape(T, -1)[both], ref["out"].reshape(T, -1)[both], TOL[dtype], "out rows")
    # a candidate below row_lo is the caller's error; the window itself is checked
    with pytest.raises(Bd.DyllmError):
        lay.layer_step_approx(lay.upload(x1), lay.make_list(idx, off), tau, full, None, row_lo=L)
    lay.close()


def _stack_refs(s, n_layers, B, L, seed, keep_lse=False):
    cfg = oracle_cfg(s)
    ws = [rand_weights(s, seed + l, std=0.08) for l in range(n_layers)]
    st = Stack(s, n_layers, B, L, keep_lse=keep_lse)
    for one, w in zip(st.layers, ws):
        one.set_weights(w)
    return cfg, ws, st


def _teacher_force(st, refs, dtype):
    out = []
    for one, ref in zip(st.layers, refs):
        start = {k: (_round(v, dtype) if k != "lse" else v.astype(np.float32)) for k, v in ref.items()}
        one.set_caches(start)
        out.append({k: v.astype(np.float64) for k, v in start.items()})
    return out


@pytest.mark.parametrize("dtype,approx", [("f32", 0), ("f32", 1), ("bf16", 0), ("bf16", 1), ("f32", 2), ("bf16", 2)])
def test_generation_loop_steps_against_oracle(dtype, approx):
    """Steps 0..8 with two dense steps, a period of four and two decoded tokens per sequence and step;
    every sparse step starts from the oracle's caches (rounded to the storage type)."""
    _say("denoise steps", dtype, ("exact", "approx", "approx with reused normalisers")[approx])
    s = small_shape(dtype, gqa=True)
    B, L, LP, NL = 2, 96, 40, 2
    T = B * L
    cached = approx == 2
    cfg, ws, st = _stack_refs(s, NL, B, L, 101, keep_lse=cached)
    tau = 0.9 if approx else 0.99
    sched_o = O.Schedule(t_full=2, full_period=4, prompt_len=LP, approx=bool(approx), tau=tau, cached_norm=cached)
    sched_g = Bd.Schedule(2, 4, LP, int(approx), tau)
    refs = [O.new_caches(B, L, cfg) for _ in range(NL)]
    if cached:
        for r_ in refs:
            r_["lse"] = np.zeros((B, L, cfg.n_heads))
    x = _round(W.philox(102, "x").standard_normal((B, L, s.hidden), dtype=np.float32), dtype)
    cand = Bd.IndexList.empty(T, B)
    carry_o, carry_g = None, None
    decoded = np.zeros(0, np.int32)
    kinds, compared, unfirm_steps = [], 0, 0
    for t in range(9):
        if t >= 2:
            refs = _teacher_force(st, refs, dtype)
        dl = st.make_list(decoded, _offsets(decoded, B, L)) if decoded.size else None
        if carry_o is not None:
            # both sides carry the oracle's set, so that one step is compared at a time
            carry_g = st.make_list(carry_o.astype(np.int32), _offsets(carry_o, B, L))
        # per-layer cosines of this step, from a copy, to know which tokens sit near the threshold
        firm = True
        kind_o = O.step_kind(t, sched_o)
        lo = 0 if kind_o != "response" else LP
        before = [{k: v.copy() for k, v in r.items()} for r in refs]
        if kind_o != "dense":
            cp = [{k: v.copy() for k, v in r.items()} for r in refs]
            c0 = O.merge_lists(carry_o, decoded, L, lo)
            per = (O.stack_step_approx(x, c0, ws, cfg, cp, tau, lo, cached) if approx else O.stack_step(x, c0, ws, cfg, cp, tau))
            firm = all(np.all(np.abs(np.asarray(c) - tau) > BAND) for _, _, c in per)
        new_carry = O.denoise_step(t, sched_o, x, decoded, carry_o, ws, cfg, refs)
        xd = st.upload(x)
        kind, out = st.denoise_step(sched_g, t, xd, dl, carry_g, cand)
        kinds.append(kind)
        assert st.ctx.poll_status() == 0
        if new_carry is None:
            assert kind == Bd.STEP_DENSE and out is None
        else:
            idx_g, off_g = st.layers[0].read_list(out)
            if firm:
                assert np.array_equal(idx_g, new_carry), "step %d" % t
                assert np.array_equal(off_g, _offsets(new_carry, B, L))
            else:
                unfirm_steps += 1
        # every layer against the oracle's layer on the inputs the GPU's layer read (the output cache
        # and the list of the GPU's layer above; the caches both sides held before the step), at the
        # one-layer tolerance
        h, cl = to_host(xd), (None if kind_o == "dense" else c0)
        step_rows = np.flatnonzero(np.arange(T) % L >= lo)
        for l, one in enumerate(st.layers):
            got = one.get_caches()
            what = "step %d layer %d" % (t, l)
            if kind_o == "dense":
                ref = O.new_caches(B, L, cfg)
                O.full_step(h, ws[l], cfg, ref)
                swapped = np.zeros(0, np.int64)
            else:
                ref = before[l]
                if approx:
                    idx_ref, _, cos_ref = O.layer_step_approx(h, cl, ws[l], cfg, ref, tau, lo, cached)
                    pool, cos_pool = step_rows, cos_ref[step_rows]
                else:
                    idx_ref, _, cos_ref = O.layer_step(h, cl, ws[l], cfg, ref, tau)
                    pool, cos_pool = cl, cos_ref
                idx_l, off_l = one.read_list(st.idx_outs[l])
                assert np.array_equal(off_l, _offsets(idx_l, B, L))
                assert_index_sets_match(idx_l, idx_ref, pool, cos_pool, tau, what)
                swapped = np.setxor1d(idx_l, idx_ref)  # inside the band: their output rows may differ
                cl = idx_l
            for name in ("k", "v", "c"):
                assert_close(got[name], ref[name], TOL[dtype], "%s %s" % (what, name))
            keep = np.setdiff1d(np.arange(T), swapped)
            assert_close(got["out"].reshape(T, -1)[keep], ref["out"].reshape(T, -1)[keep], TOL[dtype], what + " out")
            h = got["out"]
        compared += 1
        carry_o = new_carry
        # the next step's input: two freshly decoded response positions per sequence get a new row
        g = W.philox(103, "dec", t)
        decoded = np.sort(np.concatenate([b * L + LP + g.choice(L - LP, size=2, replace=False) for b in range(B)])).astype(np.int32)
        x = x.copy().reshape(T, -1)
        x[decoded] = g.standard_normal((decoded.size, s.hidden), dtype=np.float32)
        x = _round(x, dtype).reshape(B, L, -1)
    assert compared == 9 and unfirm_steps <= 4, (compared, unfirm_steps)
    assert kinds == [Bd.STEP_DENSE] * 2 + [Bd.STEP_RESPONSE] * 2 + [Bd.STEP_FULL] + [Bd.STEP_RESPONSE] * 3 + [Bd.STEP_FULL]
    st.close()


@pytest.mark.parametrize("approx", [False, True])
def test_stack_step_replays_from_a_captured_graph(approx):
    """The layer loop is one enqueue of kernels with no allocation, copy or wait in it, so a caller may
    capture it once and replay it with new inputs in the same buffers.  Every replay (with eager work
    and synchronisations in between) must give what the eager call gives on the same inputs."""
    _say("graph replay", "approx" if approx else "exact")
    dtype = "bf16"
    s = small_shape(dtype, gqa=True)
    B, L, NL, CAP = 2, 96, 3, 40
    T = B * L
    cfg, ws, st = _stack_refs(s, NL, B, L, 111)
    x0 = _round(W.philox(112, "x").standard_normal((B, L, s.hidden), dtype=np.float32), dtype)
    st.full_step(st.upload(x0))
    torch.cuda.synchronize()
    snap = [{k: getattr(one, k).clone() for k in ("k", "v", "c", "out")} for one in st.layers]

    def restore():
        for one, sn in zip(st.layers, snap):
            for k, v in sn.items():
                getattr(one, k).copy_(v)

    def run(xd, il):
        if approx:
            st.stack_step_approx(xd, il, 0.9)
        else:
            st.stack_step(xd, il, 0.99, want_cos=False)

    def state():
        torch.cuda.synchronize()
        lists = [tuple(a.copy() for a in st.layers[0].read_list(o)) for o in st.idx_outs]
        return [one.get_caches() for one in st.layers], lists

    # three inputs with different candidate counts, all within one list capacity
    cases = []
    for k, counts in enumerate(([20, 15], [3, 0], [11, 29])):
        idx, off = rand_rows(113 + k, B, L, counts)
        x = x0.copy().reshape(T, -1)
        x[idx] = W.perturbed_rows(x[idx], np.full(idx.size, 1.0), 120 + k)
        cases.append((_round(x, dtype).reshape(B, L, -1), idx, off))
    eager = []
    for x, idx, off in cases:
        restore()
        run(st.upload(x), st.make_list(idx, off, cap=CAP))
        eager.append(state())
    # persistent input buffers for the captured call
    xd = st.upload(cases[0][0]).clone()
    il = st.make_list(cases[0][1], cases[0][2], cap=CAP)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        restore()
        run(xd, il)  # warm-up on the capture stream (one-time function attributes are set here)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(xd, il)
    torch.cuda.synchronize()
    for rep in range(2):
        for k, (x, idx, off) in enumerate(cases):
            restore()
            xd.copy_(st.upload(x))
            buf = np.zeros(CAP, np.int32)
            buf[:idx.size] = idx
            il.idx.copy_(torch.from_numpy(buf).cuda())
            il.offsets.copy_(torch.from_numpy(off.astype(np.int32)).cuda())
            torch.cuda.synchronize()
            graph.replay()
            got_c, got_l = state()
            want_c, want_l = eager[k]
            for l in range(NL):
                assert np.array_equal(got_l[l][0], want_l[l][0]) and np.array_equal(got_l[l][1], want_l[l][1]), (rep, k, l)
                for name in ("k", "v", "c", "out"):
                    assert np.array_equal(got_c[l][name], want_c[l][name]), (rep, k, l, name)
    assert st.ctx.poll_status() == 0
    st.close()
