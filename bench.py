#!/usr/bin/env python3
"""Benchmark of the sparse layer step on one MI355X.

A "step" is one dyllm_layer_step (the whole hot path: gather+norm, q/k/v GEMM, rotation and K/V
merge, partial attention, cosine saliency + commit, compaction, out-projection, FFN, scatter-back)
over one batch of synthetic input that is already resident in HBM; for the 32-layer configuration
(c5) a step is one dyllm_stack_step, i.e. 32 such layer steps chained through the output caches and
the salient sets.  Prints ONE JSON line.

The headline workload is c3 at a salient fraction of 10 % (LLaDA-8B-shaped layer, 16 sequences of
1280 tokens: the regime where the gathered GEMMs are bound by the matrix pipes); the same line
carries a "sweep" over the other 8B-shaped configurations (c2, c3 at 2 / 5 / 10 / 25 %, c4, c5).  The
dense step has three comparators: the library's own dyllm_full_step, a plain torch layer (library
GEMMs + SDPA, harness only), and a composite of the best parts on the box -- the vendor library's four
GEMMs per layer (which run at 1.5-1.6 PFLOP/s, faster than this library's) plus this library's own
dense step without its GEMM stages.  The speed-up is quoted against the fastest of the three.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c2|c3|c4|c5] [--frac 0.10] [--no-sweep]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
FP32_VALU_PEAK_TFLOPS = 157.3
RIDGE = MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)  # flop per byte


def stage_work(shape, B, L, M_in, M_out, esz):
    """Algorithmic flops and HBM bytes of each stage for one step (M_in candidates, M_out salient)."""
    d, dq, dkv, F = shape.hidden, shape.dq, shape.dkv, shape.ffn
    nq = dq + 2 * dkv
    w = {}
    w["gather_rmsnorm"] = (4.0 * M_in * d, M_in * d * esz * 2 + d * esz)
    w["gemm_qkv"] = (2.0 * M_in * d * nq, nq * d * esz + M_in * d * esz + M_in * nq * 4)
    w["rope_scatter"] = (6.0 * M_in * nq, M_in * nq * 4 + M_in * nq * esz)
    w["partial_attention"] = (4.0 * M_in * L * dq, 2 * B * L * dkv * esz + 2 * M_in * dq * esz)
    w["saliency_compact"] = (6.0 * M_in * dq, 3 * M_in * dq * esz + M_in + 4 * M_out)
    w["marker_overhead"] = (0.0, 0.0)  # two stream events with no work between them
    w["gemm_oproj"] = (2.0 * M_out * dq * d, d * dq * esz + M_out * dq * esz + M_out * d * (esz + 4))
    w["rmsnorm_ffn"] = (4.0 * M_out * d, M_out * d * (4 + esz))
    w["gemm_swiglu"] = (4.0 * M_out * d * F, 2 * F * d * esz + M_out * d * esz + M_out * F * esz)
    w["gemm_down"] = (2.0 * M_out * F * d, d * F * esz + M_out * F * esz + M_out * d * (4 + esz))
    return w


def standalone_kernels(s, torch, rows=32768, iters=20):
    """The bandwidth-bound kernels on their own, over `rows` token rows (the token count of the 32-layer
    configuration): all-rows temporal cosine + salient test (Sec. 3.1-3.2), compaction of all flags
    (the where(...) of Alg. 3).  Times from events on the launch stream; bytes = both context buffers
    read once (+ outputs) / one flag byte in and four index bytes out per selected token."""
    from paper_2603_08026_amd import binding as Bd
    td = torch.float32 if s.dtype == "f32" else torch.bfloat16
    esz = 4 if s.dtype == "f32" else 2
    B = 16
    L = rows // B
    T = B * L
    # a context of its own: these calls need the batch and sequence bounds, not the row workspace
    ctx = Bd.Context(Bd.LayerCfg(s.hidden, s.n_heads, s.n_kv_heads, s.head_dim, s.ffn, B, L, 128,
                                 Bd.F32 if s.dtype == "f32" else Bd.BF16, s.rms_eps, s.rope_theta))
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    old = torch.randn(T, s.dq, generator=g, device="cuda").to(td)
    new = old.clone()
    moved = torch.rand(T, generator=g, device="cuda") < 0.1  # a tenth of the contexts changed
    new[moved] = torch.randn(int(moved.sum()), s.dq, generator=g, device="cuda").to(td)
    cos = torch.empty(T, dtype=torch.float32, device="cuda")
    flag = torch.empty(T, dtype=torch.uint8, device="cuda")
    outl = Bd.IndexList.empty(T, B)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    ms_sal = timed(lambda: ctx.saliency(new, old, None, B, L, 0.99, cos, flag, False))
    ms_cmp = timed(lambda: ctx.compact(flag, None, B, L, outl))
    n_sel = int(outl.offsets[-1].item())
    by_sal = 2.0 * T * s.dq * esz + 5.0 * T
    by_cmp = 1.0 * T + 4.0 * n_sel + 4.0 * (B + 1)
    ctx.close()
    return {"rows": T, "selected": n_sel,
            "saliency_all_rows": {"ms": round(ms_sal, 5), "gbps": round(by_sal / ms_sal / 1e6, 1),
                                  "frac_of_hbm_peak": round(by_sal / ms_sal / 1e6 / HBM_PEAK_GBS, 3)},
            "compact_all_rows": {"ms": round(ms_cmp, 5), "gbps": round(by_cmp / ms_cmp / 1e6, 2)}}


def cpu_baseline(wl, budget_s=20.0):
    """Times the CPU oracle as it stands on a bounded sample of the same workload."""
    import numpy as np
    from dataclasses import replace
    from oracle import dyllm_oracle as O
    from synth import workload as W
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    nb = min(wl.batch, 2)
    sub = replace(wl, batch=nb, t_full=1)
    s = sub.shape
    cfg = O.LayerCfg(s.hidden, s.n_heads, s.n_kv_heads, s.head_dim, s.ffn, s.rms_eps, s.rope_theta)
    w = W.make_weights(s)
    caches = O.new_caches(nb, sub.seq, cfg)
    times = []
    t_begin = time.time()
    for st in W.step_stream(sub, 12):
        if st.dense:
            O.full_step(st.x, w, cfg, caches)
            continue
        t0 = time.time()
        O.layer_step(st.x, st.idx, w, cfg, caches, sub.tau)
        times.append(time.time() - t0)
        if time.time() - t_begin > budget_s and len(times) >= 2:
            break
    t = float(np.median(times))
    return {
        "value": nb * sub.seq / t, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
        "sample": "%d sparse layer steps of %s on the first %d of %d sequences after one dense warm-up step "
                  "(numpy float64 oracle, median %.3f s per step)" % (len(times), wl.name, nb, wl.batch, t),
    }


def vendor_gemms_ms(s, B, L, torch, iters=10, seed=6):
    """The four GEMMs of a dense layer of this shape (q|k|v, out-projection, gate|up, down) through
    torch.nn.functional.linear, i.e. the vendor library's kernels, back to back: the strongest GEMM
    comparator on the box.  Harness only.  Returns milliseconds per layer."""
    import torch.nn.functional as Fn
    td = torch.float32 if s.dtype == "f32" else torch.bfloat16
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    d, dq, dkv, F = s.hidden, s.dq, s.dkv, s.ffn
    T = B * L

    def mat(n, k):
        return (torch.randn(n, k, generator=g, device="cuda") * 0.02).to(td)

    wqkv, wo, wgu, wd = mat(dq + 2 * dkv, d), mat(d, dq), mat(2 * F, d), mat(d, F)
    x, c, a = mat(T, d), mat(T, dq), mat(T, F)

    def four():
        Fn.linear(x, wqkv); Fn.linear(c, wo); Fn.linear(x, wgu); Fn.linear(a, wd)

    with torch.no_grad():
        four(); four()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            four()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / iters * 1e3


GEMM_STAGES = ("gemm_qkv", "gemm_oproj", "gemm_swiglu", "gemm_down")


def composite_dense_ms(lay_ctx, run_dense, n_calls, vendor_ms, NL, torch):
    """A dense step made of the best parts on the box: the vendor library's four GEMMs per layer plus
    this library's own dense step WITHOUT its GEMM stages (attention, norms, rotary embedding, merges,
    measured with stage events on the launch stream).  Not a runnable step: a lower bound for a dense
    implementation, and the comparator the sparse step's speed-up is finally quoted against."""
    lay_ctx.profile_begin(n_calls * NL)
    for _ in range(n_calls):
        run_dense()
    torch.cuda.synchronize()
    st, _ = lay_ctx.profile_end()
    ev = st.get("marker_overhead", 0.0)
    rest = sum(max(ms - ev, 0.0) for n, ms in st.items() if n not in GEMM_STAGES and n != "marker_overhead")
    return (vendor_ms + rest) * NL, rest * NL


def torch_dense_layer_ms(s, B, L, torch, iters=3, seed=5):
    """A dense layer step of the same shape written with torch's library calls (F.linear, SDPA,
    elementwise ops): the comparator the library's own dense step is checked against.  It is
    harness code, outside the product path, and produces the same four outputs (K after rotation,
    V, attention context, layer output).  Returns milliseconds per layer step."""
    import torch.nn.functional as Fn
    td = torch.float32 if s.dtype == "f32" else torch.bfloat16
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    d, dq, dkv, F, H, Hkv, dh = s.hidden, s.dq, s.dkv, s.ffn, s.n_heads, s.n_kv_heads, s.head_dim

    def mat(n, k):
        return (torch.randn(n, k, generator=g, device="cuda") * 0.02).to(td)

    wqkv, wo, wgu, wd = mat(dq + 2 * dkv, d), mat(d, dq), mat(2 * F, d), mat(d, F)
    ga = torch.ones(d, dtype=td, device="cuda")
    gf = torch.ones(d, dtype=td, device="cuda")
    x = torch.randn(B, L, d, generator=g, device="cuda").to(td)
    half = dh // 2
    ang = torch.arange(L, device="cuda", dtype=torch.float32)[:, None] * \
        (s.rope_theta ** (-2.0 * torch.arange(half, device="cuda", dtype=torch.float32) / dh))[None, :]
    cs, sn = ang.cos().to(td)[None, :, None, :], ang.sin().to(td)[None, :, None, :]

    def rot(t):  # [B, L, heads, dh], half-split pairing
        a, b = t[..., :half], t[..., half:]
        return torch.cat([a * cs - b * sn, a * sn + b * cs], dim=-1)

    def layer():
        n = Fn.rms_norm(x, (d,), ga, s.rms_eps)
        qkv = Fn.linear(n, wqkv)
        q = rot(qkv[..., :dq].view(B, L, H, dh))
        k = rot(qkv[..., dq:dq + dkv].view(B, L, Hkv, dh))
        v = qkv[..., dq + dkv:].view(B, L, Hkv, dh)
        c = Fn.scaled_dot_product_attention(q.transpose(1, 2), k.transpose(1, 2), v.transpose(1, 2),
                                            enable_gqa=(H != Hkv)).transpose(1, 2).reshape(B, L, dq)
        h = x + Fn.linear(c, wo)
        f = Fn.rms_norm(h, (d,), gf, s.rms_eps)
        gu = Fn.linear(f, wgu)
        y = h + Fn.linear(Fn.silu(gu[..., :F]) * gu[..., F:], wd)
        return k, v, c, y

    with torch.no_grad():
        layer()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            layer()
        torch.cuda.synchronize()
    return (time.perf_counter() - t0) / iters * 1e3


def roofline_of(stage_ms, work, dtype):
    """The stage with the largest time against the roof that bounds it."""
    dom = max((n for n in stage_ms if n != "marker_overhead"), key=lambda n: stage_ms[n])
    fl, by = work[dom]
    ms = stage_ms[dom]
    is_gemm_or_attn = dom.startswith("gemm") or dom == "partial_attention"
    if dtype == "bf16" and is_gemm_or_attn and fl / by >= RIDGE:
        roof = {"bound": "mfma", "achieved": fl / (ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s"}
    elif dtype == "f32" and is_gemm_or_attn and fl / by >= FP32_VALU_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBS:
        roof = {"bound": "alu", "achieved": fl / (ms * 1e-3) / 1e12, "peak": FP32_VALU_PEAK_TFLOPS, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": by / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["kernel"] = dom
    roof["launch_ms"] = ms
    return roof


class Bench:
    """One workload on the device: layers (or the stack), its inputs, and the timed legs."""

    def __init__(self, wl, variant, torch, np, host_inputs, n_sparse):
        from paper_2603_08026_amd.layer import Layer, Stack
        from synth import workload as W
        self.wl, self.torch, self.np, self.variant = wl, torch, np, variant
        s = wl.shape
        self.NL = NL = wl.n_layers
        td = torch.float32 if s.dtype == "f32" else torch.bfloat16
        if NL == 1 and host_inputs:
            lay = Layer.from_shape(s, wl.batch, wl.seq)
            lay.set_weights(W.make_weights(s))
            self.layers = [lay]
        else:
            # weights drawn on the device (same distribution as the host generator: N(0, 0.02^2)
            # matrices, gains 1 + 0.1 N(0,1)); a stack's 14 GB would take minutes on the host
            lay = Stack(s, NL, wl.batch, wl.seq) if NL > 1 else Layer.from_shape(s, wl.batch, wl.seq)
            self.layers = lay.layers if NL > 1 else [lay]
            shapes = {"wq": (s.dq, s.hidden), "wk": (s.dkv, s.hidden), "wv": (s.dkv, s.hidden),
                      "wo": (s.hidden, s.dq), "w_gate": (s.ffn, s.hidden), "w_up": (s.ffn, s.hidden),
                      "w_down": (s.hidden, s.ffn)}
            for l, one in enumerate(self.layers):
                g = torch.Generator(device="cuda")
                g.manual_seed(W.SEED_W + l)
                wt = {n: (torch.randn(*sh, generator=g, device="cuda") * 0.02).to(td) for n, sh in shapes.items()}
                for n in ("g_attn", "g_ffn"):
                    wt[n] = (1 + 0.1 * torch.randn(s.hidden, generator=g, device="cuda")).to(td)
                one.set_device_weights(wt)
        self.lay, self.last = lay, self.layers[-1]
        if NL == 1:
            self.full = lay.full_step
            self.sparse = lambda xd, il: lay.layer_step(xd, il, wl.tau, want_cos=False)
        else:
            self.full = lay.full_step
            self.sparse = lambda xd, il: lay.stack_step(xd, il, wl.tau, want_cos=False)
        self.dense_x, self.steps = [], []
        all_idx = np.arange(wl.tokens, dtype=np.int32)
        all_off = np.arange(wl.batch + 1, dtype=np.int32) * wl.seq
        if host_inputs:
            # the seeded host generator the parity tests use
            for st in W.step_stream(wl, wl.t_full + n_sparse):
                xd = lay.upload(st.x)
                if st.dense:
                    self.dense_x.append(xd)
                elif variant == "salient-ablation":
                    self.steps.append((xd, lay.make_list(all_idx, all_off), wl.tokens))
                else:
                    self.steps.append((xd, lay.make_list(st.idx, st.offsets), int(st.idx.size)))
        else:
            # same candidate lists as the host generator (W.step_rows), hidden states drawn on the
            # device: N(0,1) start, candidates redrawn N(0,1) per step.  (A sparse step reads only
            # the candidates' rows of x, so the tiny drift of the other rows is left out here.)
            g = torch.Generator(device="cuda")
            g.manual_seed(W.SEED_X)
            x = torch.randn(wl.batch, wl.seq, s.hidden, generator=g, device="cuda").to(td)
            self.dense_x.append(x)
            for t in range(1, n_sparse + 1):
                idx, off = W.step_rows(wl, t)
                x = x.clone()
                sel = torch.from_numpy(idx.astype(np.int64)).cuda()
                x.view(wl.tokens, -1)[sel] = torch.randn(idx.size, s.hidden, generator=g, device="cuda").to(td)
                self.steps.append((x, lay.make_list(idx, off), int(idx.size)))

    def warm_caches(self):
        for xd in self.dense_x:  # dense warm-up steps (Sec. 3.2)
            self.full(xd)
        self.torch.cuda.synchronize()

    def run(self, range_):
        for i in range_:
            xd, il, _ = self.steps[i]
            self.sparse(xd, il)

    def snapshot(self):
        return [{k: getattr(one, k).clone() for k in ("k", "v", "c", "out")} for one in self.layers]

    def restore(self, snap):
        for one, sn in zip(self.layers, snap):
            for k_, v_ in sn.items():
                getattr(one, k_).copy_(v_)
        self.torch.cuda.synchronize()

    def time_sparse(self, Wu, K):
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.run(range(Wu, Wu + K))
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / K

    def time_stages(self, Wu, K):
        """The same K steps with one HIP event after every stage, recorded on the launch stream."""
        self.lay.ctx.profile_begin(K * self.NL)
        t0 = time.perf_counter()
        self.run(range(Wu, Wu + K))
        self.torch.cuda.synchronize()
        t = (time.perf_counter() - t0) / K
        stage_ms, calls = self.lay.ctx.profile_end()
        # every stage time runs from one stream event to the next; the cost of the event itself is
        # measured by the stage that has no kernel and taken off the others
        ev = stage_ms.get("marker_overhead", 0.0)
        stage_ms = {n: (max(ms - ev, 1e-6) if n != "marker_overhead" else ms) for n, ms in stage_ms.items()}
        return t, stage_ms, calls

    def time_dense(self, iters):
        torch = self.torch
        xd = self.dense_x[-1]
        self.full(xd)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            self.full(xd)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / iters

    def close(self):
        self.lay.close()


def sweep_entry(wl, torch, np, K, Wu, dense_iters):
    """One line of the sweep: sparse step, both dense steps, dominant stage and its roofline fraction."""
    s = wl.shape
    esz = 4 if s.dtype == "f32" else 2
    # One layer: the stage-timing pass repeats the timed steps from a snapshot of the caches.  A stack
    # (whose snapshot would be tens of GB) times its stages on the NEXT K steps instead: repeating
    # steps on caches that have already seen them would select fewer rows in the deeper layers.
    stack = wl.n_layers > 1
    b = Bench(wl, "sparse", torch, np, host_inputs=False, n_sparse=Wu + (2 * K if stack else K))
    b.warm_caches()
    b.run(range(Wu))
    snap = None if stack else b.snapshot()
    t_step = b.time_sparse(Wu, K)
    if snap is not None:
        b.restore(snap)
    s0 = Wu + K if stack else Wu
    _, stage_ms, _ = b.time_stages(s0, K)
    t_dense = b.time_dense(dense_iters)
    m_in = float(np.mean([m for _, _, m in b.steps[s0:s0 + K]]))
    t_comp = None
    try:
        vg = vendor_gemms_ms(s, wl.batch, wl.seq, torch, iters=(3 if stack else 6))
        comp_ms, _ = composite_dense_ms(b.lay.ctx, lambda: b.full(b.dense_x[-1]), 1, vg, wl.n_layers, torch)
        t_comp = comp_ms * 1e-3
    except Exception as e:
        sys.stderr.write("bench.py: composite dense comparator failed for %s: %r\n" % (wl.name, e))
    b.close()
    del b, snap
    torch.cuda.empty_cache()
    t_torch = torch_dense_layer_ms(s, wl.batch, wl.seq, torch, iters=dense_iters) * wl.n_layers * 1e-3
    roof = roofline_of(stage_ms, stage_work(s, wl.batch, wl.seq, m_in, m_in, esz), s.dtype)
    torch.cuda.empty_cache()
    return {"workload": wl.name, "frac": wl.frac, "layers": wl.n_layers, "salient_rows_mean": m_in,
            "ms_per_step": t_step * 1e3, "tokens_per_s": wl.tokens * wl.n_layers / t_step,
            "dense_ms": t_dense * 1e3, "dense_torch_ms": t_torch * 1e3,
            "dense_composite_ms": None if t_comp is None else t_comp * 1e3,
            "speedup": min(t for t in (t_dense, t_torch, t_comp) if t is not None) / t_step,
            "dominant": roof["kernel"], "bound": roof["bound"], "achieved": round(roof["achieved"], 1),
            "unit": roof["unit"], "frac_of_peak": round(roof["frac"], 4),
            "stage_ms": {n: round(ms, 5) for n, ms in stage_ms.items()}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 20; 6 for c5)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps (default 5; 2 for c5)")
    ap.add_argument("--config", default="c3", choices=["c1", "c2", "c3", "c4", "c5", "c6"])
    ap.add_argument("--layers", type=int, default=None, help="stack depth override for c5")
    ap.add_argument("--frac", type=float, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--dense-iters", type=int, default=3)
    ap.add_argument("--variant", default="sparse", choices=["sparse", "salient-ablation"],
                    help="salient-ablation: every token is a candidate (exact attention and the cosine test "
                         "over all rows), out-projection and FFN for the selected ones only (Table 1, 'Salient')")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the graph-replay, approximate-step and stand-alone-kernel legs (profiling runs)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the sweep over the other configurations")
    ap.add_argument("--device-inputs", action="store_true",
                    help="draw weights and hidden states on the device (as the sweep entries do) instead of "
                         "taking them from the seeded host generator")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on exactly one GPU (sequences are independent, so the path "
                         "would shard along the batch with no exchange); --gpus %d is not supported\n" % args.gpus)
        sys.exit(2)

    import numpy as np
    import torch
    from dataclasses import replace
    from paper_2603_08026_amd.layer import Layer
    from synth import workload as W

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible\n")
        sys.exit(2)
    torch.cuda.set_device(0)
    wl = W.CONFIGS[args.config]
    if args.frac is not None:
        wl = W.with_frac(wl, args.frac)
    if args.layers is not None:
        wl = replace(wl, n_layers=args.layers)
    s = wl.shape
    esz = 4 if s.dtype == "f32" else 2
    NL = wl.n_layers
    K = args.steps if args.steps is not None else (20 if NL == 1 else 6)
    Wu = args.warmup if args.warmup is not None else (5 if NL == 1 else 2)

    # traffic calibration dispatch: one plain device copy of a known size, larger than every cache
    # (512 MiB read + 512 MiB written), so that a counter run can scale FETCH_SIZE / WRITE_SIZE
    calib_src = torch.ones(512 << 20, dtype=torch.uint8, device="cuda")
    calib_dst = torch.empty_like(calib_src)
    calib_dst.copy_(calib_src)
    torch.cuda.synchronize()
    del calib_src, calib_dst

    host_inputs = (NL == 1) and not args.device_inputs
    bn = Bench(wl, args.variant, torch, np, host_inputs, Wu + K)
    lay, layers, last, steps, sparse, dense_x = bn.lay, bn.layers, bn.last, bn.steps, bn.sparse, bn.dense_x
    bn.warm_caches()
    bn.run(range(Wu))
    torch.cuda.synchronize()
    snap = bn.snapshot()
    t_step = bn.time_sparse(Wu, K)
    m_out_last = int(last.idx_out.offsets[-1].item())

    # the same K steps again, from the same cache state, with one HIP event after every stage
    bn.restore(snap)
    t_step_instr, stage_ms, calls = bn.time_stages(Wu, K)

    # The same K steps from HIP graphs (the step path only enqueues kernels, so a caller may capture
    # it).  Two legs, to separate the cost of the graph launch from that of feeding a graph:
    #  (a) one graph PER STEP, each captured on that step's own resident inputs and replayed in turn --
    #      the same work as the eager loop and nothing else in the timed region;
    #  (b) ONE graph on persistent input buffers, the step's candidate list and the candidates' input
    #      rows (all that a sparse step reads of x) copied into them before every replay, copies timed.
    graph_info = None
    try:
        if args.no_extras:
            raise RuntimeError("skipped (--no-extras)")
        side = torch.cuda.Stream()
        bn.restore(snap)
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            sparse(steps[Wu][0], steps[Wu][1])  # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graphs = []
        for i in range(Wu, Wu + K):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                sparse(steps[i][0], steps[i][1])
            graphs.append(g)
        torch.cuda.synchronize()
        bn.restore(snap)
        t0 = time.perf_counter()
        for g in graphs:
            g.replay()
        torch.cuda.synchronize()
        t_per_step_graphs = (time.perf_counter() - t0) / K
        rows_a = int(last.idx_out.offsets[-1].item())
        del graphs
        # (b)
        bn.restore(snap)
        T_, cap = wl.tokens, max(m for _, _, m in steps[Wu:Wu + K])
        feeds = []
        for i in range(Wu, Wu + K):
            xd_i, il_i, m_i = steps[i]
            sel = il_i.idx[:m_i].long()
            feeds.append((sel, xd_i.view(T_, -1)[sel].clone(), il_i.idx[:m_i], il_i.offsets))
        xg = steps[Wu][0].clone()
        ilg = lay.make_list(np.zeros(0, np.int32), np.zeros(wl.batch + 1, np.int32), cap=cap)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            sparse(xg, ilg)
        torch.cuda.synchronize()

        def feed(f):
            sel, rows_i, idx_i, off_i = f
            xg.view(T_, -1).index_copy_(0, sel, rows_i)
            ilg.idx[:idx_i.numel()].copy_(idx_i)
            ilg.offsets.copy_(off_i)

        t0 = time.perf_counter()
        for f in feeds:
            feed(f)
        torch.cuda.synchronize()
        t_feed_only = (time.perf_counter() - t0) / K
        bn.restore(snap)
        t0 = time.perf_counter()
        for f in feeds:
            feed(f)
            graph.replay()
        torch.cuda.synchronize()
        graph_info = {"ms_per_step": t_per_step_graphs * 1e3, "replays": K,
                      "what": "one captured graph per step, replayed in turn (no copies in the timed region)",
                      "salient_rows_out_last": rows_a,
                      "fed_graph_ms_per_step": (time.perf_counter() - t0) / K * 1e3,
                      "feed_copies_only_ms_per_step": t_feed_only * 1e3,
                      "fed_graph_salient_rows_out_last": int(last.idx_out.offsets[-1].item())}
        del graph, feeds, xg
    except Exception as e:  # reported, never hidden: the figure is an extra, not the metric
        graph_info = {"error": repr(e)}

    # single layer: the same K steps once more with the approximate update of all other tokens
    # (Sec. 3.3, Alg. 4) in place of leaving their contexts untouched
    approx = None
    if NL == 1 and not args.no_extras:
        def restore():
            for k_, v_ in snap[0].items():
                getattr(lay, k_).copy_(v_)
        restore()
        lay.layer_step_approx(steps[Wu][0], steps[Wu][1], wl.tau)
        restore()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(Wu, Wu + K):
            lay.layer_step_approx(steps[i][0], steps[i][1], wl.tau)
        torch.cuda.synchronize()
        t_approx = (time.perf_counter() - t0) / K
        approx = {"ms_per_step": t_approx * 1e3, "tokens_per_s": wl.tokens / t_approx,
                  "salient_rows_out_last": int(lay.idx_out.offsets[-1].item())}
        # the same with a threshold no cosine falls below: nothing is selected, the out-projection and
        # FFN see an empty list, what remains is q of all tokens, k/v of the candidates, both
        # attention passes and the cosine test over all tokens
        restore()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(Wu, Wu + K):
            lay.layer_step_approx(steps[i][0], steps[i][1], -2.0)
        torch.cuda.synchronize()
        approx["ms_per_step_nothing_selected"] = (time.perf_counter() - t0) / K * 1e3
        # ... and as a response-only step (Sec. 3.5): the step's tokens are the last resp_len positions
        # of every sequence, the candidates are cut down to them, keys and values span the sequence
        row_lo = wl.seq - wl.resp_len
        if 0 < row_lo < wl.seq:
            resp_lists = []
            for i in range(Wu, Wu + K):
                cut = lay.make_list(np.zeros(0, np.int32), np.zeros(wl.batch + 1, np.int32), cap=steps[i][2])
                lay.ctx.merge_lists(steps[i][1], None, wl.batch, wl.seq, row_lo, cut)
                resp_lists.append(cut)
            restore()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(Wu, Wu + K):
                lay.layer_step_approx(steps[i][0], resp_lists[i - Wu], -2.0, row_lo=row_lo)
            torch.cuda.synchronize()
            approx["ms_per_step_response_only_nothing_selected"] = (time.perf_counter() - t0) / K * 1e3
            approx["response_rows"] = wl.batch * wl.resp_len
        # the variant with reused softmax normalisers (only the candidates' keys are scored): a second
        # layer object with the fifth cache, same weights, warmed by the same dense steps
        lay2 = Layer.from_shape(s, wl.batch, wl.seq, keep_lse=True)
        lay2.set_device_weights(lay.wt, packed=True)
        for xd_ in dense_x:
            lay2.full_step(xd_)
        lay2.layer_step_approx(steps[Wu][0], steps[Wu][1], -2.0, cached_norm=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(Wu, Wu + K):
            lay2.layer_step_approx(steps[i][0], steps[i][1], -2.0, cached_norm=True)
        torch.cuda.synchronize()
        approx["ms_per_step_reused_normalisers_nothing_selected"] = (time.perf_counter() - t0) / K * 1e3
        if 0 < row_lo < wl.seq:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(Wu, Wu + K):
                lay2.layer_step_approx(steps[i][0], resp_lists[i - Wu], -2.0, row_lo=row_lo, cached_norm=True)
            torch.cuda.synchronize()
            approx["ms_per_step_reused_normalisers_response_only_nothing_selected"] = (time.perf_counter() - t0) / K * 1e3
        lay2.close()
        del lay2
    del snap

    # dense step of the same shape on the same GPU: the library's own, and the torch comparator
    t_dense = bn.time_dense(args.dense_iters)
    try:
        t_dense_torch = torch_dense_layer_ms(s, wl.batch, wl.seq, torch, iters=args.dense_iters) * NL * 1e-3
        torch.cuda.empty_cache()
    except Exception as e:
        sys.stderr.write("bench.py: torch dense comparator failed: %r\n" % (e,))
        t_dense_torch = None
    # third comparator: the vendor library's GEMMs + this library's non-GEMM dense stages
    t_dense_comp = t_vendor_gemms = None
    try:
        t_vendor_gemms = vendor_gemms_ms(s, wl.batch, wl.seq, torch) * 1e-3
        torch.cuda.empty_cache()
        comp_ms, _ = composite_dense_ms(lay.ctx, lambda: bn.full(bn.dense_x[-1]), 2, t_vendor_gemms * 1e3, NL, torch)
        t_dense_comp = comp_ms * 1e-3
    except Exception as e:
        sys.stderr.write("bench.py: composite dense comparator failed: %r\n" % (e,))
    t_dense_best = min(t for t in (t_dense, t_dense_torch, t_dense_comp) if t is not None)

    m_in = float(np.mean([m for _, _, m in steps[Wu:Wu + K]]))
    # (sparse variant: every candidate passes the test on this workload; ablation: the last step's count)
    work = stage_work(s, wl.batch, wl.seq, m_in, m_in if args.variant == "sparse" else float(m_out_last), esz)
    stages = {}
    for name, ms in stage_ms.items():
        fl, by = work[name]
        stages[name] = {"ms": round(ms, 5), "gbps": round(by / (ms * 1e-3) / 1e9, 1) if by else None,
                        "tflops": round(fl / (ms * 1e-3) / 1e12, 2) if fl else None}
    roof = roofline_of(stage_ms, work, s.dtype)
    dom = roof["kernel"]
    # HBM bytes of the dominant stage's kernels: from a separate counter run of this command (two
    # rocprofv3 --pmc passes), kept as a file; it is NOT measured in this run
    roof["traffic"] = None
    tag = args.config + ("" if args.frac is None else "_%g" % args.frac)
    tr = os.path.join(ROOT, "profiles", "traffic_%s.json" % tag)
    if os.path.exists(tr):
        try:
            roof["traffic"] = json.load(open(tr)).get(dom)
            roof["traffic_source"] = "static: profiles/traffic_%s.json (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE " \
                                     "runs of this command, not measured in this run)" % tag
        except Exception:
            roof["traffic"] = None

    out = {
        "metric": "denoised tokens/s per layer-step at 8B shape; speedup vs dense step",
        # tokens advanced through one layer per second: a stack step advances every token through NL layers
        "value": wl.tokens * NL / t_step, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wu,
        "ms_per_step": t_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": s.dtype, "data": "synthetic",
        "config": {"workload": wl.name + ("" if args.variant == "sparse" else "+" + args.variant), "batch": wl.batch, "seq_len": wl.seq, "salient_frac": wl.frac,
                   "salient_rows_mean": m_in, "salient_rows_out_last": m_out_last, "tau": wl.tau,
                   "hidden": s.hidden, "n_heads": s.n_heads, "n_kv_heads": s.n_kv_heads, "ffn": s.ffn,
                   "layers": NL},
        "dense_ms_per_step": t_dense * 1e3,
        "dense_torch_ms_per_step": None if t_dense_torch is None else t_dense_torch * 1e3,
        "dense_composite_ms_per_step": None if t_dense_comp is None else t_dense_comp * 1e3,
        "dense_vendor_gemms_ms_per_layer": None if t_vendor_gemms is None else t_vendor_gemms * 1e3,
        # against the fastest of the three dense comparators (own step, torch layer, vendor GEMMs + own rest)
        "speedup_vs_dense": t_dense_best / t_step,
        "speedup_vs_composite_dense": None if t_dense_comp is None else t_dense_comp / t_step,
        "speedup_vs_own_dense": t_dense / t_step,
        "speedup_vs_torch_dense": None if t_dense_torch is None else t_dense_torch / t_step,
        "salient_rows_per_s": m_in / t_step,
        "ms_per_step_with_stage_events": t_step_instr * 1e3, "stage_calls": calls, "stages": stages,
        "roofline": roof,
    }
    out["graph_replay"] = graph_info
    if approx is not None:
        approx["speedup_vs_dense"] = t_dense_best * 1e3 / approx["ms_per_step"]
        out["approx_step"] = approx
    if NL > 1:
        # stack only: generated tokens per second of the paper's kind over the layer stack alone
        # (no embedding, logits or sampling): B * L_R over T_full dense and the remaining sparse steps
        total = wl.t_full * t_dense + (wl.steps - wl.t_full) * t_step
        out["ms_per_layer_step"] = t_step * 1e3 / NL
        out["stack_generated_tokens_per_s"] = wl.batch * wl.resp_len / total
        out["stack_generated_tokens_per_s_dense_only"] = wl.batch * wl.resp_len / (wl.steps * t_dense)
        out["data"] = "synthetic (weights drawn on the device)"
    elif not host_inputs:
        out["data"] = "synthetic (weights and hidden states drawn on the device)"
    bn.close()
    del bn, lay, layers, last, steps, sparse, dense_x
    torch.cuda.empty_cache()
    if not args.no_extras:
        out["standalone"] = standalone_kernels(s, torch)
        torch.cuda.empty_cache()
    if not args.no_sweep:
        # the other 8B-shaped configurations, with fewer steps each; inputs drawn on the device
        sweep = []
        # (c3 at 2 %: the share of salient tokens the paper's own runs average, 1.3 .. 8.4 % per layer
        # [App. D.2, Table 4: average salient tokens per layer])
        for name, frac in (("c2", None), ("c3", 0.02), ("c3", 0.05), ("c3", 0.10), ("c3", 0.25), ("c4", None),
                           ("c5", None)):
            w2 = W.CONFIGS[name] if frac is None else W.with_frac(W.CONFIGS[name], frac)
            deep = w2.n_layers > 1
            try:
                sweep.append(sweep_entry(w2, torch, np, K=(min(K, 4) if deep else min(K, 10)),
                                         Wu=(1 if deep else 2), dense_iters=(1 if deep else 2)))
            except Exception as e:
                sweep.append({"workload": w2.name, "frac": w2.frac, "error": repr(e)})
            torch.cuda.empty_cache()
        out["sweep"] = sweep
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
