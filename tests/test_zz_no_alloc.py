"""dyllm_compact_static, the entry point that allocates nothing, against dyllm_compact through the C
ABI: same lists and offsets bit for bit, on consecutive calls that share the library's fixed device
words (the second call smaller than the first), with and without a row list, and its size limit."""
import numpy as np
import pytest
import torch

from paper_2603_08026_amd import binding as Bd
from synth import workload as W

pytestmark = pytest.mark.gpu


def _say(*a):
    print("[case]", *a, flush=True)


def _ctx(B, L):
    return Bd.Context(Bd.LayerCfg(256, 4, 4, 64, 384, B, L, 0, Bd.F32, 1e-5, 10000.0))


def _lists_equal(a: Bd.IndexList, b: Bd.IndexList):
    off_a, off_b = a.offsets.cpu().numpy(), b.offsets.cpu().numpy()
    assert np.array_equal(off_a, off_b)
    n = int(off_a[-1])
    assert np.array_equal(a.idx[:n].cpu().numpy(), b.idx[:n].cpu().numpy())
    return n


def test_compact_static_matches_compact_on_consecutive_calls():
    _say("compact_static: consecutive calls, second one smaller")
    g = W.philox(501, "flags")
    # (B, L, share of flagged tokens, with a row list): large first, then smaller, then ragged sizes
    cases = [(16, 2048, 0.1, False), (3, 700, 0.5, False), (16, 2048, 0.02, True), (2, 100, 0.3, True),
             (1, 1, 1.0, False), (5, 333, 0.0, False), (4, 4096, 1.0, False)]
    for B, L, share, with_rows in cases:
        T = B * L
        ctx = _ctx(B, L)
        if with_rows:
            m = max(1, T // 3)
            rows_np = np.sort(g.choice(T, size=m, replace=False)).astype(np.int32)
            off = np.searchsorted(rows_np, np.arange(B + 1) * L).astype(np.int32)
            cap = m + 5
            buf = np.zeros(cap, np.int32)
            buf[:m] = rows_np
            rows = Bd.IndexList(torch.from_numpy(buf).cuda(), torch.from_numpy(off).cuda())
            n_flags = cap
        else:
            rows, n_flags = None, T
        flag = torch.from_numpy((g.random(n_flags) < share).astype(np.uint8)).cuda()
        want, got = Bd.IndexList.empty(n_flags, B), Bd.IndexList.empty(n_flags, B)
        ctx.compact(flag, rows, B, L, want)
        Bd.compact_static(flag, rows, B, L, got)
        torch.cuda.synchronize()
        n = _lists_equal(got, want)
        # and against the definition: the flagged entries, in order
        f = flag.cpu().numpy().astype(bool)
        ref = (rows_np[f[:rows_np.size]] if with_rows else np.flatnonzero(f)).astype(np.int32)
        assert n == ref.size and np.array_equal(got.idx[:n].cpu().numpy(), ref)
        assert ctx.poll_status() == 0
        ctx.close()


def test_compact_static_overflow_and_limits():
    _say("compact_static: overflow word, size limit, argument checks")
    B, L = 2, 600
    T = B * L
    flag = torch.ones(T, dtype=torch.uint8, device="cuda")
    short = Bd.IndexList.empty(100, B)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    Bd.compact_static(flag, None, B, L, short, status)
    torch.cuda.synchronize()
    assert int(status.item()) == Bd.ERR_CAPACITY
    assert np.array_equal(short.idx.cpu().numpy(), np.arange(100)) and int(short.offsets[-1].item()) == 100
    # without a status word the overflow is dropped silently and the next call is unaffected
    Bd.compact_static(flag, None, B, L, short, None)
    full = Bd.IndexList.empty(T, B)
    status.zero_()
    Bd.compact_static(flag, None, B, L, full, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0 and np.array_equal(full.idx.cpu().numpy(), np.arange(T))
    assert full.offsets.cpu().numpy().tolist() == [0, L, T]
    # beyond the stated maximum: refused before any launch
    big_B, big_L = 2, Bd.COMPACT_STATIC_MAX_ROWS // 2 + 1
    with pytest.raises(Bd.DyllmError) as e:
        Bd.compact_static(flag, None, big_B, big_L, full, None)
    assert e.value.code == Bd.ERR_CAPACITY
    with pytest.raises(Bd.DyllmError) as e:
        Bd.compact_static(flag, None, 0, L, full, None)
    assert e.value.code == Bd.ERR_INVALID_ARG
    # the largest size it takes
    Bm, Lm = 16, Bd.COMPACT_STATIC_MAX_ROWS // 16
    fm = (torch.arange(Bm * Lm, device="cuda") % 7 == 3).to(torch.uint8)
    outm = Bd.IndexList.empty(Bm * Lm, Bm)
    Bd.compact_static(fm, None, Bm, Lm, outm, status)
    torch.cuda.synchronize()
    n = int(outm.offsets[-1].item())
    ref = torch.nonzero(fm).view(-1).to(torch.int32)
    assert n == ref.numel() and torch.equal(outm.idx[:n], ref) and int(status.item()) == 0
