"""The synthetic input recipe: deterministic, well-formed index lists, stated sizes."""
import numpy as np

from synth import workload as W


def test_streams_are_reproducible_and_independent():
    a = W.philox(1, "x", 3).standard_normal(8)
    b = W.philox(1, "x", 3).standard_normal(8)
    c = W.philox(1, "x", 4).standard_normal(8)
    assert np.array_equal(a, b) and not np.array_equal(a, c)


def test_round_bf16_is_nearest_even_and_idempotent():
    # bf16 spacing near 1 is 2^-7
    x = np.array([1.0, 1.0 + 2 ** -9, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -9, 1.0 + 3 * 2 ** -8, -3.14159, 0.0],
                 dtype=np.float32)
    r = W.round_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0
    assert r[2] == 1.0  # tie: even mantissa (0) wins
    assert r[3] == np.float32(1.0 + 2 ** -7)
    assert r[4] == np.float32(1.0 + 2 ** -6)  # tie: even mantissa (2) wins
    assert np.array_equal(W.round_bf16(r), r)
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    assert np.max(np.abs(r - x) / np.maximum(np.abs(x), 1e-30)) <= 2 ** -8


def test_step_rows_sorted_unique_with_offsets():
    for name in ("c1", "c2", "c3"):
        w = W.CONFIGS[name]
        for t in (1, 2, 7):
            idx, off = W.step_rows(w, t)
            assert idx.dtype == np.int32 and off.dtype == np.int32 and off.shape == (w.batch + 1,)
            assert np.all(np.diff(idx) > 0)
            assert off[0] == 0 and off[-1] == idx.size
            for b in range(w.batch):
                seg = idx[off[b]:off[b + 1]]
                assert np.all((seg >= b * w.seq) & (seg < (b + 1) * w.seq))
            idx2, off2 = W.step_rows(w, t)
            assert np.array_equal(idx, idx2) and np.array_equal(off, off2)


def test_salient_counts_follow_the_configured_fraction():
    w = W.CONFIGS["c2"]
    idx, off = W.step_rows(w, 5)
    assert round(0.10 * w.seq) <= idx.size <= round(0.10 * w.seq) + w.n_unmask
    w3 = W.CONFIGS["c3"]
    idx, off = W.step_rows(w3, 5)
    counts = np.diff(off)
    assert counts.min() >= 0.5 * 0.10 * w3.seq - 1 and counts.max() <= 1.5 * 0.10 * w3.seq + w3.n_unmask + 1
    assert len(set(counts.tolist())) > 4  # ragged
    for f in (0.05, 0.25):
        idx, off = W.step_rows(W.with_frac(W.CONFIGS["c2"], f), 5)
        assert abs(idx.size - f * 1024) <= 5


def test_unmask_order_goes_block_by_block():
    w = W.CONFIGS["c2"]
    order = W.unmask_order(w, 0)
    assert sorted(order.tolist()) == list(range(w.prompt_len, w.seq))
    blocks = (order - w.prompt_len) // W.BLOCK
    assert np.all(np.diff(blocks) >= 0)


def test_hidden_drift_model():
    w = W.CONFIGS["c1"]
    steps = list(W.step_stream(w, 3))
    assert steps[0].dense and not steps[1].dense and steps[1].idx is not None
    x0, x1, idx = steps[0].x, steps[1].x, steps[1].idx
    flat0, flat1 = x0.reshape(-1, w.shape.hidden), x1.reshape(-1, w.shape.hidden)
    others = np.setdiff1d(np.arange(w.tokens), idx)
    d = flat1[others] - flat0[others]
    assert 0.5e-3 < d.std() < 2e-3
    assert np.abs(flat1[idx] - flat0[idx]).mean() > 0.5  # redrawn rows
    again = list(W.step_stream(w, 3))
    assert np.array_equal(again[2].x, steps[2].x)


def test_weights_shapes_and_bf16_rounding():
    w = W.make_weights(W.TINY)
    assert w["wq"].shape == (256, 256) and w["w_gate"].shape == (768, 256) and w["w_down"].shape == (256, 768)
    assert 0.018 < w["w_up"].std() < 0.022
    small = W.LayerShape(64, 4, 2, 16, 96, dtype="bf16")
    wb = W.make_weights(small)
    assert wb["wk"].shape == (32, 64)
    assert all(np.all((v.view(np.uint32) & 0xFFFF) == 0) for v in wb.values())


def test_second_workload_concentrates_the_redraw_in_the_response():
    w = W.CONFIGS["c6"]
    assert w.n_unmask == 2
    for t in (1, 7, 40):
        idx, off = W.step_rows(w, t)
        assert np.all(np.diff(idx) > 0) and off[-1] == idx.size
        pos = idx % w.seq
        share = np.mean(pos >= w.prompt_len)
        assert 0.85 <= share <= 0.95
        for b in range(w.batch):
            rows = idx[off[b]:off[b + 1]]
            assert np.all(rows // w.seq == b)
            assert 0.5 * 0.05 * w.seq - 2 <= rows.size <= 1.5 * 0.05 * w.seq + 2 + w.n_unmask
