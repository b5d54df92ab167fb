"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random numbers and index sets.  It holds none of the
method's arithmetic (no norm, projection, attention, cosine, selection): both
the CPU oracle's tests and the GPU harness take their inputs from here, and
neither of them is imported here.

Shapes follow the paper's evaluation setting: 1024-ish prompt tokens plus a
256-token response (Sec. 4.2.4), semi-autoregressive blocks of 32 response
positions (Sec. 2.3, App. D.3), LLaDA-8B- and Dream-7B-shaped layers
(Sec. 4.1).  Trained weights and the benchmark prompts themselves are not
available; weights are random-init and hidden states follow a drift model:
per step most tokens move by a tiny amount, a seeded random subset (plus the
newly unmasked response positions) is redrawn.

Every draw comes from a counter-based Philox stream keyed by
(seed, tensor name, layer / step / batch row), so any piece can be regenerated
on its own and is identical wherever it is generated.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field, replace
from typing import Dict, Iterator, List, Optional, Tuple

import numpy as np

SEED_W = 1234
SEED_X = 42
BLOCK = 32  # semi-AR block length used to order "newly unmasked" positions


def philox(seed: int, *key) -> np.random.Generator:
    """Counter-based generator for one (seed, key...) stream."""
    h = hashlib.blake2b(repr((int(seed),) + tuple(key)).encode(), digest_size=16).digest()
    return np.random.Generator(np.random.Philox(key=np.frombuffer(h, dtype=np.uint64)))


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of already bf16-representable fp32 values (uint16)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


@dataclass(frozen=True)
class LayerShape:
    hidden: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    dtype: str = "bf16"  # "f32" or "bf16": storage type of the GPU path
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def dq(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def dkv(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def group(self) -> int:
        return self.n_heads // self.n_kv_heads


@dataclass(frozen=True)
class Workload:
    name: str
    shape: LayerShape
    batch: int
    prompt_len: int
    resp_len: int
    steps: int
    frac: float  # salient (redrawn) fraction of the sequence per step
    ragged: bool = False  # per-sequence counts ~ frac * L * U[0.5, 1.5]
    t_full: int = 4  # dense warm-up steps (Sec. 3.2)
    tau: float = 0.99
    n_layers: int = 1
    drift_std: float = 1e-3
    resp_share: Optional[float] = None  # share of the redrawn rows taken from the response (None: uniform over L)
    unmask: Optional[int] = None        # tokens unmasked per step and sequence (None: resp_len // steps)

    @property
    def seq(self) -> int:
        return self.prompt_len + self.resp_len

    @property
    def tokens(self) -> int:
        return self.batch * self.seq

    @property
    def n_unmask(self) -> int:
        return max(1, self.resp_len // self.steps) if self.unmask is None else self.unmask


TINY = LayerShape(hidden=256, n_heads=4, n_kv_heads=4, head_dim=64, ffn=768, dtype="f32")
LLADA = LayerShape(hidden=4096, n_heads=32, n_kv_heads=32, head_dim=128, ffn=12288, dtype="bf16")
DREAM = LayerShape(hidden=3584, n_heads=28, n_kv_heads=4, head_dim=128, ffn=18944, dtype="bf16")

CONFIGS: Dict[str, Workload] = {
    # tiny fp32 layer the oracle finishes in seconds
    "c1": Workload("c1-tiny-f32", TINY, 1, 96, 32, 8, 0.10, t_full=1, tau=0.99),
    # LLaDA-8B-shaped layer, batch 1, 768 + 256
    "c2": Workload("c2-llada8b-b1-l1024", LLADA, 1, 768, 256, 64, 0.10, tau=0.99),
    # LLaDA-8B-shaped layer, batch 16, 1024 + 256, ragged per-sequence counts
    "c3": Workload("c3-llada8b-b16-l1280", LLADA, 16, 1024, 256, 64, 0.10, ragged=True, tau=0.99),
    # Dream-7B-shaped layer (GQA 28/4), batch 16
    "c4": Workload("c4-dream7b-b16-l1280", DREAM, 16, 1024, 256, 64, 0.10, tau=0.995),
    # 32-layer LLaDA-shaped stack, batch 16, 1536 + 512
    "c5": Workload("c5-llada8b-stack32-b16-l2048", LLADA, 16, 1536, 512, 128, 0.10,
                   ragged=True, tau=0.99, n_layers=32),
    # second workload: salient tokens concentrated in the response (Sec. 3.5; App. D.1: context
    # updates cluster around the latest unmasked tokens), two tokens unmasked per step (Sec. 4.2.4)
    "c6": Workload("c6-llada8b-b16-l1280-resp", LLADA, 16, 1024, 256, 128, 0.05, ragged=True, tau=0.99,
                   resp_share=0.9, unmask=2),
}


def with_frac(w: Workload, frac: float) -> Workload:
    return replace(w, frac=frac)


def make_weights(shape: LayerShape, layer: int = 0, std: float = 0.02,
                 seed: int = SEED_W) -> Dict[str, np.ndarray]:
    """Random-init weights of one layer, fp32 arrays ([out, in] row-major).

    For a bf16 layer every value is rounded to bf16 so that both sides start
    from exactly the same numbers.  Norm gains are drawn near 1 (not exactly 1)
    so that a dropped gain is visible.
    """
    d, dq, dkv, f = shape.hidden, shape.dq, shape.dkv, shape.ffn
    spec = {
        "wq": (dq, d), "wk": (dkv, d), "wv": (dkv, d), "wo": (d, dq),
        "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
    }
    out = {}
    for name, shp in spec.items():
        g = philox(seed + layer, "w", name)
        w = g.standard_normal(shp, dtype=np.float32) * np.float32(std)
        out[name] = w
    for name in ("g_attn", "g_ffn"):
        g = philox(seed + layer, "w", name)
        out[name] = (1.0 + 0.1 * g.standard_normal(d, dtype=np.float32)).astype(np.float32)
    if shape.dtype == "bf16":
        out = {k: round_bf16(v) for k, v in out.items()}
    return out


def _count_for(w: Workload, t: int, b: int, seed: int) -> int:
    base = w.frac * w.seq
    if w.ragged:
        u = philox(seed, "count", t, b).uniform(0.5, 1.5)
        base *= u
    return int(min(w.seq, max(0, round(base))))


def unmask_order(w: Workload, b: int, seed: int = SEED_X) -> np.ndarray:
    """Order in which response positions get unmasked for sequence b.

    Blocks of 32 response positions are taken left to right; inside a block
    the order is a seeded permutation.  Returns sequence positions (prompt
    offset included), length resp_len.
    """
    order = []
    for blk, start in enumerate(range(0, w.resp_len, BLOCK)):
        n = min(BLOCK, w.resp_len - start)
        perm = philox(seed, "unmask", b, blk).permutation(n)
        order.append(w.prompt_len + start + perm)
    return np.concatenate(order).astype(np.int64) if order else np.zeros(0, np.int64)


def step_rows(w: Workload, t: int, seed: int = SEED_X) -> Tuple[np.ndarray, np.ndarray]:
    """Redrawn + newly unmasked positions of step t (t >= 1).

    Returns (idx, offsets): flat token ids b*L+i, ascending and unique, and
    the per-sequence offsets [B+1] into idx.
    """
    idx: List[np.ndarray] = []
    offsets = np.zeros(w.batch + 1, dtype=np.int32)
    nu = w.n_unmask
    for b in range(w.batch):
        n = _count_for(w, t, b, seed)
        g = philox(seed, "redraw", t, b)
        if w.resp_share is None:
            red = g.choice(w.seq, size=n, replace=False)
        else:  # n_r of the n rows from the response positions, the others from the prompt
            n_r = min(w.resp_len, int(round(w.resp_share * n)))
            n_p = min(w.prompt_len, n - n_r)
            red = np.concatenate([w.prompt_len + g.choice(w.resp_len, size=n_r, replace=False),
                                  g.choice(w.prompt_len, size=n_p, replace=False)])
        order = unmask_order(w, b, seed)
        lo = ((t - 1) * nu) % max(1, w.resp_len)
        newly = order[lo:lo + nu]
        rows = np.unique(np.concatenate([red.astype(np.int64), newly]))
        idx.append(rows + b * w.seq)
        offsets[b + 1] = offsets[b] + rows.size
    flat = np.concatenate(idx).astype(np.int32) if idx else np.zeros(0, np.int32)
    return flat, offsets


def initial_hidden(w: Workload, seed: int = SEED_X) -> np.ndarray:
    """X_0 ~ N(0,1), fp32 [B, L, hidden] (rounded to bf16 for a bf16 layer)."""
    x = np.empty((w.batch, w.seq, w.shape.hidden), dtype=np.float32)
    for b in range(w.batch):
        x[b] = philox(seed, "x0", b).standard_normal((w.seq, w.shape.hidden), dtype=np.float32)
    return round_bf16(x) if w.shape.dtype == "bf16" else x


def next_hidden(w: Workload, x_prev: np.ndarray, t: int, idx: np.ndarray,
                seed: int = SEED_X) -> np.ndarray:
    """X_t from X_{t-1}: rows in idx are redrawn N(0,1); the rest drift by N(0, drift_std^2)."""
    x = np.empty_like(x_prev, dtype=np.float32)
    L = w.seq
    for b in range(w.batch):
        g = philox(seed, "drift", t, b)
        x[b] = x_prev[b] + g.standard_normal((L, w.shape.hidden), dtype=np.float32) * np.float32(w.drift_std)
        rows = idx[(idx >= b * L) & (idx < (b + 1) * L)] - b * L
        if rows.size:
            g2 = philox(seed, "fresh", t, b)
            x[b, rows] = g2.standard_normal((rows.size, w.shape.hidden), dtype=np.float32)
    return round_bf16(x) if w.shape.dtype == "bf16" else x


@dataclass
class Step:
    t: int
    dense: bool
    x: np.ndarray  # [B, L, hidden] fp32
    idx: Optional[np.ndarray]  # flat ids (None on dense steps)
    offsets: Optional[np.ndarray]  # [B+1]


def step_stream(w: Workload, n_steps: Optional[int] = None, seed: int = SEED_X) -> Iterator[Step]:
    """Steps 0..n_steps-1: the first t_full are dense (cache warm-up), the rest sparse."""
    n = w.steps if n_steps is None else n_steps
    x = initial_hidden(w, seed)
    for t in range(n):
        if t == 0:
            idx, off = None, None
        else:
            idx, off = step_rows(w, t, seed)
            x = next_hidden(w, x, t, idx, seed)
        if t < w.t_full:
            yield Step(t, True, x, None, None)
        else:
            yield Step(t, False, x, idx, off)


def perturbed_rows(base: np.ndarray, sigmas: np.ndarray, seed: int, *key) -> np.ndarray:
    """base + sigma_i * N(0,1) per row: used to make cosines straddle a threshold."""
    g = philox(seed, "perturb", *key)
    noise = g.standard_normal(base.shape, dtype=np.float32)
    return (base + noise * sigmas.astype(np.float32)[:, None]).astype(np.float32)
