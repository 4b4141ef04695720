"""Seeded synthetic inputs for the five benchmark configurations.

Harness code, not part of the library package: tests, ``bench.py`` and the smoke run
import it; the package imports nothing from it.  It holds no arithmetic of the attention
path: it draws floating-point Q, K, V with the stated distributions and turns them into
the INT8 tensors the path starts from with the workload recipe (``s_X = max|X| / 127``,
``numpy.rint``, clamp to [-127, 127] -- the same operation as Sec. 2.1, Eq. quant, written
with numpy; a CPU test checks this recipe against the pinned oracle quantizer, never the
other way round).  The quantizer tests of the oracle and of the HIP library draw their own
floating-point tensors and do not come here.  It imports neither the oracle nor the library.

The shapes stand in for the paper's language models (causal, long L) and vision
transformers (non-causal, L = 197) by shape only.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class Problem:
    name: str
    B: int
    Hq: int
    Hkv: int
    L: int
    d: int
    causal: bool
    per_head: bool
    q: np.ndarray  # int8 [B,Hq,L,d]
    k: np.ndarray  # int8 [B,Hkv,L,d]
    v: np.ndarray  # int8 [B,Hkv,L,d]
    s_q: np.ndarray  # float32 [1] or [Hq]
    s_k: np.ndarray  # float32 [1] or [Hkv]
    s_v: np.ndarray  # float32 [1] or [Hkv]
    meta: dict = field(default_factory=dict)

    @property
    def pairs(self) -> int:
        return self.L * (self.L + 1) // 2 if self.causal else self.L * self.L

    @property
    def ops(self) -> int:
        """Counted int8 work: the two contractions only, 2 ops per multiply-accumulate."""
        return 4 * self.d * self.pairs * self.B * self.Hq

    @property
    def algorithmic_bytes(self) -> int:
        """Q + out (query heads) and K + V (KV heads), one byte per element."""
        return (2 * self.B * self.Hq + 2 * self.B * self.Hkv) * self.L * self.d


CONFIGS = {
    # name: (B, Hq, Hkv, L, d, causal, per_head, seed)
    "c1_single_head": (1, 1, 1, 128, 64, False, False, 0),
    "c2_vit_b16": (8, 12, 12, 197, 64, False, False, 1),
    "c3_llm_prefill_2k": (1, 16, 16, 2048, 64, True, False, 2),
    "c4_gqa_prefill_8k": (1, 32, 8, 8192, 128, True, False, 3),
    "c5_batched_prefill_4k": (16, 32, 32, 4096, 128, True, True, 4),
}


def quantize(x: np.ndarray, per_head: bool):
    """Eq. quant.  per_head=False: one scale for the tensor; True: one scale per head index
    (axis 1), shared over the batch."""
    if per_head:
        amax = np.abs(x).max(axis=(0, 2, 3)).astype(np.float32)
        amax = np.maximum(amax, np.float32(1e-12))
        s = (amax / np.float32(127.0)).astype(np.float32)
        xs = x / s[None, :, None, None]
    else:
        amax = np.float32(max(float(np.abs(x).max()), 1e-12))
        s = np.asarray([amax / np.float32(127.0)], dtype=np.float32)
        xs = x / s[0]
    xq = np.clip(np.rint(xs), -127, 127).astype(np.int8)
    return np.ascontiguousarray(xq), s


def _normal(rng, shape):
    return rng.standard_normal(shape, dtype=np.float32)


def _rotary(x: np.ndarray) -> np.ndarray:
    """Rotate channel pairs (2i, 2i+1) by angle p * 10000^(-2i/d) at position p."""
    B, H, L, d = x.shape
    i = np.arange(d // 2, dtype=np.float64)
    freq = 10000.0 ** (-2.0 * i / d)
    ang = np.arange(L, dtype=np.float64)[:, None] * freq[None, :]
    cos, sin = np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
    xe, xo = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = xe * cos - xo * sin
    out[..., 1::2] = xe * sin + xo * cos
    return out


def make_problem(name: str, *, B=None, Hq=None, Hkv=None, L=None, d=None, seed=None) -> Problem:
    """Build one of the named configurations; the keyword overrides shrink (or grow) it while
    keeping its distribution, masking and quantization recipe."""
    cB, cHq, cHkv, cL, cd, causal, per_head, cseed = CONFIGS[name]
    B = cB if B is None else B
    Hq = cHq if Hq is None else Hq
    Hkv = cHkv if Hkv is None else Hkv
    L = cL if L is None else L
    d = cd if d is None else d
    seed = cseed if seed is None else seed
    rng = np.random.default_rng(seed)
    qs, ks = (B, Hq, L, d), (B, Hkv, L, d)
    meta = {"seed": seed}

    if name == "c5_batched_prefill_4k":
        q = rng.standard_t(4, size=qs).astype(np.float32)
        k = rng.standard_t(4, size=ks).astype(np.float32)
        v = rng.standard_t(4, size=ks).astype(np.float32)
    else:
        q, k, v = _normal(rng, qs), _normal(rng, ks), _normal(rng, ks)

    if name == "c2_vit_b16":
        # 2% of the channels of every head (at least one) carry x8 outliers in Q, K and V.
        n_out = max(1, int(round(0.02 * d)))
        ch = np.stack([rng.choice(d, size=n_out, replace=False) for _ in range(Hkv)])
        g = Hq // Hkv
        for h in range(Hq):
            q[:, h, :, ch[h // g]] *= 8.0
        for h in range(Hkv):
            k[:, h, :, ch[h]] *= 8.0
            v[:, h, :, ch[h]] *= 8.0
        meta["outlier_channels"] = ch.tolist()
    elif name == "c3_llm_prefill_2k":
        q, k = _rotary(q), _rotary(k)
    elif name == "c4_gqa_prefill_8k":
        # 1% of the K channels of every KV head (at least one) scaled x10: heavy-tailed logits.
        n_out = max(1, int(round(0.01 * d)))
        ch = np.stack([rng.choice(d, size=n_out, replace=False) for _ in range(Hkv)])
        for h in range(Hkv):
            k[:, h, :, ch[h]] *= 10.0
        meta["outlier_channels"] = ch.tolist()

    q8, s_q = quantize(q, per_head)
    k8, s_k = quantize(k, per_head)
    v8, s_v = quantize(v, per_head)
    return Problem(name, B, Hq, Hkv, L, d, causal, per_head, q8, k8, v8, s_q, s_k, s_v, meta)


def random_problem(seed: int, B: int, Hq: int, Hkv: int, L: int, d: int, causal: bool,
                   per_head: bool = False, spread: float = 1.0, name: str = "random") -> Problem:
    """Plain N(0, spread^2) inputs of an arbitrary shape, for edge-case and ragged-shape tests."""
    rng = np.random.default_rng(seed)
    q = _normal(rng, (B, Hq, L, d)) * np.float32(spread)
    k = _normal(rng, (B, Hkv, L, d)) * np.float32(spread)
    v = _normal(rng, (B, Hkv, L, d))
    if per_head:
        # make the heads differ in range so that per-head scales actually differ
        q *= (1.0 + np.arange(Hq, dtype=np.float32))[None, :, None, None]
        k *= (1.0 + 0.5 * np.arange(Hkv, dtype=np.float32))[None, :, None, None]
    q8, s_q = quantize(q, per_head)
    k8, s_k = quantize(k, per_head)
    v8, s_v = quantize(v, per_head)
    return Problem(name, B, Hq, Hkv, L, d, causal, per_head, q8, k8, v8, s_q, s_k, s_v, {"seed": seed})


def calibrated_out_scale(p: Problem, sample_rows: int = 64) -> np.ndarray:
    """An output scale s_O (per tensor or per query head) from max|O| of fp64 softmax attention on
    a few sampled rows of the dequantized inputs -- so that the INT8 output uses its range.  This
    is calibration of a *parameter*, done in floating point outside the integer path."""
    rng = np.random.default_rng(p.meta.get("seed", 0) + 1000)
    g = p.Hq // p.Hkv
    amax = np.zeros(p.Hq, dtype=np.float64)
    for h in range(p.Hq):
        kv = h // g
        sq = float(p.s_q[h] if p.per_head else p.s_q[0])
        sk = float(p.s_k[kv] if p.per_head else p.s_k[0])
        sv = float(p.s_v[kv] if p.per_head else p.s_v[0])
        b = int(rng.integers(p.B))
        rows = rng.integers(0, p.L, size=min(sample_rows, p.L))
        qf = p.q[b, h, rows].astype(np.float64) * sq
        kf = p.k[b, kv].astype(np.float64) * sk
        vf = p.v[b, kv].astype(np.float64) * sv
        a = qf @ kf.T / np.sqrt(p.d)
        if p.causal:
            a = np.where(np.arange(p.L)[None, :] <= rows[:, None], a, -np.inf)
        a -= a.max(axis=1, keepdims=True)
        w = np.exp(a)
        w /= w.sum(axis=1, keepdims=True)
        amax[h] = np.abs(w @ vf).max()
    amax = np.maximum(amax, 1e-12)
    if p.per_head:
        return (amax / 127.0).astype(np.float32)
    return np.asarray([amax.max() / 127.0], dtype=np.float32)
