"""Seeded synthetic inputs for the DMA forward path.

This module only draws random numbers and shapes them; it holds none of the method's arithmetic
and imports neither the GPU binding nor the CPU oracle, so both sides can be fed the same bits.

All tensors are generated on the host in float32 with ``numpy.random.Generator(Philox(seed))``,
transformed, rounded to bf16 (round to nearest even) and returned as ``numpy.uint16`` bit patterns
with layout q[B, Hq, S, D], k[B, Hkv, S, D], v[B, Hkv, S, D].  Draw order: Q, K, V, then outlier
channel indices, then outlier factors.

The value structure follows what the paper describes for its LLaMA workloads: channel-wise outliers
in Q and K (Sec. 4 "Challenges") and attention-sink-like first keys (Sec. 5.2, sink window); the
shapes follow LLaMA-3.1-8B attention (32 query heads, 8 kv heads, head dimension 128) at the
paper's 2.5K-30K token lengths (Sec. 5.1).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    S: int
    D: int
    tile: int
    band: int
    seed: int
    kind: str                      # "fixed_channels" | "random_channels" | "sink" | "student_t"
    extra: dict = field(default_factory=dict)

    @property
    def causal_flops(self) -> float:
        """2*B*Hq*S^2*D: the flash-attention convention for a causal forward."""
        return 2.0 * self.B * self.Hq * float(self.S) ** 2 * self.D


# The five configurations of the build's baseline description.
CONFIGS = {
    "tiny": Workload("tiny", 1, 2, 2, 256, 64, 64, 1, 1001, "fixed_channels",
                     {"channels": (5, 22, 41, 58), "factor": 15.0}),
    "prefill_8k": Workload("prefill_8k", 1, 32, 32, 8192, 128, 128, 2, 2002, "random_channels"),
    "gqa_32k": Workload("gqa_32k", 1, 32, 8, 32768, 128, 128, 2, 3003, "sink"),
    "batched_4k": Workload("batched_4k", 8, 32, 32, 4096, 128, 128, 2, 4004, "random_channels"),
    "heavy_tail_16k": Workload("heavy_tail_16k", 1, 40, 8, 16384, 128, 128, 2, 5005, "student_t"),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(rng, shape):
    return rng.standard_normal(size=shape, dtype=np.float32)


def generate(w: Workload):
    """Returns (q_bits, k_bits, v_bits) as uint16 arrays for workload ``w``."""
    rng = np.random.Generator(np.random.Philox(w.seed))
    qs, ks = (w.B, w.Hq, w.S, w.D), (w.B, w.Hkv, w.S, w.D)
    group = w.Hq // w.Hkv
    if w.kind == "student_t":
        nu = 3.0
        q = (rng.standard_t(nu, size=qs) / np.sqrt(nu)).astype(np.float32)
        k = (rng.standard_t(nu, size=ks) / np.sqrt(nu)).astype(np.float32)
        v = (rng.standard_t(nu, size=ks) / np.sqrt(nu)).astype(np.float32)
    else:
        q, k, v = _normal(rng, qs), _normal(rng, ks), _normal(rng, ks)

    if w.kind == "fixed_channels":
        ch = list(w.extra["channels"])
        q[..., ch] *= np.float32(w.extra["factor"])
        k[..., ch] *= np.float32(w.extra["factor"])
    elif w.kind in ("random_channels", "sink"):
        n_out = int(np.ceil(0.02 * w.D))
        chans = np.stack([rng.choice(w.D, size=n_out, replace=False) for _ in range(w.Hkv)])
        fq = rng.uniform(10.0, 20.0, size=(w.Hkv, n_out)).astype(np.float32)
        fk = rng.uniform(10.0, 20.0, size=(w.Hkv, n_out)).astype(np.float32)
        for h in range(w.Hkv):
            for c in range(n_out):
                q[:, h * group:(h + 1) * group, :, chans[h, c]] *= fq[h, c]
                k[:, h, :, chans[h, c]] *= fk[h, c]
        if w.kind == "sink":
            # first four key positions get 5x the mean key norm of their head
            norms = np.sqrt((k.astype(np.float64) ** 2).sum(-1))          # [B, Hkv, S]
            mean_norm = norms.mean(-1, keepdims=True)                      # [B, Hkv, 1]
            scale = (5.0 * mean_norm / norms[..., :4]).astype(np.float32)  # [B, Hkv, 4]
            k[:, :, :4, :] *= scale[..., None]
    return f32_to_bf16_bits(q), f32_to_bf16_bits(k), f32_to_bf16_bits(v)


def small_variant(w: Workload, *, S: int, Hq: int | None = None, Hkv: int | None = None, B: int | None = None,
                  seed: int | None = None) -> Workload:
    """Same recipe at a reduced size (for element-by-element parity against the oracle)."""
    return Workload(w.name + f"_S{S}", B or w.B, Hq or w.Hq, Hkv or w.Hkv, S, w.D, w.tile, w.band,
                    seed if seed is not None else w.seed, w.kind, dict(w.extra))


def sample_rows(w: Workload, q_tiles, heads, n_random: int, seed: int) -> np.ndarray:
    """(b, hq, i) triples: every row of the listed query tiles for the listed (b, hq) pairs, plus
    n_random uniformly drawn rows."""
    rows = []
    for (b, h) in heads:
        for t in q_tiles:
            for i in range(t * w.tile, (t + 1) * w.tile):
                rows.append((b, h, i))
    rng = np.random.Generator(np.random.Philox(seed))
    for _ in range(n_random):
        rows.append((int(rng.integers(w.B)), int(rng.integers(w.Hq)), int(rng.integers(w.S))))
    return np.asarray(rows, dtype=np.int64).reshape(-1, 3)
