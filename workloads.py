"""Seeded synthetic jagged batches shared by the tests, the smoke check and the benchmark.

This module draws lengths and values and nothing else: it holds none of the
attention arithmetic, so both the GPU path's callers and the CPU oracle's
callers can take inputs from it without sharing any of the method's code.

The paper measures on production recommendation data that is not public
(section 3); these batches take the shapes it states (jagged sequences of
highly variable length, section 2.3; maximum lengths of 3K to 16K, table 1;
CP sizes 2/4/8) and stand in for it.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    lengths: tuple          # per-sequence lengths
    num_heads: int
    d_qk: int
    d_v: int
    max_len: int            # the 1/max_len normaliser
    dtype: str              # "bf16" | "f32"
    scale: float            # values ~ N(0,1) * scale
    seed: int               # torch generator seed for the values
    backward: bool
    cp_size: int = 0        # > 0: context-parallel emulation with this many ranks

    @property
    def batch(self) -> int:
        return len(self.lengths)

    @property
    def total_rows(self) -> int:
        return int(sum(self.lengths))

    @property
    def alpha(self) -> float:
        return 1.0 / float(np.sqrt(self.d_qk))

    @property
    def pairs_per_head(self) -> int:
        """Causally visible (query, key) pairs of one head."""
        return int(sum(l * (l + 1) // 2 for l in self.lengths))

    def seq_offsets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.lengths)]).astype(np.int32)

    def flops(self, backward: Optional[bool] = None) -> Dict[str, float]:
        """Algorithmic flops over visible pairs only (d = d_qk = d_v case generalised).

        forward: 2*d_qk (QK^T) + 2*d_v (PV) per pair; backward: S recompute
        2*d_qk, dP 2*d_v, dV 2*d_v, dK 2*d_qk, dQ 2*d_qk per pair.
        """
        pairs = self.pairs_per_head * self.num_heads
        f = (2 * self.d_qk + 2 * self.d_v) * pairs
        b = (6 * self.d_qk + 4 * self.d_v) * pairs
        return {"fwd": float(f), "bwd": float(b)}


def _lengths(cfg: int) -> List[int]:
    rng = np.random.default_rng(0)
    if cfg == 1:
        return [int(x) for x in rng.integers(1, 64, endpoint=True, size=4)]
    if cfg == 2:
        return [int(x) for x in rng.integers(1, 1024, endpoint=True, size=32)]
    if cfg == 3:
        return [int(x) for x in rng.integers(512, 4096, endpoint=True, size=16)]
    if cfg == 4:
        raw = rng.integers(4096, 16384, endpoint=True, size=8)
        return [int((x + 7) // 8 * 8) for x in raw]
    if cfg == 5:
        raw = rng.lognormal(np.log(8192.0), 0.8, 8)
        return [int(x) for x in np.clip(np.rint(raw), 64, 32768)]
    raise ValueError("unknown config %r" % (cfg,))


# Lengths the generators above must reproduce (the workload is pinned: a numpy
# change that altered the stream would otherwise silently change the benchmark).
_PINNED = {
    1: (55, 41, 33, 18),
    4: (14552, 11928, 10384, 7416, 7880, 4600, 5024, 4304),
    5: (9059, 7370, 13674, 8909, 5337, 10940, 23251, 17476),
}
_PINNED_TOTAL = {1: 147, 2: 17286, 3: 37117, 4: 66088, 5: 96016}


def config(cfg: int) -> Workload:
    """The five benchmark/test configurations, numbered from 1."""
    lengths = tuple(_lengths(cfg))
    if cfg in _PINNED:
        assert lengths == _PINNED[cfg], "config %d lengths changed: %r" % (cfg, lengths)
    assert sum(lengths) == _PINNED_TOTAL[cfg], "config %d total rows changed" % cfg
    if cfg == 1:
        return Workload("cfg1_tiny_f32", lengths, 2, 32, 32, 64, "f32", 1.0, 2, True)
    if cfg == 2:
        return Workload("cfg2_fwd_B32_L1-1024", lengths, 4, 128, 128, 1024, "bf16", 0.5, 3, False)
    if cfg == 3:
        return Workload("cfg3_B16_L512-4096", lengths, 4, 128, 128, 4096, "bf16", 0.5, 4, True)
    if cfg == 4:
        return Workload("cfg4_cp4_B8_L4096-16384", lengths, 4, 128, 128, 16384, "bf16", 0.5, 5,
                        True, cp_size=4)
    return Workload("cfg5_skewed_B8_lognormal", lengths, 8, 128, 128, 32768, "bf16", 0.5, 6, True)


def large_batch(kind: str) -> Workload:
    """Large batches of short sequences (the regime the paper's section 3 contrasts with long
    sequences), H = 4, d = 128, bf16, forward and backward:
    "short": 8192 sequences of 16..64 rows; "mid": 1536 sequences of 300..600 rows."""
    rng = np.random.default_rng(7)
    if kind == "short":
        lengths = rng.integers(16, 64, endpoint=True, size=8192)
        return Workload("short_B8192_L16-64", tuple(int(x) for x in lengths), 4, 128, 128, 64, "bf16", 0.5, 7, True)
    if kind == "mid":
        lengths = rng.integers(300, 600, endpoint=True, size=1536)
        return Workload("mid_B1536_L300-600", tuple(int(x) for x in lengths), 4, 128, 128, 600, "bf16", 0.5, 8, True)
    raise ValueError("unknown large batch %r" % (kind,))


def custom(name: str, lengths, num_heads: int, d_qk: int, d_v: int, max_len: int,
           dtype: str = "bf16", scale: float = 0.5, seed: int = 0, backward: bool = True,
           cp_size: int = 0) -> Workload:
    return Workload(name, tuple(int(x) for x in lengths), num_heads, d_qk, d_v, max_len, dtype,
                    scale, seed, backward, cp_size)


def torch_dtype(w: Workload) -> torch.dtype:
    return torch.bfloat16 if w.dtype == "bf16" else torch.float32


def values(w: Workload) -> Dict[str, torch.Tensor]:
    """q, k, v, d_o on the CPU in the workload's storage dtype (rounded once)."""
    g = torch.Generator(device="cpu").manual_seed(w.seed)
    T, H = w.total_rows, w.num_heads
    out = {}
    for name, d in (("q", w.d_qk), ("k", w.d_qk), ("v", w.d_v), ("d_o", w.d_v)):
        x = torch.randn((T, H, d), generator=g, dtype=torch.float32) * w.scale
        out[name] = x.to(torch_dtype(w))
    return out


def device_values(w: Workload, device: str = "cuda", rows_per_chunk: int = 1 << 19) -> Dict[str, torch.Tensor]:
    """q, k, v, d_o drawn on the device (seeded device generator, the same distribution as
    values()), for workloads whose tensors are too large to draw on the host and copy: several
    GiB each.  The values differ from values(w): a test takes what it gives the oracle from these
    tensors."""
    g = torch.Generator(device=device).manual_seed(w.seed)
    T, H = w.total_rows, w.num_heads
    out = {}
    for name, d in (("q", w.d_qk), ("k", w.d_qk), ("v", w.d_v), ("d_o", w.d_v)):
        x = torch.empty((T, H, d), dtype=torch_dtype(w), device=device)
        for r0 in range(0, T, rows_per_chunk):
            r1 = min(T, r0 + rows_per_chunk)
            x[r0:r1] = (torch.randn((r1 - r0, H, d), generator=g, dtype=torch.float32, device=device)
                        * w.scale).to(x.dtype)
        out[name] = x
    return out


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of stored values (bf16 or fp32) to float64 for the oracle."""
    return t.detach().cpu().to(torch.float64).numpy()


def timestamps(w: Workload, kind: str = "events", seed: int = 0) -> np.ndarray:
    """One int32 timestamp per row, for the attention with timestamp bias.

    "events": per sequence a random start plus cumulative heavy-tailed gaps (log-normal seconds
    with a median of a minute: bursts of activity separated by idle hours), non-decreasing
    inside a sequence, as a user's interaction history is; "shuffled": values drawn the same way
    but in random order inside each sequence (nothing sorted: every block of pairs spans many buckets);
    "equal": one value per sequence (every difference zero); "wide": differences up to the
    whole int32 range.
    """
    rng = np.random.default_rng(1000 + seed)
    out = []
    for L in w.lengths:
        if kind == "equal":
            t = np.full(L, rng.integers(0, 2 ** 30), dtype=np.int64)
        elif kind == "wide":
            t = np.sort(rng.integers(-2 ** 31, 2 ** 31 - 1, size=L, dtype=np.int64))
        else:
            gaps = np.exp(rng.normal(np.log(60.0), 2.0, size=L)).astype(np.int64)
            t = rng.integers(0, 2 ** 28) + np.cumsum(np.minimum(gaps, 10 ** 6))
            if kind == "shuffled":
                t = rng.permutation(t)
            elif kind != "events":
                raise ValueError(kind)
        out.append(t)
    out.append(np.zeros(0, dtype=np.int64))
    return np.concatenate(out).astype(np.int32)


def bias_table(num_buckets: int, seed: int = 0, scale: float = 1.0) -> np.ndarray:
    """A bucket table of the timestamp bias: fp32 values ~ N(0,1) * scale."""
    rng = np.random.default_rng(2000 + seed)
    return (rng.standard_normal(num_buckets) * scale).astype(np.float32)
