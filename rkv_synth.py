"""Seeded synthetic KV workloads with the shapes and structure of the paper's keys and values.

This module only draws random inputs; it holds none of the method's arithmetic, so that the CPU
oracle and the HIP path can both be fed from it without sharing any code of the method.

Structure copied from what the paper reports about real LLaMA keys (arXiv 2501.16383, Sec. 1 and
Fig. 1-2, Sec. 4.2, Sec. 4.3): a few channels per head carry much larger magnitudes, different
channels in different heads, consistent across tokens before RoPE; a handful of sink tokens carry
massive activations; values have no such outliers.

Recipe: K, V ~ N(0,1) rounded to fp16; in every KV head `n_out` channels (drawn without
replacement) of K are multiplied by a factor; sink tokens multiply their whole K and V rows by
`sink_gain`; queries ~ N(0,1).  The "offset" variant adds a per-channel mean of +-factor instead
of multiplying (the only variant in which a signed channel sum says anything about a channel).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int
    layers: int
    rot_heads: int
    n_sinks: int
    rope_theta: float
    outlier_count: Tuple[int, int]      # inclusive range of outlier channels per head
    outlier_gain: Tuple[float, float]   # range of the multiplicative factor
    sink_gain: float = 100.0
    seed: int = 1000


# The five configurations the build is measured and tested on.
WORKLOADS = {
    "cfg0": Workload("cfg0", 1, 32, 32, 128, 512, 1, 2, 1, 10000.0, (4, 4), (20.0, 20.0), seed=1000),
    "cfg1": Workload("cfg1", 8, 32, 32, 128, 4096, 32, 4, 4, 10000.0, (4, 8), (10.0, 50.0), seed=1001),
    "cfg2": Workload("cfg2", 16, 40, 40, 128, 4096, 40, 4, 4, 10000.0, (4, 8), (10.0, 50.0), seed=1002),
    "cfg3": Workload("cfg3", 1, 32, 32, 128, 32768, 1, 4, 4, 10000.0, (4, 8), (10.0, 50.0), seed=1003),
    "cfg4": Workload("cfg4", 32, 32, 8, 128, 8192, 32, 4, 4, 500000.0, (4, 8), (10.0, 50.0), seed=1004),
    # not one of the benchmark configurations: one sequence of config 1's model, the latency-bound end of decoding
    "single": Workload("single", 1, 32, 32, 128, 4096, 32, 4, 4, 10000.0, (4, 8), (10.0, 50.0), seed=1005),
}


def head_outliers(w: Workload, layer: int = 0):
    """Per KV head: (channel indices, gains), fixed for a (workload, layer)."""
    rng = np.random.Generator(np.random.PCG64(w.seed * 7919 + layer))
    chans, gains = [], []
    for _ in range(w.n_kv_heads):
        cnt = int(rng.integers(w.outlier_count[0], w.outlier_count[1] + 1))
        chans.append(rng.choice(w.head_dim, size=cnt, replace=False))
        gains.append(rng.uniform(w.outlier_gain[0], w.outlier_gain[1], size=cnt))
    return chans, gains


def make_kv(w: Workload, n_tokens: int, batch: Optional[int] = None, layer: int = 0, stream: int = 0,
            sink_positions=None, offset_variant: bool = False):
    """K, V [batch, n_tokens, n_kv_heads, head_dim] fp16 and the sink mask [batch, n_tokens] uint8.

    `stream` separates independent draws of the same (workload, layer): 0 = the cache contents,
    1 = calibration tokens, 2.. = appended decode tokens.
    """
    B = w.batch if batch is None else batch
    rng = np.random.Generator(np.random.PCG64([w.seed + layer, stream]))
    k = rng.standard_normal((B, n_tokens, w.n_kv_heads, w.head_dim))
    v = rng.standard_normal((B, n_tokens, w.n_kv_heads, w.head_dim))
    chans, gains = head_outliers(w, layer)
    sign_rng = np.random.Generator(np.random.PCG64(w.seed * 31 + layer))
    for h in range(w.n_kv_heads):
        if offset_variant:
            sgn = sign_rng.choice([-1.0, 1.0], size=len(chans[h]))
            k[:, :, h, chans[h]] += sgn * gains[h]
        else:
            k[:, :, h, chans[h]] *= gains[h]
    mask = np.zeros((B, n_tokens), dtype=np.uint8)
    if sink_positions is None:
        sink_positions = list(range(w.n_sinks)) if stream == 0 else []
    for p in sink_positions:
        if 0 <= p < n_tokens:
            k[:, p] *= w.sink_gain
            v[:, p] *= w.sink_gain
            mask[:, p] = 1
    return k.astype(np.float16), v.astype(np.float16), mask


def make_q(w: Workload, batch: Optional[int] = None, layer: int = 0, step: int = 0) -> np.ndarray:
    B = w.batch if batch is None else batch
    rng = np.random.Generator(np.random.PCG64([w.seed + layer, 1_000_003 + step]))
    return rng.standard_normal((B, w.n_q_heads, w.head_dim)).astype(np.float16)


def make_kv_torch(w: Workload, n_tokens: int, device, batch: Optional[int] = None, layer: int = 0, stream: int = 0):
    """Same recipe drawn on the device with torch's generator, for full-size throughput inputs
    (values differ from make_kv; distribution and structure are the same)."""
    import torch
    B = w.batch if batch is None else batch
    g = torch.Generator(device=device)
    g.manual_seed((w.seed + layer) * 1_000_003 + stream)
    shape = (B, n_tokens, w.n_kv_heads, w.head_dim)
    k = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    v = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    chans, gains = head_outliers(w, layer)
    for h in range(w.n_kv_heads):
        idx = torch.as_tensor(np.asarray(chans[h]), device=device, dtype=torch.long)
        gn = torch.as_tensor(np.asarray(gains[h]), device=device, dtype=torch.float32)
        k[:, :, h, idx] *= gn
    mask = torch.zeros((B, n_tokens), dtype=torch.uint8, device=device)
    if stream == 0:
        for p in range(min(w.n_sinks, n_tokens)):
            k[:, p] *= w.sink_gain
            v[:, p] *= w.sink_gain
            mask[:, p] = 1
    return k.to(torch.float16), v.to(torch.float16), mask


def make_q_torch(w: Workload, device, batch: Optional[int] = None, layer: int = 0, step: int = 0):
    import torch
    B = w.batch if batch is None else batch
    g = torch.Generator(device=device)
    g.manual_seed((w.seed + layer) * 1_000_003 + 999_983 + step)
    return torch.randn((B, w.n_q_heads, w.head_dim), generator=g, device=device, dtype=torch.float32).to(torch.float16)
