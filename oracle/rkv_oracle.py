"""RotateKV oracle: a plain, slow, float64 CPU statement of what the hot path computes.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module; only the
test-suite, the smoke check and the benchmark's CPU-baseline leg call it.  It shares no code,
tables or helpers with the HIP library and imports nothing from the package.

Every function follows a passage of the paper (arXiv 2501.16383) and says which one.  The method
is a lossy encoding, so the write half (rotate, reorder, quantize) is the algorithm's steps in the
paper's order; the read half ends in the textbook attention of Eq. 5, evaluated on the
dequantized, inverse-reordered, inverse-rotated, RoPE'd keys.  No blocking, fusion or reordering
of steps: rotations are explicit dense matrix products with the Walsh-Hadamard matrix built from
its recursion (Eq. 10), everything in float64.

Conventions shared by all functions
  * a token's keys (values) are a row of E = n_kv_heads * head_dim channels, head-major
    (the reshape of Alg. 1 step 2);
  * a rotation group is `rot_heads` consecutive KV heads, n = rot_heads * head_dim channels
    (Sec. 4.2, grouped-head rotation);
  * `perm` P is an index vector over the E rotated channels, z[i] = y[P[i]]: position i of the
    reordered row takes rotated channel P[i] (Sec. 4.1);
  * quantization is per token, in blocks of `quant_group` consecutive reordered channels
    (Sec. 5.1, quantization settings), Eq. 6-9 with round-half-to-even and no clipping;
  * scale is stored in fp16 and the stored value is the one used to quantize, so that the write
    and the read agree; zero-point is an integer kept in fp16 (|zero| <= 2048).  16 + 16 bits of
    metadata per 128 two-bit codes is the 2.25 average bits of Table `tab:gsm8k`.
  * meta_format = 1 is the storage named in Sec. 5.1 (quantization settings) and the last row of
    Table `tab:ablation`: scale in FP8, zero-point in INT8, 2.125 average bits.  The paper names
    neither the FP8 flavour nor the rounding; here it is E4M3 (the OCP format with 448 as its
    largest number) and the scale is rounded UP to the next representable number, so that
    2^bits - 1 steps still cover the block's range and the half-step error bound of the rounding
    in Eq. 6 holds with the stored scale.  Zero-points beyond the INT8 range are clamped.

Parity pins: tests/test_oracle_*.py.  Unpinned (needs real model keys, absent here): the
absolute reconstruction-MSE values of Table `tab:quantizeerror`; only their ordering is checked.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

F16_MAX = 65504.0
ZERO_LIMIT = 2048.0
E4M3_MAX = 448.0


@dataclass
class OracleConfig:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int = 128
    rot_heads: int = 4
    quant_group: int = 128
    bits: int = 2
    perm_span: int = 128
    rope_style: int = 0          # 0: pairs (j, j + d/2); 1: pairs (2j, 2j + 1)
    v_rotate: int = 0            # 1: per-head Hadamard on V before quantization
    rope_theta: float = 10000.0
    max_sinks: int = 4
    meta_format: int = 0         # 0: fp16 scale + fp16 zero; 1: FP8 (E4M3) scale + INT8 zero

    @property
    def E(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def n(self) -> int:
        return self.rot_heads * self.head_dim


# --------------------------------------------------------------------------------------------
# Hadamard matrix and rotation (Sec. 3.3, Eq. 10; Sec. 4.2 grouped-head rotation)
# --------------------------------------------------------------------------------------------

def hadamard(n: int) -> np.ndarray:
    """Walsh-Hadamard matrix of order n by the recursion of Eq. 10 (1/sqrt(2) per level)."""
    if n < 1 or (n & (n - 1)) != 0:
        raise ValueError("order must be a power of two")
    H = np.array([[1.0]])
    while H.shape[0] < n:
        H = np.block([[H, H], [H, -H]]) / np.sqrt(2.0)
    return H


def rotate_groups(x: np.ndarray, n: int) -> np.ndarray:
    """y_r = H_n x_r for every block r of n consecutive channels of the last axis (Sec. 4.2)."""
    x = np.asarray(x, dtype=np.float64)
    E = x.shape[-1]
    if E % n != 0:
        raise ValueError("rotation size must divide the row")
    H = hadamard(n)
    y = np.empty_like(x)
    for r in range(E // n):
        y[..., r * n:(r + 1) * n] = x[..., r * n:(r + 1) * n] @ H.T
    return y


# --------------------------------------------------------------------------------------------
# Reorder (Sec. 4.1) and its calibration (Alg. 1)
# --------------------------------------------------------------------------------------------

def reorder(y: np.ndarray, perm: np.ndarray) -> np.ndarray:
    """z[..., i] = y[..., P[i]]."""
    return np.asarray(y)[..., np.asarray(perm)]


def reorder_inverse(z: np.ndarray, perm: np.ndarray) -> np.ndarray:
    """y[..., P[i]] = z[..., i]."""
    z = np.asarray(z)
    y = np.empty_like(z)
    y[..., np.asarray(perm)] = z
    return y


def calibrate_perm(k_cal: np.ndarray, cfg: OracleConfig) -> np.ndarray:
    """Alg. 1: rotate the calibration keys, sum every channel over all tokens (signed), argsort.

    k_cal: [n_tok, n_kv_heads, head_dim].  The sort is ascending and stable, and is taken inside
    each block of `perm_span` channels (perm_span = E is the algorithm as printed).
    """
    E = cfg.E
    rows = np.asarray(k_cal, dtype=np.float64).reshape(-1, E)
    rotated = rotate_groups(rows, cfg.n)            # the algorithm's input: keys already rotated
    channel_sum = rotated.sum(axis=0)               # step 3
    perm = np.empty(E, dtype=np.int32)
    span = cfg.perm_span
    if E % span != 0:
        raise ValueError("perm_span must divide the row")
    for s in range(E // span):
        block = channel_sum[s * span:(s + 1) * span]
        perm[s * span:(s + 1) * span] = np.argsort(block, kind="stable") + s * span   # step 4
    return perm


# --------------------------------------------------------------------------------------------
# Quantizer (Sec. 3.2, Eq. 6-9)
# --------------------------------------------------------------------------------------------

def _to_f16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest fp16 (ties to even), returned as float64."""
    with np.errstate(over="ignore"):
        return np.asarray(x, dtype=np.float64).astype(np.float16).astype(np.float64)


def e4m3_values() -> np.ndarray:
    """The 127 non-negative finite numbers of FP8 E4M3 in ascending order, from the format's
    definition: 1 sign, 4 exponent bits (bias 7), 3 mantissa bits; exponent field 0 holds the
    subnormals m * 2^-9; the all-ones pattern is NaN, so the largest number is 1.75 * 2^8 = 448."""
    vals = []
    for code in range(0x7F):
        e, m = code >> 3, code & 7
        vals.append(m * 2.0 ** -9 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7))
    return np.array(vals)


def _to_e4m3_up(x: np.ndarray) -> np.ndarray:
    """Smallest E4M3 number >= x (x >= 0), saturating at 448; returned as float64."""
    tab = e4m3_values()
    x = np.asarray(x, dtype=np.float64)
    idx = np.searchsorted(tab, x, side="left")
    return tab[np.minimum(idx, len(tab) - 1)]


def quantize(z: np.ndarray, group: int = 128, bits: int = 2, meta_format: int = 0):
    """Eq. 6, 8, 9 on blocks of `group` consecutive elements of the last axis.

    Returns (codes uint8 [..., C], scale float64 [..., C/group], zero float64 [..., C/group]).
    scale = (max - min) / (2^bits - 1) rounded to fp16 and clamped to the fp16 range;
    zero = -round(min / scale) clamped to +-2048; code = clamp(round(x / scale) + zero, 0, 2^bits-1).
    A block whose scale rounds to 0 (constant block, or a range below fp16's smallest number)
    takes scale = fp16(|min|), or 1 if that is 0 too: every code is then 0 and the block
    reconstructs to its own (fp16-rounded) constant.

    meta_format = 1: scale = the same quotient rounded up to the next E4M3 number (at most 448; a
    positive range never rounds to 0, so only a constant block takes the |min| rule, with |min|
    rounded up the same way), zero clamped to the INT8 range -128 .. 127.
    """
    z = np.asarray(z, dtype=np.float64)
    C = z.shape[-1]
    if C % group != 0:
        raise ValueError("group must divide the row")
    qmax = float(2 ** bits - 1)
    blocks = z.reshape(z.shape[:-1] + (C // group, group))
    mn = blocks.min(axis=-1)
    mx = blocks.max(axis=-1)
    if meta_format == 1:
        scale = _to_e4m3_up((mx - mn) / qmax)                         # Eq. 8, stored in FP8
        alt = _to_e4m3_up(np.abs(mn))
        zlo, zhi = -128.0, 127.0
    else:
        scale = np.minimum(_to_f16((mx - mn) / qmax), F16_MAX)        # Eq. 8, stored in fp16
        alt = np.minimum(_to_f16(np.abs(mn)), F16_MAX)
        zlo, zhi = -ZERO_LIMIT, ZERO_LIMIT
    degenerate = scale == 0.0
    alt = np.where(alt == 0.0, 1.0, alt)
    scale = np.where(degenerate, alt, scale)
    zero = np.clip(-np.rint(mn / scale), zlo, zhi)                     # Eq. 9
    q = np.rint(blocks / scale[..., None]) + zero[..., None]           # Eq. 6
    codes = np.clip(q, 0.0, qmax).astype(np.uint8)
    return codes.reshape(z.shape), scale, zero + 0.0


def dequantize(codes: np.ndarray, scale: np.ndarray, zero: np.ndarray, group: int = 128) -> np.ndarray:
    """Eq. 7: x' = scale * (code - zero)."""
    codes = np.asarray(codes)
    C = codes.shape[-1]
    blocks = codes.reshape(codes.shape[:-1] + (C // group, group)).astype(np.float64)
    x = np.asarray(scale)[..., None] * (blocks - np.asarray(zero)[..., None])
    return x.reshape(codes.shape)


def pack_canonical(codes: np.ndarray, bits: int = 2) -> np.ndarray:
    """Canonical byte image of a logical code array: byte k holds codes 4k..4k+3, code 4k+r in
    bits [2r, 2r+1]; 3- and 4-bit codes take a nibble each, byte k holding code 2k in its low and
    code 2k+1 in its high nibble.  (The packing is not fixed by the paper; this is the reference
    image that a physical layout must be a documented bijection of.)"""
    c = np.asarray(codes, dtype=np.uint8)
    if bits in (3, 4):
        c2 = c.reshape(c.shape[:-1] + (c.shape[-1] // 2, 2))
        return (c2[..., 0] | (c2[..., 1] << 4)).astype(np.uint8)
    if bits != 2:
        raise ValueError("canonical packing is defined for 2-, 3- and 4-bit codes")
    c4 = c.reshape(c.shape[:-1] + (c.shape[-1] // 4, 4))
    return (c4[..., 0] | (c4[..., 1] << 2) | (c4[..., 2] << 4) | (c4[..., 3] << 6)).astype(np.uint8)


def unpack_canonical(packed: np.ndarray, bits: int = 2) -> np.ndarray:
    p = np.asarray(packed, dtype=np.uint8)
    if bits in (3, 4):
        out = np.stack([p & 15, p >> 4], axis=-1)
        return out.reshape(p.shape[:-1] + (p.shape[-1] * 2,)).astype(np.uint8)
    out = np.stack([(p >> (2 * r)) & 3 for r in range(4)], axis=-1)
    return out.reshape(p.shape[:-1] + (p.shape[-1] * 4,)).astype(np.uint8)


# --------------------------------------------------------------------------------------------
# RoPE (Sec. 4.2: it acts on channel pairs; the cache holds pre-RoPE keys)
# --------------------------------------------------------------------------------------------

def rope(x: np.ndarray, pos: np.ndarray, theta: float, style: int = 0) -> np.ndarray:
    """Rotate channel pairs of the last axis (one head, d channels) by pos * theta^(-2j/d).

    x: [..., d]; pos broadcastable to x.shape[:-1] (0-based token index).
    style 0 pairs channel j with j + d/2; style 1 pairs 2j with 2j + 1.
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    half = d // 2
    j = np.arange(half, dtype=np.float64)
    freq = theta ** (-2.0 * j / d)
    ang = np.asarray(pos, dtype=np.float64)[..., None] * freq
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    if style == 0:
        a, b = x[..., :half], x[..., half:]
        out[..., :half] = a * c - b * s
        out[..., half:] = a * s + b * c
    else:
        a, b = x[..., 0::2], x[..., 1::2]
        out[..., 0::2] = a * c - b * s
        out[..., 1::2] = a * s + b * c
    return out


# --------------------------------------------------------------------------------------------
# Attention-sink selection (Fig. 3 caption, Sec. 4.3)
# --------------------------------------------------------------------------------------------

def select_sinks(block_output: np.ndarray, k: int) -> np.ndarray:
    """Token indices of the k most massive activations of the previous decoder block's output.

    block_output: [T, C].  A token's score is its largest |activation|; ties go to the lower
    index; the result is ascending.
    """
    a = np.abs(np.asarray(block_output, dtype=np.float64)).max(axis=1)
    order = np.lexsort((np.arange(a.shape[0]), -a))
    return np.sort(order[:k]).astype(np.int64)


# --------------------------------------------------------------------------------------------
# The cache: write half (Sec. 4.4) and read half (decoding procedure, Eq. 4-5)
# --------------------------------------------------------------------------------------------

@dataclass
class OracleCache:
    cfg: OracleConfig
    perm: np.ndarray
    length: int = 0
    k_codes: Optional[np.ndarray] = None      # [B, T, E] logical (reordered) order
    k_scale: Optional[np.ndarray] = None      # [B, T, E/group]
    k_zero: Optional[np.ndarray] = None
    v_codes: Optional[np.ndarray] = None
    v_scale: Optional[np.ndarray] = None
    v_zero: Optional[np.ndarray] = None
    k_rot: Optional[np.ndarray] = None        # [B, T, E] rotated + reordered keys before Eq. 6 (for tie analysis)
    v_in: Optional[np.ndarray] = None         # [B, T, E] values entering Eq. 6
    sink_pos: List[List[int]] = field(default_factory=list)          # per sequence
    sink_k: List[List[np.ndarray]] = field(default_factory=list)     # per sequence, rows [Hkv, d] fp16 values
    sink_v: List[List[np.ndarray]] = field(default_factory=list)


def cache_new(cfg: OracleConfig, perm: Optional[np.ndarray] = None) -> OracleCache:
    E = cfg.E
    if perm is None:
        perm = np.arange(E, dtype=np.int32)
    perm = np.asarray(perm, dtype=np.int64)
    if sorted(perm.tolist()) != list(range(E)):
        raise ValueError("perm is not a permutation")
    span = cfg.perm_span
    if np.any(perm // span != np.arange(E) // span):
        raise ValueError("perm crosses a perm_span block")
    B = cfg.batch
    return OracleCache(cfg=cfg, perm=perm, sink_pos=[[] for _ in range(B)],
                       sink_k=[[] for _ in range(B)], sink_v=[[] for _ in range(B)])


def _cat(a, b):
    return b if a is None else np.concatenate([a, b], axis=1)


def fold_rotation(w: np.ndarray, cfg: OracleConfig, perm: Optional[np.ndarray] = None) -> np.ndarray:
    """Offline folding of the key rotation and reorder into a projection (Sec. 4.2, Sec. 4.4).

    w: [rows, E], the key projection with the E output channels along the last axis, so that
    keys = x @ w.  Returns w' with x @ w' = reorder(rotate(x @ w)): rotation and reorder are
    linear maps on the output channels, so they act on every row of w.  (For the value rotation
    call it with rot_heads = 1 and no perm.)
    """
    w = np.asarray(w, dtype=np.float64)
    out = rotate_groups(w, cfg.n)
    if perm is not None:
        out = reorder(out, np.asarray(perm))
    return out


def quantize_append(cache: OracleCache, k: np.ndarray, v: np.ndarray,
                    sink_mask: Optional[np.ndarray] = None, keys_rotated: bool = False) -> None:
    """Write half.  k, v: [B, n_new, Hkv, d] holding fp16 values, keys pre-RoPE.

    keys_rotated: the keys come from a projection with the rotation and the reorder folded in
    (fold_rotation), i.e. they already are what enters Eq. 6; a retained sink row is then brought
    back to the original basis (inverse reorder, the same rotation again) and rounded to fp16.

    Keys: grouped-head rotation, then reorder, then Eq. 6-9 per token per block (Sec. 4.1-4.2,
    Table `tab:smooth`: rotate first, reorder second).  Values: optional per-head rotation, then
    the same quantizer, no reorder (Sec. 4.4).  Tokens flagged in sink_mask keep their original
    fp16 rows (Sec. 4.3) while the sequence has fewer than max_sinks of them; later flagged
    tokens are treated as ordinary tokens.  Every token, flagged or not, also gets codes so that
    slots stay aligned; the read half ignores the codes of retained sinks.
    """
    cfg = cache.cfg
    B, n_new = k.shape[0], k.shape[1]
    E = cfg.E
    k16 = np.asarray(k, dtype=np.float16)
    v16 = np.asarray(v, dtype=np.float16)
    x = k16.astype(np.float64).reshape(B, n_new, E)
    if keys_rotated:
        z = x
        k_orig = rotate_groups(reorder_inverse(z, cache.perm), cfg.n)
        k_sink16 = k_orig.astype(np.float16).reshape(k16.shape)
    else:
        y = rotate_groups(x, cfg.n)
        z = reorder(y, cache.perm)
        k_sink16 = k16
    kc, ks, kz = quantize(z, cfg.quant_group, cfg.bits, cfg.meta_format)
    u = v16.astype(np.float64).reshape(B, n_new, E)
    if cfg.v_rotate:
        u = rotate_groups(u, cfg.head_dim)
    vc, vs, vz = quantize(u, cfg.quant_group, cfg.bits, cfg.meta_format)
    if sink_mask is not None:
        m = np.asarray(sink_mask).astype(bool)
        for b in range(B):
            for t in range(n_new):
                if m[b, t] and len(cache.sink_pos[b]) < cfg.max_sinks:
                    cache.sink_pos[b].append(cache.length + t)
                    cache.sink_k[b].append(k_sink16[b, t].copy())
                    cache.sink_v[b].append(v16[b, t].copy())
    cache.k_codes, cache.k_scale, cache.k_zero = _cat(cache.k_codes, kc), _cat(cache.k_scale, ks), _cat(cache.k_zero, kz)
    cache.v_codes, cache.v_scale, cache.v_zero = _cat(cache.v_codes, vc), _cat(cache.v_scale, vs), _cat(cache.v_zero, vz)
    cache.k_rot, cache.v_in = _cat(cache.k_rot, z), _cat(cache.v_in, u)
    cache.length += n_new


def dequantize_cache(cache: OracleCache, substitute_sinks: bool = False):
    """Reconstructed keys and values in the original basis, keys pre-RoPE: [B, T, Hkv, d].

    Keys: Eq. 7, inverse reorder, then the same grouped rotation again (H is symmetric and
    orthogonal, so it is its own inverse) - the two online steps that Sec. 4.4 undoes before
    attention.  Values: Eq. 7, and the per-head rotation undone when v_rotate is set.
    """
    cfg = cache.cfg
    B, T, E = cache.k_codes.shape
    zq = dequantize(cache.k_codes, cache.k_scale, cache.k_zero, cfg.quant_group)
    yq = reorder_inverse(zq, cache.perm)
    k_hat = rotate_groups(yq, cfg.n).reshape(B, T, cfg.n_kv_heads, cfg.head_dim)
    v_hat = dequantize(cache.v_codes, cache.v_scale, cache.v_zero, cfg.quant_group)
    if cfg.v_rotate:
        v_hat = rotate_groups(v_hat, cfg.head_dim)
    v_hat = v_hat.reshape(B, T, cfg.n_kv_heads, cfg.head_dim)
    if substitute_sinks:
        for b in range(B):
            for pos, kr, vr in zip(cache.sink_pos[b], cache.sink_k[b], cache.sink_v[b]):
                k_hat[b, pos] = kr.astype(np.float64)
                v_hat[b, pos] = vr.astype(np.float64)
    return k_hat, v_hat


def decode_attention(cache: OracleCache, q: np.ndarray, q_pos: Optional[np.ndarray] = None,
                     k_cur: Optional[np.ndarray] = None, v_cur: Optional[np.ndarray] = None):
    """Read half: Eq. 5 over the cache as stored.

    k_cur, v_cur ([B, Hkv, d] fp16 values, key pre-RoPE), if given, are the token being decoded,
    not yet in the cache: it is attended in full precision at position T (the decoding procedure
    that concatenates the new key and value to the dequantized cache before quantizing them);
    q_pos then defaults to T.

    q: [B, Hq, d] fp16 values, pre-RoPE.  Keys are reconstructed (dequantize_cache), retained
    sink rows replace their reconstructions, RoPE is applied to every key at its token index and
    to the query at q_pos (default: last cached index), and
        out = softmax(q~ . K~^T / sqrt(d)) . V
    per query head; query head h reads KV head h // (Hq / Hkv).
    Returns (out [B, Hq, d], lse [B, Hq]) in float64.
    """
    cfg = cache.cfg
    B, T = cache.k_codes.shape[0], cache.length
    d = cfg.head_dim
    k_hat, v_hat = dequantize_cache(cache, substitute_sinks=True)
    if k_cur is not None:
        kc = np.asarray(k_cur, dtype=np.float16).astype(np.float64).reshape(B, 1, cfg.n_kv_heads, d)
        vc = np.asarray(v_cur, dtype=np.float16).astype(np.float64).reshape(B, 1, cfg.n_kv_heads, d)
        k_hat = np.concatenate([k_hat, kc], axis=1)
        v_hat = np.concatenate([v_hat, vc], axis=1)
        T = T + 1
    if q_pos is None:
        q_pos = np.full(B, T - 1, dtype=np.int64)
    q_pos = np.asarray(q_pos, dtype=np.int64)
    qf = np.asarray(q, dtype=np.float16).astype(np.float64)
    rep = cfg.n_q_heads // cfg.n_kv_heads
    out = np.empty((B, cfg.n_q_heads, d))
    lse = np.empty((B, cfg.n_q_heads))
    tpos = np.arange(T)
    for b in range(B):
        for h in range(cfg.n_q_heads):
            kv = h // rep
            q_r = rope(qf[b, h], q_pos[b], cfg.rope_theta, cfg.rope_style)
            k_r = rope(k_hat[b, :, kv, :], tpos, cfg.rope_theta, cfg.rope_style)
            s = (k_r @ q_r) / np.sqrt(float(d))
            m = s.max()
            p = np.exp(s - m)
            l = p.sum()
            out[b, h] = (p / l) @ v_hat[b, :, kv, :]
            lse[b, h] = m + np.log(l)
    return out, lse


def decode_attention_multi(cache: OracleCache, q: np.ndarray, q_pos: np.ndarray):
    """Several query tokens per sequence in one step (speculative or chunked decoding): query i of
    sequence b sits at position q_pos[b, i] and attends the cached tokens 0 .. q_pos[b, i] - Eq. 5
    with the causal mask of the decoding phase.  q: [B, nq, Hq, d]; returns (out [B, nq, Hq, d],
    lse [B, nq, Hq]).  Each query is one single-query read of the cache cut at its position (a
    position past the last cached token sees the whole cache and only sets the RoPE angle).
    """
    cfg = cache.cfg
    q = np.asarray(q)
    q_pos = np.asarray(q_pos, dtype=np.int64)
    B, nq = q.shape[0], q.shape[1]
    out = np.empty((B, nq, cfg.n_q_heads, cfg.head_dim))
    lse = np.empty((B, nq, cfg.n_q_heads))
    for b in range(B):
        for i in range(nq):
            T = min(int(q_pos[b, i]) + 1, cache.length)
            cut = OracleCache(cfg=OracleConfig(**{**cfg.__dict__, "batch": 1}), perm=cache.perm, length=T)
            for name in ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero"):
                setattr(cut, name, getattr(cache, name)[b:b + 1, :T])
            keep = [s for s, pos in enumerate(cache.sink_pos[b]) if pos < T]
            cut.sink_pos = [[cache.sink_pos[b][s] for s in keep]]
            cut.sink_k = [[cache.sink_k[b][s] for s in keep]]
            cut.sink_v = [[cache.sink_v[b][s] for s in keep]]
            o, l = decode_attention(cut, q[b:b + 1, i], np.array([q_pos[b, i]]))
            out[b, i], lse[b, i] = o[0], l[0]
    return out, lse


def average_bits(cfg: OracleConfig) -> float:
    """Stored bits per cached element: codes plus the scale and the zero-point of each block (fp16
    each, or FP8 and INT8 with meta_format = 1)."""
    return cfg.bits + (16.0 if cfg.meta_format == 1 else 32.0) / cfg.quant_group
