"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without the GPU.

Each test is chosen so that a plausible slip in oracle/rkv_oracle.py (a dropped term, a wrong
sign or index, a transposed operand, the wrong order of rotate and reorder) fails at least one.
"""
import itertools
import os

import numpy as np
import pytest
import scipy.linalg

from oracle import rkv_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                out.append(line.split())
    return out


# ----------------------------------------------------------------------------- Hadamard (Eq. 10)

@pytest.mark.parametrize("n", [1, 2, 4, 128, 256, 512])
def test_hadamard_closed_form_and_library(n):
    H = O.hadamard(n)
    i = np.arange(n)
    pop = np.array([[bin(a & b).count("1") for b in i] for a in i])
    closed = (-1.0) ** pop / np.sqrt(n)
    assert np.allclose(H, closed, atol=1e-15)
    assert np.allclose(H, scipy.linalg.hadamard(n) / np.sqrt(n), atol=1e-15)


@pytest.mark.parametrize("n", [2, 128, 512])
def test_hadamard_orthogonal_symmetric_self_inverse(n):
    H = O.hadamard(n)
    assert np.array_equal(H, H.T)
    assert np.allclose(H @ H, np.eye(n), atol=1e-12)
    Hi = np.rint(H * np.sqrt(n)).astype(np.int64)          # un-normalised: exactly n*I in integers
    assert np.array_equal(Hi @ Hi, n * np.eye(n, dtype=np.int64))
    e0 = np.zeros(n)
    e0[0] = 1.0
    assert np.allclose(H @ e0, 1.0 / np.sqrt(n))


def test_rotation_parseval_and_group_locality():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 1024))
    y = O.rotate_groups(x, 256)
    for r in range(4):
        assert np.allclose((y[:, r * 256:(r + 1) * 256] ** 2).sum(1), (x[:, r * 256:(r + 1) * 256] ** 2).sum(1))
    x2 = x.copy()
    x2[:, 300] += 1.0                         # a change in group 1 must stay in group 1
    d = O.rotate_groups(x2, 256) - y
    assert np.all(d[:, :256] == 0) and np.all(d[:, 512:] == 0) and np.all(np.abs(d[:, 256:512]) > 0)


def _fwht_counting(x):
    """Textbook in-place butterfly FWHT (un-normalised) that counts its additions."""
    x = np.array(x, dtype=np.float64)
    n, h, adds = x.shape[0], 1, 0
    while h < n:
        for i in range(0, n, 2 * h):
            for j in range(i, i + h):
                a, b = x[j], x[j + h]
                x[j], x[j + h] = a + b, a - b
                adds += 2
        h *= 2
    return x, adds


def test_fwht_cost_matches_paper_table():
    """The dense rotation equals a butterfly FWHT whose add count is the table's FLOPs column."""
    rng = np.random.default_rng(1)
    for heads, n, flops in _rows("fwht_flops_per_layer.txt"):
        heads, n, flops = int(heads), int(n), int(flops)
        assert n == heads * 128
        if n <= 1024:
            x = rng.standard_normal(n)
            y, adds = _fwht_counting(x)
            assert np.allclose(y / np.sqrt(n), O.rotate_groups(x[None], n)[0], atol=1e-10)
        else:
            adds = n * int(np.log2(n))
        assert adds * (4096 // n) == flops


# ----------------------------------------------------------------------------- reorder, Alg. 1

def test_reorder_roundtrip_and_direction():
    rng = np.random.default_rng(2)
    P = rng.permutation(64)
    y = rng.standard_normal((5, 64))
    z = O.reorder(y, P)
    for i in range(64):
        assert np.array_equal(z[:, i], y[:, P[i]])
    assert np.array_equal(O.reorder_inverse(z, P), y)


def test_calibrate_bruteforce_tiny():
    """Alg. 1 on a tiny layer, against an O(n^2) rank count; signed sum, ascending, stable."""
    cfg = O.OracleConfig(batch=1, n_q_heads=2, n_kv_heads=2, head_dim=4, rot_heads=2, perm_span=8, quant_group=4)
    rng = np.random.default_rng(3)
    k = rng.standard_normal((6, 2, 4))
    P = O.calibrate_perm(k, cfg)
    H8 = scipy.linalg.hadamard(8) / np.sqrt(8.0)
    sums = sum(H8 @ k[t].reshape(8) for t in range(6))
    rank = [sum(1 for j in range(8) if sums[j] < sums[i] or (sums[j] == sums[i] and j < i)) for i in range(8)]
    expect = np.empty(8, dtype=int)
    for i, r in enumerate(rank):
        expect[r] = i
    assert np.array_equal(P, expect)
    assert sorted(P.tolist()) == list(range(8))
    # sign matters: negating the keys reverses the order of distinct sums
    assert np.array_equal(O.calibrate_perm(-k, cfg), expect[::-1])


def test_calibrate_span_closed_and_stable_ties():
    cfg = O.OracleConfig(batch=1, n_q_heads=4, n_kv_heads=4, head_dim=128, rot_heads=2, perm_span=128)
    rng = np.random.default_rng(4)
    P = O.calibrate_perm(rng.standard_normal((16, 4, 128)), cfg)
    assert sorted(P.tolist()) == list(range(512))
    assert np.array_equal(P // 128, np.arange(512) // 128)
    Pz = O.calibrate_perm(np.zeros((3, 4, 128)), cfg)        # all sums equal: stable => identity
    assert np.array_equal(Pz, np.arange(512))


# ----------------------------------------------------------------------------- quantizer (Eq. 6-9)

def test_quantizer_nearest_level_bruteforce():
    """For every element the chosen code is a nearest reconstruction level among the four."""
    rng = np.random.default_rng(5)
    for trial in range(200):
        g = int(rng.choice([4, 8]))
        x = rng.standard_normal((1, g)) * rng.uniform(0.1, 30) + rng.uniform(-5, 5)
        c, s, z = O.quantize(x, group=g)
        levels = s[0, 0] * (np.arange(4) - z[0, 0])
        for e in range(g):
            dist = np.abs(levels - x[0, e])
            assert dist[c[0, e]] <= dist.min() + 1e-12
        assert c[0, np.argmin(x[0])] == 0 and c[0, np.argmax(x[0])] == 3


def test_quantizer_reproduces_all_grid_patterns():
    """All 4^4 code patterns placed exactly on a grid come back unchanged (Eq. 6 inverts Eq. 7)."""
    s, z = 0.75, 1.0
    for pat in itertools.product(range(4), repeat=4):
        if min(pat) != 0 or max(pat) != 3:
            continue                      # the grid is anchored by the block's own min and max
        x = s * (np.array(pat, dtype=np.float64)[None] - z)
        c, sc, ze = O.quantize(x, group=4)
        assert sc[0, 0] == s and ze[0, 0] == z
        assert tuple(c[0]) == pat
        assert np.array_equal(O.dequantize(c, sc, ze, group=4), x)


def test_quantizer_half_step_bound_and_metadata():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((64, 1024)) * np.exp(rng.uniform(-3, 3, size=(64, 1)))
    c, s, z = O.quantize(x, group=128)
    xh = O.dequantize(c, s, z, group=128)
    step = np.repeat(s, 128, axis=-1)
    assert np.all(np.abs(x - xh) <= 0.5 * step * (1 + 2.0 ** -8))
    assert c.max() == 3 and c.min() == 0
    assert np.array_equal(s.astype(np.float16).astype(np.float64), s)     # scale is an fp16 number
    assert np.array_equal(z, np.rint(z)) and np.abs(z).max() <= 2048
    raw = (x.reshape(64, 8, 128).max(-1) - x.reshape(64, 8, 128).min(-1)) / 3.0
    assert np.all(np.abs(s - raw) <= raw * 2.0 ** -11)                     # nearest fp16 of Eq. 8


def test_quantizer_rounds_half_to_even():
    # scale 1, zero 0: 0.5 -> 0, 1.5 -> 2, 2.5 -> 2
    x = np.array([[0.0, 0.5, 1.5, 2.5, 3.0, 1.0, 2.0, 0.25]])
    c, s, z = O.quantize(x, group=8)
    assert s[0, 0] == 1.0 and z[0, 0] == 0.0
    assert c[0].tolist() == [0, 0, 2, 2, 3, 1, 2, 0]


def test_quantizer_degenerate_blocks():
    for val in [0.0, 2.5, -0.125]:
        x = np.full((1, 8), val)
        c, s, z = O.quantize(x, group=8)
        assert np.all(c == 0)
        assert np.allclose(O.dequantize(c, s, z, group=8), val)
        assert np.isfinite(s).all() and s[0, 0] > 0


def test_fp16_metadata_clamps_written_out_by_hand():
    """The stored zero-point is an integer in an fp16 field: beyond +-2048 fp16 no longer holds
    every integer, so Eq. 9's value is clamped there; the stored scale cannot exceed the largest
    fp16 number 65504.  Expected metadata and codes below are Eq. 6, 8, 9 worked by hand."""
    # range 0.3 at offset 1000: Eq. 8 gives 0.1 -> fp16 0.0999755859375; Eq. 9 gives
    # -rint(1000 / 0.09998) = -10002, stored as -2048; Eq. 6: rint(x / s) - 2048 > 3 for every x -> 3
    x = np.array([[1000.0, 1000.1, 1000.2, 1000.3]])
    c, s, z = O.quantize(x, group=4)
    assert s[0, 0] == float(np.float16(0.1)) == 0.0999755859375
    assert z[0, 0] == -2048.0
    assert c[0].tolist() == [3, 3, 3, 3]
    # the mirror image: Eq. 9 gives +10005 (-1000.3 / s = -10005.4), stored as +2048; codes clamp to 0
    c, s, z = O.quantize(-x, group=4)
    assert s[0, 0] == 0.0999755859375 and z[0, 0] == 2048.0
    assert c[0].tolist() == [0, 0, 0, 0]
    # just inside the limit nothing is clamped: min -204.6, range 0.3 -> zero = rint(204.6 / s) = 2046
    y = np.array([[-204.6, -204.5, -204.4, -204.3]])
    c, s, z = O.quantize(y, group=4)
    assert z[0, 0] == 2046.0 == np.rint(204.6 / 0.0999755859375)
    assert c[0].tolist() == [0, 1, 2, 3]
    # range 300000: Eq. 8 gives 100000, beyond fp16 -> stored 65504; Eq. 9: -rint(-150000 / 65504) = 2;
    # Eq. 6: rint(x / 65504) + 2 = 0, 2, 3, 4 -> 0, 2, 3, 3
    w = np.array([[-150000.0, 0.0, 60000.0, 150000.0]])
    c, s, z = O.quantize(w, group=4)
    assert s[0, 0] == 65504.0 and z[0, 0] == 2.0
    assert c[0].tolist() == [0, 2, 3, 3]
    assert np.all(np.isfinite(O.dequantize(c, s, z, group=4)))
    # the largest range that needs no clamp: 3 * 65504
    # (x / s = -1.5, -0.61, 0.61, 1.5; halves go to the even neighbour: -2, -1, 1, 2; plus zero = 2)
    w = np.array([[-98256.0, -40000.0, 40000.0, 98256.0]])
    c, s, z = O.quantize(w, group=4)
    assert s[0, 0] == 65504.0 and z[0, 0] == 2.0 and c[0].tolist() == [0, 1, 3, 3]


def test_pack_roundtrip_all_bytes():
    allb = np.arange(256, dtype=np.uint8)
    codes = O.unpack_canonical(allb[None])
    assert codes.shape == (1, 1024) and codes.max() == 3
    assert np.array_equal(O.pack_canonical(codes)[0], allb)
    assert O.pack_canonical(np.array([[1, 0, 0, 0, 0, 2, 0, 0, 0, 0, 0, 3]], dtype=np.uint8))[0].tolist() == [1, 8, 192]
    # wider codes: a nibble each, the even-numbered code in the low one
    nib = O.unpack_canonical(allb[None], bits=4)
    assert nib.shape == (1, 512) and nib.max() == 15 and nib[0, :6].tolist() == [0, 0, 1, 0, 2, 0]
    assert np.array_equal(O.pack_canonical(nib, bits=4)[0], allb)
    assert O.pack_canonical(np.array([[7, 1, 0, 5]], dtype=np.uint8), bits=3)[0].tolist() == [0x17, 0x50]


def test_average_bits_matches_paper():
    (val,), = _rows("average_bits.txt")
    cfg = O.OracleConfig(batch=1, n_q_heads=32, n_kv_heads=32)
    assert O.average_bits(cfg) == float(val)
    # and from the stored arrays themselves
    rng = np.random.default_rng(7)
    c, s, z = O.quantize(rng.standard_normal((4, 4096)), group=128)
    bits = O.pack_canonical(c).size * 8 + (s.size + z.size) * 16
    assert bits / c.size == float(val)


# ----------------------------------------------------------------------------- 3- and 4-bit codes, groups of 64 and 32 (Sec. 5.1; Tables tab:ablation, tab:quantgrani)

@pytest.mark.parametrize("bits", [3, 4])
def test_wider_codes_nearest_level_bruteforce(bits):
    """Every element takes a nearest of the 2^bits reconstruction levels; the block's minimum and
    maximum take the first and the last code."""
    rng = np.random.default_rng(70 + bits)
    top = 2 ** bits - 1
    for trial in range(200):
        g = int(rng.choice([4, 8, 32]))
        x = rng.standard_normal((1, g)) * rng.uniform(0.1, 30) + rng.uniform(-5, 5)
        c, s, z = O.quantize(x, group=g, bits=bits)
        levels = s[0, 0] * (np.arange(top + 1) - z[0, 0])
        dist = np.abs(levels[None, :] - x[0][:, None])
        assert np.all(dist[np.arange(g), c[0]] <= dist.min(axis=1) + 1e-12)
        assert c[0, np.argmin(x[0])] == 0 and c[0, np.argmax(x[0])] == top


@pytest.mark.parametrize("bits", [3, 4])
def test_wider_codes_reproduce_grid_patterns(bits):
    """Code patterns placed exactly on a grid with 2^bits levels come back unchanged, with the
    grid's own step and zero-point as metadata."""
    rng = np.random.default_rng(80 + bits)
    top = 2 ** bits - 1
    s, z = 0.375, 5.0
    for trial in range(300):
        pat = rng.integers(0, top + 1, size=8)
        pat[rng.integers(0, 4)] = 0
        pat[4 + rng.integers(0, 4)] = top
        x = s * (pat.astype(np.float64)[None] - z)
        c, sc, ze = O.quantize(x, group=8, bits=bits)
        assert sc[0, 0] == s and ze[0, 0] == z
        assert np.array_equal(c[0], pat)
        assert np.array_equal(O.dequantize(c, sc, ze, group=8), x)


@pytest.mark.parametrize("bits,group", [(2, 64), (2, 32), (3, 128), (3, 64), (4, 128), (4, 32)])
def test_wider_codes_and_smaller_groups_error_law(bits, group):
    """Half-step bound per element with the block's own stored step = fp16(range / (2^bits - 1));
    on uniformly distributed data the rounding error is uniform over one step, so its mean square
    is step^2 / 12."""
    rng = np.random.default_rng(90 + bits + group)
    top = 2 ** bits - 1
    # a random offset per block, so that the grid (anchored at an integer zero-point) sits anywhere
    # relative to the block's minimum
    x = (rng.uniform(-1.0, 1.0, size=(256, 1024)) + np.repeat(rng.uniform(-3, 3, size=(256, 1024 // group)), group, axis=-1))
    x = x * np.exp(rng.uniform(-2, 2, size=(256, 1)))
    c, s, z = O.quantize(x, group=group, bits=bits)
    assert s.shape == (256, 1024 // group) and z.shape == s.shape
    assert c.max() == top and c.min() == 0
    xh = O.dequantize(c, s, z, group=group)
    step = np.repeat(s, group, axis=-1)
    # the stored step is the exact one within 2^-11; over 2^bits - 1 steps that moves the top level
    assert np.all(np.abs(x - xh) <= step * (0.5 + top * 2.0 ** -11 + 1e-12))
    blocks = x.reshape(256, 1024 // group, group)
    raw = (blocks.max(-1) - blocks.min(-1)) / top
    assert np.all(np.abs(s - raw) <= raw * 2.0 ** -11)
    ratio = np.mean(((x - xh) / step) ** 2) * 12.0
    assert 0.96 <= ratio <= 1.04


def test_average_bits_of_the_wider_settings():
    """Codes plus 16 + 16 bits of metadata per block: 4.25 and 3.25 bits at group 128, 2.5 and 3
    bits for 2-bit codes at groups 64 and 32 (half of it with 8 + 8 bits of metadata)."""
    base = dict(batch=1, n_q_heads=32, n_kv_heads=32)
    want = {(4, 128, 0): 4.25, (3, 128, 0): 3.25, (2, 64, 0): 2.5, (2, 32, 0): 3.0, (4, 32, 0): 5.0,
            (4, 128, 1): 4.125, (2, 64, 1): 2.25, (3, 32, 1): 3.5}
    for (bits, group, mf), val in want.items():
        cfg = O.OracleConfig(bits=bits, quant_group=group, meta_format=mf, **base)
        assert O.average_bits(cfg) == val
        c, s, z = O.quantize(np.random.default_rng(3).standard_normal((2, 4096)), group=group, bits=bits, meta_format=mf)
        assert (c.size * bits + (s.size + z.size) * (8 if mf else 16)) / c.size == val


@pytest.mark.parametrize("bits,group", [(4, 128), (3, 64), (2, 32)])
def test_cache_with_wider_codes_and_smaller_groups(bits, group):
    """The cache carries bits and group through the write and the read half: metadata shapes,
    code range, half-step bound in the rotated and reordered basis, the read half equal to textbook
    attention over the reconstructed cache, and reconstructions of keys and values closer to the
    originals than the 2-bit, group-128 cache's."""
    rng = np.random.default_rng(95)
    k = rng.standard_normal((2, 48, 4, 128)).astype(np.float16)
    k[..., 7] *= 12.0                                              # an outlier channel in every head
    v = rng.standard_normal((2, 48, 4, 128)).astype(np.float16)
    q = rng.standard_normal((2, 4, 128)).astype(np.float16)
    outs = {}
    for name, (b_, g_) in {"base": (2, 128), "this": (bits, group)}.items():
        cfg = O.OracleConfig(batch=2, n_q_heads=4, n_kv_heads=4, rot_heads=2, max_sinks=0, bits=b_, quant_group=g_)
        c = O.cache_new(cfg)
        O.quantize_append(c, k, v)
        assert c.k_scale.shape == (2, 48, 512 // g_) and c.v_zero.shape == (2, 48, 512 // g_)
        assert c.k_codes.max() == 2 ** b_ - 1 and c.v_codes.max() == 2 ** b_ - 1
        zq = O.dequantize(c.k_codes, c.k_scale, c.k_zero, g_)
        assert np.all(np.abs(zq - c.k_rot) <= np.repeat(c.k_scale, g_, axis=-1) * (0.5 + (2 ** b_ - 1) * 2.0 ** -11 + 1e-12))
        k_hat, v_hat = O.dequantize_cache(c)
        out, _ = O.decode_attention(c, q)
        ref = _textbook_attention(q.astype(np.float64), k_hat, v_hat, np.array([47, 47]), 10000.0, 1)
        assert np.abs(out - ref).max() <= 1e-9
        outs[name] = (np.mean((k_hat - k.astype(np.float64)) ** 2), np.mean((v_hat - v.astype(np.float64)) ** 2))
    assert outs["this"][0] < 0.8 * outs["base"][0] and outs["this"][1] < 0.8 * outs["base"][1]


# ----------------------------------------------------------------------------- FP8 scale + INT8 zero (Sec. 5.1, Table tab:ablation last row)

def test_e4m3_table_matches_the_library_format():
    """The oracle's table, built from the format's definition, against torch's float8_e4m3fn
    decoding of the same bit patterns (a library routine the oracle does not use)."""
    import torch
    tab = O.e4m3_values()
    lib = torch.arange(0, 127, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(tab, lib)
    assert tab[0] == 0.0 and tab[1] == 2.0 ** -9 and tab[-1] == 448.0 and np.all(np.diff(tab) > 0)
    assert bool(torch.isnan(torch.tensor([0x7F], dtype=torch.uint8).view(torch.float8_e4m3fn).float()).all())


def test_fp8_scale_is_the_quotient_rounded_up():
    rng = np.random.default_rng(60)
    x = rng.standard_normal((64, 1024)) * np.exp(rng.uniform(-4, 4, size=(64, 1)))
    c, s, z = O.quantize(x, group=128, meta_format=1)
    tab = O.e4m3_values()
    raw = (x.reshape(64, 8, 128).max(-1) - x.reshape(64, 8, 128).min(-1)) / 3.0
    idx = np.searchsorted(tab, s)
    assert np.array_equal(tab[idx], s)                                # an E4M3 number ...
    assert np.all(s >= raw) and np.all(tab[idx - 1] < raw)            # ... the smallest one that covers the range
    assert np.all(s <= raw * 1.125 + 2.0 ** -9)                       # at most one 3-bit-mantissa step above
    assert np.array_equal(z, np.rint(z)) and z.min() >= -128 and z.max() <= 127
    xh = O.dequantize(c, s, z, group=128)
    assert np.all(np.abs(x - xh) <= 0.5 * np.repeat(s, 128, axis=-1) * (1 + 1e-12))     # half-step bound, stored scale
    assert c.min() == 0 and c.max() == 3
    # the block minimum always takes code 0; the maximum 3, or 2 when the scale was rounded up far enough
    blocks_c = c.reshape(64, 8, 128)
    am, aM = x.reshape(64, 8, 128).argmin(-1), x.reshape(64, 8, 128).argmax(-1)
    assert np.all(np.take_along_axis(blocks_c, am[..., None], -1) == 0)
    assert np.all(np.take_along_axis(blocks_c, aM[..., None], -1) >= 2)


def test_fp8_quantizer_nearest_level_bruteforce():
    rng = np.random.default_rng(61)
    for trial in range(200):
        g = int(rng.choice([4, 8]))
        x = rng.standard_normal((1, g)) * rng.uniform(0.1, 30) + rng.uniform(-5, 5)
        c, s, z = O.quantize(x, group=g, meta_format=1)
        levels = s[0, 0] * (np.arange(4) - z[0, 0])
        for e in range(g):
            dist = np.abs(levels - x[0, e])
            assert dist[c[0, e]] <= dist.min() + 1e-12


def test_fp8_saturation_and_clamps():
    tab = O.e4m3_values()
    # a range beyond 3 * 448: the scale saturates
    c, s, z = O.quantize(np.array([[0.0, 3000.0, 10.0, 20.0]]), group=4, meta_format=1)
    assert s[0, 0] == 448.0 and z[0, 0] == 0 and c[0].tolist() == [0, 3, 0, 0]
    # a tiny positive range rounds up to the smallest subnormal instead of to 0
    c, s, z = O.quantize(np.array([[0.0, 1e-6, 0.0, 0.0]]), group=4, meta_format=1)
    assert s[0, 0] == 2.0 ** -9 and np.all(c == 0)
    # a block far from 0 compared with its range: the zero-point leaves INT8 and is clamped
    c, s, z = O.quantize(np.array([[1000.0, 1001.0, 1000.5, 1000.25]]), group=4, meta_format=1)
    assert s[0, 0] == tab[np.searchsorted(tab, 1.0 / 3.0)] and z[0, 0] == -128 and np.all(c == 3)
    c, s, z = O.quantize(-np.array([[1000.0, 1001.0, 1000.5, 1000.25]]), group=4, meta_format=1)
    assert z[0, 0] == 127 and np.all(c == 0)
    # constant blocks: |min| rounded up, code 0, reconstruction exact when |min| is an E4M3 number
    for val, exact in [(0.0, True), (2.5, True), (-0.125, True), (2.3, False)]:
        c, s, z = O.quantize(np.full((1, 8), val), group=8, meta_format=1)
        xh = O.dequantize(c, s, z, group=8)
        assert np.all(c == 0) and s[0, 0] > 0
        assert np.all(np.abs(xh - val) <= 0.5 * s[0, 0])
        if exact:
            assert np.all(xh == val)


def test_fp8_average_bits_and_effect_on_the_error():
    """2 bits + (8 + 8) / 128 = 2.125 from the stored arrays; and the coarser scale changes the
    reconstruction error only a little (the ablation table's last row reports no change in
    perplexity): between 1x and 1.3x the mean squared error of the fp16 metadata."""
    rng = np.random.default_rng(62)
    x = rng.standard_normal((64, 4096))
    c, s, z = O.quantize(x, group=128, meta_format=1)
    bits = O.pack_canonical(c).size * 8 + (s.size + z.size) * 8
    assert bits / c.size == 2.125
    cfg = O.OracleConfig(batch=1, n_q_heads=32, n_kv_heads=32, meta_format=1)
    assert O.average_bits(cfg) == 2.125
    c0, s0, z0 = O.quantize(x, group=128)
    e8 = np.mean((O.dequantize(c, s, z) - x) ** 2)
    e16 = np.mean((O.dequantize(c0, s0, z0) - x) ** 2)
    assert 1.0 <= e8 / e16 <= 1.3


def test_fp8_cache_roundtrip_and_attention():
    """End to end with meta_format = 1: the cache's metadata are E4M3 / INT8 numbers, the
    reconstruction obeys the half-step bound in the rotated basis, and with every token retained
    as a sink the read half is still the textbook attention (the format touches only the 2-bit
    stream)."""
    cfg = O.OracleConfig(batch=2, n_q_heads=4, n_kv_heads=4, rot_heads=2, max_sinks=40, meta_format=1)
    rng = np.random.default_rng(63)
    k = rng.standard_normal((2, 40, 4, 128)).astype(np.float16)
    v = rng.standard_normal((2, 40, 4, 128)).astype(np.float16)
    q = rng.standard_normal((2, 4, 128)).astype(np.float16)
    c = O.cache_new(cfg)
    O.quantize_append(c, k, v)
    tab = O.e4m3_values()
    assert np.isin(c.k_scale, tab).all() and np.isin(c.v_scale, tab).all()
    assert np.abs(c.k_zero).max() <= 128 and np.abs(c.v_zero).max() <= 128
    zq = O.dequantize(c.k_codes, c.k_scale, c.k_zero)
    assert np.all(np.abs(zq - c.k_rot) <= 0.5 * np.repeat(c.k_scale, 128, axis=-1) * (1 + 1e-12))
    q_pos = np.array([39, 39])
    out, _ = O.decode_attention(c, q)
    k_hat, v_hat = O.dequantize_cache(c)
    ref = _textbook_attention(q.astype(np.float64), k_hat, v_hat, q_pos, 10000.0, 1)
    assert np.abs(out - ref).max() <= 1e-9
    c2 = O.cache_new(cfg)
    O.quantize_append(c2, k, v, np.ones((2, 40), dtype=np.uint8))
    out2, _ = O.decode_attention(c2, q)
    ref2 = _textbook_attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), q_pos, 10000.0, 1)
    assert np.abs(out2 - ref2).max() <= 1e-9


# ----------------------------------------------------------------------------- RoPE

@pytest.mark.parametrize("style", [0, 1])
def test_rope_properties(style):
    rng = np.random.default_rng(8)
    x = rng.standard_normal((7, 128))
    pos = np.arange(7) * 13
    y = O.rope(x, pos, 10000.0, style)
    assert np.allclose((y ** 2).sum(1), (x ** 2).sum(1))
    assert np.allclose(O.rope(x, np.zeros(7), 10000.0, style), x)
    q = rng.standard_normal(128)
    s0 = O.rope(x, pos, 10000.0, style) @ O.rope(q, 100, 10000.0, style)
    s1 = O.rope(x, pos + 57, 10000.0, style) @ O.rope(q, 157, 10000.0, style)
    assert np.allclose(s0, s1, atol=1e-9)


def test_rope_matches_complex_rotation():
    """Half-split pairing (j, j+64) with angle pos * theta^(-j/64): compare with e^{i angle}."""
    rng = np.random.default_rng(9)
    x = rng.standard_normal(128)
    pos = 37
    w = (x[:64] + 1j * x[64:]) * np.exp(1j * pos * 10000.0 ** (-np.arange(64) / 64.0))
    y = O.rope(x, pos, 10000.0, 0)
    assert np.allclose(y[:64], w.real) and np.allclose(y[64:], w.imag)
    xi = rng.standard_normal(128)
    wi = (xi[0::2] + 1j * xi[1::2]) * np.exp(1j * pos * 500000.0 ** (-np.arange(64) / 64.0))
    yi = O.rope(xi, pos, 500000.0, 1)
    assert np.allclose(yi[0::2], wi.real) and np.allclose(yi[1::2], wi.imag)


# ----------------------------------------------------------------------------- sinks

def test_select_sinks():
    rng = np.random.default_rng(10)
    act = rng.standard_normal((200, 64))
    act[110, 5] = 300.0
    act[0, 7] = -250.0
    assert O.select_sinks(act, 2).tolist() == [0, 110]
    tie = np.zeros((5, 3))
    tie[1, 0] = tie[3, 2] = tie[4, 1] = 2.0
    assert O.select_sinks(tie, 2).tolist() == [1, 3]


# ----------------------------------------------------------------------------- whole path

def _cfg(**kw):
    base = dict(batch=2, n_q_heads=4, n_kv_heads=4, head_dim=128, rot_heads=2, perm_span=128, max_sinks=64)
    base.update(kw)
    return O.OracleConfig(**base)


def test_rotate_reorder_inverse_is_identity():
    """Write-order rotate->reorder and read-order reorder^-1->rotate compose to the identity."""
    cfg = _cfg(perm_span=256)
    rng = np.random.default_rng(11)
    P = np.concatenate([rng.permutation(256), 256 + rng.permutation(256)])
    x = rng.standard_normal((3, 512))
    z = O.reorder(O.rotate_groups(x, cfg.n), P)
    back = O.rotate_groups(O.reorder_inverse(z, P), cfg.n)
    assert np.allclose(back, x, atol=1e-12)
    wrong = O.reorder_inverse(O.rotate_groups(z, cfg.n), P)      # the other order is not an inverse
    assert not np.allclose(wrong, x, atol=1e-3)


def _textbook_attention(q, k, v, q_pos, theta, rep):
    import torch
    B, T, Hkv, d = k.shape
    Hq = q.shape[1]

    def rot(x, pos):
        w = (x[..., :d // 2] + 1j * x[..., d // 2:]) * np.exp(1j * np.asarray(pos)[..., None] * theta ** (-np.arange(d // 2) / (d / 2)))
        return np.concatenate([w.real, w.imag], axis=-1)
    kr = np.stack([rot(k[:, :, h], np.arange(T)[None, :]) for h in range(Hkv)], axis=1)     # [B,Hkv,T,d]
    qr = np.stack([rot(q[:, h], q_pos) for h in range(Hq)], axis=1)[:, :, None, :]          # [B,Hq,1,d]
    kr = np.repeat(kr, rep, axis=1)
    vv = np.repeat(np.transpose(v, (0, 2, 1, 3)), rep, axis=1)
    out = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(qr), torch.from_numpy(kr), torch.from_numpy(vv))
    return out[:, :, 0, :].numpy()


@pytest.mark.parametrize("hq,hkv", [(4, 4), (8, 2)])
def test_all_sink_cache_is_textbook_attention(hq, hkv):
    """With every token retained in fp16 the read half must equal plain attention (library SDPA),
    which pins RoPE, softmax, the 1/sqrt(d) scale and the GQA head mapping without the codec."""
    cfg = _cfg(n_q_heads=hq, n_kv_heads=hkv, rot_heads=2)
    rng = np.random.default_rng(12)
    T = 40
    k = rng.standard_normal((2, T, hkv, 128)).astype(np.float16)
    v = rng.standard_normal((2, T, hkv, 128)).astype(np.float16)
    q = rng.standard_normal((2, hq, 128)).astype(np.float16)
    cache = O.cache_new(cfg)
    O.quantize_append(cache, k, v, np.ones((2, T), dtype=np.uint8))
    q_pos = np.array([T - 1, T + 5])
    out, lse = O.decode_attention(cache, q, q_pos)
    ref = _textbook_attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), q_pos, 10000.0, hq // hkv)
    assert np.allclose(out, ref, atol=1e-10)
    assert np.allclose(lse, _library_lse(q, k.astype(np.float64), q_pos, 10000.0, hq // hkv), rtol=0, atol=1e-10)


def _library_lse(q, k_hat, q_pos, theta, rep):
    """Eq. 5's normaliser by a library log-sum-exp: log sum_t exp(q~ . k~_t / sqrt(d)) for keys
    k_hat [B, T, Hkv, d] (pre-RoPE), RoPE written as a complex rotation."""
    from scipy.special import logsumexp
    B, T, Hkv, d = k_hat.shape
    w = theta ** (-np.arange(d // 2) / (d / 2))
    kz = (k_hat[..., :d // 2] + 1j * k_hat[..., d // 2:]) * np.exp(1j * np.arange(T)[None, :, None, None] * w)
    qf = np.asarray(q, dtype=np.float64)
    qz = (qf[..., :d // 2] + 1j * qf[..., d // 2:]) * np.exp(1j * np.asarray(q_pos)[:, None, None] * w)
    out = np.empty(qf.shape[:2])
    for b in range(B):
        for h in range(qf.shape[1]):
            scores = (kz[b, :, h // rep] * np.conj(qz[b, h])).real.sum(-1) / np.sqrt(d)
            out[b, h] = logsumexp(scores)
    return out


def test_lse_of_a_quantized_cache_is_the_log_sum_exp_of_its_scores():
    """The second result of the read half is Eq. 5's normaliser, max included: against a library
    log-sum-exp over the scores of the reconstructed keys (retained rows substituted).  The keys
    are scaled so that the largest score is far from 0 - a normaliser without its max term, or
    with the sum taken before the shift, is then off by tens."""
    cfg = _cfg(n_q_heads=8, n_kv_heads=4, rot_heads=2, max_sinks=2)
    rng = np.random.default_rng(31)
    T = 48
    k = (rng.standard_normal((2, T, 4, 128)) * 6.0).astype(np.float16)
    v = rng.standard_normal((2, T, 4, 128)).astype(np.float16)
    q = rng.standard_normal((2, 8, 128)).astype(np.float16)
    mask = np.zeros((2, T), np.uint8)
    mask[:, 3] = 1
    cache = O.cache_new(cfg)
    O.quantize_append(cache, k, v, mask)
    q_pos = np.array([T - 1, T + 2])
    out, lse = O.decode_attention(cache, q, q_pos)
    k_hat, v_hat = O.dequantize_cache(cache, substitute_sinks=True)
    ref = _library_lse(q, k_hat, q_pos, 10000.0, 2)
    assert np.abs(ref).min() > 3.0                      # the max term matters in every head
    assert np.allclose(lse, ref, rtol=0, atol=1e-9)
    # and the first result is the softmax-weighted mean that goes with that normaliser
    ref_out = _textbook_attention(q.astype(np.float64), k_hat, v_hat, q_pos, 10000.0, 2)
    assert np.allclose(out, ref_out, rtol=0, atol=1e-10)


def test_no_quantization_error_on_grid_data():
    """Keys whose rotated image lies exactly on a 2-bit grid survive the whole write+read path."""
    cfg = _cfg(batch=1, rot_heads=2, perm_span=256)
    rng = np.random.default_rng(13)
    P = np.concatenate([rng.permutation(256), 256 + rng.permutation(256)])
    codes = rng.integers(0, 4, size=(1, 6, 512))
    codes[..., 0::128] = 0
    codes[..., 1::128] = 3
    z = 0.5 * (codes - 1.0)                                   # scale 0.5, zero 1 in every block
    x = O.rotate_groups(O.reorder_inverse(z, P), 256)        # keys whose rotate+reorder image is z
    xr = np.rint(x * 32.0) / 32.0                              # multiples of 1/32 below 16: exact in fp16
    assert np.abs(xr - x).max() < 1e-12
    x16 = xr.astype(np.float16)
    assert np.array_equal(x16.astype(np.float64), xr)
    cache = O.cache_new(cfg, P)
    O.quantize_append(cache, x16.reshape(1, 6, 4, 128), np.zeros((1, 6, 4, 128), np.float16))
    assert np.array_equal(cache.k_codes, codes)
    k_hat, _ = O.dequantize_cache(cache)
    assert np.allclose(k_hat.reshape(1, 6, 512), xr, atol=1e-12)


def test_decode_stream_error_is_bounded_and_sinks_are_exact():
    cfg = _cfg(max_sinks=1)
    rng = np.random.default_rng(14)
    T = 64
    k = rng.standard_normal((2, T, 4, 128)).astype(np.float16)
    v = rng.standard_normal((2, T, 4, 128)).astype(np.float16)
    mask = np.zeros((2, T), np.uint8)
    mask[:, 0] = 1
    mask[:, 5] = 1                                             # second flag exceeds max_sinks: ignored
    cache = O.cache_new(cfg)
    O.quantize_append(cache, k, v, mask)
    assert cache.sink_pos == [[0], [0]]
    k_hat, v_hat = O.dequantize_cache(cache, substitute_sinks=True)
    assert np.array_equal(k_hat[:, 0], k[:, 0].astype(np.float64))
    assert np.array_equal(v_hat[:, 0], v[:, 0].astype(np.float64))
    # per-element bound in the rotated domain carries to an L2 bound per rotation group
    step = np.repeat(cache.k_scale, 128, axis=-1)
    err = (k_hat.reshape(2, T, 512) - k.astype(np.float64).reshape(2, T, 512))[:, 1:]
    bound = np.sqrt(((0.5 * step[:, 1:] * (1 + 2.0 ** -8)) ** 2).reshape(2, T - 1, 2, 256).sum(-1))
    assert np.all(np.sqrt((err.reshape(2, T - 1, 2, 256) ** 2).sum(-1)) <= bound + 1e-9)


def test_append_in_pieces_equals_bulk():
    cfg = _cfg()
    rng = np.random.default_rng(15)
    k = rng.standard_normal((2, 20, 4, 128)).astype(np.float16)
    v = rng.standard_normal((2, 20, 4, 128)).astype(np.float16)
    a, b = O.cache_new(cfg), O.cache_new(cfg)
    O.quantize_append(a, k, v)
    O.quantize_append(b, k[:, :13], v[:, :13])
    O.quantize_append(b, k[:, 13:], v[:, 13:])
    assert np.array_equal(a.k_codes, b.k_codes) and np.array_equal(a.v_scale, b.v_scale)
    q = rng.standard_normal((2, 4, 128)).astype(np.float16)
    assert np.allclose(O.decode_attention(a, q)[0], O.decode_attention(b, q)[0])


def test_v_rotate_roundtrip():
    cfg0, cfg1 = _cfg(v_rotate=0), _cfg(v_rotate=1)
    rng = np.random.default_rng(16)
    k = rng.standard_normal((2, 8, 4, 128)).astype(np.float16)
    v = rng.standard_normal((2, 8, 4, 128)).astype(np.float16)
    c1 = O.cache_new(cfg1)
    O.quantize_append(c1, k, v)
    _, v_hat = O.dequantize_cache(c1)
    step = np.repeat(c1.v_scale, 128, axis=-1).reshape(2, 8, 4, 128)
    err = np.sqrt(((v_hat - v.astype(np.float64)) ** 2).sum(-1))
    assert np.all(err <= np.sqrt(((0.5 * step * (1 + 2.0 ** -8)) ** 2).sum(-1)) + 1e-9)
    assert not np.array_equal(c1.v_codes, O.quantize(v.astype(np.float64).reshape(2, 8, 512))[0])


def test_v_rotate_is_a_rotation_of_each_head_on_its_own():
    """The value rotation of Sec. 4.4 is a Hadamard of the head dimension, head by head (the
    grouped rotation is the keys').  A value row that is non-zero in one head only must leave
    every other head's block constant (all codes 0), and a head that holds one constant c becomes
    c sqrt(128) e_0 - codes (3, 0, 0, ...), scale fp16(c sqrt(128) / 3), zero 0 - and reads back
    as the constant."""
    cfg = _cfg(batch=1, v_rotate=1, rot_heads=4)
    k = np.zeros((1, 2, 4, 128), np.float16)
    v = np.zeros((1, 2, 4, 128), np.float16)
    v[0, 0, 1, :] = 0.75                       # token 0: head 1 constant
    rng = np.random.default_rng(33)
    v[0, 1, 2, :] = rng.standard_normal(128).astype(np.float16)   # token 1: head 2 only
    cache = O.cache_new(cfg)
    O.quantize_append(cache, k, v)
    codes = cache.v_codes.reshape(1, 2, 4, 128)
    for t, live in ((0, 1), (1, 2)):
        for h in range(4):
            if h != live:
                assert not codes[0, t, h].any(), (t, h)
    assert codes[0, 0, 1].tolist() == [3] + [0] * 127
    assert cache.v_scale[0, 0, 1] == float(np.float16(0.75 * np.sqrt(128.0) / 3.0)) and cache.v_zero[0, 0, 1] == 0.0
    _, v_hat = O.dequantize_cache(cache)
    assert np.allclose(v_hat[0, 0, 1], 3.0 * cache.v_scale[0, 0, 1] / np.sqrt(128.0), atol=1e-12)
    assert np.abs(v_hat[0, 0, 1] - 0.75).max() < 1e-3
    assert not v_hat[0, 0, [0, 2, 3]].any() and not v_hat[0, 1, [0, 1, 3]].any()
    # token 1, head 2: codes are those of H_128 applied to that head alone
    u = O.rotate_groups(v[0, 1, 2].astype(np.float64)[None], 128)
    assert np.array_equal(codes[0, 1, 2], O.quantize(u, 128)[0][0])


def test_reorder_lowers_error_on_offset_outliers():
    """Ordering of the paper's key-reconstruction table (rotation alone vs rotation + reorder),
    on synthetic keys with per-channel offsets.  The table's absolute values need real model
    keys: parity unpinned."""
    import rkv_synth as S
    w = S.WORKLOADS["cfg1"]
    k, v, _ = S.make_kv(w, 64, batch=1, offset_variant=True, sink_positions=[])
    kc, _, _ = S.make_kv(w, 256, batch=1, stream=1, offset_variant=True, sink_positions=[])
    base = dict(batch=1, n_q_heads=32, n_kv_heads=32, rot_heads=4, perm_span=512)
    cfg = O.OracleConfig(**base)
    P = O.calibrate_perm(kc[0], cfg)
    mses = []
    for perm in (None, P):
        c = O.cache_new(cfg, perm)
        O.quantize_append(c, k, v)
        k_hat, _ = O.dequantize_cache(c)
        mses.append(((k_hat - k.astype(np.float64)) ** 2).mean())
    assert mses[1] < mses[0]


def test_select_sinks_brute_force():
    """The selector against a literal reading of its definition on tiny inputs: score = largest
    |activation| of a token; take the k best, lower index first among equals; return ascending."""
    rng = np.random.default_rng(5)
    for trial in range(200):
        T, C = int(rng.integers(1, 9)), int(rng.integers(1, 5))
        x = rng.integers(-3, 4, size=(T, C)).astype(np.float64)      # many exact ties
        k = int(rng.integers(1, T + 1))
        scores = [max(abs(v) for v in row) for row in x]
        chosen = []
        for _ in range(k):
            best = None
            for t in range(T):
                if t in chosen:
                    continue
                if best is None or scores[t] > scores[best]:
                    best = t
            chosen.append(best)
        assert O.select_sinks(x, k).tolist() == sorted(chosen)


def test_fold_rotation_is_the_rotation_moved_into_the_weights():
    """Linearity pin: projecting with the folded matrix equals projecting, rotating and reordering
    (matrix products associate), for each rotation size and with a reorder."""
    rng = np.random.default_rng(21)
    for g in (1, 2, 4):
        cfg = O.OracleConfig(batch=1, n_q_heads=4, n_kv_heads=4, rot_heads=g)
        E = cfg.E
        w = rng.standard_normal((24, E))
        x = rng.standard_normal((5, 24))
        perm = np.concatenate([128 * blk + rng.permutation(128) for blk in range(E // 128)])
        direct = O.reorder(O.rotate_groups(x @ w, cfg.n), perm)
        folded = x @ O.fold_rotation(w, cfg, perm)
        assert np.allclose(direct, folded, rtol=0, atol=1e-12)
        # folding twice with the inverse order gives the matrix back (H is an involution)
        back = O.rotate_groups(O.reorder_inverse(O.fold_rotation(w, cfg, perm), perm), cfg.n)
        assert np.allclose(back, w, rtol=0, atol=1e-12)


def test_append_of_rotated_keys_equals_append_of_plain_keys():
    """With a rotation over 2 heads the Hadamard entries are +-1/16, so keys that are multiples of
    16 have rotated images that are integers below 2048, exact in fp16: the folded-weights path fed
    with them must build the very same cache, sink rows included."""
    rng = np.random.default_rng(22)
    cfg = O.OracleConfig(batch=2, n_q_heads=4, n_kv_heads=4, rot_heads=2, max_sinks=2)
    E = cfg.E
    perm = np.concatenate([128 * blk + rng.permutation(128) for blk in range(E // 128)])
    k = (16.0 * rng.integers(-40, 41, size=(2, 9, 4, 128))).astype(np.float16)    # a wide range keeps x / scale off exact ties
    v = rng.standard_normal((2, 9, 4, 128)).astype(np.float16)
    mask = np.zeros((2, 9), dtype=np.uint8)
    mask[0, 0] = mask[1, 4] = 1
    a = O.cache_new(cfg, perm)
    O.quantize_append(a, k, v, mask)
    rot = O.reorder(O.rotate_groups(k.astype(np.float64).reshape(2, 9, E), cfg.n), perm)
    assert np.abs(rot - np.rint(rot)).max() < 1e-12          # integers, up to the recursion's 1/sqrt(2) factors
    rot = np.rint(rot)
    assert np.array_equal(rot, rot.astype(np.float16).astype(np.float64))        # exact in fp16
    b = O.cache_new(cfg, perm)
    O.quantize_append(b, rot.reshape(2, 9, 4, 128).astype(np.float16), v, mask, keys_rotated=True)
    for name in ("k_scale", "k_zero", "v_codes", "v_scale", "v_zero"):
        assert np.array_equal(getattr(a, name), getattr(b, name)), name
    # codes: equal, except where the exact integer key sits on a rounding tie of Eq. 6 (x / scale
    # an exact half-integer), which the 1e-13 noise of the plain path's rotation may tip either way
    ratio = b.k_rot / np.repeat(b.k_scale, 128, axis=-1)
    tie = (ratio - np.floor(ratio)) == 0.5
    assert np.array_equal(a.k_codes[~tie], b.k_codes[~tie]) and tie.mean() < 0.01
    assert np.abs(a.k_codes.astype(int) - b.k_codes.astype(int)).max() <= 1
    for s in range(2):
        assert a.sink_pos[s] == b.sink_pos[s]
        for ra, rb in zip(a.sink_k[s], b.sink_k[s]):
            assert np.array_equal(ra, rb)


def test_current_token_operand_equals_a_retained_row():
    """Attending the token being decoded in full precision is the same as having appended it as a
    retained (fp16) row: both put its exact key and value at position T."""
    rng = np.random.default_rng(23)
    cfg = O.OracleConfig(batch=2, n_q_heads=8, n_kv_heads=4, rot_heads=2, max_sinks=3)
    k = rng.standard_normal((2, 21, 4, 128)).astype(np.float16)
    v = rng.standard_normal((2, 21, 4, 128)).astype(np.float16)
    q = rng.standard_normal((2, 8, 128)).astype(np.float16)
    mask = np.zeros((2, 21), dtype=np.uint8)
    mask[:, 0] = 1
    a = O.cache_new(cfg)
    O.quantize_append(a, k[:, :20], v[:, :20], mask[:, :20])
    out_a, lse_a = O.decode_attention(a, q, None, k[:, 20], v[:, 20])
    b = O.cache_new(cfg)
    mask[:, 20] = 1
    O.quantize_append(b, k, v, mask)
    out_b, lse_b = O.decode_attention(b, q)
    assert np.allclose(out_a, out_b, rtol=0, atol=1e-12) and np.allclose(lse_a, lse_b, rtol=0, atol=1e-12)
    # and it differs from attending the quantized token
    c = O.cache_new(cfg)
    mask[:, 20] = 0
    O.quantize_append(c, k, v, mask)
    out_c, _ = O.decode_attention(c, q)
    assert np.abs(out_c - out_a).max() > 1e-4


def test_multi_query_decode_is_a_sequence_of_single_steps():
    """Decoding several tokens at once must give what token-by-token decoding gives: append token
    i, decode with query i over the cache so far - for every i."""
    rng = np.random.default_rng(24)
    cfg = O.OracleConfig(batch=2, n_q_heads=4, n_kv_heads=2, rot_heads=2, max_sinks=2)
    T0, nq = 13, 3
    k = rng.standard_normal((2, T0 + nq, 2, 128)).astype(np.float16)
    v = rng.standard_normal((2, T0 + nq, 2, 128)).astype(np.float16)
    q = rng.standard_normal((2, nq, 4, 128)).astype(np.float16)
    mask = np.zeros((2, T0 + nq), dtype=np.uint8)
    mask[:, 0] = 1
    mask[0, T0 + 1] = 1                       # a retained row among the new tokens: later queries see it, earlier ones do not
    step = O.cache_new(cfg)
    O.quantize_append(step, k[:, :T0], v[:, :T0], mask[:, :T0])
    ref = []
    for i in range(nq):
        O.quantize_append(step, k[:, T0 + i:T0 + i + 1], v[:, T0 + i:T0 + i + 1], mask[:, T0 + i:T0 + i + 1])
        ref.append(O.decode_attention(step, q[:, i]))
    full = O.cache_new(cfg)
    O.quantize_append(full, k, v, mask)
    pos = np.tile(np.arange(T0, T0 + nq), (2, 1))
    out, lse = O.decode_attention_multi(full, q, pos)
    for i in range(nq):
        assert np.allclose(out[:, i], ref[i][0], rtol=0, atol=1e-12)
        assert np.allclose(lse[:, i], ref[i][1], rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------- properties over random shapes

from hypothesis import given, settings, strategies as st   # noqa: E402


@settings(max_examples=40, deadline=None)
@given(st.integers(0, 2 ** 31 - 1), st.sampled_from([1, 2, 4]), st.sampled_from([1, 2, 4, 8]), st.sampled_from([128, "n", "E"]))
def test_write_then_read_views_are_consistent(seed, rot_heads, heads_mult, span_kind):
    """For random head counts, rotation sizes and reorder spans: the reorder from calibration is a
    permutation closed under its span; reorder and rotation invert exactly; every reconstructed
    element of the rotated, reordered row lies within half a stored step of what was quantized;
    and the dequantized cache is that reconstruction carried back (inverse reorder, rotation)."""
    hkv = rot_heads * heads_mult
    cfg = O.OracleConfig(batch=1, n_q_heads=hkv, n_kv_heads=hkv, rot_heads=rot_heads)
    span = {128: 128, "n": cfg.n, "E": cfg.E}[span_kind]
    cfg = O.OracleConfig(batch=1, n_q_heads=hkv, n_kv_heads=hkv, rot_heads=rot_heads, perm_span=span, max_sinks=0)
    rng = np.random.default_rng(seed)
    perm = O.calibrate_perm(rng.standard_normal((8, hkv, 128)) + rng.standard_normal((1, hkv, 128)), cfg)
    assert sorted(perm.tolist()) == list(range(cfg.E))
    assert np.array_equal(perm // span, np.arange(cfg.E) // span)
    k = (rng.standard_normal((1, 5, hkv, 128)) * np.exp(rng.uniform(-2, 2))).astype(np.float16)
    v = rng.standard_normal((1, 5, hkv, 128)).astype(np.float16)
    c = O.cache_new(cfg, perm)
    O.quantize_append(c, k, v)
    z = c.k_rot
    back = O.rotate_groups(O.reorder_inverse(z, perm), cfg.n).reshape(k.shape)
    assert np.allclose(back, k.astype(np.float64), atol=1e-9 * max(1.0, float(np.abs(k).max())))
    zq = O.dequantize(c.k_codes, c.k_scale, c.k_zero)
    assert np.all(np.abs(zq - z) <= 0.5 * np.repeat(c.k_scale, 128, axis=-1) * (1 + 2.0 ** -8))
    k_hat, v_hat = O.dequantize_cache(c)
    assert np.allclose(k_hat, O.rotate_groups(O.reorder_inverse(zq, perm), cfg.n).reshape(k.shape), atol=1e-9 * max(1.0, float(np.abs(k).max())))
    assert np.all(np.abs(v_hat.reshape(1, 5, -1) - v.astype(np.float64).reshape(1, 5, -1)) <= 0.5 * np.repeat(c.v_scale, 128, axis=-1) * (1 + 2.0 ** -8))


@settings(max_examples=25, deadline=None)
@given(st.integers(0, 2 ** 31 - 1), st.integers(1, 40), st.sampled_from([(4, 4), (8, 2), (6, 3)]), st.integers(0, 3))
def test_attention_is_a_convex_combination_and_shift_invariant(seed, T, heads, n_sink):
    """Eq. 5 for random lengths and GQA ratios: every output lies in the hull of the values the
    read half sees; the log-sum-exp bounds the largest score; shifting the query position and all
    key positions together is impossible to express through the interface, but a query far away
    changes nothing when every key sits at position 0 (T = 1)."""
    hq, hkv = heads
    cfg = O.OracleConfig(batch=1, n_q_heads=hq, n_kv_heads=hkv, rot_heads=1, max_sinks=4)
    rng = np.random.default_rng(seed)
    k = rng.standard_normal((1, T, hkv, 128)).astype(np.float16)
    v = rng.standard_normal((1, T, hkv, 128)).astype(np.float16)
    q = rng.standard_normal((1, hq, 128)).astype(np.float16)
    mask = np.zeros((1, T), np.uint8)
    mask[0, :min(n_sink, T)] = 1
    c = O.cache_new(cfg)
    O.quantize_append(c, k, v, mask)
    out, lse = O.decode_attention(c, q)
    _, v_hat = O.dequantize_cache(c, substitute_sinks=True)
    rep = hq // hkv
    for h in range(hq):
        vals = v_hat[0, :, h // rep, :]
        assert np.all(out[0, h] <= vals.max(0) + 1e-9) and np.all(out[0, h] >= vals.min(0) - 1e-9)
    assert np.isfinite(lse).all()
    if T == 1:
        out2, _ = O.decode_attention(c, q, np.array([12345]))
        assert np.allclose(out, out2, atol=1e-12)       # softmax over one key: its value, wherever the query sits
