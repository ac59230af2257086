"""Do the oracle's pins bite?  Each entry below plants one plausible mistake in a copy of
oracle/rkv_oracle.py (a dropped term, a wrong sign or index, a swapped order, the wrong rounding)
and runs tests/test_oracle_pins.py against that copy in a child process: at least one pin must
fail.  The mistakes live only in the child's memory; nothing here touches the GPU path.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle", "rkv_oracle.py")

# (what is planted, text in the oracle, replacement) - the text must occur exactly once; a tuple
# of texts and a tuple of replacements plant one mistake in several places
MUTANTS = [
    ("Hadamard recursion without the minus sign", "np.block([[H, H], [H, -H]])", "np.block([[H, H], [H, H]])"),
    ("rotation without its normalisation", "x[..., r * n:(r + 1) * n] @ H.T", "x[..., r * n:(r + 1) * n] @ H.T * np.sqrt(n)"),
    ("reorder applied in the inverse direction", "    return np.asarray(y)[..., np.asarray(perm)]\n",
     "    out = np.empty_like(np.asarray(y))\n    out[..., np.asarray(perm)] = np.asarray(y)\n    return out\n"),
    ("calibration sorts magnitudes instead of signed sums", "channel_sum = rotated.sum(axis=0)", "channel_sum = np.abs(rotated).sum(axis=0)"),
    ("calibration sorts in descending order", 'np.argsort(block, kind="stable") + s * span', 'np.argsort(-block, kind="stable") + s * span'),
    ("Eq. 6 rounds half up instead of half to even", "q = np.rint(blocks / scale[..., None]) + zero[..., None]",
     "q = np.floor(blocks / scale[..., None] + 0.5) + zero[..., None]"),
    ("Eq. 9 zero-point with the wrong sign", "zero = np.clip(-np.rint(mn / scale), zlo, zhi)", "zero = np.clip(np.rint(mn / scale), zlo, zhi)"),
    ("Eq. 8 divides the range by 2^bits", "qmax = float(2 ** bits - 1)", "qmax = float(2 ** bits)"),
    ("Eq. 8 with the step count of 2-bit codes whatever the width", "qmax = float(2 ** bits - 1)", "qmax = 3.0"),
    ("the cache quantizes with 2-bit codes whatever the configuration",
     "kc, ks, kz = quantize(z, cfg.quant_group, cfg.bits, cfg.meta_format)", "kc, ks, kz = quantize(z, cfg.quant_group, 2, cfg.meta_format)"),
    ("the read half dequantizes keys in blocks of 128 whatever the configuration",
     "zq = dequantize(cache.k_codes, cache.k_scale, cache.k_zero, cfg.quant_group)", "zq = dequantize(cache.k_codes, cache.k_scale, cache.k_zero, 128)"),
    ("average bits without the metadata's dependence on the group", "/ cfg.quant_group", "/ 128.0"),
    ("scale not rounded to the stored fp16 number", "scale = np.minimum(_to_f16((mx - mn) / qmax), F16_MAX)        # Eq. 8, stored in fp16",
     "scale = np.minimum((mx - mn) / qmax, F16_MAX)"),
    ("Eq. 7 without the scale on the zero-point", "x = np.asarray(scale)[..., None] * (blocks - np.asarray(zero)[..., None])",
     "x = np.asarray(scale)[..., None] * blocks - np.asarray(zero)[..., None]"),
    ("FP8 scale rounded down instead of up", 'idx = np.searchsorted(tab, x, side="left")', 'idx = np.maximum(np.searchsorted(tab, x, side="right") - 1, 0)'),
    ("INT8 zero-point not clamped", "zlo, zhi = -128.0, 127.0", "zlo, zhi = -ZERO_LIMIT, ZERO_LIMIT"),
    ("packed bytes with the codes in the opposite order", "(c4[..., 0] | (c4[..., 1] << 2) | (c4[..., 2] << 4) | (c4[..., 3] << 6))",
     "(c4[..., 3] | (c4[..., 2] << 2) | (c4[..., 1] << 4) | (c4[..., 0] << 6))"),
    ("RoPE turning the wrong way", "        out[..., :half] = a * c - b * s\n        out[..., half:] = a * s + b * c\n",
     "        out[..., :half] = a * c + b * s\n        out[..., half:] = -a * s + b * c\n"),
    ("RoPE frequencies with half the exponent", "freq = theta ** (-2.0 * j / d)", "freq = theta ** (-1.0 * j / d)"),
    ("sink selection breaks ties towards the higher index", "order = np.lexsort((np.arange(a.shape[0]), -a))", "order = np.lexsort((-np.arange(a.shape[0]), -a))"),
    ("rotate and reorder in the wrong order on the write side", "        y = rotate_groups(x, cfg.n)\n        z = reorder(y, cache.perm)\n",
     "        y = reorder(x, cache.perm)\n        z = rotate_groups(y, cfg.n)\n"),
    ("scores scaled by the rotation size instead of the head dimension", "s = (k_r @ q_r) / np.sqrt(float(d))", "s = (k_r @ q_r) / np.sqrt(float(cfg.n))"),
    ("GQA: query head h reads KV head h mod n_kv_heads", "            kv = h // rep\n", "            kv = h % cfg.n_kv_heads\n"),
    ("retained sink rows not substituted in the read half", "k_hat, v_hat = dequantize_cache(cache, substitute_sinks=True)", "k_hat, v_hat = dequantize_cache(cache, substitute_sinks=False)"),
    ("several query tokens: a sink behind the query is still seen", "keep = [s for s, pos in enumerate(cache.sink_pos[b]) if pos < T]",
     "keep = [s for s, pos in enumerate(cache.sink_pos[b])]"),
    ("current token put in front of the cache instead of behind it", "k_hat = np.concatenate([k_hat, kc], axis=1)", "k_hat = np.concatenate([kc, k_hat], axis=1)"),
    ("log-sum-exp without the maximum that was taken out of the exponentials", "lse[b, h] = m + np.log(l)", "lse[b, h] = np.log(l)"),
    ("fp16 zero-point not clamped to the integers fp16 holds", "        zlo, zhi = -ZERO_LIMIT, ZERO_LIMIT\n", "        zlo, zhi = -1e9, 1e9\n"),
    ("fp16 scale not clamped to the largest fp16 number", "scale = np.minimum(_to_f16((mx - mn) / qmax), F16_MAX)", "scale = _to_f16((mx - mn) / qmax)"),
    ("value rotation over the keys' rotation group instead of each head (write side)", "u = rotate_groups(u, cfg.head_dim)", "u = rotate_groups(u, cfg.n)"),
    ("value rotation over the keys' rotation group instead of each head (read side)", "v_hat = rotate_groups(v_hat, cfg.head_dim)", "v_hat = rotate_groups(v_hat, cfg.n)"),
    ("value rotation over the keys' rotation group instead of each head (both sides)",
     ("u = rotate_groups(u, cfg.head_dim)", "v_hat = rotate_groups(v_hat, cfg.head_dim)"),
     ("u = rotate_groups(u, cfg.n)", "v_hat = rotate_groups(v_hat, cfg.n)")),
]


def _find(src, needle):
    return src.count(needle)


def _run_mutant(i):
    what, old, new = MUTANTS[i]
    olds, news = (old, new) if isinstance(old, tuple) else ((old,), (new,))
    code = (
        "import sys, types\n"
        f"sys.path.insert(0, {ROOT!r}); sys.path.insert(0, {os.path.join(ROOT, 'tests')!r})\n"
        f"src = open({ORACLE!r}).read()\n"
        f"olds, news = {olds!r}, {news!r}\n"
        "for old in olds:\n"
        "    assert src.count(old) == 1, 'mutation site not found exactly once'\n"
        "for old, new in zip(olds, news):\n"
        "    src = src.replace(old, new)\n"
        "import oracle\n"
        "mod = types.ModuleType('oracle.rkv_oracle'); mod.__file__ = 'mutant'\n"
        "sys.modules['oracle.rkv_oracle'] = mod\n"
        f"exec(compile(src, {ORACLE!r}, 'exec'), mod.__dict__)\n"
        "oracle.rkv_oracle = mod\n"
        "import pytest\n"
        f"sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', {os.path.join(ROOT, 'tests', 'test_oracle_pins.py')!r}]))\n"
    )
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, cwd=ROOT, timeout=600)
    return what, r.returncode, (r.stdout + r.stderr)[-1500:]


def test_unmutated_copy_passes_the_pins():
    """The harness itself: a copy with no change planted passes (so a failure below is the mutant's)."""
    global MUTANTS
    saved = MUTANTS
    try:
        MUTANTS = [("no change", '"""RotateKV oracle', '"""RotateKV oracle')]
        what, rc, tail = _run_mutant(0)
    finally:
        MUTANTS = saved
    assert rc == 0, tail


def test_every_planted_mistake_fails_a_pin():
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(_run_mutant, range(len(MUTANTS))))
    survivors = []
    for what, rc, tail in results:
        assert "mutation site not found" not in tail, f"{what}: the oracle's text changed, update the mutation"
        assert rc in (0, 1), f"{what}: the pin run itself broke\n{tail}"
        if rc == 0:
            survivors.append(what)
    assert not survivors, f"no pin noticed: {survivors}"
