"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and rejects
unsupported configurations without touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2501_16383_amd as R
from paper_2501_16383_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(R.library_path()):
        from paper_2501_16383_amd.build import build_library
        build_library()
    return R.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "rkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rkv_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert "rkv_quantize_append" in names and "rkv_decode_attention" in names and "rkv_calibrate_perm" in names
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == names


def test_query_sizes_and_average_bits(lib):
    cfg = R.RkvConfig(batch=16, n_q_heads=40, n_kv_heads=40, max_tokens=4096)
    cache_bytes, scratch_bytes = R.query_sizes(cfg)
    payload = 16 * 4096 * (2 * 5120 // 4 + 2 * 40 * 4)        # codes + fp16 scale/zero for K and V
    assert payload * 8 / (2 * 16 * 4096 * 5120) == 2.25
    assert payload <= cache_bytes <= payload * 1.03
    assert scratch_bytes > 0


@pytest.mark.parametrize("field,value", [
    ("head_dim", 64), ("quant_group", 16), ("quant_group", 96), ("bits", 1), ("bits", 5), ("rot_heads", 3), ("rot_heads", 16), ("perm_span", 256),
    ("clip_ratio", 0.9), ("max_sinks", 65), ("max_tokens", 0), ("batch", 0), ("rope_style", 2), ("v_rotate", 2),
    ("n_q_heads", 41), ("rope_theta", 0.5),
])
def test_unsupported_configs_are_rejected(lib, field, value):
    cfg = R.RkvConfig(batch=2, n_q_heads=40, n_kv_heads=40, max_tokens=128)
    setattr(cfg, field, value)
    with pytest.raises(R.RkvError) as ei:
        R.query_sizes(cfg)
    assert ei.value.code == binding.RKV_EINVAL


@pytest.mark.parametrize("bits,group,fmt,avg", [(4, 128, 0, 4.25), (3, 128, 0, 3.25), (2, 64, 0, 2.5), (2, 32, 1, 2.5), (4, 32, 0, 5.0)])
def test_sizes_of_wider_codes_and_smaller_groups(lib, bits, group, fmt, avg):
    """The cache's payload is bits + (32 or 16) / group bits per element (codes, scale, zero-point)."""
    cfg = R.RkvConfig(batch=16, n_q_heads=32, n_kv_heads=32, max_tokens=1024, max_sinks=0, bits=bits, quant_group=group,
                      meta_format=fmt)
    cache_bytes, _ = R.query_sizes(cfg)
    payload = 2 * 16 * 1024 * 4096 * avg / 8
    assert payload <= cache_bytes <= payload * 1.03
    rot = R.RkvConfig(batch=4, n_q_heads=32, n_kv_heads=32, max_tokens=1024, bits=bits, quant_group=group, keys_rotated=1,
                      rot_heads=4, meta_format=fmt)
    # folded-in rotation is a path of the matrix-core append kernel, which takes every code width and group size
    R.query_sizes(rot)


def test_null_arguments(lib):
    assert lib.rkv_cache_length(None) == binding.RKV_EINVAL
    assert lib.rkv_cache_reset(None, None) == binding.RKV_EINVAL
    assert lib.rkv_quantize_append(None, None, None, 1, None, None) == binding.RKV_EINVAL
    assert lib.rkv_decode_attention(None, None, None, None, None, None, None) == binding.RKV_EINVAL
    out = ctypes.c_void_p()
    cc = R.RkvConfig(batch=1, n_q_heads=4, n_kv_heads=4, max_tokens=16).to_c()
    assert lib.rkv_cache_create(ctypes.byref(cc), None, 1 << 30, None, ctypes.byref(out)) == binding.RKV_EINVAL
    assert lib.rkv_strerror(binding.RKV_EPERM).decode().startswith("reorder")


@pytest.mark.parametrize("g,heads,tokens", [(1, 2, 40), (2, 4, 70), (4, 4, 300), (8, 8, 33)])
def test_physical_layout_is_a_bijection(lib, g, heads, tokens):
    """Every (sequence, token, rotated channel) owns its own 2 bits inside the K-code and the
    V-code regions: no two codes share a slot and every slot index is in range."""
    cfg = R.RkvConfig(batch=2, n_q_heads=heads, n_kv_heads=heads, max_tokens=tokens, rot_heads=g)
    E = cfg.E
    for is_v in (False, True):
        seen = set()
        n_words = None
        for b in range(2):
            for t in list(range(0, tokens, 7)) + [tokens - 1]:
                for c in range(E):
                    w, sh, n_words = R.layout_locate(cfg, is_v, b, t, c)
                    assert 0 <= w < n_words and sh % 2 == 0 and 0 <= sh < 32
                    key = (w, sh)
                    assert key not in seen
                    seen.add(key)
        # one token's codes of one rotation group fill whole words: 16 codes per word
        words = {}
        for c in range(g * 128):
            w, sh, _ = R.layout_locate(cfg, is_v, 0, 3, c)
            words.setdefault(w, set()).add(sh)
        if not is_v:
            assert all(len(v) == 16 for v in words.values()) and len(words) == g * 128 // 16
        else:
            assert all(len(v) == 1 for v in words.values()) and len(words) == g * 128     # token-minor: one word per channel


@pytest.mark.parametrize("heads,bits,group,ok", [(52, 2, 128, True), (124, 2, 128, True), (128, 2, 128, False), (44, 4, 128, True),
                                                 (124, 3, 128, True), (128, 4, 128, False), (52, 2, 64, True), (56, 2, 64, False),
                                                 (40, 4, 32, True), (44, 4, 32, False), (52, 3, 64, False), (40, 3, 32, True)])
def test_whole_row_reorder_is_bounded_by_the_append_kernels_lds(lib, heads, bits, group, ok):
    """A reorder over the whole row with groups of 64 / 32 runs on the append kernel that stages the
    row in LDS: shapes beyond a compute unit's 160 KB fail at rkv_query_sizes, not at the first
    append.  With groups of 128 the matrix-core append kernel for such a reorder serves up to 127
    KV heads, whatever the code width."""
    cfg = R.RkvConfig(batch=1, n_q_heads=heads, n_kv_heads=heads, max_tokens=128, perm_span=heads * 128, bits=bits, quant_group=group)
    if ok:
        R.query_sizes(cfg)
    else:
        with pytest.raises(R.RkvError) as ei:
            R.query_sizes(cfg)
        assert ei.value.code == binding.RKV_EINVAL
    # the same head count is fine when the reorder stays inside the rotation groups
    R.query_sizes(R.RkvConfig(batch=1, n_q_heads=heads, n_kv_heads=heads, max_tokens=128, perm_span=512, bits=bits, quant_group=group))
