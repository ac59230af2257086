"""GPU parity: the HIP path, called through the C ABI, against the float64 oracle on the same
seeded inputs.  Bars: codes, scales, zeros, permutations and sink rows bit-exact (rounding ties as
documented in parity_utils); dequantized tensors within 1e-3 absolute (+2e-6 of the row's largest
magnitude, for the x100 sink rows); attention outputs within 2e-3 of max|ref| per (sequence,
head), log-sum-exp within 1e-3."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import rkv_oracle as O
import paper_2501_16383_amd as R
import rkv_synth as S
import parity_utils as P
from paper_2501_16383_amd import binding as RB

pytestmark = pytest.mark.gpu

ATT_TOL = 2e-3
LSE_TOL = 1e-3


def small(wname, **kw):
    return dataclasses.replace(S.WORKLOADS[wname], **kw)


def build_pair(w, cfg, T, perm=None, sink_positions=None, chunks=None, layer=0):
    """Fill a GPU cache and an oracle cache with the same tokens (optionally in several appends)."""
    k, v, mask, q = P.make_case(w, cfg, T, sink_positions=sink_positions, layer=layer)
    cache = R.RkvCache(cfg)
    oc = O.cache_new(P.oracle_cfg(cfg), perm)
    if perm is not None:
        cache.set_perm(P.gpu(np.asarray(perm, dtype=np.int32)))
    bounds = [0, T] if chunks is None else chunks
    use_mask = cfg.max_sinks > 0
    for a, b in zip(bounds[:-1], bounds[1:]):
        print(f"[case] append tokens {a}:{b} B={cfg.batch} Hkv={cfg.n_kv_heads} g={cfg.rot_heads} span={cfg.perm_span}", flush=True)
        cache.quantize_append(P.gpu(k[:, a:b]), P.gpu(v[:, a:b]), P.gpu(mask[:, a:b]) if use_mask else None)
        O.quantize_append(oc, k[:, a:b], v[:, a:b], mask[:, a:b] if use_mask else None)
    torch.cuda.synchronize()
    assert cache.length == T
    return cache, oc, q


def oracle_from_export(oc, g):
    oc2 = O.cache_new(oc.cfg, oc.perm)
    oc2.length = oc.length
    for name in ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero"):
        setattr(oc2, name, g[name])
    oc2.sink_pos, oc2.sink_k, oc2.sink_v = oc.sink_pos, oc.sink_k, oc.sink_v
    return oc2


def check_sinks(cache, oc):
    s = {k: v.cpu().numpy() for k, v in cache.export_sinks().items()}
    B, E = oc.cfg.batch, oc.cfg.E
    for b in range(B):
        assert s["count"][b] == len(oc.sink_pos[b])
        for i, pos in enumerate(oc.sink_pos[b]):
            assert s["pos"][b, i] == pos
            assert np.array_equal(s["k"][b, i], oc.sink_k[b][i].reshape(E))
            assert np.array_equal(s["v"][b, i], oc.sink_v[b][i].reshape(E))


def check_dequant(cache, oc_same_codes):
    kh, vh = cache.dequantize()
    torch.cuda.synchronize()
    kr, vr = O.dequantize_cache(oc_same_codes)
    for got, ref, name in ((kh.cpu().numpy().astype(np.float64), kr, "K"), (vh.cpu().numpy().astype(np.float64), vr, "V")):
        B, T = ref.shape[:2]
        n = oc_same_codes.cfg.n if name == "K" else oc_same_codes.cfg.head_dim
        rowmax = np.abs(ref).reshape(B, T, -1, n).max(-1, keepdims=True)
        err = np.abs(got - ref).reshape(B, T, -1, n)
        assert np.all(err <= 1e-3 + 2e-6 * rowmax), f"dequantized {name}: max err {err.max()}"
        print(f"[parity] dequantized {name}: max abs err {err.max():.3e}")


def check_decode(cache, oc_same_codes, q, q_pos=None, tag="", lse_relative=False, lse_bar=None):
    qp = None if q_pos is None else P.gpu(np.asarray(q_pos, dtype=np.int32))
    out, lse = cache.decode_attention(P.gpu(q), qp, want_lse=True)
    torch.cuda.synchronize()
    ref, lse_ref = O.decode_attention(oc_same_codes, q, q_pos)
    e = P.attention_error(out.cpu().numpy().astype(np.float64), ref)
    le = np.abs(lse.cpu().numpy() - lse_ref)
    if lse_relative:        # scores in the thousands (keys at the end of the fp16 range): fp32 carries them to ~1e-7 of their size
        le = le / np.maximum(1.0, np.abs(lse_ref))
    le = float(le.max())
    print(f"[parity] decode {tag}: out err {e:.3e}  lse err {le:.3e}", flush=True)
    assert e <= ATT_TOL and le <= (LSE_TOL if lse_bar is None else lse_bar(lse_ref))
    return e


def full_check(w, cfg, T, perm=None, sink_positions=None, chunks=None, q_pos=None, paths=(1,), lse_bar=None):
    cache, oc, q = build_pair(w, cfg, T, perm, sink_positions, chunks)
    g, _, _ = P.check_cache_against_oracle(cache, oc, f"{w.name} T={T}")
    check_sinks(cache, oc)
    oc_g = oracle_from_export(oc, g)
    check_dequant(cache, oc_g)
    for path in paths:
        cache.set_decode_path(path)
        check_decode(cache, oc_g, q, q_pos, tag=f"own codes path={path}", lse_bar=lse_bar)
    # the oracle's codes through the GPU read half
    P.import_oracle_codes(cache, oc)
    for path in paths:
        cache.set_decode_path(path)
        check_decode(cache, oc, q, q_pos, tag=f"oracle codes path={path}", lse_bar=lse_bar)
    return cache, oc, q


def calibrated_perm(w, cfg, offset_variant=False):
    kc, _, _ = S.make_kv(w, 256, batch=1, stream=1, sink_positions=[], offset_variant=offset_variant)
    perm_gpu = R.calibrate_perm(cfg, P.gpu(kc[0]))
    torch.cuda.synchronize()
    perm_ref = O.calibrate_perm(kc[0], P.oracle_cfg(cfg))
    pg = perm_gpu.cpu().numpy()
    assert sorted(pg.tolist()) == list(range(cfg.E))
    if not np.array_equal(pg, perm_ref):
        # only channels whose float64 sums are closer than 1e-9 relative may swap
        rows = kc[0].astype(np.float64).reshape(-1, cfg.E)
        sums = O.rotate_groups(rows, cfg.rot_heads * 128).sum(0)
        diff = np.nonzero(pg != perm_ref)[0]
        for i in diff:
            a, b = sums[pg[i]], sums[perm_ref[i]]
            assert abs(a - b) <= 1e-9 * max(abs(a), abs(b), 1e-300), "permutation differs beyond float64 ties"
    return perm_ref


def test_cfg0_full():
    """Config 0 in full: 1 x 32 heads x 512 tokens, rotation over 2 heads, 1 sink, calibrated per-head reorder."""
    w = S.WORKLOADS["cfg0"]
    cfg = R.RkvConfig(batch=1, n_q_heads=32, n_kv_heads=32, max_tokens=512, max_sinks=1, rot_heads=2, perm_span=128)
    perm = calibrated_perm(w, cfg)
    full_check(w, cfg, 512, perm=perm, paths=(1, 2))


def test_cfg1_slice_ragged():
    """LLaMA-2-7B-shaped slice: rotation over 4 heads, 4 sinks, a ragged length spanning several tiles."""
    w = small("cfg1", n_q_heads=8, n_kv_heads=8)
    cfg = R.RkvConfig(batch=2, n_q_heads=8, n_kv_heads=8, max_tokens=700, max_sinks=4, rot_heads=4, perm_span=128)
    perm = calibrated_perm(w, cfg)
    full_check(w, cfg, 613, perm=perm, paths=(1, 2))


def test_no_sinks_and_query_position():
    """Without sinks nothing hides errors of the 2-bit stream; the query sits past the cache."""
    w = small("cfg2", n_q_heads=8, n_kv_heads=8, n_sinks=0)
    cfg = R.RkvConfig(batch=2, n_q_heads=8, n_kv_heads=8, max_tokens=400, max_sinks=0, rot_heads=4, perm_span=128)
    full_check(w, cfg, 389, sink_positions=[], q_pos=[400, 1234], paths=(1, 2))


def test_sinks_at_other_positions_and_overflow():
    """Sinks away from the start of the sequence, more flagged tokens than max_sinks."""
    w = small("cfg1", n_q_heads=4, n_kv_heads=4)
    cfg = R.RkvConfig(batch=2, n_q_heads=4, n_kv_heads=4, max_tokens=256, max_sinks=3, rot_heads=4, perm_span=128)
    full_check(w, cfg, 200, sink_positions=[0, 17, 110, 150, 199], chunks=[0, 100, 200], paths=(1, 2))


@pytest.mark.parametrize("span_kind", ["group", "row"])
def test_reorder_across_blocks(span_kind):
    """perm_span = rotation size and = whole row (Alg. 1 as printed): the reorder changes the blocks."""
    w = small("cfg1", n_q_heads=8, n_kv_heads=8)
    span = 512 if span_kind == "group" else 1024
    cfg = R.RkvConfig(batch=1, n_q_heads=8, n_kv_heads=8, max_tokens=128, max_sinks=4, rot_heads=4, perm_span=span)
    perm = calibrated_perm(w, cfg, offset_variant=True)
    assert not np.array_equal(perm // 128, np.arange(cfg.E) // 128)
    # a reorder inside the rotation group has a variant of both matrix-core kernels, and so has one across groups
    # (read half: the scores from a kernel of their own; write half: the keys from one that sees whole token rows)
    cache, _, _ = full_check(w, cfg, 100, perm=perm, paths=(1, 2), sink_positions=[])
    cache.set_decode_path(0)
    if span_kind == "group":
        assert cache.decode_kernel() == RB.KERNEL_MFMA_CROSS and cache.append_kernel() == RB.KERNEL_MFMA_CROSS
    else:
        assert cache.decode_kernel() == RB.KERNEL_MFMA_ROW and cache.append_kernel() == RB.KERNEL_MFMA_ROW


def check_two_query_tokens(cache, oc, q, hq, hkv, tag):
    """Two causal query tokens per sequence on a configuration without the plain matrix-core kernel:
    rkv_decode_attention_multi takes the configuration's own route (the scores kernel sees the query
    tokens as further query heads; at most 8 (query token, query head) pairs per KV head, refused
    beyond), and the general kernel when that is forced.  Both against the oracle on the GPU's own codes."""
    q2 = np.stack([q, q[::-1].copy()], axis=1)
    q_pos = np.array([[600, 601], [300, 612]], dtype=np.int32)
    if (hq // hkv) * 2 > 8:
        with pytest.raises(R.RkvError):
            cache.decode_attention_multi(P.gpu(q2), P.gpu(q_pos))
        return
    ref, lse_ref = O.decode_attention_multi(oracle_from_export(oc, P.export_numpy(cache)), q2, q_pos)
    for path in (0, 1):
        cache.set_decode_path(path)
        assert cache.decode_kernel(2) == (cache.decode_kernel() if path == 0 else RB.KERNEL_GENERAL)
        assert path == 1 or cache.decode_kernel(2) != RB.KERNEL_GENERAL
        out, lse = cache.decode_attention_multi(P.gpu(q2), P.gpu(q_pos), want_lse=True)
        torch.cuda.synchronize()
        e = P.attention_error(out.cpu().numpy().astype(np.float64), ref)
        le = float(np.abs(lse.cpu().numpy() - lse_ref).max())
        print(f"[parity] {tag}: two query tokens, path {path}: out err {e:.3e} lse err {le:.3e}", flush=True)
        assert e <= ATT_TOL and le <= LSE_TOL
    cache.set_decode_path(0)


@pytest.mark.parametrize("g,hq,style", [(4, 8, 0), (2, 8, 0), (4, 32, 0), (2, 16, 1), (4, 8, 1), (4, 64, 0)])
def test_reorder_over_the_whole_row_on_matrix_cores(g, hq, style):
    """perm_span = the whole token row (Alg. 1 as printed): a rotated channel belongs to any of the
    row's quantization blocks.  The read half's path for it - scores from k_scores_row (elements
    dequantized, split into two fp16 parts, rotated on the matrix cores), softmax and values from
    the matrix-core decode kernel - against the oracle and the general kernel: rotation over 4 and 2
    heads, GQA up to 8 query heads per KV head, both RoPE pairings, several chunks and a ragged
    tail, with and without retained sink rows, the current token as an exact row, single-token
    steps, sequences of different lengths, the work space built into the library.  The write half
    of this setting: k_append_row_keys (the quantization blocks span all rotation groups of a token)."""
    w = small("cfg1", n_q_heads=hq, n_kv_heads=8)
    cfg = R.RkvConfig(batch=2, n_q_heads=hq, n_kv_heads=8, max_tokens=700, max_sinks=4, rot_heads=g, perm_span=1024, rope_style=style)
    perm = calibrated_perm(w, cfg, offset_variant=True)
    assert not np.array_equal(perm // (128 * g), np.arange(cfg.E) // (128 * g))       # channels leave their rotation groups
    cache, oc, q = full_check(w, cfg, 613, perm=perm, chunks=[0, 300, 301, 613], paths=(1, 2),
                              sink_positions=None if (g, hq, style) in ((4, 8, 0), (2, 16, 1)) else [])
    cache.set_decode_path(2)
    assert cache.decode_kernel() == RB.KERNEL_MFMA_ROW and cache.append_kernel() == RB.KERNEL_MFMA_ROW
    k1, v1, _ = S.make_kv(w, 1, batch=2, stream=5, sink_positions=[])
    out = cache.decode_attention(P.gpu(q), k_cur=P.gpu(k1[:, 0]), v_cur=P.gpu(v1[:, 0]))      # the cache holds the oracle's codes here
    torch.cuda.synchronize()
    ref, _ = O.decode_attention(oc, q, None, k1[:, 0], v1[:, 0])
    assert P.attention_error(out.cpu().numpy().astype(np.float64), ref) <= ATT_TOL
    out = cache.decode_step(P.gpu(k1), P.gpu(v1), P.gpu(q))
    torch.cuda.synchronize()
    O.quantize_append(oc, k1, v1, None)
    ref, _ = O.decode_attention(oracle_from_export(oc, P.export_numpy(cache)), q)
    assert P.attention_error(out.cpu().numpy().astype(np.float64), ref) <= ATT_TOL
    cache.set_decode_path(0)
    check_two_query_tokens(cache, oc, q, hq, 8, f"whole-row reorder g={g} hq={hq}")
    # against the general kernel on the same cache, and on the work space built into the library
    cache.set_decode_path(1)
    o_gen, l_gen = cache.decode_attention(P.gpu(q), want_lse=True)
    cache.set_decode_path(0)
    o_row, l_row = cache.decode_attention(P.gpu(q), want_lse=True)
    o_st = torch.empty_like(o_row)
    cache.decode_attention_static(P.gpu(q), o_st)
    torch.cuda.synchronize()
    assert P.attention_error(o_row.cpu().numpy().astype(np.float64), o_gen.cpu().numpy().astype(np.float64)) <= 1e-4
    assert float((l_row - l_gen).abs().max()) <= 1e-4
    assert torch.equal(o_st, o_row)
    # sequences of different lengths: a cache cut back, then one filled by rkv_quantize_append_ragged
    cache.truncate([500, 133])
    assert cache.lengths == [500, 133]
    o_row = cache.decode_attention(P.gpu(q))
    cache.set_decode_path(1)
    o_gen = cache.decode_attention(P.gpu(q))
    torch.cuda.synchronize()
    assert P.attention_error(o_row.cpu().numpy().astype(np.float64), o_gen.cpu().numpy().astype(np.float64)) <= 1e-4
    k, v, mask = S.make_kv(w, 60, batch=2)
    rag = R.RkvCache(cfg)
    rag.set_perm(P.gpu(np.asarray(perm, dtype=np.int32)))
    rag.quantize_append_ragged(P.gpu(k[:, :50]), P.gpu(v[:, :50]), [50, 21], P.gpu(mask[:, :50]))
    rag.quantize_append_ragged(P.gpu(k[:, 50:60]), P.gpu(v[:, 50:60]), [3, 10], None)
    assert rag.lengths == [53, 31]
    o_rag = rag.decode_attention(P.gpu(q))
    g_rag = P.export_numpy(rag)
    torch.cuda.synchronize()
    for bb, parts in enumerate([[(0, 50), (50, 53)], [(0, 21), (50, 60)]]):     # each sequence alone in the oracle
        oc1 = O.cache_new(P.oracle_cfg(dataclasses.replace(cfg, batch=1)), perm)
        for a_, b_ in parts:
            O.quantize_append(oc1, k[bb:bb + 1, a_:b_], v[bb:bb + 1, a_:b_], mask[bb:bb + 1, a_:b_] if a_ == 0 else None)
        n_b = oc1.length
        gb = {name: arr[bb:bb + 1, :n_b] for name, arr in g_rag.items()}
        P.compare_codes(oc1.k_rot, oc1.k_codes, oc1.k_scale, oc1.k_zero, gb["k_codes"], gb["k_scale"], gb["k_zero"],
                        f"whole-row ragged b={bb} K", rot_span=cfg.E)
        P.compare_codes(oc1.v_in, oc1.v_codes, oc1.v_scale, oc1.v_zero, gb["v_codes"], gb["v_scale"], gb["v_zero"], f"whole-row ragged b={bb} V")
        ref, _ = O.decode_attention(oracle_from_export(oc1, gb), q[bb:bb + 1])
        assert P.attention_error(o_rag[bb:bb + 1].cpu().numpy().astype(np.float64), ref) <= ATT_TOL


@pytest.mark.parametrize("heads,bits", [(64, 2), (60, 2), (60, 4), (64, 3)])
def test_whole_row_reorder_with_many_heads(heads, bits):
    """A row of 64 KV heads (8192 channels, 64 quantization blocks) under a reorder over the whole
    row: beyond what the general append kernel's LDS holds (53 heads), within what the matrix-core
    kernels for this reorder serve; both read paths against the oracle.  64 blocks take the scores
    kernel that stages rows in LDS, 60 the one with a table per wave (61 KB of tables: more dynamic
    LDS than a launch gets without asking).  Wider codes: the write half serves them at any of these
    sizes, the read half up to 63 blocks (64 blocks: the general decode kernel)."""
    w = small("cfg1", n_q_heads=heads, n_kv_heads=heads)
    cfg = R.RkvConfig(batch=1, n_q_heads=heads, n_kv_heads=heads, max_tokens=128, max_sinks=4, rot_heads=4, perm_span=heads * 128,
                      bits=bits)
    perm = calibrated_perm(w, dataclasses.replace(cfg, bits=2), offset_variant=True)
    fast_read = bits == 2 or heads < 64
    cache, _, _ = full_check(w, cfg, 90, perm=perm, chunks=[0, 40, 41, 90], paths=(1, 2) if fast_read else (1, 0), sink_positions=[])
    cache.set_decode_path(0)
    assert cache.decode_kernel() == (RB.KERNEL_MFMA_ROW if fast_read else RB.KERNEL_GENERAL) and cache.append_kernel() == RB.KERNEL_MFMA_ROW


@pytest.mark.parametrize("g,hq,style,fmt", [(4, 8, 0, 0), (2, 8, 0, 0), (4, 32, 0, 0), (2, 16, 1, 0), (4, 8, 1, 0), (4, 8, 0, 1), (2, 16, 0, 1)])
def test_reorder_inside_rotation_group_on_matrix_cores(g, hq, style, fmt):
    """perm_span = the rotation size: the quantization blocks mix channels of all the group's heads.
    The decode path for this setting (scores kernel with the rotation group's blocks in its table,
    then the matrix-core kernel's softmax and value phases) against the oracle and against the general kernel: rotation over 4 and 2 heads, GQA,
    both RoPE pairings, both metadata formats, several chunks and a ragged tail, sinks, single-token
    steps, the current token as an exact row."""
    w = small("cfg1", n_q_heads=hq, n_kv_heads=8)
    cfg = R.RkvConfig(batch=2, n_q_heads=hq, n_kv_heads=8, max_tokens=700, max_sinks=4, rot_heads=g, perm_span=128 * g,
                      rope_style=style, meta_format=fmt)
    perm = calibrated_perm(w, cfg, offset_variant=True)
    assert not np.array_equal(perm // 128, np.arange(cfg.E) // 128)
    # all but the first case without retained fp16 rows, so that the compressed stream alone decides the outputs
    cache, oc, q = full_check(w, cfg, 613, perm=perm, chunks=[0, 300, 301, 302, 613], paths=(1, 2),
                              sink_positions=None if (g, hq, style, fmt) == (4, 8, 0, 0) else [])
    cache.set_decode_path(2)
    assert cache.decode_kernel() == RB.KERNEL_MFMA_CROSS and cache.append_kernel() == RB.KERNEL_MFMA_CROSS
    k1, v1, _ = S.make_kv(w, 1, batch=2, stream=5, sink_positions=[])
    out = cache.decode_attention(P.gpu(q), k_cur=P.gpu(k1[:, 0]), v_cur=P.gpu(v1[:, 0]))      # the cache holds the oracle's codes here
    torch.cuda.synchronize()
    ref, _ = O.decode_attention(oc, q, None, k1[:, 0], v1[:, 0])
    assert P.attention_error(out.cpu().numpy().astype(np.float64), ref) <= ATT_TOL
    out = cache.decode_step(P.gpu(k1), P.gpu(v1), P.gpu(q))
    torch.cuda.synchronize()
    O.quantize_append(oc, k1, v1, None)
    ref, _ = O.decode_attention(oracle_from_export(oc, P.export_numpy(cache)), q)
    assert P.attention_error(out.cpu().numpy().astype(np.float64), ref) <= ATT_TOL
    cache.set_decode_path(0)
    check_two_query_tokens(cache, oc, q, hq, 8, f"cross-block reorder g={g} hq={hq} fmt={fmt}")
    cache.set_decode_path(2)
    if (hq // 8) * 2 > 8:                                        # (beyond 8 rows per KV head: refused, not mis-computed)
        with pytest.raises(R.RkvError):
            cache.decode_attention_multi(P.gpu(np.stack([q, q], axis=1)), P.gpu(np.array([[600, 601], [600, 601]], dtype=np.int32)))
    # sequences of different lengths, and the one-call step against the two calls, bit for bit
    k, v, mask = S.make_kv(w, 40, batch=2)
    a, b = R.RkvCache(cfg), R.RkvCache(cfg)
    for c in (a, b):
        c.set_perm(P.gpu(np.asarray(perm, dtype=np.int32)))
        c.quantize_append_ragged(P.gpu(k[:, :33]), P.gpu(v[:, :33]), [33, 21], P.gpu(mask[:, :33]))
    for s_ in range(4):
        qq = P.gpu(S.make_q(w, batch=2, step=s_))
        kk, vv = P.gpu(k[:, 33 + s_:34 + s_]), P.gpu(v[:, 33 + s_:34 + s_])
        o1 = a.decode_step(kk, vv, qq)
        b.quantize_append(kk, vv)
        o2 = b.decode_attention(qq)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2), f"step {s_}"
    ea, eb = a.export_codes(), b.export_codes()
    torch.cuda.synchronize()
    assert a.lengths == [37, 25] and all(torch.equal(ea[name], eb[name]) for name in ea)
    oc1 = O.cache_new(P.oracle_cfg(dataclasses.replace(cfg, batch=1)), perm)                 # sequence 1 alone in the oracle
    O.quantize_append(oc1, np.concatenate([k[1:2, :21], k[1:2, 33:37]], axis=1), np.concatenate([v[1:2, :21], v[1:2, 33:37]], axis=1),
                      np.concatenate([mask[1:2, :21], np.zeros((1, 4), np.uint8)], axis=1))
    g1 = {name: arr[1:2, :25].cpu().numpy() for name, arr in ea.items()}
    for name in ("k_codes", "v_codes"):
        g1[name] = O.unpack_canonical(g1[name])
    P.compare_codes(oc1.k_rot, oc1.k_codes, oc1.k_scale, oc1.k_zero, g1["k_codes"], g1["k_scale"].astype(np.float64),
                    g1["k_zero"].astype(np.float64), "cross-block ragged K", rot_span=128 * g, meta_format=fmt)


def test_gqa_llama3_shape():
    """Config 4's geometry on a slice: 4 query heads per KV head, rope base 500000."""
    w = small("cfg4", n_q_heads=16, n_kv_heads=4)
    cfg = R.RkvConfig(batch=2, n_q_heads=16, n_kv_heads=4, max_tokens=300, max_sinks=4, rot_heads=4, perm_span=128,
                      rope_theta=500000.0)
    full_check(w, cfg, 270, paths=(1, 2))
    full_check(w, cfg, 270, paths=(1, 2), sink_positions=[])       # and with nothing but the compressed stream


@pytest.mark.parametrize("g,style,vrot", [(1, 0, 1), (2, 1, 0), (8, 0, 1), (4, 1, 1), (4, 1, 0), (1, 1, 0)])
def test_variants(g, style, vrot):
    """Other rotation sizes, interleaved RoPE pairing, library-side value rotation."""
    w = small("cfg1", n_q_heads=8, n_kv_heads=8)
    cfg = R.RkvConfig(batch=1, n_q_heads=8, n_kv_heads=8, max_tokens=160, max_sinks=2, rot_heads=g, perm_span=128,
                      rope_style=style, v_rotate=vrot)
    cache, _, _ = full_check(w, cfg, 150, sink_positions=[0, 3], paths=(1, 2) if g in (2, 4) else (1, 0))
    cache.set_decode_path(0)
    assert cache.decode_kernel() == (RB.KERNEL_MFMA if g in (2, 4) else RB.KERNEL_GENERAL)
    assert cache.append_kernel() == (RB.KERNEL_GENERAL if g in (1, 8) else RB.KERNEL_SHUFFLE if vrot else RB.KERNEL_MFMA)


def test_incremental_append_matches_bulk():
    """Prefill in uneven pieces, then single-token decode steps: same cache as one bulk append."""
    w = small("cfg1", n_q_heads=4, n_kv_heads=4)
    cfg = R.RkvConfig(batch=2, n_q_heads=4, n_kv_heads=4, max_tokens=128, max_sinks=4, rot_heads=4, perm_span=128)
    chunks = [0, 37] + list(range(38, 60)) + [111]
    cache, oc, q = build_pair(w, cfg, 111, chunks=chunks)
    bulk, oc_b, _ = build_pair(w, cfg, 111)
    a, b = cache.export_codes(), bulk.export_codes()
    torch.cuda.synchronize()
    for name in a:
        assert torch.equal(a[name], b[name]), name
    P.check_cache_against_oracle(cache, oc, "incremental")
    check_sinks(cache, oc)


def test_reset_and_reuse():
    w = small("cfg1", n_q_heads=4, n_kv_heads=4)
    cfg = R.RkvConfig(batch=1, n_q_heads=4, n_kv_heads=4, max_tokens=64, max_sinks=4, rot_heads=4)
    cache, oc, q = build_pair(w, cfg, 50)
    cache.reset()
    assert cache.length == 0
    k, v, mask, q = P.make_case(w, cfg, 33, layer=3)
    cache.quantize_append(P.gpu(k), P.gpu(v), P.gpu(mask))
    oc2 = O.cache_new(P.oracle_cfg(cfg))
    O.quantize_append(oc2, k, v, mask)
    g, _, _ = P.check_cache_against_oracle(cache, oc2, "after reset")
    check_sinks(cache, oc2)
    check_decode(cache, oracle_from_export(oc2, g), q, tag="after reset")


def test_error_codes():
    w = small("cfg1", n_q_heads=4, n_kv_heads=4)
    cfg = R.RkvConfig(batch=1, n_q_heads=4, n_kv_heads=4, max_tokens=20, max_sinks=1, rot_heads=4)
    cache = R.RkvCache(cfg)
    q = P.gpu(S.make_q(w, batch=1))
    with pytest.raises(R.RkvError) as ei:
        cache.decode_attention(q)
    assert ei.value.code == -5
    k, v, mask, _ = P.make_case(w, cfg, 21)
    with pytest.raises(R.RkvError) as ei:
        cache.quantize_append(P.gpu(k), P.gpu(v))
    assert ei.value.code == -2
    bad = np.arange(cfg.E, dtype=np.int32)
    bad[0] = 1
    with pytest.raises(R.RkvError) as ei:
        cache.set_perm(P.gpu(bad))
    assert ei.value.code == -3
    cross = np.arange(cfg.E, dtype=np.int32)
    cross[0], cross[200] = 200, 0
    with pytest.raises(R.RkvError) as ei:
        cache.set_perm(P.gpu(cross))
    assert ei.value.code == -3
    cache.quantize_append(P.gpu(k[:, :5]), P.gpu(v[:, :5]))
    with pytest.raises(R.RkvError) as ei:
        cache.set_perm(P.gpu(np.arange(cfg.E, dtype=np.int32)))
    assert ei.value.code == -5


def check_slice(exp, out, lse, b, rg, ks, vs, ms, q, perm=None, max_sinks=4, tag="", meta_format=0, rep=1, rope_theta=10000.0,
                bits=2, group=128, span=128):
    """One (sequence, rotation group of 4 heads) slice of a full-size run against the oracle: a
    rotation group's codes and attention outputs depend on nothing outside the slice.  The codes
    must equal the oracle's outside the documented rounding ties; the attention output is then
    compared on the GPU's own codes, so that a tie cannot hide in (or leak into) the tolerance.
    exp: export_codes() tensors already on the host (numpy)."""
    ocfg = O.OracleConfig(batch=1, n_q_heads=4 * rep, n_kv_heads=4, rot_heads=4, perm_span=span, max_sinks=max_sinks,
                          meta_format=meta_format, rope_theta=rope_theta, bits=bits, quant_group=group)
    hq = slice(4 * rep * rg, 4 * rep * (rg + 1))               # the query heads of the group's four KV heads
    oc = O.cache_new(ocfg, None if perm is None else perm[512 * rg:512 * (rg + 1)] - 512 * rg)
    O.quantize_append(oc, ks, vs, ms)
    nb = 512 // (4 if bits == 2 else 2)                         # canonical bytes of the group's 512 codes
    nm = 512 // group                                           # metadata entries of the group
    sl_c, sl_m = slice(nb * rg, nb * (rg + 1)), slice(nm * rg, nm * (rg + 1))
    g = {}
    for name in ("k", "v"):
        g[name + "_codes"] = O.unpack_canonical(exp[name + "_codes"][b:b + 1, :, sl_c], bits)
        g[name + "_scale"] = exp[name + "_scale"][b:b + 1, :, sl_m].astype(np.float64)
        g[name + "_zero"] = exp[name + "_zero"][b:b + 1, :, sl_m].astype(np.float64)
    P.compare_codes(oc.k_rot, oc.k_codes, oc.k_scale, oc.k_zero, g["k_codes"], g["k_scale"], g["k_zero"],
                    f"{tag} b={b} rg={rg} K", rot_span=512, meta_format=meta_format, bits=bits, group=group)
    P.compare_codes(oc.v_in, oc.v_codes, oc.v_scale, oc.v_zero, g["v_codes"], g["v_scale"], g["v_zero"],
                    f"{tag} b={b} rg={rg} V", meta_format=meta_format, bits=bits, group=group)
    for name, val in g.items():                                # attention on the GPU's own codes
        setattr(oc, name, val)
    ref, lse_ref = O.decode_attention(oc, q[b:b + 1, hq])
    e = P.attention_error(out[b:b + 1, hq], ref)
    le = float(np.abs(lse[b:b + 1, hq] - lse_ref).max())
    print(f"[parity] {tag} b={b} rg={rg}: out err {e:.3e} lse err {le:.3e}", flush=True)
    assert e <= ATT_TOL and le <= LSE_TOL


def export_host(cache):
    exp = cache.export_codes()
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in exp.items()}


@pytest.mark.parametrize("meta_format,bits,with_sinks,group,span", [(0, 2, True, 128, 128), (0, 2, False, 128, 128), (1, 2, True, 128, 128),
                                                                   (0, 4, True, 128, 128), (1, 3, False, 128, 128), (0, 2, False, 64, 128),
                                                                   (0, 2, True, 32, 128), (0, 2, False, 128, 512), (1, 3, False, 64, 128),
                                                                   (0, 4, False, 32, 128)])
def test_full_size_config2_sampled(meta_format, bits, with_sinks, group, span):
    """Configuration 2 (the throughput target) at full size (batch 16, 40 heads, context 4096), in the launch
    configuration bench.py times: bulk append of 4095 tokens, then one rkv_decode_step (the last
    token's append and the attention on the matrix-core path).  The oracle recomputes sampled (sequence, rotation group) slices - a
    rotation group's codes and attention outputs depend on nothing outside the slice.  Once with
    fp16 metadata, once with the FP8 scale / INT8 zero-point storage, once with 4-bit codes, once with 3-bit codes and FP8 / INT8 metadata,
    with quantization groups of 64 and 32 (Table tab:quantgrani: the sub-group variants of both matrix-core kernels),
    and with the reorder over the rotation group (span 512: quantization blocks mix the group's four heads).
    With the workload's four fp16 sink rows, as bench.py runs it, and with no retained rows at
    all: the sink keys are a hundred times the rest and take nearly all the softmax weight, so only
    the run without them lets the compressed stream decide the outputs."""
    w = S.WORKLOADS["cfg2"]
    T = w.context
    n_keep = 4 if with_sinks else 0
    cfg = R.RkvConfig(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, max_tokens=T, max_sinks=n_keep,
                      rot_heads=4, perm_span=span, meta_format=meta_format, bits=bits, quant_group=group)
    perm = calibrated_perm(w, cfg, offset_variant=span != 128)
    assert span == 128 or not np.array_equal(perm // 128, np.arange(cfg.E) // 128)
    cache = R.RkvCache(cfg)
    cache.set_perm(P.gpu(np.asarray(perm, dtype=np.int32)))
    samples = [(0, 0), (7, 3), (15, 9)]
    keep = {}
    print("[case] full-size config 2: generating inputs per sequence", flush=True)
    k_parts, v_parts, m_parts = [], [], []
    rng_w = dataclasses.replace(w)
    for b in range(w.batch):
        kb, vb, mb = S.make_kv(dataclasses.replace(rng_w, seed=w.seed + 100 * b), T, batch=1, sink_positions=None if with_sinks else [])
        for (sb, rg) in samples:
            if sb == b:
                keep[(sb, rg)] = (kb[:, :, 4 * rg:4 * rg + 4].copy(), vb[:, :, 4 * rg:4 * rg + 4].copy(), mb.copy())
        k_parts.append(torch.from_numpy(kb))
        v_parts.append(torch.from_numpy(vb))
        m_parts.append(torch.from_numpy(mb))
    k = torch.cat(k_parts).cuda()
    v = torch.cat(v_parts).cuda()
    mask = torch.cat(m_parts).cuda()
    del k_parts, v_parts
    q = S.make_q(w)
    print("[case] full-size config 2: bulk append 4095 + one decode step (append 1 + attention, as bench.py does)", flush=True)
    cache.quantize_append(k[:, :T - 1].contiguous(), v[:, :T - 1].contiguous(), mask[:, :T - 1].contiguous() if with_sinks else None)
    cache.set_decode_path(2)
    # the kernels bench.py times, not a fall-back to the general ones
    want_kind = RB.KERNEL_MFMA_CROSS if span != 128 else RB.KERNEL_MFMA if group == 128 else RB.KERNEL_MFMA_SUB
    assert cache.decode_kernel() == want_kind and cache.append_kernel() == want_kind
    assert not bool(mask[:, T - 1:].any())                  # the step's token is an ordinary one
    out, lse = cache.decode_step(k[:, T - 1:].contiguous(), v[:, T - 1:].contiguous(), P.gpu(q), want_lse=True)
    exp = export_host(cache)
    assert cache.length == T
    out = out.cpu().numpy().astype(np.float64)
    lse = lse.cpu().numpy().astype(np.float64)
    assert np.isfinite(out).all()
    for (b, rg) in samples:
        ks, vs, ms = keep[(b, rg)]
        check_slice(exp, out, lse, b, rg, ks, vs, ms if with_sinks else None, q, perm=perm, max_sinks=n_keep,
                    tag=f"full-size meta_format={meta_format} bits={bits} sinks={with_sinks} group={group} span={span}",
                    meta_format=meta_format, bits=bits, group=group, span=span)


@pytest.mark.parametrize("with_sinks,bits,group", [(False, 2, 128), (True, 2, 128), (False, 4, 128), (False, 3, 128), (False, 2, 64)])
def test_full_size_config2_whole_row_reorder_sampled(with_sinks, bits, group):
    """Configuration 2's geometry with the reorder over the whole token row (perm_span = 5120:
    Alg. 1 as printed), at full size: bulk append, then decode attention on the path bench.py
    times for this setting (scores kernel + matrix-core decode kernel).  With such a reorder a
    quantization block mixes channels of every rotation group, so the oracle recomputes whole
    sequences (two of the sixteen, all 40 heads): codes under the tie protocol, then attention on
    the GPU's own codes.  Also with 4- and 3-bit codes (the scores kernel then runs once per plane
    of code bits) and with groups of 64 (once per share of the row's 80 blocks)."""
    w = S.WORKLOADS["cfg2"]
    T = w.context
    n_keep = 4 if with_sinks else 0
    cfg = R.RkvConfig(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, max_tokens=T, max_sinks=n_keep,
                      rot_heads=4, perm_span=w.n_kv_heads * 128, bits=bits, quant_group=group)
    perm = calibrated_perm(w, dataclasses.replace(cfg, bits=2, quant_group=128), offset_variant=True)
    assert not np.array_equal(perm // 512, np.arange(cfg.E) // 512)
    cache = R.RkvCache(cfg)
    cache.set_perm(P.gpu(np.asarray(perm, dtype=np.int32)))
    assert cache.decode_kernel() == RB.KERNEL_MFMA_ROW and cache.append_kernel() == RB.KERNEL_MFMA_ROW
    sampled = (3, 15)
    keep, k_parts, v_parts, m_parts = {}, [], [], []
    print("[case] full-size config 2, whole-row reorder: generating inputs per sequence", flush=True)
    for b in range(w.batch):
        kb, vb, mb = S.make_kv(dataclasses.replace(w, seed=w.seed + 100 * b), T, batch=1, sink_positions=None if with_sinks else [])
        if b in sampled:
            keep[b] = (kb.copy(), vb.copy(), mb.copy())
        k_parts.append(torch.from_numpy(kb))
        v_parts.append(torch.from_numpy(vb))
        m_parts.append(torch.from_numpy(mb))
    k, v, mask = torch.cat(k_parts).cuda(), torch.cat(v_parts).cuda(), torch.cat(m_parts).cuda()
    del k_parts, v_parts
    q = S.make_q(w)
    print("[case] full-size config 2, whole-row reorder: bulk append 4096 + decode attention", flush=True)
    cache.quantize_append(k, v, mask if with_sinks else None)
    out, lse = cache.decode_attention(P.gpu(q), want_lse=True)
    exp = export_host(cache)
    out = out.cpu().numpy().astype(np.float64)
    lse = lse.cpu().numpy().astype(np.float64)
    assert np.isfinite(out).all() and cache.length == T
    ocfg = P.oracle_cfg(dataclasses.replace(cfg, batch=1))
    for b in sampled:
        kb, vb, mb = keep[b]
        oc = O.cache_new(ocfg, perm)
        O.quantize_append(oc, kb, vb, mb if with_sinks else None)
        g = {}
        for name in ("k", "v"):
            g[name + "_codes"] = O.unpack_canonical(exp[name + "_codes"][b:b + 1], bits)
            g[name + "_scale"] = exp[name + "_scale"][b:b + 1].astype(np.float64)
            g[name + "_zero"] = exp[name + "_zero"][b:b + 1].astype(np.float64)
        P.compare_codes(oc.k_rot, oc.k_codes, oc.k_scale, oc.k_zero, g["k_codes"], g["k_scale"], g["k_zero"],
                        f"whole-row full size b={b} K", rot_span=cfg.E, bits=bits, group=group)    # (a block's members come from any rotation group)
        P.compare_codes(oc.v_in, oc.v_codes, oc.v_scale, oc.v_zero, g["v_codes"], g["v_scale"], g["v_zero"], f"whole-row full size b={b} V",
                        bits=bits, group=group)
        for name, val in g.items():                            # attention on the GPU's own codes
            setattr(oc, name, val)
        ref, lse_ref = O.decode_attention(oc, q[b:b + 1])
        e = P.attention_error(out[b:b + 1], ref)
        le = float(np.abs(lse[b:b + 1] - lse_ref).max())
        print(f"[parity] whole-row full size sinks={with_sinks} b={b}: out err {e:.3e} lse err {le:.3e}", flush=True)
        assert e <= ATT_TOL and le <= LSE_TOL


def test_full_size_long_context_sampled():
    """Configuration 3's shape: one sequence of 32768 tokens, 32 heads; prefill-size quantize, then
    split-K decode over 128 chunks.  One rotation group is recomputed by the oracle."""
    w = S.WORKLOADS["cfg3"]
    T = w.context
    cfg = R.RkvConfig(batch=1, n_q_heads=32, n_kv_heads=32, max_tokens=T, max_sinks=4, rot_heads=4, perm_span=128)
    cache = R.RkvCache(cfg)
    k, v, mask = S.make_kv(w, T)
    q = S.make_q(w)
    print("[case] long context: bulk append 32768 + decode", flush=True)
    cache.quantize_append(P.gpu(k), P.gpu(v), P.gpu(mask))
    assert cache.decode_kernel() == RB.KERNEL_MFMA and cache.append_kernel() == RB.KERNEL_MFMA
    out, lse = cache.decode_attention(P.gpu(q), want_lse=True)
    exp = export_host(cache)
    out = out.cpu().numpy().astype(np.float64)
    lse = lse.cpu().numpy().astype(np.float64)
    rg = 5
    check_slice(exp, out, lse, 0, rg, k[:, :, 4 * rg:4 * rg + 4], v[:, :, 4 * rg:4 * rg + 4], mask, q, tag="long context")


@pytest.mark.parametrize("with_sinks", [True, False])
def test_full_size_config4_gqa_sampled(with_sinks):
    """(With the workload's four fp16 sink rows, as bench.py runs it, and without any, so that the
    compressed stream alone decides the outputs.)  Configuration 4 at full size (batch 32, 32 query / 8 KV heads, context 8192, RoPE base
    500000) in the launch configuration bench.py times: bulk append of 8191 tokens, then one
    rkv_decode_step on the matrix-core path, where a workgroup serves two of the four query heads of
    each KV head.  Two (sequence, rotation group) slices - four KV heads, sixteen query heads each -
    are recomputed by the oracle."""
    w = S.WORKLOADS["cfg4"]
    T = w.context
    cfg = R.RkvConfig(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, max_tokens=T, max_sinks=4 if with_sinks else 0,
                      rot_heads=4, perm_span=128, rope_theta=w.rope_theta)
    rep = w.n_q_heads // w.n_kv_heads
    perm = calibrated_perm(w, cfg)
    cache = R.RkvCache(cfg)
    cache.set_perm(P.gpu(np.asarray(perm, dtype=np.int32)))
    samples = [(0, 1), (31, 0)]
    keep = {}
    print("[case] full-size config 4: generating inputs per sequence", flush=True)
    k = torch.empty((w.batch, T, w.n_kv_heads, 128), dtype=torch.float16, device="cuda")
    v = torch.empty_like(k)
    mask = torch.empty((w.batch, T), dtype=torch.uint8, device="cuda")
    for b in range(w.batch):
        kb, vb, mb = S.make_kv(dataclasses.replace(w, seed=w.seed + 100 * b), T, batch=1, sink_positions=None if with_sinks else [])
        for (sb, rg) in samples:
            if sb == b:
                keep[(sb, rg)] = (kb[:, :, 4 * rg:4 * rg + 4].copy(), vb[:, :, 4 * rg:4 * rg + 4].copy(), mb.copy())
        k[b:b + 1].copy_(torch.from_numpy(kb))
        v[b:b + 1].copy_(torch.from_numpy(vb))
        mask[b:b + 1].copy_(torch.from_numpy(mb))
    q = S.make_q(w)
    print("[case] full-size config 4: bulk append 8191 + one decode step", flush=True)
    cache.quantize_append(k[:, :T - 1].contiguous(), v[:, :T - 1].contiguous(), mask[:, :T - 1].contiguous() if with_sinks else None)
    cache.set_decode_path(2)
    assert cache.decode_kernel() == RB.KERNEL_MFMA and cache.append_kernel() == RB.KERNEL_MFMA
    assert not bool(mask[:, T - 1:].any())
    out, lse = cache.decode_step(k[:, T - 1:].contiguous(), v[:, T - 1:].contiguous(), P.gpu(q), want_lse=True)
    exp = export_host(cache)
    assert cache.length == T
    out = out.cpu().numpy().astype(np.float64)
    lse = lse.cpu().numpy().astype(np.float64)
    assert np.isfinite(out).all()
    for (b, rg) in samples:
        ks, vs, ms = keep[(b, rg)]
        check_slice(exp, out, lse, b, rg, ks, vs, ms if with_sinks else None, q, perm=perm, max_sinks=4 if with_sinks else 0,
                    tag=f"full-size config 4 sinks={with_sinks}", rep=rep, rope_theta=w.rope_theta)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_full_size_config1_shape_without_sinks(bits):
    """Configuration 1's full shape (batch 8, 32 heads, context 4096) with no sink tokens, so that
    nothing hides the compressed stream's contribution; sampled slices against the oracle.  With
    2-, 3- and 4-bit codes."""
    w = small("cfg1", n_sinks=0)
    T = w.context
    cfg = R.RkvConfig(batch=w.batch, n_q_heads=32, n_kv_heads=32, max_tokens=T, max_sinks=0, rot_heads=4, perm_span=128, bits=bits)
    cache = R.RkvCache(cfg)
    k, v, _ = S.make_kv(w, T, sink_positions=[])
    q = S.make_q(w)
    print("[case] config 1 shape, no sinks: bulk append 4096 + decode", flush=True)
    cache.quantize_append(P.gpu(k), P.gpu(v))
    cache.set_decode_path(2)
    out, lse = cache.decode_attention(P.gpu(q), want_lse=True)
    exp = export_host(cache)
    out = out.cpu().numpy().astype(np.float64)
    lse = lse.cpu().numpy().astype(np.float64)
    for (b, rg) in [(0, 0), (3, 5), (7, 7)]:
        check_slice(exp, out, lse, b, rg, k[b:b + 1, :, 4 * rg:4 * rg + 4], v[b:b + 1, :, 4 * rg:4 * rg + 4], None, q,
                    max_sinks=0, tag=f"config 1 shape bits={bits}", bits=bits)


def test_large_zero_points():
    """Blocks whose rotated values all sit far from zero get zero-points in the hundreds; the
    matrix-core kernel must treat them exactly (they do not fit its fp16 operand).  Keys are built
    from a chosen rotated image: H is its own inverse, so rotating that image gives the keys."""
    w = small("cfg1", n_q_heads=8, n_kv_heads=8, n_sinks=0)
    cfg = R.RkvConfig(batch=2, n_q_heads=8, n_kv_heads=8, max_tokens=300, max_sinks=0, rot_heads=4, perm_span=128)
    T = 290
    rng = np.random.default_rng(77)
    y = rng.standard_normal((2, T, 1024))
    offs = rng.choice([0.0, 40.0, -75.0, 300.0], size=(2, T, 8), p=[0.4, 0.2, 0.2, 0.2])
    y += np.repeat(offs, 128, axis=-1)
    k = O.rotate_groups(y, 512).reshape(2, T, 8, 128).astype(np.float16)
    v = (rng.standard_normal((2, T, 8, 128)) + 5.0).astype(np.float16)       # values with an offset too
    q = S.make_q(w, batch=2)
    cache = R.RkvCache(cfg)
    oc = O.cache_new(P.oracle_cfg(cfg))
    cache.quantize_append(P.gpu(k), P.gpu(v))
    O.quantize_append(oc, k, v)
    g = P.export_numpy(cache)
    # values of magnitude 300 against block ranges of ~6: more blocks sit inside the (wider) tie windows - 11 % observed
    P.compare_codes(oc.k_rot, oc.k_codes, oc.k_scale, oc.k_zero, g["k_codes"], g["k_scale"], g["k_zero"], "large zero-points K",
                    rot_span=512, max_ambiguous=0.2)
    P.compare_codes(oc.v_in, oc.v_codes, oc.v_scale, oc.v_zero, g["v_codes"], g["v_scale"], g["v_zero"], "large zero-points V")
    assert np.abs(g["k_zero"]).max() > 100
    oc_g = oracle_from_export(oc, g)
    check_dequant(cache, oc_g)
    for path in (1, 2):
        cache.set_decode_path(path)
        check_decode(cache, oc_g, q, tag=f"large zero-points path={path}")


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_degenerate_and_extreme_blocks(bits):
    """Blocks the quantizer has special rules for, in keys and values alike (keys arrive rotated,
    so both are quantized exactly as given): all zeros, constants, a range that rounds to a zero
    scale, ranges of a few fp16 subnormals, values at the end of the fp16 range, and an offset so
    far from zero that the zero-point is clamped.  Metadata and codes against the oracle (exact
    outside ties), then the read half on those codes on both kernels."""
    w = small("cfg1", n_q_heads=8, n_kv_heads=8, n_sinks=0)
    cfg = R.RkvConfig(batch=1, n_q_heads=8, n_kv_heads=8, max_tokens=64, max_sinks=0, rot_heads=4, keys_rotated=1, bits=bits)
    T = 40
    rng = np.random.default_rng(123 + bits)
    x = rng.standard_normal((1, T, 8, 128)).astype(np.float16)
    def special(a):
        a = a.copy()
        a[0, 0] = 0.0                                              # a token of zeros: every block degenerate, scale 1
        a[0, 1, :, :] = np.float16(2.5)                            # constants
        a[0, 2, :, :] = np.float16(-0.125)
        a[0, 3, 0, :] = 0.0
        a[0, 3, 0, 5] = np.float16(6e-8)                           # range of one fp16 subnormal: the scale rounds to 0 or to it
        a[0, 4, 1, :] = np.float16(1e-7) * rng.integers(0, 4, size=128).astype(np.float16)   # a few subnormals
        a[0, 5, 2, :] = np.where(rng.random(128) < 0.5, 65504.0, -65504.0).astype(np.float16)   # the ends of the fp16 range
        a[0, 5, 2, :2] = [65504.0, -65504.0]
        a[0, 6, 3, :] = (30000.0 + 16.0 * rng.integers(0, 2, size=128)).astype(np.float16)   # one fp16 step of range on a large
        a[0, 6, 3, :2] = [30000.0, 30016.0]                                                   # offset: zero-point beyond its clamp
        a[0, 7, 4, :] = (-30000.0 - 16.0 * rng.integers(0, 2, size=128)).astype(np.float16)
        a[0, 7, 4, :2] = [-30000.0, -30016.0]
        a[0, 8, 5, :] = 1000.0
        a[0, 8, 5, 7] = 1000.5                                     # tiny range on a large offset
        return a
    k, v = special(x), special(rng.standard_normal((1, T, 8, 128)).astype(np.float16))
    perm = np.concatenate([128 * blk + rng.permutation(128) for blk in range(8)]).astype(np.int32)
    cache = R.RkvCache(cfg)
    cache.set_perm(P.gpu(perm))
    oc = O.cache_new(P.oracle_cfg(cfg), perm)
    for a, b in ((0, 9), (9, 10), (10, T)):
        cache.quantize_append(P.gpu(k[:, a:b]), P.gpu(v[:, a:b]))
        with np.errstate(over="ignore"):        # the oracle also forms every token's fp16 sink row, which overflows here and is not used
            O.quantize_append(oc, k[:, a:b], v[:, a:b], None, keys_rotated=True)
    torch.cuda.synchronize()
    # (the planted blocks with a range near zero count as ties in the comparison: their metadata
    # and codes are checked one by one below instead: 13 % of the blocks here)
    g, sk, sv = P.check_cache_against_oracle(cache, oc, f"special blocks bits={bits}", max_ambiguous=0.25)
    top = 2 ** bits - 1
    for name in ("k", "v"):
        sc, ze, co = g[name + "_scale"][0], g[name + "_zero"][0], g[name + "_codes"][0].reshape(T, 8, 128)
        assert np.all(sc[0] == 1.0) and np.all(ze[0] == 0.0) and np.all(co[0] == 0)          # zeros: scale 1
        assert np.all(sc[1] == 2.5) and np.all(ze[1] == -1.0) and np.all(co[1] == 0)         # constant c: scale |c|, zero -c/|c|
        assert np.all(sc[2] == 0.125) and np.all(ze[2] == 1.0) and np.all(co[2] == 0)
        assert np.abs(ze[6, 3]) == 2048 and np.abs(ze[7, 4]) == 2048                         # clamped
        # the whole fp16 range in one block: -65504 / scale lies just above -(top / 2) - 1/2 (the fp16 scale is rounded up
        # here), so the zero-point is (top - 1) / 2 and the codes are 0 and top - 1
        oco = getattr(oc, name + "_codes")[0].reshape(T, 8, 128)
        assert np.array_equal(co[5, 2], oco[5, 2]) and co[5, 2].min() == 0 and co[5, 2].max() == top - 1 and sc[5, 2] > 8000.0
    assert np.array_equal(g["k_scale"], oc.k_scale) and np.array_equal(g["v_zero"], oc.v_zero)
    oc_g = oracle_from_export(oc, g)
    check_dequant(cache, oc_g)
    q = S.make_q(w, batch=1)
    for path in (1, 2):
        cache.set_decode_path(path)
        check_decode(cache, oc_g, q, tag=f"special blocks bits={bits} path={path}", lse_relative=True)


def test_select_sinks_matches_oracle():
    """rkv_select_sinks against the oracle's selector: planted massive-activation tokens (also at
    non-initial positions), exact ties between tokens (lower index wins), k = 1 .. 8, and the mask
    form that rkv_quantize_append takes.  fp16 maxima are exact, so indices must be equal."""
    rng = np.random.default_rng(77)
    B, T, C = 3, 1003, 4096
    x = rng.standard_normal((B, T, C)).astype(np.float16)
    x[0, 0] *= 100.0
    x[0, 517] *= 100.0
    x[1, 3, 100] = np.float16(900.0)
    x[1, 999, 7] = np.float16(-900.0)          # same score as token 3: the lower index must win first
    x[1, 400, 9] = np.float16(900.0)
    x[2, T - 1] *= 50.0
    xg = P.gpu(x)
    for k in (1, 2, 3, 4, 8):
        print(f"[case] select sinks k={k}", flush=True)
        idx, mask = R.select_sinks(xg, k)
        torch.cuda.synchronize()
        idx, mask = idx.cpu().numpy(), mask.cpu().numpy()
        for b in range(B):
            ref = O.select_sinks(x[b], k)
            assert idx[b].tolist() == ref.tolist(), (k, b, idx[b], ref)
            want = np.zeros(T, dtype=np.uint8)
            want[ref] = 1
            assert np.array_equal(mask[b], want)
    with pytest.raises(R.RkvError):
        R.select_sinks(xg, 65)
    # the mask feeds the write half directly
    w = small("cfg1", n_q_heads=4, n_kv_heads=4)
    cfg = R.RkvConfig(batch=2, n_q_heads=4, n_kv_heads=4, max_tokens=64, max_sinks=4, rot_heads=4)
    k_, v_, _, _ = P.make_case(w, cfg, 40, sink_positions=[])
    act = rng.standard_normal((2, 40, 512)).astype(np.float16)
    act[0, 5] *= 100.0
    act[1, 17] *= 100.0
    idx, mask = R.select_sinks(P.gpu(act), 1)
    cache = R.RkvCache(cfg)
    cache.quantize_append(P.gpu(k_), P.gpu(v_), mask)
    s = {kk: vv.cpu().numpy() for kk, vv in cache.export_sinks().items()}
    assert s["count"].tolist() == [1, 1] and s["pos"][0, 0] == 5 and s["pos"][1, 0] == 17


@pytest.mark.parametrize("T,sinks", [(1, []), (1, [0]), (2, [1]), (17, [0, 16])])
def test_tiny_caches(T, sinks):
    """Degenerate lengths: a cache of one or two tokens, the only token being a sink, a sink on a
    tile boundary."""
    w = small("cfg1", n_q_heads=4, n_kv_heads=4)
    cfg = R.RkvConfig(batch=2, n_q_heads=4, n_kv_heads=4, max_tokens=32, max_sinks=2, rot_heads=4)
    full_check(w, cfg, T, sink_positions=sinks, paths=(1, 2))


def test_cache_filled_to_capacity_and_many_sinks():
    """A capacity that is no multiple of any tile size, filled exactly; the maximum number of sink
    rows (64), spread over the sequence; one more token must be refused without changing the cache."""
    w = small("cfg1", n_q_heads=8, n_kv_heads=8)
    T = 333
    cfg = R.RkvConfig(batch=1, n_q_heads=8, n_kv_heads=8, max_tokens=T, max_sinks=64, rot_heads=4)
    sinks = list(range(0, 5 * 64, 5))
    cache, oc, q = full_check(w, cfg, T, sink_positions=sinks, chunks=[0, 100, 332, 333], paths=(1, 2))
    k, v, mask, _ = P.make_case(w, cfg, 1, layer=9)
    before = cache.export_codes()
    with pytest.raises(R.RkvError) as ei:
        cache.quantize_append(P.gpu(k), P.gpu(v))
    assert ei.value.code == -2 and cache.length == T
    after = cache.export_codes()
    torch.cuda.synchronize()
    for name in before:
        assert torch.equal(before[name], after[name]), name


def test_empty_append_is_a_no_op():
    w = small("cfg1", n_q_heads=4, n_kv_heads=4)
    cfg = R.RkvConfig(batch=1, n_q_heads=4, n_kv_heads=4, max_tokens=64, max_sinks=1, rot_heads=4)
    cache, oc, q = build_pair(w, cfg, 9)
    empty = torch.empty(1, 0, 4, 128, dtype=torch.float16, device="cuda")
    cache.quantize_append(empty, empty)
    assert cache.length == 9
    P.check_cache_against_oracle(cache, oc, "after empty append")


def test_fold_rotation_matches_oracle():
    """rkv_fold_rotation against the oracle: a projection with rotation and reorder folded in, for
    the key rotation over 4 and 2 heads with a calibrated-style reorder and for the per-head value
    rotation (rot_heads = 1, no reorder); fp32 butterflies against float64."""
    rng = np.random.default_rng(31)
    for g, hkv, with_perm in ((4, 8, True), (2, 4, True), (1, 4, False)):
        cfg = R.RkvConfig(batch=1, n_q_heads=hkv, n_kv_heads=hkv, max_tokens=16, rot_heads=g)
        E = cfg.E
        w = rng.standard_normal((37, E)).astype(np.float32)
        perm = np.concatenate([128 * blk + rng.permutation(128) for blk in range(E // 128)]).astype(np.int32) if with_perm else None
        print(f"[case] fold rotation g={g} E={E} perm={with_perm}", flush=True)
        got = R.fold_rotation(cfg, P.gpu(w), None if perm is None else P.gpu(perm))
        torch.cuda.synchronize()
        ref = O.fold_rotation(w.astype(np.float64), P.oracle_cfg(cfg), perm)
        err = np.abs(got.cpu().numpy().astype(np.float64) - ref).max()
        print(f"[parity] fold rotation: max abs err {err:.3e}")
        assert err <= 2e-6 * np.abs(ref).max()


@pytest.mark.parametrize("g,bits,group,fmt", [(4, 2, 128, 0), (2, 2, 128, 0), (4, 4, 128, 0), (2, 3, 128, 0), (4, 2, 64, 0), (2, 2, 32, 0),
                                              (4, 2, 32, 0), (4, 2, 64, 1), (2, 2, 32, 1), (4, 4, 64, 0), (2, 3, 32, 1)])
def test_rotated_keys_path(g, bits, group, fmt):
    """The deployment shape of Sec. 4.2: keys arrive already rotated and reordered (folded weights),
    the write half only quantizes and packs.  Codes under the tie protocol (the input is exact, so
    only exact ties of Eq. 6 remain), sink rows brought back to the original basis (fp32 on the
    GPU, float64 in the oracle: equal up to one fp16 ulp at rounding ties), decode on both paths."""
    w = small("cfg1", n_q_heads=8, n_kv_heads=8)
    T = 150
    cfg = R.RkvConfig(batch=2, n_q_heads=8, n_kv_heads=8, max_tokens=T, max_sinks=4, rot_heads=g, keys_rotated=1, bits=bits,
                      quant_group=group, meta_format=fmt)
    ocfg = P.oracle_cfg(cfg)
    rng = np.random.default_rng(32)
    perm = np.concatenate([128 * blk + rng.permutation(128) for blk in range(cfg.E // 128)]).astype(np.int32)
    k, v, mask, q = P.make_case(w, cfg, T, sink_positions=[0, 1, 77, 149])
    # what a projection with folded weights would emit: rotated, reordered, rounded to fp16
    k_rot = O.reorder(O.rotate_groups(k.astype(np.float64).reshape(2, T, cfg.E), ocfg.n), perm).astype(np.float16)
    k_rot = k_rot.reshape(k.shape)
    cache = R.RkvCache(cfg)
    cache.set_perm(P.gpu(perm))
    assert cache.append_kernel() == (RB.KERNEL_MFMA if group == 128 else RB.KERNEL_MFMA_SUB)
    oc = O.cache_new(ocfg, perm)
    for a, b in ((0, 70), (70, 71), (71, T)):
        print(f"[case] rotated keys g={g}: append {a}:{b}", flush=True)
        cache.quantize_append(P.gpu(k_rot[:, a:b]), P.gpu(v[:, a:b]), P.gpu(mask[:, a:b]))
        O.quantize_append(oc, k_rot[:, a:b], v[:, a:b], mask[:, a:b], keys_rotated=True)
    torch.cuda.synchronize()
    gexp, sk, sv = P.check_cache_against_oracle(cache, oc, f"rotated keys g={g}")
    # (Eq. 8's division by 3 is a multiplication by the rounded reciprocal on the GPU: within 2^-23 of an
    # fp16 rounding boundary the stored scale may differ by one ulp, which the protocol allows in the
    # blocks it marks ambiguous; with four times the blocks, groups of 32 meet a couple of those)
    # (FP8 scales are rounded up: where a block's range is exactly 7 or 15 times an E4M3 number - the input is fp16 here,
    # 30 of this case's 9600 blocks - the product with 1/7 or 1/15 rounded to fp32, 0.75 and 0.87 ulp above the
    # quotient, can land just above that number and take the next step; 1/3 rounded lies 2^-25 above, which the
    # product's own rounding always absorbs.  The protocol counts such blocks as ambiguous.)
    cap = 4 if bits == 2 or fmt == 0 else 40
    assert sk["mismatched_scales"] <= (0 if group == 128 else min(cap, sk["ambiguous_groups"]))
    s = {kk: vv.cpu().numpy() for kk, vv in cache.export_sinks().items()}
    for b in range(2):
        assert s["count"][b] == len(oc.sink_pos[b])
        for i, pos in enumerate(oc.sink_pos[b]):
            assert s["pos"][b, i] == pos
            ref16 = oc.sink_k[b][i].reshape(cfg.E)
            got16 = s["k"][b, i]
            ulp = np.abs(np.spacing(ref16)).astype(np.float64)
            assert np.all(np.abs(got16.astype(np.float64) - ref16.astype(np.float64)) <= ulp), "sink key row off by more than one fp16 ulp"
            assert np.mean(got16 != ref16) < 0.05        # sums of fp16 values often sit exactly on fp16 ties
            assert np.array_equal(s["v"][b, i], oc.sink_v[b][i].reshape(cfg.E))
    # decode: the oracle takes the GPU's codes and the GPU's sink rows
    oc_g = oracle_from_export(oc, gexp)
    oc_g.sink_k = [[s["k"][b, i].reshape(8, 128) for i in range(len(oc.sink_pos[b]))] for b in range(2)]
    check_dequant(cache, oc_g)
    for path in (1, 2):
        cache.set_decode_path(path)
        check_decode(cache, oc_g, q, tag=f"rotated keys path={path}")


def test_rotated_keys_config_is_checked():
    for bad in (dict(rot_heads=1), dict(rot_heads=8, n_kv_heads=8, n_q_heads=8), dict(v_rotate=1), dict(perm_span=512)):
        kw = dict(batch=1, n_q_heads=4, n_kv_heads=4, max_tokens=16, rot_heads=4, keys_rotated=1)
        kw.update(bad)
        with pytest.raises(R.RkvError):
            R.RkvCache(R.RkvConfig(**kw))


@pytest.mark.parametrize("T", [0, 1, 77])
def test_current_token_attended_in_full_precision(T):
    """rkv_decode_attention_with_current: the token being decoded takes part as an exact fp16 row at
    position `length`, also on an empty cache and with GQA; then it is appended and the next step
    sees it quantized."""
    w = small("cfg1", n_q_heads=16, n_kv_heads=8)
    cfg = R.RkvConfig(batch=2, n_q_heads=16, n_kv_heads=8, max_tokens=128, max_sinks=2, rot_heads=4)
    k, v, mask, q = P.make_case(w, cfg, T + 1, sink_positions=[0] if T == 1 else [])
    cache = R.RkvCache(cfg)
    oc = O.cache_new(P.oracle_cfg(cfg))
    if T > 0:
        cache.quantize_append(P.gpu(k[:, :T]), P.gpu(v[:, :T]), P.gpu(mask[:, :T]))
        O.quantize_append(oc, k[:, :T], v[:, :T], mask[:, :T])
        gexp = P.export_numpy(cache)
        oc = oracle_from_export(oc, gexp)                      # same codes on both sides
    kc, vc = k[:, T], v[:, T]
    for path in (1, 2):
        cache.set_decode_path(path)
        print(f"[case] current token T={T} path={path}", flush=True)
        out, lse = cache.decode_attention(P.gpu(q), want_lse=True, k_cur=P.gpu(kc), v_cur=P.gpu(vc))
        torch.cuda.synchronize()
        if T == 0:
            ref = np.repeat(vc.astype(np.float64), 2, axis=1)  # softmax over one row: the value itself
            assert np.abs(out.cpu().numpy() - ref).max() <= 1e-6 * np.abs(ref).max() + 1e-7
            continue
        ref, lse_ref = O.decode_attention(oc, q, None, kc, vc)
        e = P.attention_error(out.cpu().numpy().astype(np.float64), ref)
        le = float(np.abs(lse.cpu().numpy() - lse_ref).max())
        print(f"[parity] current token T={T} path={path}: out err {e:.3e} lse err {le:.3e}", flush=True)
        assert e <= ATT_TOL and le <= LSE_TOL
    cache.quantize_append(P.gpu(k[:, T:]), P.gpu(v[:, T:]))
    assert cache.length == T + 1


def test_maximum_context_length():
    """The largest cache the library accepts (65536 tokens): 256 chunks on the matrix-core path and
    512 - the merge kernel's limit - on the general one; one rotation group, both paths against
    the oracle on the GPU's own codes, and one more token must be refused."""
    w = small("cfg3", n_q_heads=4, n_kv_heads=4)
    T = 65536
    cfg = R.RkvConfig(batch=1, n_q_heads=4, n_kv_heads=4, max_tokens=T, max_sinks=4, rot_heads=4)
    with pytest.raises(R.RkvError):
        R.RkvCache(R.RkvConfig(batch=1, n_q_heads=4, n_kv_heads=4, max_tokens=T + 1, max_sinks=4, rot_heads=4))
    k, v, mask = S.make_kv(w, T, batch=1)
    q = S.make_q(w, batch=1)
    cache = R.RkvCache(cfg)
    print("[case] 65536 tokens: bulk append 65535 + 1", flush=True)
    cache.quantize_append(P.gpu(k[:, :T - 1]), P.gpu(v[:, :T - 1]), P.gpu(mask[:, :T - 1]))
    cache.quantize_append(P.gpu(k[:, T - 1:]), P.gpu(v[:, T - 1:]), P.gpu(mask[:, T - 1:]))
    assert cache.length == T
    with pytest.raises(R.RkvError) as ei:
        cache.quantize_append(P.gpu(k[:, :1]), P.gpu(v[:, :1]))
    assert ei.value.code == -2
    exp = export_host(cache)
    for path in (2, 1):
        cache.set_decode_path(path)
        print(f"[case] 65536 tokens: decode path {path}", flush=True)
        out, lse = cache.decode_attention(P.gpu(q), want_lse=True)
        torch.cuda.synchronize()
        check_slice(exp, out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64), 0, 0, k, v, mask, q,
                    tag=f"65536 tokens path={path}")


@pytest.mark.parametrize("hq,hkv,g,nq,bits", [(8, 8, 4, 4, 2), (8, 8, 4, 3, 2), (16, 4, 4, 2, 2), (4, 4, 2, 2, 2), (8, 8, 4, 1, 2),
                                              (8, 8, 4, 4, 4), (16, 4, 4, 2, 3), (4, 4, 2, 3, 4)])
def test_several_query_tokens_per_step(hq, hkv, g, nq, bits):
    """rkv_decode_attention_multi: the tokens of a multi-token step are appended, then all of them
    read the cache in one call, each blind to what lies behind its own position (one of the new
    tokens is a retained sink row, which the earlier ones must not see).  Checked against the
    oracle on the GPU's own codes; sequence 1 uses scattered positions, one past the cache."""
    w = small("cfg1", n_q_heads=hq, n_kv_heads=hkv)
    T = 333
    cfg = R.RkvConfig(batch=2, n_q_heads=hq, n_kv_heads=hkv, max_tokens=400, max_sinks=4, rot_heads=g, bits=bits)
    sinks = [0, T - 2] if nq > 1 else [0]
    if (hq, nq, bits) in ((8, 3, 2), (16, 2, 2), (8, 4, 4), (16, 2, 3)):
        sinks = []                                             # nothing but the compressed stream behind every query
    cache, oc, _ = build_pair(w, cfg, T, sink_positions=sinks, chunks=[0, T - nq, T])
    oc_g = oracle_from_export(oc, P.export_numpy(cache))
    q = np.stack([S.make_q(w, batch=2, step=i) for i in range(nq)], axis=1)          # [B, nq, Hq, d]
    q_pos = np.stack([np.arange(T - nq, T), np.array([5, 255, 256, 700])[:nq]]).astype(np.int32)
    if nq == 1:
        q_pos = np.array([[T - 1], [T - 1]], dtype=np.int32)
    print(f"[case] multi-query Hq={hq} Hkv={hkv} g={g} nq={nq} q_pos={q_pos.tolist()}", flush=True)
    out, lse = cache.decode_attention_multi(P.gpu(q), P.gpu(q_pos), want_lse=True)
    torch.cuda.synchronize()
    ref, lse_ref = O.decode_attention_multi(oc_g, q, q_pos)
    e = P.attention_error(out.cpu().numpy().astype(np.float64), ref)
    le = float(np.abs(lse.cpu().numpy() - lse_ref).max())
    print(f"[parity] multi-query nq={nq}: out err {e:.3e} lse err {le:.3e}", flush=True)
    assert e <= ATT_TOL and le <= LSE_TOL
    if nq == 1:   # one query at the last position is the ordinary decode step
        cache.set_decode_path(2)
        out1 = cache.decode_attention(P.gpu(q[:, 0]))
        torch.cuda.synchronize()
        assert float((out1 - out[:, 0]).abs().max()) <= 1e-6 * float(out1.abs().max())
    # the general kernel serves the same call (up to 8 (query token, query head) pairs per KV head)
    cache.set_decode_path(1)
    assert (hq // hkv) * nq <= 8 and cache.decode_kernel(nq) == RB.KERNEL_GENERAL
    out_g, lse_g = cache.decode_attention_multi(P.gpu(q), P.gpu(q_pos), want_lse=True)
    torch.cuda.synchronize()
    assert P.attention_error(out_g.cpu().numpy().astype(np.float64), ref) <= ATT_TOL
    assert float(np.abs(lse_g.cpu().numpy() - lse_ref).max()) <= LSE_TOL
    # what the entry point refuses there: more pairs than that
    q9 = np.repeat(q[:, :1], 9, axis=1)
    with pytest.raises(R.RkvError):
        cache.decode_attention_multi(P.gpu(q9), P.gpu(np.repeat(q_pos[:, :1], 9, axis=1)))


@pytest.mark.parametrize("hq,hkv,g,style", [(8, 8, 4, 0), (4, 4, 2, 0), (16, 4, 4, 0), (8, 8, 1, 0), (8, 8, 4, 1), (8, 8, 8, 0)])
def test_fp8_scale_int8_zero_metadata(hq, hkv, g, style):
    """meta_format = 1 (FP8 E4M3 scale rounded up, INT8 zero-point: Sec. 5.1 quantization settings)
    through every write and read kernel: matrix-core and general decode, GQA, rotation sizes that
    take the general append kernels, interleaved RoPE pairs; appended in pieces with single-token
    steps; the smaller cache is checked through rkv_query_sizes."""
    w = small("cfg1", n_q_heads=hq, n_kv_heads=hkv)
    kw = dict(batch=2, n_q_heads=hq, n_kv_heads=hkv, max_tokens=700, max_sinks=4, rot_heads=g, rope_style=style)
    cfg = R.RkvConfig(meta_format=1, **kw)
    b8, _ = R.query_sizes(cfg)
    b16, _ = R.query_sizes(R.RkvConfig(**kw))
    Tpad = 768
    assert b16 - b8 == 2 * 2 * Tpad * hkv * 2                     # K and V, 2 bytes less per (token, block)
    paths = (1, 2) if g in (2, 4) else (1, 0)
    # (the cases with half-split RoPE pairs without retained fp16 rows: the compressed stream alone decides the outputs)
    full_check(w, cfg, 613, chunks=[0, 300, 301, 302, 613], paths=paths, sink_positions=[] if style == 0 else None)


def test_fp8_metadata_saturation_and_clamps():
    """Blocks whose range or offset leaves what FP8 / INT8 hold: scale saturates at 448, zero-points
    clamp at -128 / 127, a tiny range rounds up to the smallest subnormal; the GPU must store the
    same metadata and codes as the oracle (inputs are exact in fp32 and far from rounding ties)."""
    cfg = R.RkvConfig(batch=1, n_q_heads=4, n_kv_heads=4, max_tokens=16, max_sinks=0, rot_heads=4, v_rotate=0, meta_format=1)
    rng = np.random.default_rng(77)
    T = 8
    v = rng.standard_normal((1, T, 4, 128)).astype(np.float16)
    v[0, 0, 0] = (v[0, 0, 0].astype(np.float32) * 600).astype(np.float16)        # range ~4000: scale saturates
    v[0, 1, 1] = (1000.0 + rng.integers(0, 3, 128)).astype(np.float16)         # offset >> range: zero clamps at -128
    v[0, 2, 2] = (-1000.0 - rng.integers(0, 3, 128)).astype(np.float16)        # ... and at 127
    v[0, 3, 3] = (rng.integers(0, 2, 128) * 2.0 ** -12).astype(np.float16)     # tiny range: smallest subnormal scale
    v[0, 4, 0] = np.float16(2.3)                                               # constant block
    v[0, 5, 1] = np.float16(0.0)
    k = rng.standard_normal((1, T, 4, 128)).astype(np.float16)
    k[0, 6] = (k[0, 6].astype(np.float32) * 2.0 ** -11).astype(np.float16)      # a token whose key blocks get subnormal FP8 scales
    k[0, 7] = (k[0, 7].astype(np.float32) * 300.0).astype(np.float16)          # ... and one whose scales saturate
    cache = R.RkvCache(cfg)
    oc = O.cache_new(P.oracle_cfg(cfg))
    q = rng.standard_normal((1, 4, 128)).astype(np.float16)
    # first without the saturated key token, whose huge scores would take all of the softmax's mass
    cache.quantize_append(P.gpu(k[:, :7]), P.gpu(v[:, :7]))
    O.quantize_append(oc, k[:, :7], v[:, :7])
    oc7 = oracle_from_export(oc, P.export_numpy(cache))
    for path in (1, 2):
        cache.set_decode_path(path)
        check_decode(cache, oc7, q, tag=f"special blocks, 7 tokens, path={path}")
    cache.quantize_append(P.gpu(k[:, 7:]), P.gpu(v[:, 7:]))
    O.quantize_append(oc, k[:, 7:], v[:, 7:])
    g = P.export_numpy(cache)
    P.compare_codes(oc.k_rot, oc.k_codes, oc.k_scale, oc.k_zero, g["k_codes"], g["k_scale"], g["k_zero"], "special blocks K",
                    rot_span=512, meta_format=1)
    assert oc.k_scale[0, 6].max() < 2.0 ** -6 and oc.k_scale[0, 7].max() == 448.0
    assert np.array_equal(g["v_scale"], oc.v_scale)
    assert np.array_equal(g["v_zero"], oc.v_zero)
    P.compare_codes(oc.v_in, oc.v_codes, oc.v_scale, oc.v_zero, g["v_codes"], g["v_scale"], g["v_zero"], "special blocks V",
                    meta_format=1)
    gc = g["v_codes"].reshape(1, T, 4, 128)
    assert np.all(gc[0, 1, 1] == 3) and np.all(gc[0, 2, 2] == 0) and np.all(gc[0, 3, 3] == 0)
    assert np.all(gc[0, 4, 0] == 0) and np.all(gc[0, 5, 1] == 0)
    assert oc.v_scale[0, 0, 0] == 448.0 and oc.v_zero[0, 1, 1] == -128 and oc.v_zero[0, 2, 2] == 127
    assert oc.v_scale[0, 3, 3] == 2.0 ** -9
    # the read half on these codes: subnormal and saturated scales, clamped zero-points, both kernels
    oc_g = oracle_from_export(oc, g)
    for path in (1, 2):
        cache.set_decode_path(path)
        check_decode(cache, oc_g, q, tag=f"special blocks path={path}")


def test_shared_scratch_reused_across_caches():
    """Two caches with different contents share one scratch block (as the layers of a model do) and
    are decoded alternately, many times: every result must equal the first one bit for bit and
    agree with the general kernel - partial results or prepared queries left over from the other
    cache's call must never leak into a result."""
    w = small("cfg2", n_q_heads=16, n_kv_heads=16)
    T = 4096
    cfg = R.RkvConfig(batch=8, n_q_heads=16, n_kv_heads=16, max_tokens=T, max_sinks=4, rot_heads=4)
    dev = torch.device("cuda:0")
    _, scratch_bytes = R.query_sizes(cfg)
    scratch = torch.empty(scratch_bytes, dtype=torch.uint8, device=dev)
    caches, qs, refs = [], [], []
    for i in range(2):
        c = R.RkvCache(cfg, scratch=scratch)
        k, v, mask = S.make_kv_torch(w, T, dev, batch=8, layer=i)
        c.quantize_append(k, v, mask)
        q = S.make_q_torch(w, dev, batch=8, layer=i)
        c.set_decode_path(1)
        ref = c.decode_attention(q).clone()
        c.set_decode_path(2)
        first = c.decode_attention(q).clone()
        torch.cuda.synchronize()
        err = float((first - ref).abs().max() / ref.abs().max())
        print(f"[parity] cache {i}: matrix-core vs general kernel {err:.3e}", flush=True)
        assert err <= 1e-4
        caches.append(c); qs.append(q); refs.append(first)
    for rep in range(40):
        for i in range(2):
            out = caches[i].decode_attention(qs[i])
            assert torch.equal(out, refs[i]), f"repetition {rep}, cache {i}"


@pytest.mark.parametrize("bits,group", [(2, 128), (3, 128), (4, 128), (2, 64), (2, 32), (3, 32), (4, 64)])
def test_sequences_of_different_lengths(bits, group):
    """(With 2-bit codes and with 3- and 4-bit codes, which the matrix-core kernels read as two planes;
    with 2-bit codes in groups of 64 and 32, which take their sub-group variants.)
    rkv_quantize_append_ragged: three sequences are prefilled with 300 / 37 / 513 tokens in one
    call, extended by 5 / 0 / 40 in a second, then take three ordinary single-token steps.  Each
    sequence is compared with an oracle cache of its own (batch 1): codes under the tie protocol,
    sink rows, and - on the GPU's own codes - decode attention on both kernels with the default
    query position (each sequence's own last token), the current-token variant and two causal
    query tokens per step."""
    w = small("cfg1", n_q_heads=8, n_kv_heads=8)
    B = 3
    cfg = R.RkvConfig(batch=B, n_q_heads=8, n_kv_heads=8, max_tokens=600, max_sinks=4, rot_heads=4, bits=bits, quant_group=group)
    steps = [[300, 37, 513], [5, 0, 40], [1, 1, 1], [1, 1, 1], [1, 1, 1]]
    total = [sum(st[b] for st in steps) for b in range(B)]
    # (with 2-bit codes the sequences keep their fp16 sink rows; the wider codes run on the compressed stream alone)
    data = [S.make_kv(w, total[b] + 1, batch=1, layer=b, sink_positions=None if bits == 2 else []) for b in range(B)]   # one spare token for the current-token call
    cache = R.RkvCache(cfg)
    ocs = [O.cache_new(P.oracle_cfg(dataclasses.replace(cfg, batch=1))) for _ in range(B)]
    done = [0] * B
    for st in steps:
        n_max = max(st)
        k = np.zeros((B, n_max, 8, 128), np.float16)
        v = np.zeros_like(k)
        m = np.zeros((B, n_max), np.uint8)
        for b in range(B):
            kb, vb, mb = data[b]
            sl = slice(done[b], done[b] + st[b])
            k[b, :st[b]], v[b, :st[b]], m[b, :st[b]] = kb[0, sl], vb[0, sl], mb[0, sl]
            if st[b]:
                O.quantize_append(ocs[b], kb[:, sl], vb[:, sl], mb[:, sl])
            done[b] += st[b]
        print(f"[case] ragged append {st}", flush=True)
        if len(set(st)) == 1:
            cache.quantize_append(P.gpu(k), P.gpu(v), P.gpu(m))
        else:
            cache.quantize_append_ragged(P.gpu(k), P.gpu(v), st, P.gpu(m))
    torch.cuda.synchronize()
    assert cache.lengths == total and cache.length == max(total)
    g = P.export_numpy(cache)
    sinks = {kk: vv.cpu().numpy() for kk, vv in cache.export_sinks().items()}
    ocg = []
    for b in range(B):
        gb = {name: arr[b:b + 1, :total[b]] for name, arr in g.items()}
        P.compare_codes(ocs[b].k_rot, ocs[b].k_codes, ocs[b].k_scale, ocs[b].k_zero, gb["k_codes"], gb["k_scale"], gb["k_zero"],
                        f"ragged b={b} K", rot_span=512, bits=bits, group=group)
        P.compare_codes(ocs[b].v_in, ocs[b].v_codes, ocs[b].v_scale, ocs[b].v_zero, gb["v_codes"], gb["v_scale"], gb["v_zero"],
                        f"ragged b={b} V", bits=bits, group=group)
        assert sinks["count"][b] == len(ocs[b].sink_pos[0])
        for i, pos in enumerate(ocs[b].sink_pos[0]):
            assert sinks["pos"][b, i] == pos
            assert np.array_equal(sinks["k"][b, i], ocs[b].sink_k[0][i].reshape(-1))
        ocg.append(oracle_from_export(ocs[b], gb))
    q = S.make_q(w, batch=B)
    for path in (2, 1):
        cache.set_decode_path(path)
        out, lse = cache.decode_attention(P.gpu(q), want_lse=True)
        torch.cuda.synchronize()
        for b in range(B):
            ref, lse_ref = O.decode_attention(ocg[b], q[b:b + 1])
            e = P.attention_error(out[b:b + 1].cpu().numpy().astype(np.float64), ref)
            le = float(np.abs(lse[b:b + 1].cpu().numpy() - lse_ref).max())
            print(f"[parity] ragged decode path={path} b={b} len={total[b]}: out err {e:.3e} lse err {le:.3e}", flush=True)
            assert e <= ATT_TOL and le <= LSE_TOL
        kc = np.concatenate([data[b][0][:, total[b]] for b in range(B)])
        vc = np.concatenate([data[b][1][:, total[b]] for b in range(B)])
        out = cache.decode_attention(P.gpu(q), k_cur=P.gpu(kc), v_cur=P.gpu(vc))
        torch.cuda.synchronize()
        for b in range(B):
            ref, _ = O.decode_attention(ocg[b], q[b:b + 1], None, kc[b:b + 1], vc[b:b + 1])
            e = P.attention_error(out[b:b + 1].cpu().numpy().astype(np.float64), ref)
            assert e <= ATT_TOL, f"current token, path {path}, b={b}: {e}"
    cache.set_decode_path(0)
    assert cache.append_kernel() == (RB.KERNEL_MFMA if group == 128 else RB.KERNEL_MFMA_SUB)
    q2 = np.stack([S.make_q(w, batch=B, step=i) for i in range(2)], axis=1)
    q_pos = np.array([[total[b] - 2, total[b] - 1] for b in range(B)], dtype=np.int32)
    if group == 128:
        out = cache.decode_attention_multi(P.gpu(q2), P.gpu(q_pos))
        torch.cuda.synchronize()
        for b in range(B):
            ref, _ = O.decode_attention_multi(ocg[b], q2[b:b + 1], q_pos[b:b + 1])
            e = P.attention_error(out[b:b + 1].cpu().numpy().astype(np.float64), ref)
            assert e <= ATT_TOL, f"two query tokens, b={b}: {e}"
    else:                       # the sub-group variant: the scores kernel takes the query tokens as further query heads
        assert cache.decode_kernel(2) == RB.KERNEL_MFMA_SUB
        out = cache.decode_attention_multi(P.gpu(q2), P.gpu(q_pos))
        torch.cuda.synchronize()
        for b in range(B):
            ref, _ = O.decode_attention_multi(ocg[b], q2[b:b + 1], q_pos[b:b + 1])
            e = P.attention_error(out[b:b + 1].cpu().numpy().astype(np.float64), ref)
            assert e <= ATT_TOL, f"two query tokens on the sub-group variant, b={b}: {e}"
    # what the entry point refuses
    with pytest.raises(R.RkvError) as ei:
        cache.quantize_append_ragged(P.gpu(np.zeros((B, 50, 8, 128), np.float16)), P.gpu(np.zeros((B, 50, 8, 128), np.float16)), [1, 1, 50])
    assert ei.value.code == -2 and cache.lengths == total          # sequence 2 would pass max_tokens; nothing appended
    with pytest.raises(R.RkvError):
        cache.quantize_append_ragged(P.gpu(np.zeros((B, 2, 8, 128), np.float16)), P.gpu(np.zeros((B, 2, 8, 128), np.float16)), [1, 3, 0])
    cache.reset()
    assert cache.lengths == [0, 0, 0]


@pytest.mark.parametrize("hq,hkv,g,ragged,bits", [(8, 8, 4, False, 2), (16, 4, 4, False, 2), (4, 4, 2, True, 2), (8, 8, 8, False, 2),
                                                  (8, 8, 4, True, 4), (8, 4, 2, False, 4), (8, 8, 4, True, 3), (8, 4, 2, False, 3), (8, 8, 8, False, 3)])
def test_one_call_decode_step_equals_the_two_calls(hq, hkv, g, ragged, bits):
    """rkv_decode_step (append + attention in one call; on the matrix-core configurations the
    token's compression and the query's preparation share a launch) against rkv_quantize_append
    followed by rkv_decode_attention on a second cache with the same contents: outputs, codes and
    metadata bit for bit, over several steps that cross a tile and a slab boundary; also with
    sequences of different lengths, explicit query positions, and on a configuration that falls
    back to the two calls (rotation over 8 heads).  3- and 4-bit codes take the one-launch path
    like 2-bit ones."""
    w = small("cfg1", n_q_heads=hq, n_kv_heads=hkv)
    B, T0, steps = 2, 29, 6
    cfg = R.RkvConfig(batch=B, n_q_heads=hq, n_kv_heads=hkv, max_tokens=128, max_sinks=4, rot_heads=g, bits=bits)
    k, v, mask = S.make_kv(w, T0 + steps, batch=B)
    a, b = R.RkvCache(cfg), R.RkvCache(cfg)
    for c in (a, b):
        if ragged:
            c.quantize_append_ragged(P.gpu(k[:, :T0]), P.gpu(v[:, :T0]), [T0, T0 - 12], P.gpu(mask[:, :T0]))
        else:
            c.quantize_append(P.gpu(k[:, :T0]), P.gpu(v[:, :T0]), P.gpu(mask[:, :T0]))
    for s_ in range(steps):
        q = P.gpu(S.make_q(w, batch=B, step=s_))
        kk, vv = P.gpu(k[:, T0 + s_:T0 + s_ + 1]), P.gpu(v[:, T0 + s_:T0 + s_ + 1])
        q_pos = None if s_ % 2 == 0 else P.gpu(np.array([200 + s_, 7], dtype=np.int32))
        print(f"[case] decode step {s_} Hq={hq} Hkv={hkv} g={g} ragged={ragged}", flush=True)
        o1, l1 = a.decode_step(kk, vv, q, q_pos, want_lse=True)
        b.quantize_append(kk, vv)
        o2, l2 = b.decode_attention(q, q_pos, want_lse=True)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2) and torch.equal(l1, l2), f"step {s_}"
    assert a.lengths == b.lengths
    ea, eb = a.export_codes(), b.export_codes()
    torch.cuda.synchronize()
    for name in ea:
        assert torch.equal(ea[name], eb[name]), name
    with pytest.raises(R.RkvError) as ei:                     # a full cache refuses the step
        full = R.RkvCache(dataclasses.replace(cfg, max_tokens=T0))
        full.quantize_append(P.gpu(k[:, :T0]), P.gpu(v[:, :T0]))
        full.decode_step(P.gpu(k[:, :1]), P.gpu(v[:, :1]), P.gpu(S.make_q(w, batch=B)))
    assert ei.value.code == -2


@pytest.mark.parametrize("hq,hkv,g,fmt", [(24, 8, 4, 0), (32, 4, 4, 1), (8, 4, 2, 0), (12, 4, 2, 1)])
def test_gqa_ratios_and_metadata_formats(hq, hkv, g, fmt):
    """Query heads per KV head of 3 (one per workgroup), 8 (four workgroups of two per KV head) and
    2, with rotation over 4 and over 2 heads, in both metadata formats; both decode kernels."""
    w = small("cfg4", n_q_heads=hq, n_kv_heads=hkv)
    cfg = R.RkvConfig(batch=2, n_q_heads=hq, n_kv_heads=hkv, max_tokens=600, max_sinks=4, rot_heads=g, meta_format=fmt,
                      rope_theta=500000.0)
    # three of the four without retained fp16 rows: the compressed stream alone decides the outputs
    full_check(w, cfg, 531, paths=(1, 2), sink_positions=None if hq == 8 else [])


def test_rotated_keys_with_fp8_metadata_and_one_call_steps():
    """Features together: keys from a projection with the rotation folded in, FP8 / INT8 metadata,
    no sink rows, prefill followed by one-call decode steps; codes against the oracle under the
    tie protocol, attention on the GPU's own codes."""
    w = small("cfg1", n_q_heads=8, n_kv_heads=8, n_sinks=0)
    cfg = R.RkvConfig(batch=2, n_q_heads=8, n_kv_heads=8, max_tokens=128, max_sinks=0, rot_heads=4, keys_rotated=1, meta_format=1)
    ocfg = P.oracle_cfg(cfg)
    T0, steps = 70, 3
    k, v, _ = S.make_kv(w, T0 + steps, batch=2, sink_positions=[])
    # what the folded projection hands over: rotated, (identity-)reordered, rounded to fp16
    kz = O.fold_rotation(k.astype(np.float64).reshape(-1, cfg.E), ocfg).astype(np.float16).reshape(k.shape)
    cache = R.RkvCache(cfg)
    oc = O.cache_new(ocfg)
    cache.quantize_append(P.gpu(kz[:, :T0]), P.gpu(v[:, :T0]))
    O.quantize_append(oc, kz[:, :T0], v[:, :T0], None, keys_rotated=True)
    for s_ in range(steps):
        q = S.make_q(w, batch=2, step=s_)
        t = T0 + s_
        print(f"[case] rotated keys + fp8 metadata, one-call step {s_}", flush=True)
        out = cache.decode_step(P.gpu(kz[:, t:t + 1]), P.gpu(v[:, t:t + 1]), P.gpu(q))
        O.quantize_append(oc, kz[:, t:t + 1], v[:, t:t + 1], None, keys_rotated=True)
        torch.cuda.synchronize()
        g, _, _ = P.check_cache_against_oracle(cache, oc, f"rotated keys + fp8, step {s_}")
        ref, _ = O.decode_attention(oracle_from_export(oc, g), q)
        e = P.attention_error(out.cpu().numpy().astype(np.float64), ref)
        print(f"[parity] step {s_}: out err {e:.3e}", flush=True)
        assert e <= ATT_TOL


@pytest.mark.parametrize("bits,group,g,hq,fmt,span", [(4, 128, 4, 8, 0, 128), (3, 128, 4, 8, 0, 128), (2, 64, 4, 8, 0, 128),
                                                      (2, 32, 2, 8, 0, 128), (4, 32, 1, 8, 1, 128), (3, 64, 8, 16, 1, 128),
                                                      (4, 64, 4, 8, 0, 512), (3, 32, 2, 8, 0, 1024), (4, 128, 2, 16, 1, 128),
                                                      (4, 128, 4, 32, 0, 128), (3, 128, 2, 16, 1, 128), (3, 128, 4, 32, 0, 128),
                                                      (2, 32, 4, 16, 0, 128), (2, 64, 2, 8, 0, 128), (4, 64, 4, 8, 0, 128),
                                                      (3, 32, 2, 8, 1, 128), (4, 32, 4, 16, 1, 128), (3, 64, 4, 8, 0, 128),
                                                      (4, 32, 2, 16, 0, 128), (3, 64, 2, 16, 1, 128), (4, 128, 4, 8, 0, 512),
                                                      (3, 128, 2, 16, 1, 256), (3, 128, 4, 32, 0, 512), (4, 128, 2, 8, 1, 256),
                                                      (2, 64, 4, 8, 0, 512), (2, 32, 2, 16, 1, 256), (2, 32, 4, 16, 0, 512),
                                                      (3, 32, 4, 8, 1, 512), (4, 64, 2, 8, 0, 256), (4, 128, 4, 8, 0, 1024),
                                                      (3, 128, 2, 16, 1, 1024), (3, 128, 4, 32, 0, 1024), (4, 128, 2, 8, 1, 1024),
                                                      (2, 64, 4, 8, 0, 1024), (2, 32, 2, 16, 1, 1024), (4, 32, 4, 16, 0, 1024),
                                                      (3, 64, 2, 8, 1, 1024), (2, 32, 4, 32, 0, 1024)])
def test_wider_codes_and_smaller_groups(bits, group, g, hq, fmt, span):
    """3- and 4-bit codes and quantization groups of 64 and 32 channels (Sec. 5.1; Tables
    tab:ablation and tab:quantgrani) through the write half, the export and dequantize views and
    the read half: every rotation size, both metadata formats, GQA, a reorder that crosses blocks;
    appended in pieces with single-token steps.  The cache's size follows the setting."""
    w = small("cfg1", n_q_heads=hq, n_kv_heads=8)
    kw = dict(batch=2, n_q_heads=hq, n_kv_heads=8, max_tokens=256, max_sinks=4, rot_heads=g, meta_format=fmt)
    cfg = R.RkvConfig(bits=bits, quant_group=group, perm_span=span, **kw)
    mine, _ = R.query_sizes(cfg)
    base, _ = R.query_sizes(R.RkvConfig(perm_span=span, **kw))
    per_elem = (bits - 2) + (16 if fmt else 32) * (1.0 / group - 1.0 / 128)      # bits per cached element beyond 2-bit, group 128
    # K and V, batch 2, 256 token slots, 1024 channels; smaller groups also enlarge the per-cache tables of the decode kernel
    assert 0 <= (mine - base) - 2 * 2 * 256 * 1024 * per_elem / 8 <= (0 if group == 128 else 256 * 1024)
    perm = None
    if span != 128:
        perm = calibrated_perm(w, R.RkvConfig(perm_span=span, **kw), offset_variant=True)
        assert not np.array_equal(perm // group, np.arange(cfg.E) // group)
    # wider codes in groups of 128 are read by the matrix-core decode kernel as two planes, codes in
    # smaller groups by its sub-group variant (scores from the scores kernel, one table half per plane)
    on_matrix_cores = g in (2, 4)                               # (any of the spans here: 128, the rotation group, 1024 = the whole row)
    # half of the cases without any retained fp16 row, so that the compressed stream alone decides the outputs
    cache, oc, q = full_check(w, cfg, 213, perm=perm, chunks=[0, 100, 101, 102, 213], paths=(1, 2) if on_matrix_cores else (1, 0),
                              sink_positions=[] if (hq + group + bits) % 3 != 0 else None)
    assert oc.k_codes.max() == 2 ** bits - 1 and oc.k_scale.shape[-1] == 1024 // group
    if not on_matrix_cores:      # what those kernels do not cover is refused, not mis-computed
        with pytest.raises(R.RkvError):
            cache.set_decode_path(2)
            cache.decode_attention(P.gpu(q))
    cache.set_decode_path(0)
    if on_matrix_cores:
        want = (RB.KERNEL_MFMA_ROW if span == 1024 else RB.KERNEL_MFMA_SUB if group != 128 else RB.KERNEL_MFMA_CROSS if span != 128
                else RB.KERNEL_MFMA)
        assert cache.append_kernel() == want and cache.decode_kernel() == want
    # one more single-token step through rkv_decode_step (the two calls, on this setting)
    k1, v1, _ = S.make_kv(w, 1, batch=2, stream=5, sink_positions=[])
    out = cache.decode_step(P.gpu(k1), P.gpu(v1), P.gpu(q))
    torch.cuda.synchronize()
    # the cache holds the oracle's codes from full_check; the same token goes to the oracle's cache
    O.quantize_append(oc, k1, v1, None)
    g_all = P.export_numpy(cache)
    ref, _ = O.decode_attention(oracle_from_export(oc, g_all), q)
    assert P.attention_error(out.cpu().numpy().astype(np.float64), ref) <= ATT_TOL


@pytest.mark.parametrize("group,g,hq", [(32, 4, 16), (64, 2, 8)])
def test_smaller_groups_with_interleaved_rope_pairs(group, g, hq):
    """Groups of 64 / 32 with the interleaved RoPE pairing (and GQA): the scores kernel's table of the
    rotation group's own sub-blocks together with its other pairing of a lane's channels; no
    retained rows, several chunks and a ragged tail."""
    w = small("cfg1", n_q_heads=hq, n_kv_heads=8)
    cfg = R.RkvConfig(batch=2, n_q_heads=hq, n_kv_heads=8, max_tokens=700, max_sinks=4, rot_heads=g, quant_group=group, rope_style=1)
    cache, _, _ = full_check(w, cfg, 613, chunks=[0, 300, 301, 613], paths=(1, 2), sink_positions=[])
    cache.set_decode_path(0)
    assert cache.decode_kernel() == RB.KERNEL_MFMA_SUB and cache.append_kernel() == RB.KERNEL_MFMA_SUB


@pytest.mark.parametrize("setting,g,hq", [("whole row", 4, 8), ("whole row", 2, 16), ("groups of 64", 4, 8), ("groups of 32", 2, 16),
                                          ("groups of 32", 4, 8)])
def test_fp8_metadata_on_the_scores_kernel_paths(setting, g, hq):
    """FP8 scales and INT8 zero-points (Sec. 5.1) together with a reorder over the whole row (Alg. 1
    as printed) or with groups of 64 / 32 (Table tab:quantgrani): the matrix-core write half of
    each setting and the read half that takes its scores from the scores kernel, against the oracle
    and the general kernel; GQA, several chunks, a ragged tail, with and without retained rows,
    one more token through rkv_decode_step."""
    w = small("cfg1", n_q_heads=hq, n_kv_heads=8)
    kw = dict(batch=2, n_q_heads=hq, n_kv_heads=8, max_tokens=700, max_sinks=4, rot_heads=g, meta_format=1)
    perm = None
    if setting == "whole row":
        cfg, kind = R.RkvConfig(perm_span=1024, **kw), RB.KERNEL_MFMA_ROW
        perm = calibrated_perm(w, cfg, offset_variant=True)
    else:
        cfg, kind = R.RkvConfig(quant_group=int(setting.split()[-1]), **kw), RB.KERNEL_MFMA_SUB
    cache, oc, q = full_check(w, cfg, 613, perm=perm, chunks=[0, 300, 301, 613], paths=(1, 2), sink_positions=None if g == 4 and hq == 8 else [])
    cache.set_decode_path(0)
    assert cache.decode_kernel() == kind and cache.append_kernel() == kind
    k1, v1, _ = S.make_kv(w, 1, batch=2, stream=5, sink_positions=[])
    out = cache.decode_step(P.gpu(k1), P.gpu(v1), P.gpu(q))
    torch.cuda.synchronize()
    O.quantize_append(oc, k1, v1, None)                    # (the cache holds the oracle's codes from full_check)
    ref, _ = O.decode_attention(oracle_from_export(oc, P.export_numpy(cache)), q)
    assert P.attention_error(out.cpu().numpy().astype(np.float64), ref) <= ATT_TOL


@pytest.mark.parametrize("T", [1, 15, 16, 17, 64, 65])
@pytest.mark.parametrize("setting", ["groups of 32", "whole row"])
def test_scores_kernel_at_tile_and_chunk_edges(setting, T):
    """The read half that takes its scores from the scores kernel (groups of 64 / 32, a reorder over
    the whole row) with a handful of tokens: one token, one short of a 16-token tile, exactly one
    tile, one over, exactly the 64 tokens of a workgroup, one over; a sink row among them where there
    is room."""
    w = small("cfg1", n_q_heads=8, n_kv_heads=8)
    if setting == "whole row":
        cfg = R.RkvConfig(batch=2, n_q_heads=8, n_kv_heads=8, max_tokens=128, max_sinks=2, rot_heads=4, perm_span=1024)
        perm = calibrated_perm(w, cfg, offset_variant=True)
        kind = RB.KERNEL_MFMA_ROW
    else:
        cfg = R.RkvConfig(batch=2, n_q_heads=8, n_kv_heads=8, max_tokens=128, max_sinks=2, rot_heads=4, quant_group=32)
        perm, kind = None, RB.KERNEL_MFMA_SUB
    cache, _, _ = full_check(w, cfg, T, perm=perm, paths=(1, 2), sink_positions=[0] if T > 1 else [])
    cache.set_decode_path(0)
    assert cache.decode_kernel() == kind


@pytest.mark.parametrize("uniform,bits", [(True, 2), (False, 2), (False, 4), (True, 3)])
def test_truncate_rolls_back_a_multi_token_step(uniform, bits):
    """Speculative decoding's shape: four drafted tokens are appended and read the cache together
    (rkv_decode_attention_multi); some are rejected, rkv_cache_truncate rolls the cache back, and
    decoding goes on with other tokens.  The cache must then equal - codes, metadata, sink rows,
    lengths, attention outputs, all bit for bit - a cache that only ever saw the accepted tokens.
    One of the drafted tokens is a flagged sink behind the cut: it must be dropped."""
    w = small("cfg1", n_q_heads=8, n_kv_heads=8)
    B, T0 = 2, 45
    cfg = R.RkvConfig(batch=B, n_q_heads=8, n_kv_heads=8, max_tokens=128, max_sinks=4, rot_heads=4, bits=bits)
    k, v, mask = S.make_kv(w, T0 + 4 + 3, batch=B, sink_positions=[0, 1])
    mask = mask.copy()
    mask[:, T0 + 3] = 1                                        # the last drafted token is flagged as a sink
    accepted = [2, 2] if uniform else [3, 1]
    a, b = R.RkvCache(cfg), R.RkvCache(cfg)
    a.quantize_append(P.gpu(k[:, :T0 + 4]), P.gpu(v[:, :T0 + 4]), P.gpu(mask[:, :T0 + 4]))
    q4 = np.stack([S.make_q(w, batch=B, step=i) for i in range(4)], axis=1)
    pos = np.tile(np.arange(T0, T0 + 4, dtype=np.int32), (B, 1))
    a.decode_attention_multi(P.gpu(q4), P.gpu(pos))            # the verification pass
    assert int(a.export_sinks()["count"].max()) == 3
    a.truncate([T0 + n for n in accepted])
    assert a.lengths == [T0 + n for n in accepted]
    # the reference cache: prefix + accepted drafts only
    n_max = max(accepted)
    kk = np.zeros((B, T0 + n_max, 8, 128), np.float16)
    vv = np.zeros_like(kk)
    mm = np.zeros((B, T0 + n_max), np.uint8)
    for s_ in range(B):
        n = T0 + accepted[s_]
        kk[s_, :n], vv[s_, :n], mm[s_, :n] = k[s_, :n], v[s_, :n], mask[s_, :n]
    if uniform:
        b.quantize_append(P.gpu(kk), P.gpu(vv), P.gpu(mm))
    else:
        b.quantize_append_ragged(P.gpu(kk), P.gpu(vv), [T0 + n for n in accepted], P.gpu(mm))
    # both go on decoding with three fresh tokens
    for s_ in range(3):
        t = T0 + 4 + s_
        q = P.gpu(S.make_q(w, batch=B, step=10 + s_))
        oa = a.decode_step(P.gpu(k[:, t:t + 1]), P.gpu(v[:, t:t + 1]), q)
        ob = b.decode_step(P.gpu(k[:, t:t + 1]), P.gpu(v[:, t:t + 1]), q)
        torch.cuda.synchronize()
        assert torch.equal(oa, ob), f"step {s_}"
    assert a.lengths == b.lengths
    ea, eb = a.export_codes(), b.export_codes()
    sa, sb = a.export_sinks(), b.export_sinks()
    torch.cuda.synchronize()
    assert torch.equal(sa["count"], sb["count"]) and int(sa["count"].max()) == 2
    for s_ in range(B):
        n = a.lengths[s_]
        for name in ea:
            assert torch.equal(ea[name][s_, :n], eb[name][s_, :n]), (name, s_)
        c = int(sa["count"][s_])
        for name in ("pos", "k", "v"):
            assert torch.equal(sa[name][s_, :c], sb[name][s_, :c]), (name, s_)
    with pytest.raises(R.RkvError):
        a.truncate([a.lengths[0] + 1, 0])                      # cannot grow
    a.truncate(0)
    assert a.lengths == [0, 0]


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_randomly_drawn_configurations(seed):
    """Forty configurations per seed, drawn over everything a configuration may combine: rotation
    size, GQA ratio, code width, group size, metadata format, RoPE pairing, reorder span, batch,
    length (tile and chunk edges among them), retained rows, appends in pieces - most of them
    settings with a matrix-core variant.  Each goes through full_check (write half bit for bit,
    sinks, dequantize view, both decode paths on the GPU's and on the oracle's codes).
    The synthetic keys carry massive activations, so the scores here run into the thousands; a
    score is an fp32 sum over the rotation group's 128 g channels, in which the energy of the
    group's other heads cancels only up to rounding, so its error scales with the group's largest
    score and not with the head's own: the log-sum-exp bar is 1e-3, or 2e-6 (sqrt(512) 2^-24 is
    1.3e-6) of the largest log-sum-exp of the case where that is more."""
    import random
    rnd = random.Random(seed)
    lse_bar = lambda ref: max(LSE_TOL, 2e-6 * float(np.abs(ref).max()))
    seen = set()
    for i in range(40):
        g = rnd.choice([2, 4, 4, 2, 4, 2, 4, 2, 1, 8])
        hkv = rnd.choice([8, 16]) if g == 8 else rnd.choice([4, 8, 12, 16])
        if hkv % g:
            hkv = 8
        hq = hkv * rnd.choice([1, 1, 2, 3, 4])
        bits, group = rnd.choice([2, 2, 2, 3, 4]), rnd.choice([128, 128, 64, 32])
        fmt, style = rnd.choice([0, 1]), rnd.choice([0, 1])
        span = rnd.choice([128, 128, 128 * g, 128 * hkv])
        if rnd.random() < 0.85:                                # a setting with a matrix-core variant (if g is 2 or 4)
            kind = rnd.choice(["plain", "plain", "groups", "across blocks", "whole row"])
            if kind == "plain":
                group, span = 128, 128
            elif kind == "groups":
                bits, group, span = rnd.choice([2, 2, 3, 4]), rnd.choice([64, 32]), 128
            elif kind == "across blocks":
                bits, group, span = rnd.choice([2, 2, 3, 4]), rnd.choice([128, 128, 64, 32]), 128 * g
            else:
                bits, group, span = rnd.choice([2, 2, 3, 4]), rnd.choice([128, 128, 64, 32]), 128 * hkv
        B = rnd.choice([1, 2, 3])
        T = rnd.choice([1, 15, 16, 17, 63, 64, 65, 100, 255, 256, 257, rnd.randint(1, 600), rnd.randint(200, 900)])
        sinks = rnd.choice([0, 4, 2])
        w = small("cfg1", n_q_heads=hq, n_kv_heads=hkv)
        kw = dict(batch=B, n_q_heads=hq, n_kv_heads=hkv, max_tokens=T + rnd.choice([0, 1, 37]), max_sinks=sinks, rot_heads=g,
                  meta_format=fmt, rope_style=style)
        cfg = R.RkvConfig(bits=bits, quant_group=group, perm_span=span, **kw)
        print(f"[case {i}] seed={seed} g={g} hq={hq} hkv={hkv} bits={bits} group={group} fmt={fmt} style={style} span={span} "
              f"B={B} T={T} sinks={sinks}", flush=True)
        perm = None
        if span != 128 or rnd.random() < 0.8:
            perm = calibrated_perm(w, R.RkvConfig(perm_span=span, **kw), offset_variant=span != 128)
        cuts = sorted(set([0, T] + [rnd.randint(0, T) for _ in range(rnd.choice([0, 1, 3]))]))
        probe = R.RkvCache(cfg)
        if perm is not None:
            probe.set_perm(P.gpu(np.asarray(perm, dtype=np.int32)))
        kernel = probe.decode_kernel()
        del probe
        seen.add(kernel)
        full_check(w, cfg, T, perm=perm, chunks=cuts, paths=(1, 0) if kernel == RB.KERNEL_GENERAL else (1, 2),
                   sink_positions=[] if sinks == 0 or rnd.random() < 0.5 else None, lse_bar=lse_bar)
    assert seen == {RB.KERNEL_GENERAL, RB.KERNEL_MFMA, RB.KERNEL_MFMA_CROSS, RB.KERNEL_MFMA_SUB, RB.KERNEL_MFMA_ROW}


@pytest.mark.parametrize("seed", [21, 22])
def test_randomly_drawn_steps_lengths_and_query_counts(seed):
    """Forty configurations per seed, drawn as in test_randomly_drawn_configurations, through the
    other entry points: a prefill with per-sequence lengths (empty sequences among them) where the
    append kernel serves them, then one-call decode steps against the two calls on a second cache
    (outputs, log-sum-exp, codes and metadata bit for bit; explicit query positions on every other
    step), then - each sequence against an oracle cache of its own, on the GPU's codes - decode
    attention on both kernels, its current-token variant, and two to four causal query tokens
    (within the general kernel's limit of 8 rows per KV head where that kernel serves them)."""
    import random
    rnd = random.Random(seed)
    for i in range(40):
        g = rnd.choice([2, 4, 4, 2, 4, 2, 4, 2, 1, 8])
        hkv = rnd.choice([8, 16]) if g == 8 else rnd.choice([4, 8, 12, 16])
        if hkv % g:
            hkv = 8
        rep = rnd.choice([1, 1, 2, 3, 4])
        hq = hkv * rep
        bits, group = rnd.choice([2, 2, 2, 3, 4]), rnd.choice([128, 128, 64, 32])
        fmt, style = rnd.choice([0, 1]), rnd.choice([0, 1])
        span = rnd.choice([128, 128, 128 * g, 128 * hkv])
        if rnd.random() < 0.85:
            kind = rnd.choice(["plain", "plain", "groups", "across blocks", "whole row"])
            if kind == "plain":
                group, span = 128, 128
            elif kind == "groups":
                bits, group, span = rnd.choice([2, 2, 3, 4]), rnd.choice([64, 32]), 128
            elif kind == "across blocks":
                bits, group, span = rnd.choice([2, 2, 3, 4]), rnd.choice([128, 128, 64, 32]), 128 * g
            else:
                bits, group, span = rnd.choice([2, 2, 3, 4]), rnd.choice([128, 128, 64, 32]), 128 * hkv
        B, sinks = rnd.choice([1, 2, 3, 4]), rnd.choice([0, 4, 2])
        t_max = rnd.choice([1, 16, 17, 64, 65, 255, 256, 257, rnd.randint(1, 500), rnd.randint(100, 700)])
        lens = [t_max] * B
        if rnd.random() < 0.6:
            lens = [rnd.choice([t_max, rnd.randint(0, t_max), rnd.randint(0, t_max), 0]) for _ in range(B)]
            if max(lens) == 0:
                lens[0] = t_max
        n_steps = rnd.choice([1, 3, 5])
        w = small("cfg1", n_q_heads=hq, n_kv_heads=hkv)
        kw = dict(batch=B, n_q_heads=hq, n_kv_heads=hkv, max_tokens=max(lens) + n_steps + rnd.choice([0, 1, 40]), max_sinks=sinks,
                  rot_heads=g, meta_format=fmt, rope_style=style)
        cfg = R.RkvConfig(bits=bits, quant_group=group, perm_span=span, **kw)
        perm = None
        if span != 128 or rnd.random() < 0.8:
            perm = calibrated_perm(w, R.RkvConfig(perm_span=span, **kw), offset_variant=span != 128)
        a, b2 = R.RkvCache(cfg), R.RkvCache(cfg)
        if perm is not None:
            for c in (a, b2):
                c.set_perm(P.gpu(np.asarray(perm, dtype=np.int32)))
        vector_append = a.append_kernel() in (RB.KERNEL_GENERAL, RB.KERNEL_SHUFFLE)
        if vector_append:                                      # per-sequence lengths need the matrix-core append kernel
            lens = [max(lens)] * B
        total = [n + n_steps for n in lens]
        print(f"[case {i}] seed={seed} g={g} hq={hq} hkv={hkv} bits={bits} group={group} fmt={fmt} style={style} span={span} "
              f"lens={lens} steps={n_steps} sinks={sinks} kernels: decode {a.decode_kernel()} append {a.append_kernel()}", flush=True)
        sp = [] if sinks == 0 or rnd.random() < 0.5 else None
        data = [S.make_kv(w, total[s_] + 1, batch=1, layer=s_, sink_positions=sp) for s_ in range(B)]
        ocs = [O.cache_new(P.oracle_cfg(dataclasses.replace(cfg, batch=1)), perm) for _ in range(B)]
        n_max = max(lens)
        k = np.zeros((B, n_max, hkv, 128), np.float16)
        v = np.zeros_like(k)
        m = np.zeros((B, n_max), np.uint8)
        for s_ in range(B):
            kb, vb, mb = data[s_]
            n = lens[s_]
            k[s_, :n], v[s_, :n], m[s_, :n] = kb[0, :n], vb[0, :n], mb[0, :n]
            if n:
                O.quantize_append(ocs[s_], kb[:, :n], vb[:, :n], mb[:, :n] if sinks else None)
        for c in (a, b2):
            if len(set(lens)) == 1:
                c.quantize_append(P.gpu(k), P.gpu(v), P.gpu(m) if sinks else None)
            else:
                c.quantize_append_ragged(P.gpu(k), P.gpu(v), lens, P.gpu(m) if sinks else None)
        for st in range(n_steps):
            q = P.gpu(S.make_q(w, batch=B, step=st))
            kk = np.stack([data[s_][0][0, lens[s_] + st] for s_ in range(B)])[:, None]
            vv = np.stack([data[s_][1][0, lens[s_] + st] for s_ in range(B)])[:, None]
            for s_ in range(B):
                O.quantize_append(ocs[s_], kk[s_:s_ + 1], vv[s_:s_ + 1], None)
            q_pos = None if st % 2 == 0 else P.gpu(np.array([lens[s_] + st + rnd.choice([0, 5, 300]) for s_ in range(B)], dtype=np.int32))
            o1, l1 = a.decode_step(P.gpu(kk), P.gpu(vv), q, q_pos, want_lse=True)
            b2.quantize_append(P.gpu(kk), P.gpu(vv))
            o2, l2 = b2.decode_attention(q, q_pos, want_lse=True)
            torch.cuda.synchronize()
            assert torch.equal(o1, o2) and torch.equal(l1, l2), f"step {st}: one call against two"
        assert a.lengths == total and b2.lengths == total
        ea, eb = a.export_codes(), b2.export_codes()
        torch.cuda.synchronize()
        for s_ in range(B):
            for name in ea:
                assert torch.equal(ea[name][s_, :total[s_]], eb[name][s_, :total[s_]]), (name, s_)
        gexp = P.export_numpy(a)
        ocg = [oracle_from_export(ocs[s_], {name: arr[s_:s_ + 1, :total[s_]] for name, arr in gexp.items()}) for s_ in range(B)]
        q = S.make_q(w, batch=B, step=77)
        kc = np.concatenate([data[s_][0][:, total[s_]] for s_ in range(B)])
        vc = np.concatenate([data[s_][1][:, total[s_]] for s_ in range(B)])
        for path in ((1, 0) if a.decode_kernel() == RB.KERNEL_GENERAL else (1, 2)):
            a.set_decode_path(path)
            out, lse = a.decode_attention(P.gpu(q), want_lse=True)
            out_cur = a.decode_attention(P.gpu(q), k_cur=P.gpu(kc), v_cur=P.gpu(vc))
            torch.cuda.synchronize()
            for s_ in range(B):
                ref, lse_ref = O.decode_attention(ocg[s_], q[s_:s_ + 1])
                e = P.attention_error(out[s_:s_ + 1].cpu().numpy().astype(np.float64), ref)
                le = float(np.abs(lse[s_:s_ + 1].cpu().numpy() - lse_ref).max())
                # (the log-sum-exp bar: see test_randomly_drawn_configurations)
                assert e <= ATT_TOL and le <= max(LSE_TOL, 2e-6 * float(np.abs(lse_ref).max())), f"path {path} sequence {s_}: {e} {le}"
                ref, _ = O.decode_attention(ocg[s_], q[s_:s_ + 1], None, kc[s_:s_ + 1], vc[s_:s_ + 1])
                e = P.attention_error(out_cur[s_:s_ + 1].cpu().numpy().astype(np.float64), ref)
                assert e <= ATT_TOL, f"current token, path {path}, sequence {s_}: {e}"
        a.set_decode_path(0)
        nq = rnd.choice([2, 3, 4])
        try:
            a.decode_kernel(nq)
        except R.RkvError:                                     # beyond the general kernel's 8 rows per KV head: refused, not mis-computed
            with pytest.raises(R.RkvError):
                a.decode_attention_multi(P.gpu(np.zeros((B, nq, hq, 128), np.float16)), P.gpu(np.zeros((B, nq), np.int32)))
            nq = max(1, 8 // rep)
        if min(total) >= nq:
            qn = np.stack([S.make_q(w, batch=B, step=20 + j) for j in range(nq)], axis=1)
            q_pos = np.array([[total[s_] - nq + j for j in range(nq)] for s_ in range(B)], dtype=np.int32)
            out = a.decode_attention_multi(P.gpu(qn), P.gpu(q_pos))
            torch.cuda.synchronize()
            for s_ in range(B):
                ref, _ = O.decode_attention_multi(ocg[s_], qn[s_:s_ + 1], q_pos[s_:s_ + 1])
                e = P.attention_error(out[s_:s_ + 1].cpu().numpy().astype(np.float64), ref)
                assert e <= ATT_TOL, f"{nq} query tokens, sequence {s_}: {e}"


@pytest.mark.parametrize("setting,g,hq,bits,group,fmt,nq", [("whole row", 4, 8, 2, 128, 0, 4), ("whole row", 2, 16, 2, 128, 1, 3),
                                                          ("across blocks", 4, 16, 4, 128, 0, 2), ("across blocks", 2, 8, 2, 64, 1, 4),
                                                          ("inside heads", 4, 8, 3, 32, 1, 3), ("inside heads", 2, 32, 2, 64, 0, 2),
                                                          ("inside heads", 4, 8, 4, 32, 0, 8)])
def test_several_query_tokens_on_the_scores_kernel_routes(setting, g, hq, bits, group, fmt, nq):
    """rkv_decode_attention_multi where the scores come from the scores kernel (reorders across
    blocks, groups of 64 / 32, wider codes on those routes): causal query tokens at the end of the
    cache and one far behind it, GQA, sequences of different lengths, retained rows behind a query's
    position; the configuration's own route and the general kernel against the oracle on the GPU's
    codes.  Eight (query token, query head) pairs per KV head is the limit."""
    hkv = 8
    rep = hq // hkv
    w = small("cfg1", n_q_heads=hq, n_kv_heads=hkv)
    span = {"whole row": 128 * hkv, "across blocks": 128 * g, "inside heads": 128}[setting]
    kw = dict(batch=2, n_q_heads=hq, n_kv_heads=hkv, max_tokens=420, max_sinks=4, rot_heads=g, meta_format=fmt)
    cfg = R.RkvConfig(bits=bits, quant_group=group, perm_span=span, **kw)
    perm = calibrated_perm(w, R.RkvConfig(perm_span=span, **kw), offset_variant=span != 128)
    lens = [401, 150]
    data = [S.make_kv(w, lens[b], batch=1, layer=b, sink_positions=[0, 3, lens[b] - 2]) for b in range(2)]
    cache = R.RkvCache(cfg)
    cache.set_perm(P.gpu(np.asarray(perm, dtype=np.int32)))
    ocs = [O.cache_new(P.oracle_cfg(dataclasses.replace(cfg, batch=1)), perm) for _ in range(2)]
    k = np.zeros((2, max(lens), hkv, 128), np.float16)
    v = np.zeros_like(k)
    m = np.zeros((2, max(lens)), np.uint8)
    for b in range(2):
        kb, vb, mb = data[b]
        k[b, :lens[b]], v[b, :lens[b]], m[b, :lens[b]] = kb[0], vb[0], mb[0]
        O.quantize_append(ocs[b], kb, vb, mb)
    if setting == "whole row":           # (per-sequence lengths need the plain, sub-group or cross-block append kernel)
        lens = [401, 401]
        cache.quantize_append(P.gpu(np.repeat(k[:1], 2, axis=0)), P.gpu(np.repeat(v[:1], 2, axis=0)), P.gpu(np.repeat(m[:1], 2, axis=0)))
        ocs[1] = ocs[0]
    else:
        cache.quantize_append_ragged(P.gpu(k), P.gpu(v), lens, P.gpu(m))
    torch.cuda.synchronize()
    want = {"whole row": RB.KERNEL_MFMA_ROW, "across blocks": RB.KERNEL_MFMA_CROSS if group == 128 else RB.KERNEL_MFMA_SUB,
            "inside heads": RB.KERNEL_MFMA_SUB}[setting]
    gexp = P.export_numpy(cache)
    ocg = [oracle_from_export(ocs[b], {name: arr[b:b + 1, :lens[b]] for name, arr in gexp.items()}) for b in range(2)]
    qn = np.stack([S.make_q(w, batch=2, step=j) for j in range(nq)], axis=1)
    # the last query tokens of each sequence, the first of them moved far back (behind the retained row near the end)
    q_pos = np.array([[lens[b] - nq + j for j in range(nq)] for b in range(2)], dtype=np.int32)
    q_pos[:, 0] = [37, 5]
    if rep * nq > 8:
        assert want != RB.KERNEL_MFMA
        with pytest.raises(R.RkvError):
            cache.decode_attention_multi(P.gpu(qn), P.gpu(q_pos))
        nq = 8 // rep
        qn, q_pos = qn[:, :nq].copy(), q_pos[:, :nq].copy()
    refs = [O.decode_attention_multi(ocg[b], qn[b:b + 1], q_pos[b:b + 1]) for b in range(2)]
    for path in (0, 1):
        cache.set_decode_path(path)
        assert cache.decode_kernel(nq) == (want if path == 0 else RB.KERNEL_GENERAL)
        print(f"[case] {nq} query tokens, {setting}, g={g} hq={hq} bits={bits} group={group}, path {path}", flush=True)
        out, lse = cache.decode_attention_multi(P.gpu(qn), P.gpu(q_pos), want_lse=True)
        torch.cuda.synchronize()
        for b in range(2):
            ref, lse_ref = refs[b]
            e = P.attention_error(out[b:b + 1].cpu().numpy().astype(np.float64), ref)
            le = float(np.abs(lse[b:b + 1].cpu().numpy() - lse_ref).max())
            print(f"[parity] path {path} sequence {b}: out err {e:.3e} lse err {le:.3e}", flush=True)
            assert e <= ATT_TOL and le <= max(LSE_TOL, 2e-6 * float(np.abs(lse_ref).max()))
