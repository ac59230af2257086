"""rkv_decode_attention_static - the decode call that allocates nothing and takes no work space -
against rkv_decode_attention on the same caches, through the C ABI.  Same kernels, so the bar is
equality bit for bit.  Two calls in a row share the library's built-in work space, the second on a
smaller cache: nothing the first call left there may show in the second's results."""
import numpy as np
import pytest
import torch

import paper_2501_16383_amd as R
from paper_2501_16383_amd import binding as RB
import rkv_synth as S
import parity_utils as P

pytestmark = pytest.mark.gpu


def _filled(w, cfg, T, layer):
    k, v, mask, q = P.make_case(w, cfg, T, layer=layer)
    cache = R.RkvCache(cfg)
    cache.quantize_append(P.gpu(k), P.gpu(v), P.gpu(mask) if cfg.max_sinks else None)
    return cache, P.gpu(q)


@pytest.mark.parametrize("path", [0, 1])
def test_static_work_space_gives_the_same_results_twice_in_a_row(path):
    import dataclasses
    w = dataclasses.replace(S.WORKLOADS["cfg1"], n_q_heads=16, n_kv_heads=8)
    big = R.RkvConfig(batch=4, n_q_heads=16, n_kv_heads=8, max_tokens=1024, max_sinks=4, rot_heads=4)
    little = R.RkvConfig(batch=2, n_q_heads=16, n_kv_heads=8, max_tokens=512, max_sinks=0, rot_heads=4)
    print(f"[case] static work space, decode path {path}: batch 4 x 700 tokens, then batch 2 x 300 tokens", flush=True)
    a, qa = _filled(w, big, 700, 0)
    b, qb = _filled(dataclasses.replace(w, n_sinks=0), little, 300, 1)
    for c in (a, b):
        c.set_decode_path(path)
    assert a.decode_kernel() == (RB.KERNEL_MFMA if path == 0 else RB.KERNEL_GENERAL)
    ref_a, lse_ref_a = a.decode_attention(qa, want_lse=True)
    ref_b, lse_ref_b = b.decode_attention(qb, want_lse=True)
    torch.cuda.synchronize()
    out_a, lse_a = torch.full_like(ref_a, float("nan")), torch.full_like(lse_ref_a, float("nan"))
    out_b, lse_b = torch.full_like(ref_b, float("nan")), torch.full_like(lse_ref_b, float("nan"))
    a.decode_attention_static(qa, out_a, lse=lse_a)          # the larger call first ...
    b.decode_attention_static(qb, out_b, lse=lse_b)          # ... then the smaller one on the same work space
    torch.cuda.synchronize()
    assert torch.equal(out_a, ref_a) and torch.equal(lse_a, lse_ref_a)
    assert torch.equal(out_b, ref_b) and torch.equal(lse_b, lse_ref_b)
    # and once more the other way round, with a query position of the caller's
    qp = P.gpu(np.array([310, 299], dtype=np.int32))
    ref_b2 = b.decode_attention(qb, qp)
    out_b2 = torch.empty_like(ref_b2)
    b.decode_attention_static(qb, out_b2, q_pos=qp)
    a.decode_attention_static(qa, out_a)
    torch.cuda.synchronize()
    assert torch.equal(out_b2, ref_b2) and torch.equal(out_a, ref_a)
    # against the oracle too (the same bar as every decode test), on the GPU's own codes
    from oracle import rkv_oracle as O
    k, v, mask, q = P.make_case(dataclasses.replace(w, n_sinks=0), little, 300, layer=1)
    oc = O.cache_new(P.oracle_cfg(little))
    O.quantize_append(oc, k, v, None)
    g = P.export_numpy(b)
    for name in ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero"):
        setattr(oc, name, g[name])
    ref, _ = O.decode_attention(oc, q)
    assert P.attention_error(out_b.cpu().numpy().astype(np.float64), ref) <= 2e-3


@pytest.mark.parametrize("setting", ["whole row", "across blocks", "groups of 32"])
def test_static_work_space_on_the_scores_kernel_paths(setting):
    """Settings whose scores pass through the work space (a kernel of their own computes them, the
    matrix-core kernel takes them from there): the static entry point against the ordinary one,
    bit for bit, a larger cache first and a smaller one after it on the same built-in space."""
    import dataclasses
    from test_gpu_parity import calibrated_perm
    w = dataclasses.replace(S.WORKLOADS["cfg1"], n_q_heads=16, n_kv_heads=8, n_sinks=0)
    kw = dict(n_q_heads=16, n_kv_heads=8, max_sinks=0, rot_heads=4,
              perm_span={"whole row": 1024, "across blocks": 512, "groups of 32": 128}[setting],
              quant_group=32 if setting == "groups of 32" else 128)
    kind = {"whole row": RB.KERNEL_MFMA_ROW, "across blocks": RB.KERNEL_MFMA_CROSS, "groups of 32": RB.KERNEL_MFMA_SUB}[setting]
    results = []
    caches = []
    for batch, cap, T, layer in ((3, 1000, 700, 0), (2, 300, 290, 1)):
        cfg = R.RkvConfig(batch=batch, max_tokens=cap, **kw)
        perm = calibrated_perm(w, cfg, offset_variant=True)
        k, v, _, q = P.make_case(w, cfg, T, layer=layer, sink_positions=[])
        cache = R.RkvCache(cfg)
        cache.set_perm(P.gpu(np.asarray(perm, dtype=np.int32)))
        cache.quantize_append(P.gpu(k), P.gpu(v))
        assert cache.decode_kernel() == kind
        ref, lse_ref = cache.decode_attention(P.gpu(q), want_lse=True)
        caches.append((cache, P.gpu(q), ref, lse_ref))
    torch.cuda.synchronize()
    print(f"[case] static work space, {setting}: batch 3 x 700 tokens, then batch 2 x 290 tokens", flush=True)
    for cache, q, ref, lse_ref in caches:
        out, lse = torch.full_like(ref, float("nan")), torch.full_like(lse_ref, float("nan"))
        cache.decode_attention_static(q, out, lse=lse)
        results.append((out, lse))
    torch.cuda.synchronize()
    for (cache, q, ref, lse_ref), (out, lse) in zip(caches, results):
        assert torch.equal(out, ref) and torch.equal(lse, lse_ref)


def test_static_work_space_rejects_what_does_not_fit():
    """Batch 64 x 64 heads x 4096 tokens needs 37 MB of partials: RKV_ESCRATCH, nothing enqueued,
    and the call with a work space of the caller's still works."""
    cfg = R.RkvConfig(batch=64, n_q_heads=64, n_kv_heads=8, max_tokens=4096, max_sinks=0, rot_heads=4)
    cache = R.RkvCache(cfg)
    k = torch.zeros((64, 4096, 8, 128), dtype=torch.float16, device="cuda")
    cache.quantize_append(k, k)
    q = torch.zeros((64, 64, 128), dtype=torch.float16, device="cuda")
    out = torch.zeros((64, 64, 128), dtype=torch.float32, device="cuda")
    with pytest.raises(R.RkvError) as ei:
        cache.decode_attention_static(q, out)
    assert ei.value.code == RB.RKV_ESCRATCH
    cache.truncate(1024)                                      # 64 x 64 x 4 chunks: 19 MB, fits
    cache.decode_attention_static(q, out)
    ref = cache.decode_attention(q)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)
