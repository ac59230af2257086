"""ctypes binding of librkv.so.  Argument marshalling only: every step of the path runs in the
library's kernels.  torch supplies device memory and the current stream, nothing else.

The library must be present (build it with `python -m paper_2501_16383_amd.build` or
`__graft_entry__.build()`); there is no fallback of any kind.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librkv.so")
_lib = None

RKV_OK, RKV_EINVAL, RKV_ECAPACITY, RKV_EPERM, RKV_EHIP, RKV_ESTATE, RKV_ESCRATCH = 0, -1, -2, -3, -4, -5, -6
STATIC_SCRATCH_BYTES = 24 << 20
KERNEL_GENERAL, KERNEL_SHUFFLE, KERNEL_MFMA, KERNEL_MFMA_CROSS, KERNEL_MFMA_SUB, KERNEL_MFMA_ROW = 1, 2, 3, 4, 5, 6

EXPORTS = [
    "rkv_query_sizes", "rkv_cache_create", "rkv_cache_destroy", "rkv_cache_reset", "rkv_cache_length",
    "rkv_calibrate_perm", "rkv_fold_rotation", "rkv_set_perm", "rkv_select_sinks", "rkv_quantize_append", "rkv_decode_attention", "rkv_decode_attention_static", "rkv_decode_attention_with_current",
    "rkv_decode_attention_multi", "rkv_decode_step", "rkv_quantize_append_ragged", "rkv_cache_lengths", "rkv_cache_truncate",
    "rkv_set_decode_path", "rkv_decode_kernel_of", "rkv_append_kernel_of", "rkv_set_profile_events", "rkv_dequantize", "rkv_export_codes", "rkv_import_codes", "rkv_export_sinks", "rkv_layout_locate",
    "rkv_strerror",
]


class RkvError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = load_library().rkv_strerror(code).decode()
        super().__init__(f"{where}: {msg} ({code})")


class _CConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "batch", "n_q_heads", "n_kv_heads", "head_dim", "max_tokens", "max_sinks", "rot_heads",
        "quant_group", "bits", "perm_span", "rope_style", "v_rotate")] + [
        ("rope_theta", C.c_float), ("clip_ratio", C.c_float), ("keys_rotated", C.c_int32), ("meta_format", C.c_int32)]


@dataclass
class RkvConfig:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    max_tokens: int
    head_dim: int = 128
    max_sinks: int = 4
    rot_heads: int = 4
    quant_group: int = 128
    bits: int = 2
    perm_span: int = 128
    rope_style: int = 0
    v_rotate: int = 0
    rope_theta: float = 10000.0
    clip_ratio: float = 1.0
    keys_rotated: int = 0
    meta_format: int = 0

    def to_c(self) -> _CConfig:
        return _CConfig(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.max_tokens,
                        self.max_sinks, self.rot_heads, self.quant_group, self.bits, self.perm_span,
                        self.rope_style, self.v_rotate, self.rope_theta, self.clip_ratio, self.keys_rotated, self.meta_format)

    @property
    def E(self) -> int:
        return self.n_kv_heads * self.head_dim


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load librkv.so (once).  Raises if it has not been built: the product has no other path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2501_16383_amd.build`")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    cfgp = C.POINTER(_CConfig)
    lib.rkv_query_sizes.argtypes = [cfgp, C.POINTER(sz), C.POINTER(sz)]
    lib.rkv_cache_create.argtypes = [cfgp, vp, sz, vp, C.POINTER(vp)]
    lib.rkv_cache_destroy.argtypes = [vp]
    lib.rkv_cache_destroy.restype = None
    lib.rkv_cache_reset.argtypes = [vp, vp]
    lib.rkv_cache_length.argtypes = [vp]
    lib.rkv_calibrate_perm.argtypes = [cfgp, vp, i32, vp, vp, vp]
    lib.rkv_set_perm.argtypes = [vp, vp, vp]
    lib.rkv_fold_rotation.argtypes = [cfgp, vp, i32, vp, vp, vp]
    lib.rkv_select_sinks.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp]
    lib.rkv_quantize_append.argtypes = [vp, vp, vp, i32, vp, vp]
    lib.rkv_decode_attention.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.rkv_decode_attention_static.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.rkv_decode_attention_with_current.argtypes = [vp] * 9
    lib.rkv_decode_attention_multi.argtypes = [vp, vp, vp, C.c_int32, vp, vp, vp, vp]
    lib.rkv_decode_step.argtypes = [vp] * 9
    lib.rkv_quantize_append_ragged.argtypes = [vp, vp, vp, C.c_int32, vp, vp, vp]
    lib.rkv_cache_lengths.argtypes = [vp, vp]
    lib.rkv_cache_truncate.argtypes = [vp, vp, vp]
    lib.rkv_set_decode_path.argtypes = [vp, i32]
    lib.rkv_decode_kernel_of.argtypes = [vp, i32]
    lib.rkv_append_kernel_of.argtypes = [vp]
    lib.rkv_set_profile_events.argtypes = [vp, vp, vp]
    lib.rkv_dequantize.argtypes = [vp, vp, vp, vp]
    lib.rkv_export_codes.argtypes = [vp] * 8
    lib.rkv_import_codes.argtypes = [vp, i32] + [vp] * 7
    lib.rkv_export_sinks.argtypes = [vp] * 6
    lib.rkv_layout_locate.argtypes = [cfgp, i32, i32, i32, i32, C.POINTER(sz), C.POINTER(i32), C.POINTER(sz)]
    lib.rkv_strerror.argtypes = [C.c_int]
    lib.rkv_strerror.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("rkv_cache_destroy", "rkv_strerror"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(code: int, where: str) -> None:
    if code != RKV_OK:
        raise RkvError(code, where)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _dev(t, dtype, what: str):
    import torch
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{what} must be a contiguous CUDA tensor of dtype {dtype}")
    return t


def query_sizes(cfg: RkvConfig):
    lib = load_library()
    a, b = C.c_size_t(0), C.c_size_t(0)
    cc = cfg.to_c()
    _check(lib.rkv_query_sizes(C.byref(cc), C.byref(a), C.byref(b)), "rkv_query_sizes")
    return a.value, b.value


def layout_locate(cfg: RkvConfig, is_v: bool, b: int, t: int, c: int):
    """(word index, bit shift, words in the region) of a code in the physical layout (host only)."""
    lib = load_library()
    w, sh, n = C.c_size_t(0), C.c_int32(0), C.c_size_t(0)
    cc = cfg.to_c()
    _check(lib.rkv_layout_locate(C.byref(cc), int(is_v), b, t, c, C.byref(w), C.byref(sh), C.byref(n)), "rkv_layout_locate")
    return w.value, sh.value, n.value


def calibrate_perm(cfg: RkvConfig, k_cal, scratch=None):
    """rkv_calibrate_perm: k_cal [n_tok, n_kv_heads, 128] fp16 on the device -> int32 [E] on the device."""
    import torch
    lib = load_library()
    k_cal = _dev(k_cal, torch.float16, "k_cal")
    if scratch is None:
        scratch = torch.empty(cfg.E * 16 + 256, dtype=torch.uint8, device=k_cal.device)
    perm = torch.empty(cfg.E, dtype=torch.int32, device=k_cal.device)
    cc = cfg.to_c()
    _check(lib.rkv_calibrate_perm(C.byref(cc), _ptr(k_cal), k_cal.shape[0], _ptr(perm), _ptr(scratch), _stream()),
           "rkv_calibrate_perm")
    return perm


def fold_rotation(cfg: RkvConfig, w, perm=None):
    """rkv_fold_rotation: w [rows, E] fp32 on the device -> the same shape with rotation (and reorder) folded in."""
    import torch
    lib = load_library()
    w = _dev(w, torch.float32, "w")
    perm = _dev(perm, torch.int32, "perm")
    if w.dim() != 2 or w.shape[1] != cfg.E:
        raise ValueError("w must be [rows, E]")
    out = torch.empty_like(w)
    cc = cfg.to_c()
    _check(lib.rkv_fold_rotation(C.byref(cc), _ptr(w), w.shape[0], _ptr(perm), _ptr(out), _stream()), "rkv_fold_rotation")
    return out


def select_sinks(x, k: int, want_mask: bool = True):
    """rkv_select_sinks: x [batch, n_tok, width] fp16 on the device -> (int32 [batch, k], uint8 [batch, n_tok] or None)."""
    import torch
    lib = load_library()
    x = _dev(x, torch.float16, "x")
    if x.dim() != 3:
        raise ValueError("x must be [batch, n_tok, width]")
    batch, n_tok, width = x.shape
    idx = torch.empty(batch, k, dtype=torch.int32, device=x.device)
    mask = torch.empty(batch, n_tok, dtype=torch.uint8, device=x.device) if want_mask else None
    scratch = torch.empty(batch * n_tok * 4, dtype=torch.uint8, device=x.device)
    _check(lib.rkv_select_sinks(_ptr(x), batch, n_tok, width, k, _ptr(idx), _ptr(mask), _ptr(scratch), _stream()),
           "rkv_select_sinks")
    return idx, mask


class RkvCache:
    """One layer's compressed KV cache.  Owns the torch buffers that back it."""

    def __init__(self, cfg: RkvConfig, device="cuda:0", scratch=None):
        import torch
        self.cfg = cfg
        self.lib = load_library()
        self.device = torch.device(device)
        cache_bytes, scratch_bytes = query_sizes(cfg)
        self.cache_bytes, self.scratch_bytes = cache_bytes, scratch_bytes
        self.mem = torch.empty(cache_bytes, dtype=torch.uint8, device=self.device)
        self.scratch = scratch if scratch is not None else torch.empty(scratch_bytes, dtype=torch.uint8, device=self.device)
        if self.scratch.numel() < scratch_bytes:
            raise ValueError("scratch too small")
        h = C.c_void_p()
        cc = cfg.to_c()
        with torch.cuda.device(self.device):
            _check(self.lib.rkv_cache_create(C.byref(cc), self.mem.data_ptr(), cache_bytes, _stream(), C.byref(h)),
                   "rkv_cache_create")
        self.handle = h

    def __del__(self):
        h = getattr(self, "handle", None)
        if h:
            self.lib.rkv_cache_destroy(h)
            self.handle = None

    @property
    def length(self) -> int:
        return self.lib.rkv_cache_length(self.handle)

    def reset(self):
        _check(self.lib.rkv_cache_reset(self.handle, _stream()), "rkv_cache_reset")

    def set_perm(self, perm):
        import torch
        perm = _dev(perm, torch.int32, "perm")
        _check(self.lib.rkv_set_perm(self.handle, _ptr(perm), _stream()), "rkv_set_perm")

    def set_decode_path(self, path: int):
        _check(self.lib.rkv_set_decode_path(self.handle, path), "rkv_set_decode_path")

    def decode_kernel(self, n_queries: int = 0) -> int:
        """rkv_decode_kernel_of: the KERNEL_* value of the decode kernel this cache takes."""
        rc = self.lib.rkv_decode_kernel_of(self.handle, n_queries)
        if rc < 0:
            raise RkvError(rc, "rkv_decode_kernel_of")
        return rc

    def append_kernel(self) -> int:
        """rkv_append_kernel_of: the KERNEL_* value of the append kernel this cache takes."""
        rc = self.lib.rkv_append_kernel_of(self.handle)
        if rc < 0:
            raise RkvError(rc, "rkv_append_kernel_of")
        return rc

    def set_profile_events(self, ev_start, ev_stop):
        """hipEvent_t handles (ints) recorded around the main kernel of the next calls, or None, None."""
        _check(self.lib.rkv_set_profile_events(self.handle, ev_start, ev_stop), "rkv_set_profile_events")

    def quantize_append(self, k, v, sink_mask=None):
        import torch
        k = _dev(k, torch.float16, "k")
        v = _dev(v, torch.float16, "v")
        sink_mask = _dev(sink_mask, torch.uint8, "sink_mask")
        B, n_new = k.shape[0], k.shape[1]
        if k.shape != (B, n_new, self.cfg.n_kv_heads, self.cfg.head_dim) or v.shape != k.shape or B != self.cfg.batch:
            raise ValueError("k, v must be [batch, n_new, n_kv_heads, head_dim]")
        if sink_mask is not None and sink_mask.shape != (B, n_new):
            raise ValueError("sink_mask must be [batch, n_new]")
        _check(self.lib.rkv_quantize_append(self.handle, _ptr(k), _ptr(v), n_new, _ptr(sink_mask), _stream()),
               "rkv_quantize_append")

    @property
    def lengths(self):
        """Tokens cached per sequence (list of ints)."""
        arr = (C.c_int32 * self.cfg.batch)()
        _check(self.lib.rkv_cache_lengths(self.handle, arr), "rkv_cache_lengths")
        return list(arr)

    def truncate(self, new_lengths):
        """rkv_cache_truncate: an int (all sequences) or one int per sequence."""
        B = self.cfg.batch
        vals = [int(new_lengths)] * B if isinstance(new_lengths, int) else [int(x) for x in new_lengths]
        if len(vals) != B:
            raise ValueError("one length per sequence")
        arr = (C.c_int32 * B)(*vals)
        _check(self.lib.rkv_cache_truncate(self.handle, arr, _stream()), "rkv_cache_truncate")

    def quantize_append_ragged(self, k, v, n_new, sink_mask=None):
        """rkv_quantize_append_ragged: k, v [batch, n_new_max, n_kv_heads, 128] fp16; n_new: ints per sequence."""
        import torch
        k = _dev(k, torch.float16, "k")
        v = _dev(v, torch.float16, "v")
        sink_mask = _dev(sink_mask, torch.uint8, "sink_mask")
        B, n_max = k.shape[0], k.shape[1]
        if k.shape != (B, n_max, self.cfg.n_kv_heads, self.cfg.head_dim) or v.shape != k.shape or B != self.cfg.batch:
            raise ValueError("k, v must be [batch, n_new_max, n_kv_heads, head_dim]")
        if sink_mask is not None and sink_mask.shape != (B, n_max):
            raise ValueError("sink_mask must be [batch, n_new_max]")
        if len(n_new) != B:
            raise ValueError("n_new must hold one count per sequence")
        arr = (C.c_int32 * B)(*[int(x) for x in n_new])
        _check(self.lib.rkv_quantize_append_ragged(self.handle, _ptr(k), _ptr(v), n_max, arr, _ptr(sink_mask), _stream()),
               "rkv_quantize_append_ragged")

    def decode_attention(self, q, q_pos=None, out=None, lse=None, want_lse=False, k_cur=None, v_cur=None):
        import torch
        q = _dev(q, torch.float16, "q")
        q_pos = _dev(q_pos, torch.int32, "q_pos")
        k_cur = _dev(k_cur, torch.float16, "k_cur")
        v_cur = _dev(v_cur, torch.float16, "v_cur")
        cfg = self.cfg
        if (k_cur is None) != (v_cur is None):
            raise ValueError("k_cur and v_cur go together")
        if k_cur is not None and (k_cur.shape != (cfg.batch, cfg.n_kv_heads, cfg.head_dim) or v_cur.shape != k_cur.shape):
            raise ValueError("k_cur, v_cur must be [batch, n_kv_heads, head_dim]")
        if q.shape != (cfg.batch, cfg.n_q_heads, cfg.head_dim):
            raise ValueError("q must be [batch, n_q_heads, head_dim]")
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        if lse is None and want_lse:
            lse = torch.empty(q.shape[:2], dtype=torch.float32, device=q.device)
        if k_cur is not None:
            _check(self.lib.rkv_decode_attention_with_current(self.handle, _ptr(q), _ptr(q_pos), _ptr(k_cur), _ptr(v_cur), _ptr(out),
                                                              _ptr(lse), _ptr(self.scratch), _stream()),
                   "rkv_decode_attention_with_current")
            return (out, lse) if want_lse else out
        _check(self.lib.rkv_decode_attention(self.handle, _ptr(q), _ptr(q_pos), _ptr(out), _ptr(lse),
                                             _ptr(self.scratch), _stream()), "rkv_decode_attention")
        return (out, lse) if want_lse else out

    def decode_attention_static(self, q, out, q_pos=None, lse=None):
        """rkv_decode_attention_static: the library's built-in work space instead of a scratch
        tensor; the caller brings every buffer (out [batch, n_q_heads, 128] fp32, lse optional), so
        that neither this wrapper nor the library allocates."""
        import torch
        q = _dev(q, torch.float16, "q")
        q_pos = _dev(q_pos, torch.int32, "q_pos")
        out = _dev(out, torch.float32, "out")
        lse = _dev(lse, torch.float32, "lse")
        cfg = self.cfg
        if q.shape != (cfg.batch, cfg.n_q_heads, cfg.head_dim) or out.shape != q.shape:
            raise ValueError("q, out must be [batch, n_q_heads, head_dim]")
        if lse is not None and lse.shape != q.shape[:2]:
            raise ValueError("lse must be [batch, n_q_heads]")
        _check(self.lib.rkv_decode_attention_static(self.handle, _ptr(q), _ptr(q_pos), _ptr(out), _ptr(lse), _stream()),
               "rkv_decode_attention_static")
        return out

    def decode_step(self, k, v, q, q_pos=None, out=None, lse=None, want_lse=False):
        """rkv_decode_step: append one token per sequence (k, v [batch, 1, n_kv_heads, 128]) and attend."""
        import torch
        k = _dev(k, torch.float16, "k")
        v = _dev(v, torch.float16, "v")
        q = _dev(q, torch.float16, "q")
        q_pos = _dev(q_pos, torch.int32, "q_pos")
        cfg = self.cfg
        if k.shape != (cfg.batch, 1, cfg.n_kv_heads, cfg.head_dim) or v.shape != k.shape:
            raise ValueError("k, v must be [batch, 1, n_kv_heads, head_dim]")
        if q.shape != (cfg.batch, cfg.n_q_heads, cfg.head_dim):
            raise ValueError("q must be [batch, n_q_heads, head_dim]")
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        if lse is None and want_lse:
            lse = torch.empty(q.shape[:2], dtype=torch.float32, device=q.device)
        _check(self.lib.rkv_decode_step(self.handle, _ptr(k), _ptr(v), _ptr(q), _ptr(q_pos), _ptr(out), _ptr(lse),
                                        _ptr(self.scratch), _stream()), "rkv_decode_step")
        return (out, lse) if want_lse else out

    def decode_attention_multi(self, q, q_pos, want_lse=False):
        """rkv_decode_attention_multi: q [batch, n_queries, n_q_heads, 128] fp16, q_pos [batch, n_queries] int32."""
        import torch
        q = _dev(q, torch.float16, "q")
        q_pos = _dev(q_pos, torch.int32, "q_pos")
        cfg = self.cfg
        if q.dim() != 4 or q.shape[0] != cfg.batch or q.shape[2:] != (cfg.n_q_heads, cfg.head_dim):
            raise ValueError("q must be [batch, n_queries, n_q_heads, head_dim]")
        nq = q.shape[1]
        if q_pos is None or q_pos.shape != (cfg.batch, nq):
            raise ValueError("q_pos must be [batch, n_queries]")
        need = nq * self.scratch_bytes
        scratch = self.scratch
        if scratch.numel() < need:
            scratch = getattr(self, "_scratch_multi", None)
            if scratch is None or scratch.numel() < need:
                scratch = self._scratch_multi = torch.empty(need, dtype=torch.uint8, device=self.device)
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        lse = torch.empty(q.shape[:3], dtype=torch.float32, device=q.device) if want_lse else None
        _check(self.lib.rkv_decode_attention_multi(self.handle, _ptr(q), _ptr(q_pos), nq, _ptr(out), _ptr(lse), _ptr(scratch),
                                                   _stream()), "rkv_decode_attention_multi")
        return (out, lse) if want_lse else out

    def dequantize(self):
        import torch
        cfg = self.cfg
        shape = (cfg.batch, self.length, cfg.n_kv_heads, cfg.head_dim)
        k = torch.empty(shape, dtype=torch.float32, device=self.device)
        v = torch.empty(shape, dtype=torch.float32, device=self.device)
        _check(self.lib.rkv_dequantize(self.handle, _ptr(k), _ptr(v), _stream()), "rkv_dequantize")
        return k, v

    def export_codes(self):
        import torch
        cfg, T, dev = self.cfg, self.length, self.device
        kc = torch.empty((cfg.batch, T, cfg.E // (4 if cfg.bits == 2 else 2)), dtype=torch.uint8, device=dev)
        vc = torch.empty_like(kc)
        meta = [torch.empty((cfg.batch, T, cfg.E // cfg.quant_group), dtype=torch.float32, device=dev) for _ in range(4)]
        _check(self.lib.rkv_export_codes(self.handle, _ptr(kc), _ptr(meta[0]), _ptr(meta[1]), _ptr(vc), _ptr(meta[2]),
                                         _ptr(meta[3]), _stream()), "rkv_export_codes")
        return dict(k_codes=kc, k_scale=meta[0], k_zero=meta[1], v_codes=vc, v_scale=meta[2], v_zero=meta[3])

    def import_codes(self, k_codes, k_scale, k_zero, v_codes, v_scale, v_zero):
        import torch
        k_codes = _dev(k_codes, torch.uint8, "k_codes")
        v_codes = _dev(v_codes, torch.uint8, "v_codes")
        ms = [_dev(t, torch.float32, "meta") for t in (k_scale, k_zero, v_scale, v_zero)]
        _check(self.lib.rkv_import_codes(self.handle, k_codes.shape[1], _ptr(k_codes), _ptr(ms[0]), _ptr(ms[1]),
                                         _ptr(v_codes), _ptr(ms[2]), _ptr(ms[3]), _stream()), "rkv_import_codes")

    def export_sinks(self):
        import torch
        cfg, dev = self.cfg, self.device
        S = max(cfg.max_sinks, 1)
        cnt = torch.zeros(cfg.batch, dtype=torch.int32, device=dev)
        pos = torch.full((cfg.batch, S), -1, dtype=torch.int32, device=dev)
        k = torch.zeros((cfg.batch, S, cfg.E), dtype=torch.float16, device=dev)
        v = torch.zeros_like(k)
        _check(self.lib.rkv_export_sinks(self.handle, _ptr(cnt), _ptr(pos), _ptr(k), _ptr(v), _stream()),
               "rkv_export_sinks")
        return dict(count=cnt, pos=pos, k=k, v=v)
