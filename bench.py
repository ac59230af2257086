#!/usr/bin/env python3
"""Benchmark of the RotateKV hot path on one MI355X.

A step = one pass of the whole hot path over one batch: for every layer of the model shape,
append one new token per sequence (rkv_quantize_append) and run decode attention over the full
2-bit cache (rkv_decode_attention).  The workload is the LLaMA-2-13B-shaped configuration
(40 layers x 40 heads x 128, batch 16, context 4096) on synthetic keys/values with per-head
outlier channels and sink tokens.  All layers keep their own cache (7.5 GB in total), so a step
streams far more than the 256 MB of last-level cache.

Prints one JSON line: whole-job KV-tokens/s, the roofline of the dominant kernel (the
cache-streaming decode kernel, timed with HIP events on its own stream), and the CPU oracle timed
on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
SHAPES = {"cfg0": "single-layer toy", "cfg1": "LLaMA-2-7B-shaped", "cfg2": "LLaMA-2-13B-shaped", "cfg3": "long-context",
          "cfg4": "LLaMA-3-8B-shaped (GQA)"}


class Hip:
    """The few HIP runtime calls the benchmark needs for its own event timing."""

    def __init__(self):
        self.lib = ctypes.CDLL("libamdhip64.so")
        self.lib.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.lib.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def event(self):
        e = ctypes.c_void_p()
        rc = self.lib.hipEventCreate(ctypes.byref(e))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed: {rc}")
        return e

    def elapsed_ms(self, a, b) -> float:
        ms = ctypes.c_float()
        rc = self.lib.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return ms.value


def cpu_baseline(w, sample_batch: int, sample_tokens: int):
    """The oracle, as it stands, on a bounded sample of the same workload: one layer,
    `sample_batch` sequences of `sample_tokens` cached tokens; times one step (append one token,
    decode over the cache)."""
    import numpy as np
    import rkv_synth as S
    from oracle import rkv_oracle as O

    cfg = O.OracleConfig(batch=sample_batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, rot_heads=w.rot_heads,
                         perm_span=128, rope_theta=w.rope_theta, max_sinks=w.n_sinks)
    kc, _, _ = S.make_kv(w, 256, batch=1, stream=1, sink_positions=[])
    perm = O.calibrate_perm(kc[0], cfg)
    k, v, mask = S.make_kv(w, sample_tokens - 1, batch=sample_batch)
    k1, v1, _ = S.make_kv(w, 1, batch=sample_batch, stream=2, sink_positions=[])
    q = S.make_q(w, batch=sample_batch)
    cache = O.cache_new(cfg, perm)
    t0 = time.perf_counter()
    O.quantize_append(cache, k, v, mask)
    t_prefill = time.perf_counter() - t0
    t0 = time.perf_counter()
    O.quantize_append(cache, k1, v1)
    O.decode_attention(cache, q)
    t_step = time.perf_counter() - t0
    cores = len(os.sched_getaffinity(0))
    return {
        "value": sample_batch * sample_tokens / t_step, "unit": "KV-tokens/s", "cores": cores, "kind": "oracle",
        "sample": f"1 layer, {sample_batch} sequences x {sample_tokens} tokens of the same head geometry; one append+decode step "
                  f"took {t_step:.2f} s (numpy float64, dense Hadamard products; BLAS may use all {cores} cores)",
        "bulk_quantize_kv_tokens_per_s": sample_batch * (sample_tokens - 1) / t_prefill,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (0 = the workload's)")
    ap.add_argument("--path", type=int, default=0, help="decode kernel: 0 auto, 1 general, 2 matrix-core")
    ap.add_argument("--queries", type=int, default=1,
                    help="query tokens per sequence and step (above 1: that many tokens are appended, then read the cache in one multi-query call)")
    ap.add_argument("--meta-format", type=int, default=0, help="0: fp16 scale and zero-point (2.25 bits); 1: FP8 scale, INT8 zero-point (2.125 bits)")
    ap.add_argument("--bits", type=int, default=2, help="bits per code: 2, 3 or 4")
    ap.add_argument("--quant-group", type=int, default=128, help="channels per quantization block: 128, or 64 / 32 (Table tab:quantgrani; sub-group variants of the matrix-core kernels with 2-bit codes and fp16 metadata, the general kernels otherwise)")
    ap.add_argument("--perm-span", type=int, default=128,
                    help="channels the reorder may move a channel within: 128 (a head), rot_heads*128 (a rotation group) or n_kv_heads*128 (the row, Alg. 1 as printed)")
    ap.add_argument("--ragged-min", type=float, default=1.0,
                    help="below 1: sequence lengths spread evenly from this fraction of the context up to the full context")
    ap.add_argument("--separate-calls", action="store_true",
                    help="make a step of rkv_quantize_append + rkv_decode_attention instead of the one-call rkv_decode_step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=4096)
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (reference for HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2501_16383_amd as R
    import rkv_synth as S

    if not os.path.exists(R.library_path()):
        from paper_2501_16383_amd.build import build_library
        build_library()
    w = S.WORKLOADS[args.workload]
    L = args.layers or w.layers
    B, T = w.batch, w.context
    K, W, NQ = args.steps, args.warmup, args.queries
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    hip = Hip()

    cfg = R.RkvConfig(batch=B, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, max_tokens=T, max_sinks=max(w.n_sinks, 1),
                      rot_heads=w.rot_heads, perm_span=args.perm_span, rope_theta=w.rope_theta, meta_format=args.meta_format,
                      bits=args.bits, quant_group=args.quant_group)
    QB, QG = args.bits, args.quant_group
    MB = 2 if args.meta_format == 1 else 4       # bytes of metadata per (token, quantization block)
    E = cfg.E
    _, scratch_bytes = R.query_sizes(cfg)
    scratch = torch.empty(scratch_bytes * NQ, dtype=torch.uint8, device=dev)

    # ---- build the L caches: calibrate the reorder, then bulk-quantize T-1-W tokens (timed: append GB/s)
    caches, bulk_ms = [], []
    n_pre = T - (K + W) * NQ   # the last timed step decodes over exactly T tokens
    e0, e1 = hip.event(), hip.event()
    pre_lens = None
    if args.ragged_min < 1.0:      # sequence b ends the run with final_lens[b] tokens
        final_lens = [int(round(T * (args.ragged_min + (1.0 - args.ragged_min) * b / max(B - 1, 1)))) for b in range(B)]
        pre_lens = [max(fl - (K + W) * NQ, 1) for fl in final_lens]
    for l in range(L):
        c = R.RkvCache(cfg, device=dev, scratch=scratch)
        kcal, _, _ = S.make_kv_torch(w, 256, dev, batch=1, layer=l, stream=1)
        c.set_perm(R.calibrate_perm(cfg, kcal[0].contiguous()))
        k, v, mask = S.make_kv_torch(w, n_pre, dev, layer=l)
        c.set_profile_events(e0, e1)
        if pre_lens is None:
            c.quantize_append(k, v, mask)
        else:
            c.quantize_append_ragged(k, v, pre_lens, mask)
        torch.cuda.synchronize()
        bulk_ms.append(hip.elapsed_ms(e0, e1))
        c.set_profile_events(None, None)
        c.set_decode_path(args.path)
        caches.append(c)
        del k, v, mask
    n_bulk = B * n_pre if pre_lens is None else sum(pre_lens)
    bulk_bytes = n_bulk * (2 * E * 2 + 2 * E * QB // 8 + 2 * (E // QG) * MB)
    bulk_best = min(bulk_ms)
    bulk_avg = sum(bulk_ms) / len(bulk_ms)
    bulk_med = sorted(bulk_ms)[len(bulk_ms) // 2]

    # ---- per-step inputs, resident before the timed region
    n_total = K + W
    new_k = [S.make_kv_torch(w, n_total * NQ, dev, layer=l, stream=2) for l in range(L)]
    qs = [torch.stack([S.make_q_torch(w, dev, layer=l, step=s) for s in range(n_total * NQ)]) for l in range(L)]
    outs = [torch.empty((B, w.n_q_heads, 128), dtype=torch.float32, device=dev) for _ in range(L)]
    step_k = [[new_k[l][0][:, s * NQ:(s + 1) * NQ].contiguous() for s in range(n_total)] for l in range(L)]
    step_v = [[new_k[l][1][:, s * NQ:(s + 1) * NQ].contiguous() for s in range(n_total)] for l in range(L)]
    if NQ == 1:
        step_q = [[qs[l][s].contiguous() for s in range(n_total)] for l in range(L)]
    else:   # [B, NQ, Hq, 128] per step, positions = the NQ tokens just appended
        step_q = [[qs[l][s * NQ:(s + 1) * NQ].transpose(0, 1).contiguous() for s in range(n_total)] for l in range(L)]
        step_pos = [(torch.arange(NQ, dtype=torch.int32, device=dev) + (n_pre + s * NQ)).repeat(B, 1).contiguous()
                    for s in range(n_total)]

    def decode(c, l, s):
        if NQ == 1:
            c.decode_attention(step_q[l][s], out=outs[l])
        else:
            outs[l] = c.decode_attention_multi(step_q[l][s], step_pos[s])

    one_call = NQ == 1 and not args.separate_calls     # rkv_decode_step: append + attend in one library call

    def one_step(s):
        for l in range(L):
            if one_call:
                caches[l].decode_step(step_k[l][s], step_v[l][s], step_q[l][s], out=outs[l])
            else:
                caches[l].quantize_append(step_k[l][s], step_v[l][s])
                decode(caches[l], l, s)

    def decode_only_events(s, events):
        for l in range(L):
            c = caches[l]
            if one_call:                                   # the events bracket the cache-streaming kernel only
                c.set_profile_events(*events[l])
                c.decode_step(step_k[l][s], step_v[l][s], step_q[l][s], out=outs[l])
                c.set_profile_events(None, None)
                continue
            c.set_profile_events(None, None)
            c.quantize_append(step_k[l][s], step_v[l][s])
            c.set_profile_events(*events[l])
            decode(c, l, s)
            c.set_profile_events(None, None)

    if args.calib_copy_mib > 0:
        src = torch.empty(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                      # reads and writes calib_copy_mib MiB each
        torch.cuda.synchronize()
        del src, dst

    for s in range(W):
        one_step(s)
    torch.cuda.synchronize()
    # which kernels this configuration takes (RKV_KERNEL_* of the library)
    KIND_NAMES = {1: "general", 2: "shuffle", 3: "matrix-core", 4: "matrix-core, cross-block variant", 5: "matrix-core, sub-group variant",
                  6: "matrix-core, whole-row variant"}
    kinds = (caches[0].decode_kernel(NQ if NQ > 1 else 0), caches[0].append_kernel())
    assert caches[0].length == T - K * NQ
    lens_now = caches[0].lengths

    # timed region: exactly K steps, whole-job wall clock; the decode kernel of every launch is
    # bracketed by its own pair of HIP events (recorded by the library on the launch stream)
    ev = [[(hip.event(), hip.event()) for _ in range(L)] for _ in range(K)]
    kv_tokens = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(K):
        decode_only_events(W + s, ev[s])
        lens_now = [x + NQ for x in lens_now]
        kv_tokens += sum(lens_now) * L
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = [hip.elapsed_ms(a, b) for step in ev for (a, b) in step]
    avg_ms = sum(kern_ms) / len(kern_ms)
    min_ms = min(kern_ms)
    med_ms = sorted(kern_ms)[len(kern_ms) // 2]
    ctx = T - (K - 1) * NQ / 2.0
    bytes_per_tok = 2 * E * QB // 8 + 2 * (E // QG) * MB
    launch_bytes = (sum(lens_now) - B * (K - 1) * NQ / 2.0) * bytes_per_tok      # mean over the timed steps
    achieved = launch_bytes / (avg_ms * 1e-3) / 1e9

    # measured HBM traffic of the decode kernel (rocprofv3 counters, calibrated; see profiles/)
    # The counters are not read in this run: the figure is quoted from the tracked profile, and only if
    # that profile was taken on the kernel sources that are in the tree now (their hash is in the file).
    traffic = None
    traffic_source = None
    tfile = os.path.join(ROOT, "profiles", f"decode_{w.name}_hbm_traffic.md")
    default_run = (QB, QG, args.meta_format, NQ, args.path, args.perm_span) == (2, 128, 0, 1, 0, 128) and pre_lens is None   # what the counters were collected on
    if os.path.exists(tfile) and L == w.layers and default_run:
        from paper_2501_16383_amd.build import source_hash
        quoted, taken_at = None, None
        for line in open(tfile):
            if line.startswith("traffic_bytes_per_launch:"):
                quoted = float(line.split(":")[1])
            if line.startswith("csrc_sha256:"):
                taken_at = line.split(":")[1].strip()
        now = source_hash()
        traffic_source = {"file": os.path.relpath(tfile, ROOT), "csrc_sha256_of_profile": taken_at, "csrc_sha256_now": now,
                          "match": taken_at == now}
        if quoted is not None and taken_at == now:
            traffic = quoted

    # sanity: finite outputs
    assert args.path == 3 or all(bool(torch.isfinite(o).all()) for o in outs)

    # the arithmetic-only ceiling of the decode kernel: the same launches with the cache stream replaced
    # by register values (rkv_set_decode_path 3), timed with the same events; plain configurations only
    alu_only_ms = None
    if default_run and args.path == 0 and w.n_q_heads == w.n_kv_heads:      # (one query head per KV head: the variant the measurement exists for)
        tmp = torch.empty_like(outs[0])
        reps = 3
        ev_a = [[(hip.event(), hip.event()) for _ in range(L)] for _ in range(reps)]
        for c in caches:
            c.set_decode_path(3)
        for rep_ in range(reps):                             # back to back, as in the timed region
            for l in range(L):
                c = caches[l]
                c.set_profile_events(*ev_a[rep_][l])
                c.decode_attention(step_q[l][-1], out=tmp)
                c.set_profile_events(None, None)
        torch.cuda.synchronize()
        for c in caches:
            c.set_decode_path(0)
        alu = [hip.elapsed_ms(a, b) for row in ev_a[1:] for (a, b) in row]
        alu_only_ms = sum(alu) / len(alu)

    result = {
        "metric": f"{QB}-bit decode-attention KV-tokens/s (one appended token per sequence plus decode attention over the full cache, per layer)"
                  if NQ == 1 else f"{QB}-bit decode-attention KV-tokens/s ({NQ} appended tokens per sequence, then {NQ} causal queries over the full cache in one call, per layer)",
        "value": kv_tokens / wall,
        "unit": "KV-tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": wall / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",   # what the path accumulates in; storage is u2 codes + fp16 scale/zero, the rotations are exact fp4 / fp16 matrix products
        "data": "synthetic",
        "config": {"workload": f"{w.name}: {SHAPES.get(w.name, 'custom')} decode, {L} layers x {w.n_q_heads} query / {w.n_kv_heads} KV heads x 128, "
                               f"batch {B}, context {T}, rotation over {w.rot_heads} heads, reorder within {args.perm_span} channels, {QB}-bit group-{QG}, {w.n_sinks} fp16 sinks",
                   "decode_path": args.path, "queries_per_step": NQ, "calls_per_step_and_layer": 1 if one_call else 2,
                   "sequence_lengths": "all equal" if pre_lens is None else f"spread evenly from {lens_now[0]} to {lens_now[-1]} tokens",
                   "storage": f"u{QB} codes + " + ("fp16 scale / fp16 zero" if MB == 4 else "FP8 E4M3 scale / INT8 zero") +
                              f" per {QG} ({QB + 8.0 * MB / QG:g} bits per element)",
                   "arithmetic": "fp4 and fp16 matrix products (exact), fp32 vector arithmetic and accumulation"
                                 if kinds[0] != 1 else "fp32 vector arithmetic and accumulation (general kernel)",
                   "decode_kernel": KIND_NAMES.get(kinds[0], str(kinds[0])), "append_kernel": KIND_NAMES.get(kinds[1], str(kinds[1]))},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_source, "kernel": "decode (cache-streaming) kernel", "avg_launch_ms": avg_ms, "median_launch_ms": med_ms, "min_launch_ms": min_ms, "launches_timed": len(kern_ms),
                     "algorithmic_bytes_per_launch": launch_bytes, "bytes_per_kv_token": bytes_per_tok,
                     "alu_only_ms": alu_only_ms},
        "append_bulk": {"GB/s_best": bulk_bytes / (bulk_best * 1e-3) / 1e9, "GB/s_avg": bulk_bytes / (bulk_avg * 1e-3) / 1e9,
                        "GB/s_median": bulk_bytes / (bulk_med * 1e-3) / 1e9, "calls": len(bulk_ms),
                        "frac_of_hbm_peak_best": bulk_bytes / (bulk_best * 1e-3) / 1e9 / HBM_PEAK_GBS,
                        "kv_tokens_per_s_best": n_bulk / (bulk_best * 1e-3), "tokens_per_call": n_bulk,
                        "bytes_per_kv_token": 2 * E * 2 + bytes_per_tok},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, 2, args.cpu_sample_tokens)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
