#!/usr/bin/env python3
"""Benchmark of the turn-resumption hot path on one MI355X.

One step = one pass over one synthetic batch, inputs resident in HBM:
    symph_kv_pack (all layers, every session)  ->  symph_kv_unpack (into fresh free-list blocks)
    ->  symph_prefix_prefill_attn (one layer, ragged batch).
Host staging (device <-> pinned host on a side stream) is PCIe-bound and is timed on its own, outside the step.

Prints ONE JSON line.  `value` is the step's algorithmic HBM traffic divided by the step time; the per-kernel
figures (GB/s against the 8 TB/s HBM peak for pack / unpack, TFLOP/s against the 2.5 PFLOP/s dense bf16 MFMA peak
for attention) are carried next to it, each measured with events on the launch stream inside the timed region.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and scaled by the readings of the plain
# copy kernel of known size (profiles/bench_llama8b_hbm_traffic.md); other workloads have not been measured.
MEASURED_TRAFFIC_BYTES = {"llama8b": {"kv_migrate": 17.22e9, "attn": 3.92e8}}

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="llama8b", help="workload name (default: the config the metric is quoted on)")
    ap.add_argument("--only", choices=("all", "attn", "resume", "pipeline", "decode"), default="all",
                    help="attn: time symph_prefix_prefill_attn alone on a one-layer cache (per-kernel profiles); "
                         "resume: the mixed-resume workload, attention on one stream beside the unpack of arriving "
                         "sessions on a second stream (alone, alone, both); pipeline: a resume whose buffer sits in "
                         "pinned host memory, one shot against layer by layer on three streams")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-staging", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="rough budget of the CPU-baseline leg")
    return ap.parse_args()


def _cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, sess, budget_s: float):
    """Time the oracle, as it stands, on a bounded sample of the same workload on the host cores."""
    import oracle
    import workloads as W
    oracle.build()
    threads = oracle.num_threads()
    # migration sample: same shapes and length recipe, fewer layers and sessions, small pool
    mcfg = W.scaled_config(cfg, n_layers=min(cfg.n_layers, 4), n_sessions=min(cfg.n_sessions, 4), n_blocks=4096)
    msess = W.make_sessions(mcfg)
    shape = (mcfg.n_layers, mcfg.n_blocks, mcfg.block_size, mcfg.n_kv_heads, mcfg.head_dim)
    dt = np.uint16 if cfg.dtype == "bf16" else np.float32
    kp = np.arange(int(np.prod(shape)), dtype=np.uint32).astype(dt).reshape(shape)
    vp = kp[::-1].copy()
    t0 = time.perf_counter()
    buf = oracle.kv_pack(kp, vp, msess.block_table, msess.prefix_lens, msess.buf_token_offsets)
    t1 = time.perf_counter()
    oracle.kv_unpack(kp, vp, msess.dst_block_table, msess.prefix_lens, msess.buf_token_offsets, buf)
    t2 = time.perf_counter()
    mig_bytes = 2.0 * msess.payload_bytes()          # read + write
    pack_gbs = mig_bytes / (t1 - t0) / 1e9
    unpack_gbs = mig_bytes / (t2 - t1) / 1e9
    # attention sample: rows of the real batch, sized from a probe so the leg stays near the budget
    inputs = W.make_attn_inputs(cfg, sess)
    rng = np.random.default_rng(0)
    T = sess.total_new_tokens
    order = rng.permutation(T)
    keys_per_tok = np.repeat(sess.prefix_lens.astype(np.float64), sess.new_lens) + \
        np.concatenate([np.arange(1, n + 1) for n in sess.new_lens]).astype(np.float64)
    flops_tok = 4.0 * cfg.n_q_heads * cfg.head_dim * keys_per_tok
    probe = order[:4]
    t0 = time.perf_counter()
    oracle.prefix_prefill_attn(*inputs, sess.cu_new_lens, sess.prefix_lens, sess.block_table, cfg.scale,
                               token_subset=probe)
    rate = flops_tok[probe].sum() / (time.perf_counter() - t0)
    n_rows = int(np.clip(budget_s * 0.7 * rate / max(flops_tok.mean(), 1.0), 8, T))
    rows = order[:n_rows]
    t0 = time.perf_counter()
    oracle.prefix_prefill_attn(*inputs, sess.cu_new_lens, sess.prefix_lens, sess.block_table, cfg.scale,
                               token_subset=rows)
    attn_s = time.perf_counter() - t0
    attn_gflops = flops_tok[rows].sum() / attn_s / 1e9
    # the whole step on the CPU, extrapolated from the three sampled rates, in the unit of `value`
    full_mig = 2.0 * sess.payload_bytes()
    step_s = full_mig / (pack_gbs * 1e9) + full_mig / (unpack_gbs * 1e9) + sess.attn_flops() / (attn_gflops * 1e9)
    step_bytes = 2.0 * full_mig + sess.attn_bytes()
    return {
        "value": step_bytes / step_s / 1e9, "unit": "GB/s", "cores": threads, "cpu_model": _cpu_model(), "kind": "oracle",
        "sample": (f"pack+unpack of {msess.n_sessions} sessions x {mcfg.n_layers} layers "
                   f"({msess.payload_bytes() / 1e6:.0f} MB payload, same shapes and length recipe); attention on "
                   f"{n_rows} of {T} query tokens of the real batch (all heads); step extrapolated from the three rates"),
        "pack_GBps": pack_gbs, "unpack_GBps": unpack_gbs, "attn_fp64_GFLOPs": attn_gflops,
        "extrapolated_step_ms": step_s * 1e3,
    }


def attn_only(args, cfg, sess):
    """symph_prefix_prefill_attn alone on the workload's attention batch (one-layer cache): one JSON line."""
    import torch
    import paper_2412_16434_amd as S
    import workloads as W
    dev = "cuda:0"
    kh, vh, qh, knh, vnh = W.make_attn_inputs(cfg, sess)
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    cache = S.KVCache(to_dev(kh)[None], to_dev(vh)[None])
    q, k_new, v_new = to_dev(qh), to_dev(knh), to_dev(vnh)
    out = torch.empty_like(q)
    table = torch.from_numpy(sess.block_table).to(dev)
    prefix_lens = torch.from_numpy(sess.prefix_lens).to(dev)
    cu = torch.from_numpy(sess.cu_new_lens).to(dev)
    ws_bytes = S.prefix_prefill_attn_workspace_bytes(cache, sess.n_sessions, cfg.n_q_heads, sess.total_new_tokens,
                                                     sess.max_new_len, sess.max_prefix_len)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)

    def call():
        S.prefix_prefill_attn(cache, 0, q, k_new, v_new, out, cu, prefix_lens, table, sess.max_new_len,
                              sess.max_prefix_len, cfg.scale, workspace=ws if ws_bytes else None)
    for _ in range(args.warmup):
        call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        call()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms = e0.elapsed_time(e1) / args.steps
    tflops = sess.attn_flops() / ms / 1e9
    print(json.dumps({
        "metric": "prefix-prefill attn TFLOP/s", "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall_ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "n_sessions": sess.n_sessions, "new_tokens": sess.total_new_tokens,
                   "prefix_tokens": sess.total_prefix_tokens, "step": "prefix_prefill_attn(one layer)"},
        "prefix_prefill_attn": {"ms": ms, "TFLOPs": tflops, "pct_mfma_bf16_peak": 100 * tflops / MFMA_BF16_PEAK_TFLOPS,
                                "kv_GBps": sess.attn_bytes() / ms / 1e6, "flops": sess.attn_flops()},
        "roofline": {"kernel": "attn_mfma", "bound": "mfma", "achieved": tflops, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": tflops / MFMA_BF16_PEAK_TFLOPS, "traffic": None}}))


def decode_step(args):
    """A decode step: the 96 one-token rows of workload 5 (prefixes uniform in [512, 16384]) as a batch of their own.
    Such a batch is HBM-bound (every K,V byte is used for G = 4 query rows), so the figure is K,V bytes per second
    against the 8 TB/s peak; timed through the decode kernel (the default for such batches) and, with the switch off,
    through the work-item kernel that mixed batches use."""
    import torch
    import paper_2412_16434_amd as S
    import workloads as W
    dev = "cuda:0"
    cfg = W.get_config("mixed_resume")
    sess = W.make_sessions(cfg)
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    kh, vh, qh, knh, vnh = W.make_attn_inputs(cfg, sess)
    cache = S.KVCache(to_dev(kh)[None], to_dev(vh)[None])
    new_lens = np.diff(sess.cu_new_lens)
    idx = np.nonzero(new_lens == 1)[0]
    rows = sess.cu_new_lens[:-1][idx]                      # the one query row of each such session
    q, k_new, v_new = (to_dev(np.ascontiguousarray(a[rows])) for a in (qh, knh, vnh))
    out = torch.empty_like(q)
    n = len(idx)
    prefix_h = np.ascontiguousarray(sess.prefix_lens[idx])
    prefix = torch.from_numpy(prefix_h).to(dev)
    table = torch.from_numpy(np.ascontiguousarray(sess.block_table[idx])).to(dev)
    cu = torch.arange(0, n + 1, dtype=torch.int32, device=dev)
    max_prefix = int(prefix_h.max())
    ws_bytes = S.prefix_prefill_attn_workspace_bytes(cache, n, cfg.n_q_heads, n, 1, max_prefix)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    kv_bytes = float(prefix_h.sum() + n) * 2 * cfg.n_kv_heads * cfg.head_dim * 2

    def timed(tuning):
        call = lambda: S.prefix_prefill_attn(cache, 0, q, k_new, v_new, out, cu, prefix, table, 1, max_prefix, cfg.scale,
                                             workspace=ws, tuning=tuning)
        for _ in range(max(args.warmup, 2)):
            call()
        ts = []
        for _ in range(args.steps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            call()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return float(np.median(ts)), out.clone()

    dec_ms, dec_out = timed(None)
    main_ms, main_out = timed(S.AttnTuning(decode=-1))   # (needs no more workspace than the default plan)
    diff = float((dec_out.float() - main_out.float()).abs().max())
    gbs = kv_bytes / dec_ms / 1e6
    print(json.dumps({
        "metric": "decode step: K,V GB/s of prefix-prefill attention on one-token rows, as % of HBM peak",
        "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dec_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "mixed_resume, its 96 one-token rows as a batch", "n_sessions": n,
                   "prefix_tokens": int(prefix_h.sum()), "kv_bytes": kv_bytes},
        "decode_kernel": {"ms": dec_ms, "kv_GBps": gbs, "pct_hbm_peak": 100 * gbs / HBM_PEAK_GBS},
        "work_item_kernel": {"ms": main_ms, "kv_GBps": kv_bytes / main_ms / 1e6,
                             "pct_hbm_peak": 100 * kv_bytes / main_ms / 1e6 / HBM_PEAK_GBS},
        "max_abs_difference_between_the_two": diff,
        "roofline": {"kernel": "attn_decode", "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbs / HBM_PEAK_GBS, "traffic": None}}))


def resume_mix(args):
    """Mixed resume (config 5): a batch of resumed turns (96 decode-shaped rows, 32 prefill turns) runs attention while
    the K,V of 8 arriving sessions (32 layers, 4096 tokens each) are unpacked into another cache on a second stream.
    Times attention alone, the unpack alone, and both released together: one JSON line."""
    import torch
    import paper_2412_16434_amd as S
    import workloads as W
    dev = "cuda:0"
    acfg, ucfg = W.get_config("mixed_resume"), W.get_config("mixed_resume_incoming")
    asess, usess = W.make_sessions(acfg), W.make_sessions(ucfg)
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    kh, vh, qh, knh, vnh = W.make_attn_inputs(acfg, asess)
    acache = S.KVCache(to_dev(kh)[None], to_dev(vh)[None])
    q, k_new, v_new = to_dev(qh), to_dev(knh), to_dev(vnh)
    out = torch.empty_like(q)
    atable = torch.from_numpy(asess.block_table).to(dev)
    aprefix = torch.from_numpy(asess.prefix_lens).to(dev)
    cu = torch.from_numpy(asess.cu_new_lens).to(dev)
    ws_bytes = S.prefix_prefill_attn_workspace_bytes(acache, asess.n_sessions, acfg.n_q_heads, asess.total_new_tokens,
                                                     asess.max_new_len, asess.max_prefix_len)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    ushape = (ucfg.n_layers, ucfg.n_blocks, ucfg.block_size, ucfg.n_kv_heads, ucfg.head_dim)
    uk = torch.zeros(ushape, dtype=torch.bfloat16, device=dev)
    uv = torch.zeros(ushape, dtype=torch.bfloat16, device=dev)
    ucache = S.KVCache(uk, uv)
    utable = torch.from_numpy(usess.dst_block_table).to(dev)
    uprefix = torch.from_numpy(usess.prefix_lens).to(dev)
    uoff = torch.from_numpy(usess.buf_token_offsets).to(dev)
    payload = S.kv_buffer_bytes(ucache, usess.total_prefix_tokens)
    buf = torch.empty(payload // 2, dtype=torch.bfloat16, device=dev)
    buf.view(torch.int16).fill_(0x3C00)
    sa, su = torch.cuda.Stream(), torch.cuda.Stream()

    def attn():
        S.prefix_prefill_attn(acache, 0, q, k_new, v_new, out, cu, aprefix, atable, asess.max_new_len,
                              asess.max_prefix_len, acfg.scale, workspace=ws if ws_bytes else None, stream=sa)

    def unpack():
        S.kv_unpack(ucache, utable, uprefix, uoff, usess.total_prefix_tokens, buf, stream=su)

    def timed(fns):
        for f in fns:
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            for f in fns:
                f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    for _ in range(args.warmup):
        attn(); unpack()
    torch.cuda.synchronize()
    attn_ms, unpack_ms, both_ms = timed([attn]), timed([unpack]), timed([attn, unpack])
    tflops = asess.attn_flops() / attn_ms / 1e9
    print(json.dumps({
        "metric": "mixed resume: prefix-prefill attn beside kv_unpack on a second stream", "value": both_ms, "unit": "ms",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": both_ms, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "mixed_resume + mixed_resume_incoming", "attn_sessions": asess.n_sessions,
                   "attn_new_tokens": asess.total_new_tokens, "attn_prefix_tokens": asess.total_prefix_tokens,
                   "unpack_sessions": usess.n_sessions, "unpack_payload_bytes": payload},
        "attn_alone": {"ms": attn_ms, "TFLOPs": tflops, "pct_mfma_bf16_peak": 100 * tflops / MFMA_BF16_PEAK_TFLOPS,
                       "kv_GBps": asess.attn_bytes() / attn_ms / 1e6},
        "unpack_alone": {"ms": unpack_ms, "GBps": 2.0 * payload / unpack_ms / 1e6,
                         "pct_hbm_peak": 100 * 2.0 * payload / unpack_ms / 1e6 / HBM_PEAK_GBS},
        "both": {"ms": both_ms, "sum_of_alone_ms": attn_ms + unpack_ms, "max_of_alone_ms": max(attn_ms, unpack_ms)}}))


def pipelined_resume(args, cfg, sess):
    """A batch of turns resumes on this GPU while its K,V still sit in pinned host memory (Sec. 3.3).  One shot:
    host->device of the whole buffer, unpack of all layers, attention layer after layer.  Layer-wise: copy of layer
    l+1 (side stream), unpack of layer l (second stream) and attention on layer l-1 (third stream) overlap, each
    released by the event of the step before.  Reference points: the copy alone (PCIe) and the attention of all
    layers with K,V already in place.  One JSON line."""
    import torch
    import paper_2412_16434_amd as S
    import workloads as W
    dev = "cuda:0"
    L, nb, bs = cfg.n_layers, cfg.n_blocks, cfg.block_size
    k_pool = torch.zeros((L, nb, bs, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device=dev)
    v_pool = torch.zeros_like(k_pool)
    cache = S.KVCache(k_pool, v_pool)
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    _, _, qh, knh, vnh = W.make_attn_inputs(cfg, sess)
    q, k_new, v_new = to_dev(qh), to_dev(knh), to_dev(vnh)
    out = torch.empty_like(q)
    dst_table = torch.from_numpy(sess.dst_block_table).to(dev)
    prefix_lens = torch.from_numpy(sess.prefix_lens).to(dev)
    offsets = torch.from_numpy(sess.buf_token_offsets).to(dev)
    cu = torch.from_numpy(sess.cu_new_lens).to(dev)
    h_prefix, h_off = torch.from_numpy(sess.prefix_lens), torch.from_numpy(sess.buf_token_offsets)
    total = sess.total_prefix_tokens
    payload = S.kv_buffer_bytes(cache, total)
    host = torch.empty(payload // 2, dtype=torch.int16, pin_memory=True)
    host.fill_(0x3C00)
    dbuf = torch.empty(payload // 2, dtype=torch.int16, device=dev)
    ws_bytes = S.prefix_prefill_attn_workspace_bytes(cache, sess.n_sessions, cfg.n_q_heads, sess.total_new_tokens,
                                                     sess.max_new_len, sess.max_prefix_len)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    s_copy, s_unpack, s_attn = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    ev = torch.cuda.Event()
    ev_copy = [torch.cuda.Event() for _ in range(L)]
    ev_unpack = [torch.cuda.Event() for _ in range(L)]

    def attn(l, stream):
        S.prefix_prefill_attn(cache, l, q, k_new, v_new, out, cu, prefix_lens, dst_table, sess.max_new_len,
                              sess.max_prefix_len, cfg.scale, workspace=ws if ws_bytes else None, stream=stream)

    def copy_only():
        S.stage_to_device(dbuf, host, payload, s_unpack, s_copy, ev)

    def attn_only_all_layers():
        for l in range(L):
            attn(l, s_attn)

    def one_shot():
        S.stage_to_device(dbuf, host, payload, s_unpack, s_copy, ev)
        S.kv_unpack(cache, dst_table, prefix_lens, offsets, total, dbuf, stream=s_unpack)
        ev_unpack[0].record(s_unpack)
        s_attn.wait_event(ev_unpack[0])
        for l in range(L):
            attn(l, s_attn)

    def layer_wise():
        for l in range(L):
            S.stage_layer_to_device(dbuf, host, cache, l, h_prefix, h_off, s_unpack, s_copy, ev_copy[l])
            S.kv_unpack_layers(cache, l, l + 1, dst_table, prefix_lens, offsets, total, dbuf, stream=s_unpack)
            ev_unpack[l].record(s_unpack)
            s_attn.wait_event(ev_unpack[l])
            attn(l, s_attn)

    # The buffer argument of unpack / pack may itself be pinned host memory when the runtime maps it for the device at
    # the same address (checked here): the kernel then reads it over PCIe and no staging buffer in HBM is needed.
    import ctypes
    mapped = ctypes.c_void_p(0)
    rc = ctypes.CDLL("libamdhip64.so").hipHostGetDevicePointer(ctypes.byref(mapped), ctypes.c_void_p(host.data_ptr()), 0)
    host_is_mapped = rc == 0 and mapped.value == host.data_ptr()
    host_bf16 = host.view(torch.bfloat16)

    def layer_wise_direct():
        for l in range(L):
            S.kv_unpack_layers(cache, l, l + 1, dst_table, prefix_lens, offsets, total, host_bf16, stream=s_unpack)
            ev_unpack[l].record(s_unpack)
            s_attn.wait_event(ev_unpack[l])
            attn(l, s_attn)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(max(args.steps // 4, 3)):
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append((time.perf_counter() - t0) * 1e3)
        return float(np.median(ts))

    copy_ms, attn_ms = timed(copy_only), timed(attn_only_all_layers)
    shot_ms, wise_ms = timed(one_shot), timed(layer_wise)

    # ---- the other direction (Sec. 3.3: layer-wise asynchronous writes): K,V of the batch go to pinned host memory.
    # Whole sessions in one shot (pack, then one copy) and layer by layer (pack of layer l+1 overlaps the copy of layer
    # l); and only what the turn added (pack_tail of the new tokens, then one copy of that).
    src_table = torch.from_numpy(sess.table_with_room_for_the_new_turn()).to(dev)
    ev_pack = [torch.cuda.Event() for _ in range(L)]

    def write_back_one_shot():
        S.kv_pack(cache, src_table, prefix_lens, offsets, total, dbuf, stream=s_unpack)
        S.stage_to_host(host, dbuf, payload, s_unpack, s_copy, ev)

    def write_back_layer_wise():
        for l in range(L):
            S.kv_pack_layers(cache, l, l + 1, src_table, prefix_lens, offsets, total, dbuf, stream=s_unpack)
            S.stage_layer_to_host(host, dbuf, cache, l, h_prefix, h_off, s_unpack, s_copy, ev_pack[l])

    grown = torch.from_numpy((sess.prefix_lens + sess.new_lens).astype(np.int32)).to(dev)
    tail_off_h = np.concatenate([[0], np.cumsum(sess.new_lens.astype(np.int64))]).astype(np.int64)
    tail_off = torch.from_numpy(tail_off_h).to(dev)
    tail_total = int(tail_off_h[-1])
    tail_payload = S.kv_buffer_bytes(cache, tail_total)

    def write_back_tail():
        S.kv_pack_tail(cache, src_table, grown, prefix_lens, tail_off, tail_total, dbuf, stream=s_unpack)
        S.stage_to_host(host, dbuf, tail_payload, s_unpack, s_copy, ev)

    wb_shot_ms, wb_wise_ms, wb_tail_ms = timed(write_back_one_shot), timed(write_back_layer_wise), timed(write_back_tail)
    direct_ms = timed(layer_wise_direct) if host_is_mapped else None
    wb_direct_ms = timed(lambda: S.kv_pack(cache, src_table, prefix_lens, offsets, total, host_bf16, stream=s_unpack)) \
        if host_is_mapped else None
    print(json.dumps({
        "metric": "resume from pinned host memory: host->device + unpack + attention of all layers", "value": wise_ms,
        "unit": "ms", "n_gpus": 1, "steps": max(args.steps // 4, 3), "warmup": 1, "ms_per_step": wise_ms,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "n_sessions": sess.n_sessions, "n_layers": L, "payload_bytes": payload,
                   "new_tokens": sess.total_new_tokens},
        "host_to_device_alone": {"ms": copy_ms, "GBps": payload / copy_ms / 1e6},
        "attention_all_layers_kv_in_place": {"ms": attn_ms},
        "one_shot": {"ms": shot_ms, "after_the_copy_ms": shot_ms - copy_ms},
        "layer_wise": {"ms": wise_ms, "after_the_copy_ms": wise_ms - copy_ms},
        "layer_wise_unpack_straight_from_host": None if direct_ms is None else
        {"ms": direct_ms, "after_the_copy_ms": direct_ms - copy_ms, "staging_buffer_bytes": 0},
        "write_back": {"whole_sessions_one_shot_ms": wb_shot_ms, "whole_sessions_layer_wise_ms": wb_wise_ms,
                       "whole_sessions_pack_straight_to_host_ms": wb_direct_ms,
                       "new_tokens_only_ms": wb_tail_ms, "new_tokens_payload_bytes": tail_payload}}))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (sessions shard across GPUs with no exchange step; "
              "no multi-GPU figure is produced). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2412_16434_amd as S
    import workloads as W

    S.load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.only == "resume":
        resume_mix(args)
        return
    if args.only == "decode":
        decode_step(args)
        return
    cfg = W.get_config(args.config)
    if cfg.dtype != "bf16":
        print("bench.py: benchmark configs are bf16", file=sys.stderr)
        sys.exit(2)
    sess = W.make_sessions(cfg)
    if args.only == "attn":
        attn_only(args, cfg, sess)
        return
    if args.only == "pipeline":
        pipelined_resume(args, cfg, sess)
        return

    # ---- inputs, resident in HBM before anything is timed ------------------------------------------------
    L, nb, bs = cfg.n_layers, cfg.n_blocks, cfg.block_size
    shape = (L, nb, bs, cfg.n_kv_heads, cfg.head_dim)
    k_pool = torch.empty(shape, dtype=torch.bfloat16, device=dev)
    v_pool = torch.empty(shape, dtype=torch.bfloat16, device=dev)
    sent = int(np.array([W.SENTINEL16], dtype=np.uint16).view(np.int16)[0])
    k_pool.view(torch.int16).fill_(sent)
    v_pool.view(torch.int16).fill_(sent)
    W.fill_pool_blocks_device(k_pool, v_pool, cfg, sess.owned_blocks())
    # the attention layer holds the seeded Gaussian draws (owned blocks only)
    kh, vh, qh, knh, vnh = W.make_attn_inputs(cfg, sess)
    la = cfg.attn_layer
    owned = torch.from_numpy(sess.owned_blocks().astype(np.int64)).to(dev)
    for pool, host in ((k_pool, kh), (v_pool, vh)):
        src = torch.from_numpy(host.view(np.int16)[sess.owned_blocks()]).to(dev)
        pool[la].view(torch.int16).index_copy_(0, owned, src)
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    q, k_new, v_new = to_dev(qh), to_dev(knh), to_dev(vnh)
    out = torch.empty_like(q)
    table = torch.from_numpy(sess.block_table).to(dev)
    dst_table = torch.from_numpy(sess.dst_block_table).to(dev)
    prefix_lens = torch.from_numpy(sess.prefix_lens).to(dev)
    offsets = torch.from_numpy(sess.buf_token_offsets).to(dev)
    cu = torch.from_numpy(sess.cu_new_lens).to(dev)
    cache = S.KVCache(k_pool, v_pool)
    total = sess.total_prefix_tokens
    payload = S.kv_buffer_bytes(cache, total)
    assert payload == sess.payload_bytes()
    buf = torch.empty(payload // 2, dtype=torch.bfloat16, device=dev)
    ws_bytes = S.prefix_prefill_attn_workspace_bytes(cache, sess.n_sessions, cfg.n_q_heads, sess.total_new_tokens,
                                                     sess.max_new_len, sess.max_prefix_len)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)

    def step(evs=None):
        if evs: evs[0].record()
        S.kv_pack(cache, table, prefix_lens, offsets, total, buf)
        if evs: evs[1].record()
        S.kv_unpack(cache, dst_table, prefix_lens, offsets, total, buf)
        if evs: evs[2].record()
        S.prefix_prefill_attn(cache, la, q, k_new, v_new, out, cu, prefix_lens, table, sess.max_new_len,
                              sess.max_prefix_len, cfg.scale, workspace=ws if ws_bytes else None)
        if evs: evs[3].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    pack_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
    unpack_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in evs]))
    attn_ms = float(np.mean([e[2].elapsed_time(e[3]) for e in evs]))
    spread = {name: {"median_ms": float(np.median(v)), "min_ms": float(np.min(v))}
              for name, v in (("kv_pack", [e[0].elapsed_time(e[1]) for e in evs]),
                              ("kv_unpack", [e[1].elapsed_time(e[2]) for e in evs]),
                              ("prefix_prefill_attn", [e[2].elapsed_time(e[3]) for e in evs]))}

    # ---- contiguous copy of the same byte count: the practical HBM ceiling -------------------------------
    scratch = torch.empty_like(buf)
    for _ in range(2):
        S.device_copy(scratch, buf, payload)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        S.device_copy(scratch, buf, payload)
    e1.record()
    torch.cuda.synchronize()
    copy_ms = e0.elapsed_time(e1) / 5
    # the runtime's own device-to-device copy of the same bytes (torch's copy_ of contiguous tensors is hipMemcpyAsync)
    for _ in range(2):
        scratch.copy_(buf)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        scratch.copy_(buf)
    e1.record()
    torch.cuda.synchronize()
    memcpy_ms = e0.elapsed_time(e1) / 5
    del scratch

    # ---- append of the turn's K,V rows to the cache (one layer): small, outside the step, reported on its own ------
    app_table = torch.from_numpy(sess.table_with_room_for_the_new_turn()).to(dev)
    for _ in range(2):
        S.kv_append(cache, la, k_new, v_new, cu, prefix_lens, app_table)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        S.kv_append(cache, la, k_new, v_new, cu, prefix_lens, app_table)
    e1.record()
    torch.cuda.synchronize()
    append_us = e0.elapsed_time(e1) / 20 * 1e3
    append_bytes = 2.0 * 2.0 * sess.total_new_tokens * cfg.n_kv_heads * cfg.head_dim * 2   # K and V, read + written

    # ---- write-back of what the turn added (all layers): only the new tokens of every session move --------------------
    grown_h = (sess.prefix_lens + sess.new_lens).astype(np.int32)
    tail_off_h = np.concatenate([[0], np.cumsum(sess.new_lens.astype(np.int64))]).astype(np.int64)
    grown, tail_off = torch.from_numpy(grown_h).to(dev), torch.from_numpy(tail_off_h).to(dev)
    tail_total = int(tail_off_h[-1])
    tail_payload = S.kv_buffer_bytes(cache, tail_total)
    tail_buf = buf[: tail_payload // 2]
    for _ in range(2):
        S.kv_pack_tail(cache, app_table, grown, prefix_lens, tail_off, tail_total, tail_buf)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        S.kv_pack_tail(cache, app_table, grown, prefix_lens, tail_off, tail_total, tail_buf)
    e1.record()
    torch.cuda.synchronize()
    tail_ms = e0.elapsed_time(e1) / 10

    # ---- priority-based residency (Sec. 3.3): the LOWER HALF of the layers of every session moved in with one launch.
    # The same pools seen as one pool of L * n_blocks slots (slot = layer * n_blocks + block), one unit per (session,
    # layer), the chunks where they lie in the whole migration buffer.
    Lh = max(cfg.n_layers // 2, 1)
    nb_pool = k_pool.shape[1]
    slot_pool = S.KVCache(k_pool.view(1, cfg.n_layers * nb_pool, *k_pool.shape[2:]),
                          v_pool.view(1, cfg.n_layers * nb_pool, *v_pool.shape[2:]))
    units = [(s_, l_) for l_ in range(Lh) for s_ in range(sess.n_sessions)]
    u_lens_h = np.array([sess.prefix_lens[s_] for s_, _ in units], dtype=np.int32)
    u_table_h = np.stack([np.where(sess.dst_block_table[s_] >= 0, sess.dst_block_table[s_] + l_ * nb_pool, -1)
                          for s_, l_ in units]).astype(np.int32)
    u_rows_h = np.array([int(sess.buf_token_offsets[s_]) * 2 * cfg.n_layers + 2 * l_ * int(sess.prefix_lens[s_])
                         for s_, l_ in units], dtype=np.int64)
    u_off_h = np.concatenate([[0], np.cumsum(u_lens_h.astype(np.int64))]).astype(np.int64)
    u_table, u_lens, u_off, u_rows = (torch.from_numpy(a).to(dev) for a in (u_table_h, u_lens_h, u_off_h, u_rows_h))
    u_total = int(u_off_h[-1])
    u_payload = 2 * u_total * cfg.n_kv_heads * cfg.head_dim * 2
    for _ in range(2):
        S.kv_unpack_units(slot_pool, u_table, u_lens, u_off, u_rows, u_total, buf)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        S.kv_unpack_units(slot_pool, u_table, u_lens, u_off, u_rows, u_total, buf)
    e1.record()
    torch.cuda.synchronize()
    units_ms = e0.elapsed_time(e1) / 10

    # ---- the residency pool itself (host code, Sec. 3.3): 512 announced sessions of config-2 lengths, 32 layers, room for
    # a quarter of them; time of one settle from empty, of a framework demand that evicts, of the settle after it
    rng_pool = np.random.default_rng(12)
    pool_lens = rng_pool.integers(1024, 8193, size=512)
    pool_blocks = int(np.sum(-(-pool_lens // cfg.block_size))) * cfg.n_layers
    kp = S.KvPool(cfg.n_layers, pool_blocks // 4, cfg.block_size)
    for i, n in enumerate(pool_lens):
        kp.advise(i, int(n))
    import ctypes as C
    lib, n_take = S.load_library(), pool_blocks // 16
    changes = (S.PoolChange * (512 * cfg.n_layers))()
    slot_arr = (C.c_int32 * (pool_blocks // 4))()
    take_arr = (C.c_int32 * n_take)()
    nc, ns = C.c_int32(), C.c_int32()
    t0 = time.perf_counter()
    rc0 = lib.symph_pool_settle(kp.handle, changes, len(changes), slot_arr, len(slot_arr), C.byref(nc), C.byref(ns))
    t1 = time.perf_counter()
    loaded = nc.value
    rc1 = lib.symph_pool_framework_take(kp.handle, n_take, take_arr)
    t2 = time.perf_counter()
    rc2 = lib.symph_pool_settle(kp.handle, changes, len(changes), slot_arr, len(slot_arr), C.byref(nc), C.byref(ns))
    t3 = time.perf_counter()
    assert rc0 == rc1 == rc2 == 0
    pool_stats = {"sessions": 512, "layers": cfg.n_layers, "slots": pool_blocks // 4,
                  "first_settle_ms": (t1 - t0) * 1e3, "units_loaded": loaded, "slots_assigned": pool_blocks // 4 - kp.counts()[0] - n_take,
                  "framework_take_ms": (t2 - t1) * 1e3, "slots_taken": n_take,
                  "settle_after_it_ms": (t3 - t2) * 1e3, "changes_reported": nc.value}
    kp.close()

    # ---- MFMA-only reference kernel: what the matrix cores deliver here, for a launch as short as the attention
    # call (the shader clock is still ramping up) and sustained ------------------------------------------------------
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    mfma_ref = {}
    for label, iters, reps in (("short", 300, 7), ("sustained", 40000, 3)):
        ts = []
        for _ in range(reps):
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flops = S.mfma_reference(iters, sink)
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        ms = float(np.median(ts))
        mfma_ref[label] = {"ms": ms, "TFLOPs": flops / ms / 1e9, "pct_mfma_bf16_peak": flops / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS * 100}

    # ---- host staging on a side stream (PCIe) -----------------------------------------------------------------
    staging = None
    if not args.no_staging:
        nbytes = min(payload, 1 << 30)
        host = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
        side = torch.cuda.Stream()
        main_stream = torch.cuda.current_stream()
        ev = torch.cuda.Event()
        bview = buf.view(torch.uint8)
        res = {}
        for name, fn in (("d2h", lambda: S.stage_to_host(host, bview, nbytes, main_stream, side, ev)),
                         ("h2d", lambda: S.stage_to_device(bview, host, nbytes, main_stream, side, ev))):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            res[name + "_GBps"] = 3 * nbytes / (time.perf_counter() - t0) / 1e9
        res["bytes"] = nbytes
        staging = res
        del host

    mig_bytes = 2.0 * payload                 # every payload byte read once and written once
    attn_flops = sess.attn_flops()
    attn_bytes = sess.attn_bytes()
    step_bytes = 2.0 * mig_bytes + attn_bytes
    pack_gbs = mig_bytes / pack_ms / 1e6
    unpack_gbs = mig_bytes / unpack_ms / 1e6
    attn_tflops = attn_flops / attn_ms / 1e9
    dominant = "pack" if pack_ms >= unpack_ms else "unpack"
    dom_gbs = pack_gbs if dominant == "pack" else unpack_gbs

    result = {
        "metric": "prefix-prefill attn TFLOP/s + KV pack/unpack GB/s, as % of MI355X peaks",
        "value": step_bytes / ms_step / 1e6,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "n_sessions": sess.n_sessions, "n_layers": L, "n_q_heads": cfg.n_q_heads,
                   "n_kv_heads": cfg.n_kv_heads, "head_dim": cfg.head_dim, "block_size": bs, "pool_blocks": nb,
                   "prefix_tokens": total, "new_tokens": sess.total_new_tokens, "payload_bytes": payload,
                   "step": "kv_pack(all layers) + kv_unpack(all layers) + prefix_prefill_attn(one layer)"},
        "kv_pack": {"ms": pack_ms, "GBps": pack_gbs, "payload_GBps": pack_gbs / 2, "pct_hbm_peak": 100 * pack_gbs / HBM_PEAK_GBS,
                    **spread["kv_pack"]},
        "kv_unpack": {"ms": unpack_ms, "GBps": unpack_gbs, "payload_GBps": unpack_gbs / 2,
                      "pct_hbm_peak": 100 * unpack_gbs / HBM_PEAK_GBS, **spread["kv_unpack"]},
        "prefix_prefill_attn": {"ms": attn_ms, "TFLOPs": attn_tflops,
                                "pct_mfma_bf16_peak": 100 * attn_tflops / MFMA_BF16_PEAK_TFLOPS,
                                "kv_GBps": attn_bytes / attn_ms / 1e6, "flops": attn_flops,
                                **spread["prefix_prefill_attn"]},
        "contiguous_copy": {"ms": copy_ms, "GBps": mig_bytes / copy_ms / 1e6,
                            "runtime_memcpy_d2d_ms": memcpy_ms, "runtime_memcpy_d2d_GBps": mig_bytes / memcpy_ms / 1e6},
        "kv_append_one_layer": {"us": append_us, "GBps": append_bytes / append_us / 1e3, "bytes": append_bytes},
        "kv_pack_tail_new_turn": {"ms": tail_ms, "GBps": 2.0 * tail_payload / tail_ms / 1e6, "payload_bytes": tail_payload,
                                  "pct_hbm_peak": 100 * 2.0 * tail_payload / tail_ms / 1e6 / HBM_PEAK_GBS},
        "kv_unpack_units_lower_half_of_the_layers": {"ms": units_ms, "GBps": 2.0 * u_payload / units_ms / 1e6,
                                                     "payload_bytes": u_payload, "n_units": len(units),
                                                     "pct_hbm_peak": 100 * 2.0 * u_payload / units_ms / 1e6 / HBM_PEAK_GBS},
        "residency_pool_host": pool_stats,
        "mfma_reference": {**mfma_ref, "attn_pct_of_short_reference": 100 * attn_tflops / mfma_ref["short"]["TFLOPs"]},
        "host_staging": staging,
        "roofline": {"kernel": f"kv_migrate ({dominant})", "bound": "hbm", "achieved": dom_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": dom_gbs / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name, {}).get("kv_migrate")},
        "roofline_attn": {"kernel": "attn_mfma", "bound": "mfma", "achieved": attn_tflops,
                          "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": attn_tflops / MFMA_BF16_PEAK_TFLOPS,
                          "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name, {}).get("attn")},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, sess, args.cpu_seconds)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
