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

PROFILES = os.path.join(ROOT, "profiles")


def measured_traffic(workload: str) -> dict:
    """HBM bytes per launch from profiles/bench_<workload>_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    scaled by the readings of the plain copy kernel of known size; written by `bench.py --write-traffic-summary`):
    the line `traffic_bytes_per_launch: kernel=bytes ...`.  Empty if that workload has not been profiled."""
    path = os.path.join(PROFILES, f"bench_{workload}_hbm_traffic.md")
    out = {}
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    for item in line.split(":", 1)[1].split():
                        k, v = item.split("=")
                        out[k] = float(v)
    except OSError:
        pass
    return out


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
    ap.add_argument("--no-per-config", action="store_true",
                    help="leave out the other four workloads, the mixed-resume modes and the decode step")
    ap.add_argument("--write-traffic-summary", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"),
                    help="no GPU work: read the counter csv files of two `rocprofv3 --pmc FETCH_SIZE` / `--pmc "
                         "WRITE_SIZE` runs of this script and write profiles/bench_<config>_hbm_traffic.md")
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
    # migration sample: same shapes, lengths and sessions, fewer layers, small pool: a payload of more than 2 GB, far
    # beyond the host's last-level cache, so that the rate is a DRAM figure
    import dataclasses
    mcfg = dataclasses.replace(W.scaled_config(cfg, n_layers=min(cfg.n_layers, 8), n_blocks=max(8192, cfg.n_blocks // 8)),
                               fresh_tables=False)      # (the scatter goes back through the source table)
    msess = W.make_sessions(mcfg)
    shape = (mcfg.n_layers, mcfg.n_blocks, mcfg.block_size, mcfg.n_kv_heads, mcfg.head_dim)
    dt = np.uint16 if cfg.dtype == "bf16" else np.float32
    kp = np.resize(np.arange(65521, dtype=np.uint32).astype(dt), shape)      # (values do not matter to a copy)
    vp = np.resize(np.arange(65519, dtype=np.uint32).astype(dt), shape)
    t0 = time.perf_counter()
    buf = oracle.kv_pack(kp, vp, msess.block_table, msess.prefix_lens, msess.buf_token_offsets)
    t1 = time.perf_counter()
    oracle.kv_unpack(kp, vp, msess.block_table, msess.prefix_lens, msess.buf_token_offsets, buf)
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
                   f"({msess.payload_bytes() / 1e6:.0f} MB payload, same shapes and lengths); attention on "
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
    kp, vp, q, k_new, v_new = W.make_attn_inputs_device(cfg, sess, dev)
    cache = S.KVCache(kp[None], vp[None])
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
    kp, vp, q_all, kn_all, vn_all = W.make_attn_inputs_device(cfg, sess, dev)
    cache = S.KVCache(kp[None], vp[None])
    new_lens = np.diff(sess.cu_new_lens)
    idx = np.nonzero(new_lens == 1)[0]
    rows = torch.from_numpy(sess.cu_new_lens[:-1][idx].astype(np.int64)).to(dev)   # the one query row of each such session
    q, k_new, v_new = (a[rows].contiguous() for a in (q_all, kn_all, vn_all))
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
    return ({
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
                     "frac": gbs / HBM_PEAK_GBS, "traffic": None}})


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
    kp, vp, q, k_new, v_new = W.make_attn_inputs_device(acfg, asess, dev)
    acache = S.KVCache(kp[None], vp[None])
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
    return ({
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
        "both": {"ms": both_ms, "sum_of_alone_ms": attn_ms + unpack_ms, "max_of_alone_ms": max(attn_ms, unpack_ms)}})


def pipelined_resume(args, cfg, sess, brief: bool = False):
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

    def layer_wise_layer_major():
        # the buffer laid out layer -> session -> K|V -> token: one copy per layer instead of one per session and layer
        for l in range(L):
            S.stage_batch_layers_to_device(dbuf, host, cache, l, l + 1, total, s_unpack, s_copy, ev_copy[l])
            S.kv_unpack_batch_layers(cache, l, l + 1, dst_table, prefix_lens, offsets, total, dbuf, stream=s_unpack)
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
    shot_ms, wise_lm_ms = timed(one_shot), timed(layer_wise_layer_major)
    if brief:   # the part of this mode that the default run carries
        return {"payload_bytes": payload, "n_layers": L,
                "host_to_device_alone": {"ms": copy_ms, "GBps": payload / copy_ms / 1e6},
                "attention_all_layers_kv_in_place": {"ms": attn_ms},
                "one_shot": {"ms": shot_ms, "after_the_copy_ms": shot_ms - copy_ms},
                "layer_wise_layer_major_buffer": {"ms": wise_lm_ms, "after_the_copy_ms": wise_lm_ms - copy_ms, "copies": L}}
    wise_ms = timed(layer_wise)

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

    def write_back_layer_wise_layer_major():
        for l in range(L):
            S.kv_pack_batch_layers(cache, l, l + 1, src_table, prefix_lens, offsets, total, dbuf, stream=s_unpack)
            S.stage_batch_layers_to_host(host, dbuf, cache, l, l + 1, total, s_unpack, s_copy, ev_pack[l])

    grown = torch.from_numpy((sess.prefix_lens + sess.new_lens).astype(np.int32)).to(dev)
    tail_off_h = np.concatenate([[0], np.cumsum(sess.new_lens.astype(np.int64))]).astype(np.int64)
    tail_off = torch.from_numpy(tail_off_h).to(dev)
    tail_total = int(tail_off_h[-1])
    tail_payload = S.kv_buffer_bytes(cache, tail_total)

    def write_back_tail():
        S.kv_pack_tail(cache, src_table, grown, prefix_lens, tail_off, tail_total, dbuf, stream=s_unpack)
        S.stage_to_host(host, dbuf, tail_payload, s_unpack, s_copy, ev)

    wb_shot_ms, wb_wise_ms, wb_tail_ms = timed(write_back_one_shot), timed(write_back_layer_wise), timed(write_back_tail)
    wb_wise_lm_ms = timed(write_back_layer_wise_layer_major)
    direct_ms = timed(layer_wise_direct) if host_is_mapped else None
    wb_direct_ms = timed(lambda: S.kv_pack(cache, src_table, prefix_lens, offsets, total, host_bf16, stream=s_unpack)) \
        if host_is_mapped else None
    return ({
        "metric": "resume from pinned host memory: host->device + unpack + attention of all layers", "value": wise_ms,
        "unit": "ms", "n_gpus": 1, "steps": max(args.steps // 4, 3), "warmup": 1, "ms_per_step": wise_ms,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "n_sessions": sess.n_sessions, "n_layers": L, "payload_bytes": payload,
                   "new_tokens": sess.total_new_tokens},
        "host_to_device_alone": {"ms": copy_ms, "GBps": payload / copy_ms / 1e6},
        "attention_all_layers_kv_in_place": {"ms": attn_ms},
        "one_shot": {"ms": shot_ms, "after_the_copy_ms": shot_ms - copy_ms},
        "layer_wise": {"ms": wise_ms, "after_the_copy_ms": wise_ms - copy_ms, "copies": L * sess.n_sessions},
        "layer_wise_layer_major_buffer": {"ms": wise_lm_ms, "after_the_copy_ms": wise_lm_ms - copy_ms, "copies": L},
        "layer_wise_unpack_straight_from_host": None if direct_ms is None else
        {"ms": direct_ms, "after_the_copy_ms": direct_ms - copy_ms, "staging_buffer_bytes": 0},
        "write_back": {"whole_sessions_one_shot_ms": wb_shot_ms, "whole_sessions_layer_wise_ms": wb_wise_ms,
                       "whole_sessions_layer_wise_layer_major_buffer_ms": wb_wise_lm_ms,
                       "whole_sessions_pack_straight_to_host_ms": wb_direct_ms,
                       "new_tokens_only_ms": wb_tail_ms, "new_tokens_payload_bytes": tail_payload}})


def _median_event_ms(fn, warmup: int, iters: int) -> float:
    """Median time of `fn` (one library call on the current stream), events around each of `iters` calls issued back
    to back, one synchronisation at the end."""
    import torch
    for _ in range(warmup):
        fn()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for e0, e1 in evs:
        e0.record()
        fn()
        e1.record()
    torch.cuda.synchronize()
    return float(np.median([e0.elapsed_time(e1) for e0, e1 in evs]))


def _attn_figures(sess, ms: float) -> dict:
    """TFLOP/s against the matrix-core peak, K,V GB/s against the HBM peak, and which of the two roofs lies lower for
    this batch (the time each would need at its peak)."""
    flops, nbytes = sess.attn_flops(), sess.attn_bytes()
    tflops, gbs = flops / ms / 1e9, nbytes / ms / 1e6
    t_mfma, t_hbm = flops / (MFMA_BF16_PEAK_TFLOPS * 1e12), nbytes / (HBM_PEAK_GBS * 1e9)
    return {"ms": ms, "TFLOPs": tflops, "frac_mfma_bf16_peak": tflops / MFMA_BF16_PEAK_TFLOPS, "kv_GBps": gbs,
            "frac_hbm_peak": gbs / HBM_PEAK_GBS, "flops": flops, "bytes": nbytes,
            "flop_per_byte": flops / max(nbytes, 1), "binding_roof": "mfma" if t_mfma >= t_hbm else "hbm"}


def measure_config(args, name: str) -> dict:
    """pack, unpack (all layers, every session) and one-layer attention of one workload, each timed on its own with
    events on the launch stream.  Pools hold zeros for the migration legs (a copy does not look at values); the
    attention inputs are drawn on the device with the workload's shapes, lengths, tables and value distribution."""
    import torch
    import paper_2412_16434_amd as S
    import workloads as W
    dev = "cuda:0"
    cfg = W.get_config(name)
    mig_cfg = W.get_config("mixed_resume_incoming") if name == "mixed_resume" else cfg     # (the sessions that arrive)
    out = {"workload": name, "dtype": cfg.dtype}
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32

    # ---- migration legs
    msess = W.make_sessions(mig_cfg)
    shape = (mig_cfg.n_layers, mig_cfg.n_blocks, mig_cfg.block_size, mig_cfg.n_kv_heads, mig_cfg.head_dim)
    cache = S.KVCache(torch.zeros(shape, dtype=tdt, device=dev), torch.zeros(shape, dtype=tdt, device=dev))
    table = torch.from_numpy(msess.block_table).to(dev)
    dst_table = torch.from_numpy(msess.dst_block_table).to(dev)
    plens = torch.from_numpy(msess.prefix_lens).to(dev)
    offs = torch.from_numpy(msess.buf_token_offsets).to(dev)
    total = msess.total_prefix_tokens
    payload = S.kv_buffer_bytes(cache, total)
    buf = torch.zeros(max(payload // cache.k_pool.element_size(), 8), dtype=tdt, device=dev)
    # pack then unpack, alternating as in the step, events around each call
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(7)]
    for it in range(-2, 7):
        if it >= 0: evs[it][0].record()
        S.kv_pack(cache, table, plens, offs, total, buf)
        if it >= 0: evs[it][1].record()
        S.kv_unpack(cache, dst_table, plens, offs, total, buf)
        if it >= 0: evs[it][2].record()
    torch.cuda.synchronize()
    pack_ms = float(np.median([e[0].elapsed_time(e[1]) for e in evs]))
    unpack_ms = float(np.median([e[1].elapsed_time(e[2]) for e in evs]))
    for leg, ms in (("kv_pack", pack_ms), ("kv_unpack", unpack_ms)):
        gbs = 2.0 * payload / ms / 1e6
        out[leg] = {"ms": ms, "GBps": gbs, "frac_hbm_peak": gbs / HBM_PEAK_GBS, "payload_bytes": payload,
                    "sessions": msess.n_sessions, "layers": mig_cfg.n_layers}
        if 2 * payload < (256 << 20):
            out[leg]["note"] = "payload lives in the caches: no share-of-peak claim"
    del cache, buf, table, dst_table
    torch.cuda.empty_cache()

    # ---- attention on one layer
    sess = W.make_sessions(cfg)
    if cfg.dtype == "bf16":
        k_pool, v_pool, q, k_new, v_new = W.make_attn_inputs_device(cfg, sess, dev)
    else:
        k_pool, v_pool, q, k_new, v_new = (torch.from_numpy(a).to(dev) for a in W.make_attn_inputs(cfg, sess))
        k_pool.nan_to_num_(0.0); v_pool.nan_to_num_(0.0)
    acache = S.KVCache(k_pool[None], v_pool[None])
    o = torch.empty_like(q)
    atable = torch.from_numpy(sess.block_table).to(dev)
    aplens = torch.from_numpy(sess.prefix_lens).to(dev)
    cu = torch.from_numpy(sess.cu_new_lens).to(dev)
    ws_bytes = S.prefix_prefill_attn_workspace_bytes(acache, sess.n_sessions, cfg.n_q_heads, sess.total_new_tokens,
                                                     sess.max_new_len, sess.max_prefix_len)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    attn_ms = _median_event_ms(
        lambda: S.prefix_prefill_attn(acache, 0, q, k_new, v_new, o, cu, aplens, atable, sess.max_new_len,
                                      sess.max_prefix_len, cfg.scale, workspace=ws if ws_bytes else None), 3, 15)
    out["prefix_prefill_attn"] = {**_attn_figures(sess, attn_ms), "sessions": sess.n_sessions,
                                  "new_tokens": sess.total_new_tokens, "prefix_tokens": sess.total_prefix_tokens}
    if cfg.dtype != "bf16":
        out["prefix_prefill_attn"]["note"] = "fp32 runs the plain one-wave-per-row kernel: correctness path, no roofline claim"
    del acache, k_pool, v_pool, ws
    torch.cuda.empty_cache()
    return out


def write_traffic_summary(args, out_dir=None):
    """profiles/bench_<config>_hbm_traffic.md (or the same file name under out_dir) from the counter csv files of two rocprofv3 runs of this script (one with
    --pmc FETCH_SIZE, one with --pmc WRITE_SIZE).  The plain copy kernel of known size in the same runs gives the unit
    of each counter on this machine; every other kernel's readings are scaled by it."""
    import csv
    import glob
    import workloads as W
    cfg = W.get_config(args.config)
    sess = W.make_sessions(cfg)
    payload = sess.payload_bytes()

    def means(d, counter):
        """kernel name -> (mean reading, launches) over the launches with that kernel's LARGEST grid: the run also
        launches the same instantiations on smaller inputs (the write-back of a turn, the unit-wise scatter)."""
        acc = {}
        for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            with open(f) as fh:
                for r in csv.DictReader(fh):
                    if r.get("Counter_Name") == counter:
                        acc.setdefault(r["Kernel_Name"], {}).setdefault(int(r["Grid_Size"]), []).append(float(r["Counter_Value"]))
        return {k: (sum(g[max(g)]) / len(g[max(g)]), len(g[max(g)]), max(g)) for k, g in acc.items()}
    fetch, write = means(args.write_traffic_summary[0], "FETCH_SIZE"), means(args.write_traffic_summary[1], "WRITE_SIZE")

    def pick(table, *subs):
        hits = [(k, v) for k, v in table.items() if all(s in k for s in subs)]
        if not hits:
            raise SystemExit(f"no kernel matching {subs} in the counter files")
        _, v = max(hits, key=lambda kv: kv[1][2])   # of several instantiations, the one with the largest launch
        return v[0], v[1]
    copy_f, _ = pick(fetch, "device_copy_kernel")
    copy_w, _ = pick(write, "device_copy_kernel")
    unit_f, unit_w = payload / copy_f, payload / copy_w          # bytes per count
    rows, line = [], []
    for label, key, subs, algo in (
            ("kv_pack", "kv_pack", ("kv_migrate", "kernel<unsigned int __vector(4), true,"), 2.0 * payload),
            ("kv_unpack", "kv_unpack", ("kv_migrate", "kernel<unsigned int __vector(4), false,"), 2.0 * payload),
            ("prefix_prefill_attn (main kernel)", "attn_mfma", ("attn_mfma_kernel",), float(sess.attn_bytes()))):
        f, nf = pick(fetch, *subs)
        w, nw = pick(write, *subs)
        rd, wr = f * unit_f, w * unit_w
        rows.append(f"| {label} | {f:.4g} ({nf}) | {w:.4g} ({nw}) | {rd / 1e9:.3f} GB | {wr / 1e9:.3f} GB | "
                    f"{(rd + wr) / 1e9:.3f} GB | {algo / 1e9:.3f} GB | {(rd + wr) / algo:.3f} |")
        line.append(f"{key}={rd + wr:.6g}")
    text = f"""# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE: HBM traffic per launch, workload {cfg.name}, one MI355X

Commands (separate runs, from the repo root on the GPU box; the third needs no GPU):

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d gpurun_out/pmc_fetch -o f -- python3 bench.py --steps 2 --warmup 1 --no-cpu-baseline --no-staging --no-per-config
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d gpurun_out/pmc_write -o w -- python3 bench.py --steps 2 --warmup 1 --no-cpu-baseline --no-staging --no-per-config
    python3 bench.py --write-traffic-summary gpurun_out/pmc_fetch gpurun_out/pmc_write

Calibration: the plain copy kernel (`symph_device_copy`) of the same runs reads {payload} B and writes {payload} B; its
mean FETCH_SIZE is {copy_f:.5g} and its mean WRITE_SIZE {copy_w:.5g}, so one count is {unit_f:.1f} B of reads and
{unit_w:.1f} B of writes on this machine.

| kernel | FETCH_SIZE, mean (launches) | WRITE_SIZE, mean (launches) | HBM read | HBM written | total | algorithmic bytes | total / algorithmic |
|---|---|---|---|---|---|---|---|
""" + "\n".join(rows) + f"""

Algorithmic bytes: pack / unpack 2 x payload (every byte read once and written once); attention: K,V of one layer once,
Q, O, K_new, V_new.  bench.py reads the next line for `roofline.traffic`:

traffic_bytes_per_launch: {' '.join(line)}
"""
    path = os.path.join(out_dir or PROFILES, f"bench_{cfg.name}_hbm_traffic.md")
    with open(path, "w") as f:
        f.write(text)
    print(path)
    return path


def main():
    args = parse_args()
    if args.write_traffic_summary:
        write_traffic_summary(args)
        return
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
        print(json.dumps(resume_mix(args)))
        return
    if args.only == "decode":
        print(json.dumps(decode_step(args)))
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
        print(json.dumps(pipelined_resume(args, cfg, sess)))
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

    traffic = measured_traffic(cfg.name)
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
                     "traffic": traffic.get("kv_pack" if dominant == "pack" else "kv_unpack")},
        "roofline_attn": {"kernel": "attn_mfma", "bound": "mfma", "achieved": attn_tflops,
                          "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": attn_tflops / MFMA_BF16_PEAK_TFLOPS,
                          "traffic": traffic.get("attn_mfma")},
    }
    if not args.no_per_config:
        # the other workloads, each leg timed on its own; the headline workload's row repeats the step's figures
        del k_pool, v_pool, pool, cache, slot_pool, buf, tail_buf
        torch.cuda.empty_cache()
        per = {cfg.name: {"workload": cfg.name, "dtype": cfg.dtype, "measured": "inside the timed step",
                          "kv_pack": {"ms": pack_ms, "GBps": pack_gbs, "frac_hbm_peak": pack_gbs / HBM_PEAK_GBS,
                                      "payload_bytes": payload},
                          "kv_unpack": {"ms": unpack_ms, "GBps": unpack_gbs, "frac_hbm_peak": unpack_gbs / HBM_PEAK_GBS,
                                        "payload_bytes": payload},
                          "prefix_prefill_attn": _attn_figures(sess, attn_ms)}}
        for name in ("tiny_fp32", "llama70b_long", "many_short", "mixed_resume"):
            if name != cfg.name:
                per[name] = measure_config(args, name)
        result["per_config"] = per
        mix = resume_mix(args)
        result["mixed_resume"] = {k: mix[k] for k in ("attn_alone", "unpack_alone", "both")}
        if not args.no_staging:
            result["layer_wise_resume"] = pipelined_resume(args, cfg, sess, brief=True)
        dec = decode_step(args)
        result["decode_step"] = {"config": dec["config"], "decode_kernel": dec["decode_kernel"],
                                 "work_item_kernel": dec["work_item_kernel"],
                                 "max_abs_difference_between_the_two": dec["max_abs_difference_between_the_two"]}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, sess, args.cpu_seconds)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
