"""Helpers for the GPU parity tests: move seeded host inputs to the device, call the C-ABI through the Python
binding, bring results back as numpy.  The oracle is only ever given the host arrays."""
from __future__ import annotations

import numpy as np
import torch

import paper_2412_16434_amd as S
import workloads as W

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    """numpy -> device tensor; uint16 arrays are bf16 bit patterns."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a).to(DEV)


def to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def widen(a: np.ndarray) -> np.ndarray:
    return W.bf16_bits_to_f32(a).astype(np.float64) if a.dtype == np.uint16 else a.astype(np.float64)


class DeviceSessions:
    def __init__(self, sess: W.SessionBatch):
        self.sess = sess
        self.table = torch.from_numpy(sess.block_table).to(DEV)
        self.dst_table = None if sess.dst_block_table is None else torch.from_numpy(sess.dst_block_table).to(DEV)
        self.prefix_lens = torch.from_numpy(sess.prefix_lens).to(DEV)
        self.offsets = torch.from_numpy(sess.buf_token_offsets).to(DEV)
        self.cu_new_lens = torch.from_numpy(sess.cu_new_lens).to(DEV)


def gpu_pack(cache: S.KVCache, ds: DeviceSessions, dst: bool = False, stream=None) -> torch.Tensor:
    n = S.kv_buffer_bytes(cache, ds.sess.total_prefix_tokens)
    buf = torch.empty(max(n // cache.k_pool.element_size(), 1), dtype=cache.k_pool.dtype, device=DEV)
    S.kv_pack(cache, ds.dst_table if dst else ds.table, ds.prefix_lens, ds.offsets, ds.sess.total_prefix_tokens, buf,
              stream=stream)
    return buf[: n // cache.k_pool.element_size()]


def gpu_unpack(cache: S.KVCache, ds: DeviceSessions, buf: torch.Tensor, dst: bool = True, stream=None) -> None:
    S.kv_unpack(cache, ds.dst_table if dst else ds.table, ds.prefix_lens, ds.offsets, ds.sess.total_prefix_tokens,
                buf, stream=stream)


def gpu_attention(cfg: W.WorkloadConfig, sess: W.SessionBatch, inputs, layer: int = 0, scale=None, tuning=None,
                  max_new_len=None, expect_flags: int = 0) -> np.ndarray:
    """Run symph_prefix_prefill_attn on host inputs (one-layer pools) and return the output as numpy.  ``tuning``: an
    S.AttnTuning for the _tuned entry points; ``max_new_len``: the bound handed to the library when it is not the true
    one.  The scheduler's flags are read back after every call and must be ``expect_flags``."""
    k_pool, v_pool, q, k_new, v_new = inputs
    ds = DeviceSessions(sess)
    cache = S.KVCache(to_dev(k_pool)[None], to_dev(v_pool)[None])
    qd, knd, vnd = to_dev(q), to_dev(k_new), to_dev(v_new)
    out = torch.full_like(qd, float("nan"))
    mnl = sess.max_new_len if max_new_len is None else max_new_len
    ws_bytes = S.prefix_prefill_attn_workspace_bytes(cache, sess.n_sessions, cfg.n_q_heads, sess.total_new_tokens,
                                                     mnl, sess.max_prefix_len, tuning=tuning)
    ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device=DEV) if ws_bytes else None
    S.prefix_prefill_attn(cache, layer, qd, knd, vnd, out, ds.cu_new_lens, ds.prefix_lens, ds.table,
                          mnl, sess.max_prefix_len, cfg.scale if scale is None else scale, workspace=ws, tuning=tuning)
    torch.cuda.synchronize()
    assert S.debug_attn_flags(ws) == expect_flags, "the device-side scheduler reported a problem"
    return to_host(out)


def attn_errors(got: np.ndarray, ref: np.ndarray):
    """(max-abs error, relative L2 error) of a bf16/fp32 result against the fp64 oracle, over finite ref rows."""
    g = widen(got)
    mask = np.isfinite(ref)
    diff = np.where(mask, g - np.where(mask, ref, 0.0), 0.0)
    if not np.all(np.isfinite(g[mask])):
        return float("inf"), float("inf")
    max_abs = float(np.max(np.abs(diff))) if diff.size else 0.0
    denom = float(np.sqrt(np.sum(np.where(mask, ref, 0.0) ** 2)))
    rel = float(np.sqrt(np.sum(diff ** 2)) / denom) if denom > 0 else 0.0
    return max_abs, rel


# tolerances of the benchmark spec (max-abs) and the tighter relative-L2 gate that an all-zero output cannot pass
TOL = {"bf16": (2e-2, 1e-2), "fp32": (1e-5, 1e-5)}
