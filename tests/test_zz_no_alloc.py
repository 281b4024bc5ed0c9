"""symph_prefix_prefill_attn_static (the attention call that allocates nothing: its scratch is a fixed array inside the
library) against symph_prefix_prefill_attn on the same inputs, through the C ABI, on two calls in a row, the second
with a smaller batch; both also against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2412_16434_amd as S
import workloads as W
from gpu_util import DEV, TOL, DeviceSessions, attn_errors, to_dev, to_host, widen

pytestmark = pytest.mark.gpu


def _cfg(**kw):
    base = dict(name="static", index=80, dtype="bf16", n_layers=1, n_q_heads=8, n_kv_heads=2, head_dim=128,
                block_size=16, n_blocks=4096, n_sessions=6, prefix_dist=("uniform", 200, 6000),
                new_dist=("uniform", 1, 150), sigma=1.0, scale=1.0 / np.sqrt(128.0), fresh_tables=False)
    base.update(kw)
    return W.WorkloadConfig(**base)


def _both(oracle_mod, cfg, seed, label):
    sess = W.make_sessions(cfg, seed)
    k_pool, v_pool, q, k_new, v_new = W.make_attn_inputs(cfg, sess, seed)
    ds = DeviceSessions(sess)
    cache = S.KVCache(to_dev(k_pool)[None], to_dev(v_pool)[None])
    qd, knd, vnd = to_dev(q), to_dev(k_new), to_dev(v_new)
    args = (cache, 0, qd, knd, vnd)
    tail = (ds.cu_new_lens, ds.prefix_lens, ds.table, sess.max_new_len, sess.max_prefix_len, cfg.scale)
    out_static = torch.full_like(qd, float("nan"))
    S.prefix_prefill_attn_static(*args, out_static, *tail)       # no workspace, no allocation inside the library
    torch.cuda.synchronize()
    ws_bytes = S.prefix_prefill_attn_workspace_bytes(cache, sess.n_sessions, cfg.n_q_heads, sess.total_new_tokens,
                                                     sess.max_new_len, sess.max_prefix_len)
    ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device=DEV) if ws_bytes else None
    out_ws = torch.full_like(qd, float("nan"))
    S.prefix_prefill_attn(*args, out_ws, *tail, workspace=ws)
    torch.cuda.synchronize()
    a, b = to_host(out_static), to_host(out_ws)
    assert np.all(np.isfinite(widen(a))), "non-finite values in the static entry point's output"
    tol_abs, tol_rel = TOL[cfg.dtype]
    d_abs, d_rel = attn_errors(a, widen(b))
    ref = oracle_mod.prefix_prefill_attn(k_pool, v_pool, q, k_new, v_new, sess.cu_new_lens, sess.prefix_lens,
                                         sess.block_table, cfg.scale)
    o_abs, o_rel = attn_errors(a, ref)
    print(f"[no-alloc] {label}: rows={a.shape[0]} vs workspace entry: max_abs={d_abs:.3e} rel_l2={d_rel:.3e} "
          f"bitwise_equal={np.array_equal(a, b)}; vs oracle: max_abs={o_abs:.3e} rel_l2={o_rel:.3e}", flush=True)
    assert d_abs <= tol_abs and d_rel <= tol_rel
    assert o_abs <= tol_abs and o_rel <= tol_rel


def test_two_calls_in_a_row_the_second_smaller(oracle_mod):
    # a batch whose long sessions are split along the key axis (partial results, counters and the work list all live in
    # the scratch array), then a smaller one that must not see anything the first left behind
    _both(oracle_mod, _cfg(), 61, "first call: 6 sessions, prefixes up to 6000")
    _both(oracle_mod, _cfg(n_sessions=2, prefix_dist=("uniform", 1, 300), new_dist=("uniform", 1, 40)), 62,
          "second call: 2 short sessions")


def test_decode_step_then_prefill_then_fp32(oracle_mod):
    # the decode kernel's slots and lists, then the work-item path again, then a shape that needs no scratch at all
    _both(oracle_mod, _cfg(n_sessions=12, prefix_dist=("uniform", 1, 3000), new_dist=("uniform", 1, 4)), 63,
          "decode step, 12 sessions")
    _both(oracle_mod, _cfg(n_sessions=3, prefix_dist=("uniform", 1, 900), new_dist=("uniform", 30, 90)), 64,
          "prefill turns, 3 sessions")
    _both(oracle_mod, _cfg(dtype="fp32", head_dim=64, n_q_heads=4, scale=0.125, n_sessions=2,
                           prefix_dist=("uniform", 1, 200), new_dist=("uniform", 1, 30), n_blocks=64), 65, "fp32, d = 64")
