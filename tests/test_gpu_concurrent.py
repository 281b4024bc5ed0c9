"""Config 5's shape of use: a batch of resumed turns runs attention on one stream while the K,V of newly arriving
sessions are unpacked into another cache on a second stream.  Both entry points are re-entrant and share nothing but
the device, so running them side by side must give exactly what each gives alone; both are checked against the oracle.
"""
import numpy as np
import pytest
import torch

import paper_2412_16434_amd as S
import workloads as W
from gpu_util import DEV, TOL, DeviceSessions, attn_errors, to_dev, to_host

pytestmark = pytest.mark.gpu


def sentinel_like(a):
    out = np.empty_like(a)
    out[...] = W.SENTINEL16   # bf16 bit patterns
    return out


def test_attention_and_unpack_on_two_streams(oracle_mod):
    acfg = W.scaled_config(W.get_config("mixed_resume"), n_layers=1, n_sessions=16, prefix_scale=1 / 16, new_scale=1 / 4,
                           n_blocks=2048, n_decode=12)
    asess = W.make_sessions(acfg)
    k_pool, v_pool, q, k_new, v_new = W.make_attn_inputs(acfg, asess)
    ref_out = oracle_mod.prefix_prefill_attn(k_pool, v_pool, q, k_new, v_new, asess.cu_new_lens, asess.prefix_lens,
                                             asess.block_table, acfg.scale)

    ucfg = W.scaled_config(W.get_config("mixed_resume_incoming"), n_layers=4, n_sessions=3, prefix_scale=1 / 16, n_blocks=128)
    usess = W.make_sessions(ucfg)
    uk, uv = W.make_pool_host(ucfg, usess)
    buf_host = oracle_mod.kv_pack(uk, uv, usess.block_table, usess.prefix_lens, usess.buf_token_offsets)
    ref_k, ref_v = sentinel_like(uk), sentinel_like(uv)
    oracle_mod.kv_unpack(ref_k, ref_v, usess.dst_block_table, usess.prefix_lens, usess.buf_token_offsets, buf_host)

    ads, uds = DeviceSessions(asess), DeviceSessions(usess)
    acache = S.KVCache(to_dev(k_pool)[None], to_dev(v_pool)[None])
    qd, knd, vnd = to_dev(q), to_dev(k_new), to_dev(v_new)
    ws_bytes = S.prefix_prefill_attn_workspace_bytes(acache, asess.n_sessions, acfg.n_q_heads, asess.total_new_tokens,
                                                     asess.max_new_len, asess.max_prefix_len)
    ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device=DEV)
    buf = to_dev(buf_host)
    sa, su = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for rep in range(3):  # fresh outputs every time; the two streams are released together
        out = torch.full_like(qd, float("nan"))
        ucache = S.KVCache(to_dev(sentinel_like(uk)), to_dev(sentinel_like(uv)))
        torch.cuda.synchronize()
        S.prefix_prefill_attn(acache, 0, qd, knd, vnd, out, ads.cu_new_lens, ads.prefix_lens, ads.table,
                              asess.max_new_len, asess.max_prefix_len, acfg.scale, workspace=ws, stream=sa)
        S.kv_unpack(ucache, uds.dst_table, uds.prefix_lens, uds.offsets, usess.total_prefix_tokens, buf, stream=su)
        S.prefix_prefill_attn(acache, 0, qd, knd, vnd, out, ads.cu_new_lens, ads.prefix_lens, ads.table,
                              asess.max_new_len, asess.max_prefix_len, acfg.scale, workspace=ws, stream=sa)
        torch.cuda.synchronize()
        max_abs, rel = attn_errors(to_host(out), ref_out)
        print(f"[concurrent] rep {rep}: attention max_abs={max_abs:.3e} rel_l2={rel:.3e}", flush=True)
        assert max_abs <= TOL["bf16"][0] and rel <= TOL["bf16"][1]
        assert to_host(ucache.k_pool).tobytes() == ref_k.tobytes(), "unpack beside attention: K pool differs"
        assert to_host(ucache.v_pool).tobytes() == ref_v.tobytes(), "unpack beside attention: V pool differs"
