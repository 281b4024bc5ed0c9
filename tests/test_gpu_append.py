"""symph_kv_append against the oracle: the new turn's K,V rows of a layer land behind each session's prefix in the paged
cache, bit for bit, and nothing else in the pools changes (Symphony Sec. 2.1 "KV Cache", Sec. 3.3).  A whole turn cycle
closes the loop: attention of turn 1, append of its K,V, attention of turn 2 against the grown cache."""
import numpy as np
import pytest
import torch

import paper_2412_16434_amd as S
import workloads as W
from gpu_util import DEV, TOL, DeviceSessions, attn_errors, gpu_attention, to_dev, to_host

pytestmark = pytest.mark.gpu


def _cfg(**kw):
    base = dict(name="append", index=50, dtype="bf16", n_layers=3, n_q_heads=8, n_kv_heads=2, head_dim=128,
                block_size=16, n_blocks=160, n_sessions=6, prefix_dist=("uniform", 0, 120), new_dist=("uniform", 0, 45),
                sigma=1.0, scale=1.0 / np.sqrt(128.0), fresh_tables=False)
    base.update(kw)
    return W.WorkloadConfig(**base)


def new_rows(cfg, sess, seed):
    rng = np.random.default_rng(seed)
    shape = (sess.total_new_tokens, cfg.n_kv_heads, cfg.head_dim)
    if cfg.dtype == "bf16":
        return (W.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32)),
                W.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32)))
    return rng.standard_normal(shape).astype(np.float32), rng.standard_normal(shape).astype(np.float32)


@pytest.mark.parametrize("kw", [
    dict(),
    dict(prefix_dist=("const", 0), new_dist=("uniform", 1, 40)),                  # first turn: cache empty so far
    dict(prefix_dist=("const", 16), new_dist=("const", 16)),                      # exactly one more full block
    dict(prefix_dist=("const", 15), new_dist=("const", 2)),                       # crosses a block boundary
    dict(new_dist=("const", 1)),                                                  # decode steps
    dict(block_size=8, n_blocks=320),
    dict(dtype="fp32", n_kv_heads=3, head_dim=20, block_size=4, n_blocks=400),    # 240-byte rows
    dict(dtype="bf16", n_kv_heads=1, head_dim=6, block_size=4, n_blocks=400),     # 12-byte rows: 4-byte path
])
def test_append_matches_the_oracle(oracle_mod, kw):
    cfg = _cfg(**kw)
    sess = W.make_sessions(cfg, 61)
    if sess.total_new_tokens == 0:
        pytest.skip("no new tokens drawn")
    table = sess.table_with_room_for_the_new_turn()
    k_pool, v_pool = W.make_pool_host(cfg, sess, 61)
    k_new, v_new = new_rows(cfg, sess, 62)
    cache = S.KVCache(to_dev(k_pool), to_dev(v_pool))
    ds = DeviceSessions(sess)
    for layer in (cfg.n_layers - 1, 0):
        oracle_mod.kv_append(k_pool, v_pool, layer, k_new, v_new, sess.cu_new_lens, sess.prefix_lens, table)
        S.kv_append(cache, layer, to_dev(k_new), to_dev(v_new), ds.cu_new_lens, ds.prefix_lens,
                    torch.from_numpy(table).to(DEV))
        torch.cuda.synchronize()
        assert to_host(cache.k_pool).tobytes() == k_pool.tobytes(), f"append, layer {layer}: K pool differs"
        assert to_host(cache.v_pool).tobytes() == v_pool.tobytes(), f"append, layer {layer}: V pool differs"


def test_rows_with_block_ids_outside_the_cache_are_skipped(oracle_mod):
    cfg = _cfg(n_layers=1, n_sessions=3, prefix_dist=("const", 10), new_dist=("const", 30))
    sess = W.make_sessions(cfg, 63)
    table = sess.table_with_room_for_the_new_turn()
    bad = table.copy()
    bad[1, 1] = cfg.n_blocks + 5          # second block of session 1: positions 16..31
    bad[2, 2] = -1
    k_pool, v_pool = W.make_pool_host(cfg, sess, 63)
    k_new, v_new = new_rows(cfg, sess, 64)
    cache = S.KVCache(to_dev(k_pool), to_dev(v_pool))
    ds = DeviceSessions(sess)
    S.kv_append(cache, 0, to_dev(k_new), to_dev(v_new), ds.cu_new_lens, ds.prefix_lens, torch.from_numpy(bad).to(DEV))
    torch.cuda.synchronize()
    # the oracle appends the rows that do have a block: drop the others from its input
    keep = np.ones(sess.total_new_tokens, dtype=bool)
    for s, blk in ((1, 1), (2, 2)):
        for i in range(int(sess.new_lens[s])):
            if (int(sess.prefix_lens[s]) + i) // cfg.block_size == blk:
                keep[sess.cu_new_lens[s] + i] = False
    exp_k, exp_v = k_pool.copy(), v_pool.copy()
    oracle_mod.kv_append(exp_k, exp_v, 0, k_new, v_new, sess.cu_new_lens, sess.prefix_lens, table)
    for s, blk in ((1, 1), (2, 2)):        # what the oracle wrote into the blocks the GPU must skip is undone
        exp_k[0, table[s, blk]] = k_pool[0, table[s, blk]]
        exp_v[0, table[s, blk]] = v_pool[0, table[s, blk]]
    assert to_host(cache.k_pool).tobytes() == exp_k.tobytes() and to_host(cache.v_pool).tobytes() == exp_v.tobytes()
    assert not keep.all()


def test_turn_cycle_attend_append_attend(oracle_mod):
    """Turn 1 attends with its K,V alongside the cache; its K,V are appended; turn 2 (fresh queries, fresh K,V) attends
    against the grown cache.  The oracle runs the same cycle on the host."""
    cfg = _cfg(n_layers=1, n_sessions=5, prefix_dist=("uniform", 0, 200), new_dist=("uniform", 1, 60), n_blocks=256)
    sess = W.make_sessions(cfg, 65)
    table = sess.table_with_room_for_the_new_turn()
    k_pool, v_pool, q, k_new, v_new = W.make_attn_inputs(cfg, sess, 65)
    sess1 = W.SessionBatch(cfg, sess.prefix_lens, sess.new_lens, table, None, sess.buf_token_offsets, sess.cu_new_lens)
    got1 = gpu_attention(cfg, sess1, (k_pool, v_pool, q, k_new, v_new))
    ref1 = oracle_mod.prefix_prefill_attn(k_pool, v_pool, q, k_new, v_new, sess.cu_new_lens, sess.prefix_lens, table,
                                          cfg.scale)
    m1, r1 = attn_errors(got1, ref1)
    assert m1 <= TOL["bf16"][0] and r1 <= TOL["bf16"][1]

    ds = DeviceSessions(sess1)
    cache = S.KVCache(to_dev(k_pool)[None], to_dev(v_pool)[None])
    S.kv_append(cache, 0, to_dev(k_new), to_dev(v_new), ds.cu_new_lens, ds.prefix_lens, ds.table)
    torch.cuda.synchronize()
    kp, vp = k_pool[None].copy(), v_pool[None].copy()
    oracle_mod.kv_append(kp, vp, 0, k_new, v_new, sess.cu_new_lens, sess.prefix_lens, table)
    assert to_host(cache.k_pool).tobytes() == kp.tobytes() and to_host(cache.v_pool).tobytes() == vp.tobytes()

    # turn 2: one token per session against the grown cache (the table still has room only up to P + N: N2 = 0 would
    # be empty, so the turn reuses the last appended position's block when P + N is not a block boundary)
    grown = (sess.prefix_lens + sess.new_lens).astype(np.int32)
    n2 = np.ones(sess.n_sessions, dtype=np.int32)
    cu2 = np.arange(sess.n_sessions + 1, dtype=np.int32)
    rng = np.random.default_rng(66)
    shape = (sess.n_sessions, cfg.n_kv_heads, cfg.head_dim)
    q2 = W.f32_to_bf16_bits(rng.standard_normal((sess.n_sessions, cfg.n_q_heads, cfg.head_dim)).astype(np.float32))
    k2 = W.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    v2 = W.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    sess2 = W.SessionBatch(cfg, grown, n2, table, None, sess.buf_token_offsets, cu2)
    got2 = gpu_attention(cfg, sess2, (to_host(cache.k_pool)[0], to_host(cache.v_pool)[0], q2, k2, v2))
    ref2 = oracle_mod.prefix_prefill_attn(kp[0], vp[0], q2, k2, v2, cu2, grown, table, cfg.scale)
    m2, r2 = attn_errors(got2, ref2)
    print(f"[turn cycle] turn 1 max_abs={m1:.3e} rel_l2={r1:.3e}; turn 2 max_abs={m2:.3e} rel_l2={r2:.3e}", flush=True)
    assert m2 <= TOL["bf16"][0] and r2 <= TOL["bf16"][1]
