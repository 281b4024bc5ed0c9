"""symph_kv_pack_tail / symph_kv_unpack_tail (write-back of what a turn added) against the byte-copy oracle."""
import numpy as np
import pytest
import torch

import paper_2412_16434_amd as S
import workloads as W
from gpu_util import DEV, to_dev, to_host

pytestmark = pytest.mark.gpu


def _cfg(**kw):
    base = dict(name="tail", index=80, dtype="bf16", n_layers=3, n_q_heads=8, n_kv_heads=2, head_dim=128, block_size=16,
                n_blocks=256, n_sessions=6, prefix_dist=("uniform", 0, 300), new_dist=("const", 1), sigma=1.0, scale=0.1)
    base.update(kw)
    return W.WorkloadConfig(**base)


def _begins(sess, seed):
    rng = np.random.default_rng(seed)
    P = sess.prefix_lens.astype(np.int64)
    pick = rng.integers(0, 4, size=P.shape[0])
    return np.where(pick == 0, 0, np.where(pick == 1, P, rng.integers(0, P + 1))).astype(np.int32)


def _sentinel_like(a):
    out = np.empty_like(a)
    (out if a.dtype == np.uint16 else out.view(np.uint32))[...] = W.SENTINEL16 if a.dtype == np.uint16 else 0x7FC00001
    return out


@pytest.mark.parametrize("kw", [
    dict(),
    dict(prefix_dist=("uniform", 0, 40), n_sessions=40, n_blocks=512),
    dict(n_layers=1, n_sessions=1, prefix_dist=("const", 700), n_blocks=128),
    dict(n_layers=7, block_size=8, n_blocks=512, prefix_dist=("uniform", 1, 90)),
    dict(dtype="fp32", n_kv_heads=3, head_dim=20, block_size=4, n_blocks=512, prefix_dist=("uniform", 1, 50)),
    dict(dtype="bf16", n_kv_heads=1, head_dim=6, block_size=4, n_blocks=512, prefix_dist=("uniform", 1, 50)),
    dict(n_kv_heads=8, n_q_heads=32, n_sessions=70, n_blocks=2048, prefix_dist=("uniform", 0, 300)),   # planes per lane: 2
])
def test_pack_tail_and_unpack_tail_match_the_oracle(oracle_mod, kw):
    cfg = _cfg(**kw)
    sess = W.make_sessions(cfg, 51)
    k_pool, v_pool = W.make_pool_host(cfg, sess, 51)
    begins = _begins(sess, 51)
    offs = oracle_mod.tail_offsets(sess.prefix_lens, begins)
    total = int(offs[-1])
    ref = oracle_mod.kv_pack_tail(k_pool, v_pool, sess.block_table, sess.prefix_lens, begins)

    cache = S.KVCache(to_dev(k_pool), to_dev(v_pool))
    table, dst = torch.from_numpy(sess.block_table).to(DEV), torch.from_numpy(sess.dst_block_table).to(DEV)
    pl, bg, of = (torch.from_numpy(a).to(DEV) for a in (sess.prefix_lens, begins, offs))
    n_bytes = S.kv_buffer_bytes(cache, total)
    assert n_bytes == ref.nbytes
    buf = torch.zeros(max(ref.size, 1), dtype=cache.k_pool.dtype, device=DEV)
    S.kv_pack_tail(cache, table, pl, bg, of, total, buf)
    torch.cuda.synchronize()
    assert to_host(buf)[: ref.size].tobytes() == ref.tobytes(), "pack_tail differs from the oracle"
    assert to_host(cache.k_pool).tobytes() == k_pool.tobytes() and to_host(cache.v_pool).tobytes() == v_pool.tobytes()

    ks, vs = _sentinel_like(k_pool), _sentinel_like(v_pool)
    oracle_mod.kv_unpack_tail(ks, vs, sess.dst_block_table, sess.prefix_lens, begins, ref)
    dcache = S.KVCache(to_dev(_sentinel_like(k_pool)), to_dev(_sentinel_like(v_pool)))
    S.kv_unpack_tail(dcache, dst, pl, bg, of, total, buf)
    torch.cuda.synchronize()
    assert to_host(dcache.k_pool).tobytes() == ks.tobytes(), "unpack_tail: K pool differs from the oracle"
    assert to_host(dcache.v_pool).tobytes() == vs.tobytes(), "unpack_tail: V pool differs from the oracle"


def test_tail_begin_outside_the_session_is_skipped(oracle_mod):
    cfg = _cfg(n_sessions=4, prefix_dist=("const", 40))
    sess = W.make_sessions(cfg, 52)
    k_pool, v_pool = W.make_pool_host(cfg, sess, 52)
    begins = np.array([10, -3, 41, 40], dtype=np.int32)        # sessions 1 and 2 are inconsistent, 3 has nothing new
    lens = np.array([30, 0, 0, 0], dtype=np.int64)
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    good = np.array([10, 40, 40, 40], dtype=np.int32)           # what the call must behave like
    ref = oracle_mod.kv_pack_tail(k_pool, v_pool, sess.block_table, sess.prefix_lens, good)
    cache = S.KVCache(to_dev(k_pool), to_dev(v_pool))
    buf = torch.zeros(ref.size, dtype=torch.bfloat16, device=DEV)
    S.kv_pack_tail(cache, torch.from_numpy(sess.block_table).to(DEV), torch.from_numpy(sess.prefix_lens).to(DEV),
                   torch.from_numpy(begins).to(DEV), torch.from_numpy(offs).to(DEV), 30, buf)
    torch.cuda.synchronize()
    assert to_host(buf).tobytes() == ref.tobytes()


def test_turn_cycle_write_back(oracle_mod):
    """A turn: the cache holds P_old tokens and a host copy of them exists (whole pack); the turn appends its K,V rows
    (symph_kv_append, every layer); pack_tail moves only the new rows; host copy + tail, plane by plane, must equal a
    whole pack of the cache at its new length."""
    cfg = _cfg(n_layers=2, n_sessions=5, n_blocks=512, prefix_dist=("uniform", 1, 200), new_dist=("uniform", 1, 60))
    sess = W.make_sessions(cfg, 53)
    k_pool, v_pool = W.make_pool_host(cfg, sess, 53)
    table_h = sess.table_with_room_for_the_new_turn()
    P_old = sess.prefix_lens
    P_new = (sess.prefix_lens + sess.new_lens).astype(np.int32)
    L, row = cfg.n_layers, cfg.n_kv_heads * cfg.head_dim
    cache = S.KVCache(to_dev(k_pool), to_dev(v_pool))
    table = torch.from_numpy(table_h).to(DEV)
    old_off = np.concatenate([[0], np.cumsum(P_old)]).astype(np.int64)
    host_copy = torch.zeros(int(old_off[-1]) * 2 * L * row, dtype=torch.bfloat16, device=DEV)
    S.kv_pack(cache, table, torch.from_numpy(P_old).to(DEV), torch.from_numpy(old_off).to(DEV), int(old_off[-1]), host_copy)
    rng = np.random.default_rng(53)
    T = sess.total_new_tokens
    new_rows = [(rng.standard_normal((2, T, cfg.n_kv_heads, cfg.head_dim)).astype(np.float32)) for _ in range(L)]
    cu = torch.from_numpy(sess.cu_new_lens).to(DEV)
    for layer in range(L):
        kn = torch.from_numpy(new_rows[layer][0]).to(DEV).to(torch.bfloat16)
        vn = torch.from_numpy(new_rows[layer][1]).to(DEV).to(torch.bfloat16)
        S.kv_append(cache, layer, kn, vn, cu, torch.from_numpy(P_old).to(DEV), table)
    new_off = np.concatenate([[0], np.cumsum(P_new)]).astype(np.int64)
    whole = torch.zeros(int(new_off[-1]) * 2 * L * row, dtype=torch.bfloat16, device=DEV)
    S.kv_pack(cache, table, torch.from_numpy(P_new).to(DEV), torch.from_numpy(new_off).to(DEV), int(new_off[-1]), whole)
    tail_off = oracle_mod.tail_offsets(P_new, P_old)
    tail = torch.zeros(int(tail_off[-1]) * 2 * L * row, dtype=torch.bfloat16, device=DEV)
    S.kv_pack_tail(cache, table, torch.from_numpy(P_new).to(DEV), torch.from_numpy(P_old).to(DEV),
                   torch.from_numpy(tail_off).to(DEV), int(tail_off[-1]), tail)
    torch.cuda.synchronize()
    hc, wh, tl = to_host(host_copy), to_host(whole), to_host(tail)
    for s in range(sess.n_sessions):
        Po, Pn = int(P_old[s]), int(P_new[s])
        for plane in range(2 * L):
            o0 = (int(old_off[s]) * 2 * L + plane * Po) * row
            t0 = (int(tail_off[s]) * 2 * L + plane * (Pn - Po)) * row
            w0 = (int(new_off[s]) * 2 * L + plane * Pn) * row
            joined = np.concatenate([hc[o0:o0 + Po * row], tl[t0:t0 + (Pn - Po) * row]])
            assert joined.tobytes() == wh[w0:w0 + Pn * row].tobytes()
    # and the whole pack is the oracle's, so the chain is anchored
    kh, vh = to_host(cache.k_pool), to_host(cache.v_pool)
    assert oracle_mod.kv_pack(kh, vh, table_h, P_new, new_off).tobytes() == wh.tobytes()
