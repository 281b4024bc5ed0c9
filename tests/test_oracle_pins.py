"""Pins for the CPU oracle: everything here checks ``oracle/`` against something other than itself.

pack / unpack (a permutation copy; Symphony Sec. 3.2 node manager, Sec. 3.3 memory management, Sec. 3.5):
  * tagged pools: every pool element carries its own coordinates, so each buffer element can be decoded and
    checked against the layout rules without recomputing any offset;
  * a numpy route (take blocks, reshape, concatenate) for the whole buffer;
  * the identity-table special case, which is a plain memcpy;
  * round trips and sentinel bytes;
  * the cache sizes the paper prints (tests/golden/kv_cache_sizes.txt).
attention (Sec. 2.1: A_h = softmax(Q K^T / sqrt(d)), y = concat_h A_h V_h; causal because a token needs the keys
and values of all prior tokens only):
  * brute force: contiguous K,V rebuilt token by token, full (P+N)^2 causal score matrix, scipy softmax;
  * torch's scaled_dot_product_attention in fp64 (library routine), MHA (G = 1) and GQA;
  * cached-prefix result == full recompute; split-point invariance; block-id permutation invariance;
  * weights sum to one; closed forms (equal keys, constant V, one dominant key, single token).
"""
import os

import numpy as np
import pytest
import scipy.special

import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------------------------------------
# helpers that do NOT use the oracle
# --------------------------------------------------------------------------------------------------------
def to_f64(a: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns / fp32 through torch's own conversion (a library route)."""
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    return a.astype(np.float64)


def contiguous_kv(pool: np.ndarray, table_row: np.ndarray, P: int, new: np.ndarray) -> np.ndarray:
    """[P+N][H_kv][d] fp64 for one session, rebuilt token by token (slow on purpose)."""
    bs = pool.shape[1]
    rows = [pool[table_row[t // bs], t % bs] for t in range(P)]
    rows += [new[i] for i in range(new.shape[0])]
    return to_f64(np.stack(rows)) if rows else np.zeros((0,) + pool.shape[2:])


def brute_force_attention(k_pool, v_pool, q, k_new, v_new, sess: W.SessionBatch, scale: float) -> np.ndarray:
    cfg = sess.cfg
    G = cfg.group
    out = np.zeros(q.shape, dtype=np.float64)
    sc = float(np.float32(scale))
    for s in range(sess.n_sessions):
        P, N = int(sess.prefix_lens[s]), int(sess.new_lens[s])
        a, b = int(sess.cu_new_lens[s]), int(sess.cu_new_lens[s + 1])
        if N == 0:
            continue
        K = contiguous_kv(k_pool, sess.block_table[s], P, k_new[a:b])
        V = contiguous_kv(v_pool, sess.block_table[s], P, v_new[a:b])
        # queries for every position: only the last N exist; earlier rows are dummies that are discarded
        Qn = to_f64(q[a:b])
        n = P + N
        causal = np.tril(np.ones((n, n), dtype=bool))
        for h in range(cfg.n_q_heads):
            g = h // G
            Qfull = np.zeros((n, cfg.head_dim))
            Qfull[P:] = Qn[:, h]
            scores = sc * (Qfull @ K[:, g].T)
            scores = np.where(causal, scores, -np.inf)
            A = scipy.special.softmax(scores, axis=1)
            out[a:b, h] = (A @ V[:, g])[P:]
    return out


def small_cfg(dtype="bf16", **kw):
    base = dict(name="pin", index=9, dtype=dtype, n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=8, block_size=4,
                n_blocks=40, n_sessions=3, prefix_dist=("uniform", 1, 19), new_dist=("uniform", 1, 7), sigma=1.0,
                scale=1.0 / np.sqrt(8.0))
    base.update(kw)
    return W.WorkloadConfig(**base)


# --------------------------------------------------------------------------------------------------------
# pack / unpack
# --------------------------------------------------------------------------------------------------------
def tagged_pools(cfg):
    """fp32-sized pools whose 32-bit patterns encode (kv, layer, block, slot, head, dim)."""
    L, nb, bs, H, d = cfg.n_layers, cfg.n_blocks, cfg.block_size, cfg.n_kv_heads, cfg.head_dim
    l, b, o, g, c = np.meshgrid(np.arange(L), np.arange(nb), np.arange(bs), np.arange(H), np.arange(d), indexing="ij")

    def tag(kv):
        t = (((((kv * L + l) * nb + b) * bs + o) * H + g) * d + c).astype(np.uint32)
        return t.view(np.float32).copy()
    return tag(0), tag(1)


def decode_tag(t, cfg):
    L, nb, bs, H, d = cfg.n_layers, cfg.n_blocks, cfg.block_size, cfg.n_kv_heads, cfg.head_dim
    t = t.astype(np.int64)
    c = t % d; t //= d
    g = t % H; t //= H
    o = t % bs; t //= bs
    b = t % nb; t //= nb
    l = t % L; t //= L
    return t, l, b, o, g, c   # t is now kv


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_pack_tagged_pool_layout(oracle_mod, seed):
    cfg = small_cfg("fp32", n_sessions=4, prefix_dist=("uniform", 0, 23))
    sess = W.make_sessions(cfg, seed)
    k_pool, v_pool = tagged_pools(cfg)
    buf = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)
    assert buf.size * 4 == sess.payload_bytes()
    kv, l, b, o, g, c = decode_tag(buf.view(np.uint32), cfg)
    # walk the buffer in order and state what each position must hold, from the layout rules alone
    pos = 0
    H, d, bs = cfg.n_kv_heads, cfg.head_dim, cfg.block_size
    for s in range(sess.n_sessions):
        P = int(sess.prefix_lens[s])
        for layer in range(cfg.n_layers):
            for which in (0, 1):
                for t in range(P):
                    sl = slice(pos, pos + H * d)
                    assert np.all(kv[sl] == which) and np.all(l[sl] == layer)
                    assert np.all(b[sl] == sess.block_table[s, t // bs]) and np.all(o[sl] == t % bs)
                    assert np.array_equal(g[sl], np.repeat(np.arange(H), d))
                    assert np.array_equal(c[sl], np.tile(np.arange(d), H))
                    pos += H * d
    assert pos == buf.size


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_pack_matches_numpy_take_route(oracle_mod, dtype):
    cfg = small_cfg(dtype, n_sessions=5, n_layers=3, n_blocks=64, prefix_dist=("uniform", 0, 30))
    sess = W.make_sessions(cfg, 11)
    k_pool, v_pool = W.make_pool_host(cfg, sess, 5)
    pieces = []
    nblk = sess.blocks_per_session()
    for s in range(sess.n_sessions):
        P = int(sess.prefix_lens[s])
        ids = sess.block_table[s, : nblk[s]]
        for layer in range(cfg.n_layers):
            for pool in (k_pool, v_pool):
                pieces.append(np.take(pool[layer], ids, axis=0).reshape(-1, cfg.row_elems)[:P].ravel())
    expect = np.concatenate(pieces) if pieces else np.zeros(0, k_pool.dtype)
    got = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)
    assert got.tobytes() == expect.tobytes()


def test_pack_identity_table_is_memcpy(oracle_mod):
    cfg = small_cfg("bf16", n_layers=1, n_sessions=1, n_blocks=8, prefix_dist=("const", 32), fresh_tables=False)
    sess = W.make_sessions(cfg, 3)
    sess.block_table[0, :] = np.arange(8, dtype=np.int32)
    k_pool, v_pool = W.make_pool_host(cfg, sess, 3)
    got = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)
    assert got.tobytes() == k_pool.tobytes() + v_pool.tobytes()


def test_locate_against_tagged_pool(oracle_mod):
    cfg = small_cfg("fp32", n_sessions=3, prefix_dist=("uniform", 3, 23))
    sess = W.make_sessions(cfg, 4)
    k_pool, v_pool = tagged_pools(cfg)
    buf = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)
    rng = np.random.default_rng(0)
    ls, bst = cfg.layer_elems, cfg.block_elems
    for _ in range(200):
        s = int(rng.integers(sess.n_sessions))
        t = int(rng.integers(sess.prefix_lens[s]))
        layer, kv = int(rng.integers(cfg.n_layers)), int(rng.integers(2))
        pe, be = oracle_mod.kv_locate(ls, bst, cfg.n_layers, cfg.block_size, cfg.n_kv_heads, cfg.head_dim,
                                      sess.block_table, sess.prefix_lens, sess.buf_token_offsets, s, layer, kv, t)
        pool = (v_pool if kv else k_pool).ravel()
        assert np.array_equal(pool[pe: pe + cfg.row_elems].view(np.uint32), buf[be: be + cfg.row_elems].view(np.uint32))
        kvd, l, b, o, g, c = decode_tag(pool[pe: pe + 1].view(np.uint32), cfg)
        assert (kvd[0], l[0], b[0], o[0], g[0], c[0]) == (kv, layer, sess.block_table[s, t // cfg.block_size],
                                                          t % cfg.block_size, 0, 0)


def test_row_map_against_tagged_pool(oracle_mod):
    """The table form of the index function (what the full-size GPU parity tests compare whole buffers with): walk
    the buffer in order, state from the layout rules alone which (K|V, layer, block, slot) each row is, and require
    the map to name exactly that row of the tagged pool; every row is named, none twice."""
    cfg = small_cfg("fp32", n_sessions=5, n_layers=3, prefix_dist=("uniform", 0, 23))
    sess = W.make_sessions(cfg, 6)
    k_pool, v_pool = tagged_pools(cfg)
    pool_elem, kv = oracle_mod.kv_row_map(cfg.layer_elems, cfg.block_elems, cfg.n_layers, cfg.block_size,
                                          cfg.n_kv_heads, cfg.head_dim, sess.block_table, sess.prefix_lens,
                                          sess.buf_token_offsets)
    assert pool_elem.size == sess.total_prefix_tokens * 2 * cfg.n_layers and pool_elem.min() >= 0 and kv.max() <= 1
    r = 0
    for s in range(sess.n_sessions):
        for layer in range(cfg.n_layers):
            for which in (0, 1):
                for tok in range(int(sess.prefix_lens[s])):
                    pool = (v_pool if which else k_pool).ravel()
                    kvd, l, b, o, g, c = decode_tag(pool[pool_elem[r]: pool_elem[r] + 1].view(np.uint32), cfg)
                    assert kv[r] == which
                    assert (kvd[0], l[0], b[0], o[0], g[0], c[0]) == (
                        which, layer, sess.block_table[s, tok // cfg.block_size], tok % cfg.block_size, 0, 0)
                    r += 1
    assert r == pool_elem.size
    assert np.unique(pool_elem * 2 + kv).size == pool_elem.size      # (no block is shared in this batch)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_unpack_round_trips_and_leaves_other_bytes_alone(oracle_mod, dtype):
    cfg = small_cfg(dtype, n_sessions=6, n_layers=2, n_blocks=96, prefix_dist=("geometric", 9.0, 1, 29))
    sess = W.make_sessions(cfg, 21)
    assert np.all(sess.prefix_lens % cfg.block_size != 0)       # every last block partial
    k_pool, v_pool = W.make_pool_host(cfg, sess, 8)
    buf = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)

    # (a) same table: the pool does not change
    k2, v2 = k_pool.copy(), v_pool.copy()
    oracle_mod.kv_unpack(k2, v2, sess.block_table, sess.prefix_lens, sess.buf_token_offsets, buf)
    assert k2.tobytes() == k_pool.tobytes() and v2.tobytes() == v_pool.tobytes()

    # (b) fresh table into a sentinel pool: packing again gives the same buffer ...
    ks = np.empty_like(k_pool); vs = np.empty_like(v_pool)
    sent = 0x7FC1 if dtype == "bf16" else 0x7FC00001
    uview = (lambda a: a) if dtype == "bf16" else (lambda a: a.view(np.uint32))
    uview(ks)[...] = sent; uview(vs)[...] = sent
    oracle_mod.kv_unpack(ks, vs, sess.dst_block_table, sess.prefix_lens, sess.buf_token_offsets, buf)
    again = oracle_mod.kv_pack(ks, vs, sess.dst_block_table, sess.prefix_lens, sess.buf_token_offsets)
    assert again.tobytes() == buf.tobytes()
    # ... and exactly the valid token slots were written, nothing else
    written = np.zeros(ks.shape[:3], dtype=bool)      # [L][block][slot]
    for s in range(sess.n_sessions):
        for t in range(int(sess.prefix_lens[s])):
            written[:, sess.dst_block_table[s, t // cfg.block_size], t % cfg.block_size] = True
    for pool in (ks, vs):
        is_sent = np.all(uview(pool) == sent, axis=(3, 4))
        assert np.array_equal(is_sent, ~written)
    # and each written slot holds the source token's row
    for s in range(sess.n_sessions):
        for t in range(int(sess.prefix_lens[s])):
            j, o = t // cfg.block_size, t % cfg.block_size
            assert np.array_equal(ks[:, sess.dst_block_table[s, j], o], k_pool[:, sess.block_table[s, j], o])
            assert np.array_equal(vs[:, sess.dst_block_table[s, j], o], v_pool[:, sess.block_table[s, j], o])


@pytest.mark.parametrize("lo,hi", [(0, 1), (1, 3), (2, 2), (0, 4), (3, 4)])
def test_layer_range_pack_tagged_pool(oracle_mod, lo, hi):
    """Layers lo..hi-1 only (Sec. 3.3: K,V travel layer by layer).  Tagged pools again: every buffer element of a
    moved layer decodes to the coordinates the layout rules give, every other element keeps the sentinel it had, and a
    layer of a session is ONE contiguous chunk of 2*P rows at (off[s]*2L + 2*layer*P) rows (closed form)."""
    cfg = small_cfg("fp32", n_layers=4, n_sessions=4, prefix_dist=("uniform", 0, 23))
    sess = W.make_sessions(cfg, 21)
    k_pool, v_pool = tagged_pools(cfg)
    H, d, bs, L = cfg.n_kv_heads, cfg.head_dim, cfg.block_size, cfg.n_layers
    row = H * d
    sentinel = np.uint32(0xFFFFFFFF)
    buf = np.full(sess.payload_bytes() // 4, sentinel, dtype=np.uint32).view(np.float32)
    oracle_mod.kv_pack_layers(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets, buf, lo, hi)
    bits = buf.view(np.uint32)
    kv, l, b, o, g, c = decode_tag(bits, cfg)
    for s in range(sess.n_sessions):
        P = int(sess.prefix_lens[s])
        base = int(sess.buf_token_offsets[s]) * 2 * L * row
        for layer in range(L):
            chunk = slice(base + 2 * layer * P * row, base + 2 * (layer + 1) * P * row)
            if not (lo <= layer < hi):
                assert np.all(bits[chunk] == sentinel)
                continue
            assert np.all(l[chunk] == layer)
            assert np.array_equal(kv[chunk], np.repeat([0, 1], P * row))
            t = np.tile(np.repeat(np.arange(P), row), 2)
            assert np.array_equal(b[chunk], sess.block_table[s][t // bs]) and np.array_equal(o[chunk], t % bs)
            assert np.array_equal(g[chunk], np.tile(np.repeat(np.arange(H), d), 2 * P))
            assert np.array_equal(c[chunk], np.tile(np.arange(d), 2 * P * H))


def test_layer_ranges_compose_to_the_whole(oracle_mod):
    """Disjoint layer ranges, in any order, give exactly the one-shot buffer / pools; an unpacked range leaves the
    other layers of the pools untouched."""
    cfg = small_cfg("bf16", n_layers=5, n_sessions=4, n_blocks=64, prefix_dist=("uniform", 0, 30))
    sess = W.make_sessions(cfg, 22)
    k_pool, v_pool = W.make_pool_host(cfg, sess, 22)
    whole = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)
    buf = np.full_like(whole, 0x7FC1)
    for lo, hi in [(3, 5), (0, 1), (1, 3)]:
        oracle_mod.kv_pack_layers(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets, buf, lo, hi)
    assert buf.tobytes() == whole.tobytes()

    ref_k, ref_v = np.full_like(k_pool, 0x7FC1), np.full_like(v_pool, 0x7FC1)
    oracle_mod.kv_unpack(ref_k, ref_v, sess.dst_block_table, sess.prefix_lens, sess.buf_token_offsets, whole)
    got_k, got_v = np.full_like(k_pool, 0x7FC1), np.full_like(v_pool, 0x7FC1)
    oracle_mod.kv_unpack_layers(got_k, got_v, sess.dst_block_table, sess.prefix_lens, sess.buf_token_offsets, whole, 1, 3)
    assert np.all(got_k[[0, 3, 4]] == 0x7FC1) and np.all(got_v[[0, 3, 4]] == 0x7FC1)
    assert got_k[1:3].tobytes() == ref_k[1:3].tobytes() and got_v[1:3].tobytes() == ref_v[1:3].tobytes()
    for lo, hi in [(3, 5), (0, 1)]:
        oracle_mod.kv_unpack_layers(got_k, got_v, sess.dst_block_table, sess.prefix_lens, sess.buf_token_offsets, whole,
                                    lo, hi)
    assert got_k.tobytes() == ref_k.tobytes() and got_v.tobytes() == ref_v.tobytes()


def test_batch_layer_major_buffer_tagged_pool(oracle_mod):
    """The layer -> session -> K|V -> token buffer: walk it in that order and state, from the layout rule alone, which
    tagged pool row every position must hold; untouched layers keep their sentinel; a layer of the whole batch is one
    contiguous piece of 2 * total rows at row l * 2 * total."""
    cfg = small_cfg("fp32", n_sessions=4, n_layers=3, prefix_dist=("uniform", 0, 23))
    sess = W.make_sessions(cfg, 8)
    k_pool, v_pool = tagged_pools(cfg)
    H, d, bs, L = cfg.n_kv_heads, cfg.head_dim, cfg.block_size, cfg.n_layers
    row, total = H * d, sess.total_prefix_tokens
    for lo, hi in ((0, 3), (1, 2), (2, 3), (1, 1)):
        buf = np.full(total * 2 * L * row, -5.0, dtype=np.float32)
        oracle_mod.kv_pack_batch_layers(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets, buf,
                                        lo, hi)
        kv, l, b, o, g, c = decode_tag(buf.view(np.uint32), cfg)
        pos = 0
        for layer in range(L):
            assert pos == layer * 2 * total * row                       # one contiguous piece per layer
            for s in range(sess.n_sessions):
                for which in (0, 1):
                    for tok in range(int(sess.prefix_lens[s])):
                        sl = slice(pos, pos + row)
                        if lo <= layer < hi:
                            assert np.all(kv[sl] == which) and np.all(l[sl] == layer)
                            assert np.all(b[sl] == sess.block_table[s, tok // bs]) and np.all(o[sl] == tok % bs)
                            assert np.array_equal(g[sl], np.repeat(np.arange(H), d))
                            assert np.array_equal(c[sl], np.tile(np.arange(d), H))
                        else:
                            assert np.all(buf[sl] == -5.0)
                        pos += row
        assert pos == buf.size


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_batch_layer_major_buffer_is_the_session_major_one_reordered(oracle_mod, dtype):
    """Same rows, other order: cut the session-major buffer (pinned above) into its (session, layer) chunks with numpy
    and concatenate them layer by layer; scatter from the layer-major buffer into a fresh table and gather again."""
    cfg = small_cfg(dtype, n_sessions=5, n_layers=3, n_blocks=96, prefix_dist=("uniform", 0, 30), fresh_tables=True)
    sess = W.make_sessions(cfg, 12)
    k_pool, v_pool = W.make_pool_host(cfg, sess, 5)
    row, L = cfg.row_elems, cfg.n_layers
    sm = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)
    pieces = []
    for layer in range(L):
        for s in range(sess.n_sessions):
            P = int(sess.prefix_lens[s])
            a = (int(sess.buf_token_offsets[s]) * 2 * L + 2 * layer * P) * row
            pieces.append(sm[a: a + 2 * P * row])
    expect = np.concatenate(pieces)
    lm = np.zeros_like(sm)
    oracle_mod.kv_pack_batch_layers(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets, lm, 0, L)
    assert lm.tobytes() == expect.tobytes()
    # scatter through the fresh table, layer ranges one at a time, then the session-major gather from there is `sm`
    k2, v2 = k_pool.copy(), v_pool.copy()
    for layer in range(L):
        oracle_mod.kv_unpack_batch_layers(k2, v2, sess.dst_block_table, sess.prefix_lens, sess.buf_token_offsets, lm,
                                          layer, layer + 1)
    again = oracle_mod.kv_pack(k2, v2, sess.dst_block_table, sess.prefix_lens, sess.buf_token_offsets)
    assert again.tobytes() == sm.tobytes()
    # and nothing but the destination slots changed
    changed_k = np.nonzero((k2 != k_pool).reshape(L, cfg.n_blocks, -1).any(axis=2))
    assert set(changed_k[1]) <= set(sess.owned_blocks(dst=True).tolist())


def test_append_places_rows_by_position(oracle_mod):
    """Appended K,V rows land at position P_s + i of their session (checked with tagged new rows and by reading the
    pools back through the table, a numpy route), and every other element of the pools keeps its tag."""
    cfg = small_cfg("fp32", n_layers=3, n_sessions=4, n_blocks=64, prefix_dist=("uniform", 0, 23), new_dist=("uniform", 0, 9))
    sess = W.make_sessions(cfg, 31)
    table = sess.table_with_room_for_the_new_turn()
    k_pool, v_pool = tagged_pools(cfg)
    k0, v0 = k_pool.copy(), v_pool.copy()
    T, H, d, bs = sess.total_new_tokens, cfg.n_kv_heads, cfg.head_dim, cfg.block_size
    tag_new = lambda kv: (0x40000000 + (kv * T * H * d) + np.arange(T * H * d, dtype=np.uint32)).view(np.float32).reshape(T, H, d)
    k_new, v_new = tag_new(0), tag_new(1)
    layer = 1
    oracle_mod.kv_append(k_pool, v_pool, layer, k_new, v_new, sess.cu_new_lens, sess.prefix_lens, table)
    touched = np.zeros(k_pool.shape[:3], dtype=bool)
    for s in range(sess.n_sessions):
        P, a = int(sess.prefix_lens[s]), int(sess.cu_new_lens[s])
        for i in range(int(sess.new_lens[s])):
            pos = P + i
            b, o = table[s, pos // bs], pos % bs
            assert np.array_equal(k_pool[layer, b, o].view(np.uint32), k_new[a + i].view(np.uint32))
            assert np.array_equal(v_pool[layer, b, o].view(np.uint32), v_new[a + i].view(np.uint32))
            touched[layer, b, o] = True
    assert np.array_equal(k_pool.view(np.uint32)[~touched], k0.view(np.uint32)[~touched])
    assert np.array_equal(v_pool.view(np.uint32)[~touched], v0.view(np.uint32)[~touched])


def test_append_then_attend_equals_attending_the_new_rows_directly(oracle_mod):
    """The last token of a turn, computed (a) with the turn's K,V passed alongside the cache and (b) after appending
    the turn's first N-1 tokens to the cache and passing only the last one, sees the same keys: same output row."""
    cfg = small_cfg("fp32", n_layers=1, n_sessions=3, n_blocks=64, prefix_dist=("uniform", 0, 23), new_dist=("uniform", 2, 9))
    sess = W.make_sessions(cfg, 32)
    k_pool, v_pool, q, k_new, v_new = W.make_attn_inputs(cfg, sess, 32)
    direct = oracle_mod.prefix_prefill_attn(k_pool, v_pool, q, k_new, v_new, sess.cu_new_lens, sess.prefix_lens,
                                            sess.block_table, cfg.scale)
    table = sess.table_with_room_for_the_new_turn()
    # append all but the last token of every session
    head_rows = np.concatenate([np.arange(sess.cu_new_lens[s], sess.cu_new_lens[s + 1] - 1) for s in range(sess.n_sessions)])
    last_rows = sess.cu_new_lens[1:] - 1
    cu_head = np.zeros(sess.n_sessions + 1, np.int32)
    cu_head[1:] = np.cumsum(sess.new_lens - 1)
    kp, vp = k_pool[None].copy(), v_pool[None].copy()
    oracle_mod.kv_append(kp, vp, 0, k_new[head_rows], v_new[head_rows], cu_head, sess.prefix_lens, table)
    longer = (sess.prefix_lens + sess.new_lens - 1).astype(np.int32)
    cu_one = np.arange(sess.n_sessions + 1, dtype=np.int32)
    after = oracle_mod.prefix_prefill_attn(kp[0], vp[0], q[last_rows], k_new[last_rows], v_new[last_rows], cu_one, longer,
                                           table, cfg.scale)
    assert np.allclose(after, direct[last_rows], rtol=1e-12, atol=1e-14)


def test_pack_preserves_nan_payloads_and_negative_zero(oracle_mod):
    cfg = small_cfg("bf16", n_sessions=2, n_layers=1, n_blocks=16, prefix_dist=("const", 7))
    sess = W.make_sessions(cfg, 5)
    k_pool, v_pool = W.make_pool_host(cfg, sess, 5, kind="counter")    # raw bit patterns: NaNs, infs, -0 included
    k_pool[0, sess.block_table[0, 0], 0, 0, :4] = [0x8000, 0x7FC1, 0xFFFF, 0x7F80]
    buf = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)
    assert list(buf[:4]) == [0x8000, 0x7FC1, 0xFFFF, 0x7F80]


def test_buffer_bytes_match_the_papers_cache_sizes(oracle_mod):
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "kv_cache_sizes.txt")) if ln.strip() and ln[0] != "#"]
    assert len(rows) == 2
    for L, H, d, e, tokens, paper_gb in rows:
        got = oracle_mod.kv_buffer_bytes(int(L), int(H), int(d), int(e), int(tokens))
        assert got == int(paper_gb) * 2 ** 30                 # the paper's figure, read as binary gigabytes
        assert abs(got / 1e9 - float(paper_gb)) / float(paper_gb) < 0.08   # and within rounding of decimal GB
    # empty sessions occupy nothing
    assert oracle_mod.kv_buffer_bytes(32, 8, 128, 2, 0) == 0


def test_pack_empty_and_zero_length_sessions(oracle_mod):
    cfg = small_cfg("bf16", n_sessions=3, prefix_dist=("const", 0))
    sess = W.make_sessions(cfg, 1)
    k_pool, v_pool = W.make_pool_host(cfg, sess, 1)
    buf = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)
    assert buf.size == 0


# --------------------------------------------------------------------------------------------------------
# attention
# --------------------------------------------------------------------------------------------------------
def run_oracle_attn(oracle_mod, sess, inputs, **kw):
    k_pool, v_pool, q, k_new, v_new = inputs
    return oracle_mod.prefix_prefill_attn(k_pool, v_pool, q, k_new, v_new, sess.cu_new_lens, sess.prefix_lens,
                                          sess.block_table, sess.cfg.scale, **kw)


@pytest.mark.parametrize("dtype,seed", [("bf16", 1), ("bf16", 2), ("fp32", 3), ("fp32", 4)])
def test_attention_brute_force_full_matrix(oracle_mod, dtype, seed):
    cfg = small_cfg(dtype, n_sessions=4, prefix_dist=("uniform", 0, 21), new_dist=("uniform", 0, 9),
                    n_q_heads=6, n_kv_heads=2)
    sess = W.make_sessions(cfg, seed)
    inputs = W.make_attn_inputs(cfg, sess, seed)
    got = run_oracle_attn(oracle_mod, sess, inputs)
    ref = brute_force_attention(*inputs, sess, cfg.scale)
    assert got.shape == ref.shape
    if got.size:
        assert np.max(np.abs(got - ref)) < 1e-12


@pytest.mark.parametrize("G", [1, 4])
def test_attention_matches_torch_sdpa_fp64(oracle_mod, G):
    import torch
    import torch.nn.functional as F
    cfg = small_cfg("bf16", n_sessions=3, n_q_heads=2 * G, n_kv_heads=2, head_dim=16, block_size=16, n_blocks=32,
                    prefix_dist=("uniform", 5, 70), new_dist=("uniform", 1, 12), scale=0.25)
    sess = W.make_sessions(cfg, 17)
    inputs = W.make_attn_inputs(cfg, sess, 17)
    k_pool, v_pool, q, k_new, v_new = inputs
    got = run_oracle_attn(oracle_mod, sess, inputs)
    for s in range(sess.n_sessions):
        P, N = int(sess.prefix_lens[s]), int(sess.new_lens[s])
        a, b = int(sess.cu_new_lens[s]), int(sess.cu_new_lens[s + 1])
        K = torch.from_numpy(contiguous_kv(k_pool, sess.block_table[s], P, k_new[a:b])).permute(1, 0, 2)  # [H_kv][n][d]
        V = torch.from_numpy(contiguous_kv(v_pool, sess.block_table[s], P, v_new[a:b])).permute(1, 0, 2)
        Q = torch.from_numpy(to_f64(q[a:b])).permute(1, 0, 2)                                            # [H_q][N][d]
        K = K.repeat_interleave(G, dim=0)
        V = V.repeat_interleave(G, dim=0)
        mask = torch.ones(N, P + N, dtype=torch.bool).tril(diagonal=P)
        ref = F.scaled_dot_product_attention(Q[None], K[None], V[None], attn_mask=mask[None, None], scale=0.25)[0]
        assert torch.max(torch.abs(torch.from_numpy(got[a:b]).permute(1, 0, 2) - ref)).item() < 1e-12


def test_cached_prefix_equals_full_recompute_and_any_split(oracle_mod):
    """Resuming from a cached prefix must give the rows a full recompute of the session gives (Sec. 3.5:
    the mechanism changes neither model nor data)."""
    cfg = small_cfg("bf16", n_sessions=1, prefix_dist=("const", 37), new_dist=("const", 11), n_blocks=64)
    sess = W.make_sessions(cfg, 2)
    inputs = W.make_attn_inputs(cfg, sess, 2)
    k_pool, v_pool, q, k_new, v_new = inputs
    ref = run_oracle_attn(oracle_mod, sess, inputs)
    P, N = 37, 11
    kfull = np.stack([k_pool[sess.block_table[0, t // 4], t % 4] for t in range(P)] + list(k_new))
    vfull = np.stack([v_pool[sess.block_table[0, t // 4], t % 4] for t in range(P)] + list(v_new))
    for split in (0, 5, 36, 40):          # tokens [0, split) cached, the rest "new"
        c2 = small_cfg("bf16", n_sessions=1, prefix_dist=("const", split), new_dist=("const", P + N - split),
                       n_blocks=64)
        s2 = W.make_sessions(c2, 99)      # a different random table
        kp = np.full_like(k_pool, W.SENTINEL16); vp = np.full_like(v_pool, W.SENTINEL16)
        for t in range(split):
            kp[s2.block_table[0, t // 4], t % 4] = kfull[t]
            vp[s2.block_table[0, t // 4], t % 4] = vfull[t]
        n2 = P + N - split
        q2 = np.zeros((n2,) + q.shape[1:], dtype=q.dtype)
        keep = min(N, n2)                                 # earlier rows: zero queries, discarded below
        q2[n2 - keep:] = q[N - keep:]
        out = oracle_mod.prefix_prefill_attn(kp, vp, q2, np.ascontiguousarray(kfull[split:]),
                                             np.ascontiguousarray(vfull[split:]), s2.cu_new_lens, s2.prefix_lens,
                                             s2.block_table, cfg.scale)
        assert np.max(np.abs(out[n2 - keep:] - ref[N - keep:])) < 1e-13


def test_block_id_permutation_leaves_output_unchanged(oracle_mod):
    cfg = small_cfg("fp32", n_sessions=3, prefix_dist=("uniform", 4, 30), new_dist=("uniform", 1, 6), n_blocks=48)
    sess = W.make_sessions(cfg, 6)
    inputs = W.make_attn_inputs(cfg, sess, 6)
    ref = run_oracle_attn(oracle_mod, sess, inputs)
    perm = np.random.default_rng(0).permutation(cfg.n_blocks).astype(np.int32)    # old id -> new id
    k_pool, v_pool, q, k_new, v_new = inputs
    kp = np.empty_like(k_pool); vp = np.empty_like(v_pool)
    kp[perm] = k_pool; vp[perm] = v_pool
    tab = np.where(sess.block_table >= 0, perm[np.maximum(sess.block_table, 0)], -1).astype(np.int32)
    out = oracle_mod.prefix_prefill_attn(kp, vp, q, k_new, v_new, sess.cu_new_lens, sess.prefix_lens, tab, cfg.scale)
    assert np.array_equal(out, ref)


def test_softmax_weights_sum_to_one_and_are_causal(oracle_mod):
    cfg = small_cfg("bf16", n_sessions=2, prefix_dist=("uniform", 10, 40), new_dist=("const", 5), n_blocks=64)
    sess = W.make_sessions(cfg, 8)
    inputs = W.make_attn_inputs(cfg, sess, 8)
    full = run_oracle_attn(oracle_mod, sess, inputs)
    for s in range(2):
        for i in range(5):
            for h in range(cfg.n_q_heads):
                w, o = oracle_mod.attn_row_weights(*inputs, sess.cu_new_lens, sess.prefix_lens, sess.block_table,
                                                   cfg.scale, s, i, h)
                assert w.size == sess.prefix_lens[s] + i + 1      # sees the prefix and new tokens 0..i, no more
                assert abs(w.sum() - 1.0) < 1e-12 and np.all(w > 0)
                assert np.array_equal(o, full[sess.cu_new_lens[s] + i, h])


def test_attention_closed_forms(oracle_mod):
    cfg = small_cfg("fp32", n_sessions=1, prefix_dist=("const", 13), new_dist=("const", 4), n_blocks=16)
    sess = W.make_sessions(cfg, 10)
    k_pool, v_pool, q, k_new, v_new = W.make_attn_inputs(cfg, sess, 10)
    ids = sess.block_table[0, :4]
    P, N, G = 13, 4, cfg.group

    # (1) all keys equal -> uniform weights -> output = mean of the visible V rows
    kp = k_pool.copy(); kp[ids] = 0.5
    kn = np.full_like(k_new, 0.5)
    out = oracle_mod.prefix_prefill_attn(kp, v_pool, q, kn, v_new, sess.cu_new_lens, sess.prefix_lens,
                                         sess.block_table, cfg.scale)
    vfull = np.concatenate([v_pool[ids].reshape(-1, cfg.n_kv_heads, cfg.head_dim)[:P], v_new]).astype(np.float64)
    for i in range(N):
        for h in range(cfg.n_q_heads):
            assert np.allclose(out[i, h], vfull[: P + i + 1, h // G].mean(axis=0), rtol=0, atol=1e-13)

    # (2) V constant per kv-head -> output is that constant, whatever the scores
    vp = v_pool.copy(); vn = v_new.copy()
    for g in range(cfg.n_kv_heads):
        vp[ids, :, g] = 3.0 + g
        vn[:, g] = 3.0 + g
    out = oracle_mod.prefix_prefill_attn(k_pool, vp, q, k_new, vn, sess.cu_new_lens, sess.prefix_lens,
                                         sess.block_table, cfg.scale)
    for h in range(cfg.n_q_heads):
        assert np.allclose(out[:, h], 3.0 + h // G, rtol=0, atol=1e-13)

    # (3) one key dominates: q = e_0, key j* = 1000 e_0, all other keys 0  ->  output = V[j*]
    qq = np.zeros_like(q); qq[..., 0] = 1.0
    kp = k_pool.copy(); kp[ids] = 0.0
    kn = np.zeros_like(k_new)
    jstar = 6
    kp[ids[jstar // 4], jstar % 4, :, 0] = 1000.0
    out = oracle_mod.prefix_prefill_attn(kp, v_pool, qq, kn, v_new, sess.cu_new_lens, sess.prefix_lens,
                                         sess.block_table, 1.0)
    for h in range(cfg.n_q_heads):
        assert np.allclose(out[:, h], vfull[jstar, h // G][None], rtol=0, atol=1e-13)

    # (4) the scale is applied to the scores: doubling the scale == doubling q
    a = oracle_mod.prefix_prefill_attn(k_pool, v_pool, q, k_new, v_new, sess.cu_new_lens, sess.prefix_lens,
                                       sess.block_table, 2 * cfg.scale)
    b = oracle_mod.prefix_prefill_attn(k_pool, v_pool, 2 * q, k_new, v_new, sess.cu_new_lens, sess.prefix_lens,
                                       sess.block_table, cfg.scale)
    assert np.max(np.abs(a - b)) < 1e-12


def test_first_turn_single_token_returns_its_own_value(oracle_mod):
    cfg = small_cfg("bf16", n_sessions=2, prefix_dist=("const", 0), new_dist=("const", 1))
    sess = W.make_sessions(cfg, 12)
    k_pool, v_pool, q, k_new, v_new = W.make_attn_inputs(cfg, sess, 12)
    out = oracle_mod.prefix_prefill_attn(k_pool, v_pool, q, k_new, v_new, sess.cu_new_lens, sess.prefix_lens,
                                         sess.block_table, cfg.scale)
    for h in range(cfg.n_q_heads):
        assert np.array_equal(out[:, h], to_f64(v_new)[:, h // cfg.group])


def test_token_subset_matches_full(oracle_mod):
    cfg = small_cfg("bf16", n_sessions=3, prefix_dist=("uniform", 1, 19), new_dist=("uniform", 1, 7))
    sess = W.make_sessions(cfg, 14)
    inputs = W.make_attn_inputs(cfg, sess, 14)
    full = run_oracle_attn(oracle_mod, sess, inputs)
    rows = [0, sess.total_new_tokens - 1, sess.total_new_tokens // 2]
    part = run_oracle_attn(oracle_mod, sess, inputs, token_subset=rows)
    assert np.array_equal(part[rows], full[rows])
    others = np.setdiff1d(np.arange(sess.total_new_tokens), rows)
    assert np.all(np.isnan(part[others]))


# --------------------------------------------------------------------------------------------------------
# write-back of what a turn added: tokens tail_begin[s] .. P_s - 1 only (Sec. 3.3)
# --------------------------------------------------------------------------------------------------------
def _tail_begins(sess, rng):
    """Per session: 0, P_s (nothing new), or something in between."""
    P = sess.prefix_lens.astype(np.int64)
    pick = rng.integers(0, 4, size=P.shape[0])
    b = np.where(pick == 0, 0, np.where(pick == 1, P, rng.integers(0, P + 1)))
    return b.astype(np.int32)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_pack_tail_tagged_pool_layout(oracle_mod, seed):
    """Every element of a tail buffer decodes to the coordinates the layout rules give: session-major over the tail
    lengths, layer-major, K then V, token tail_begin + i."""
    cfg = small_cfg("fp32", n_layers=3, n_sessions=5, n_blocks=64, prefix_dist=("uniform", 0, 23))
    sess = W.make_sessions(cfg, seed)
    begins = _tail_begins(sess, np.random.default_rng(seed))
    k_pool, v_pool = tagged_pools(cfg)
    buf = oracle_mod.kv_pack_tail(k_pool, v_pool, sess.block_table, sess.prefix_lens, begins)
    H, d, bs = cfg.n_kv_heads, cfg.head_dim, cfg.block_size
    assert buf.size == int((sess.prefix_lens - begins).sum()) * 2 * cfg.n_layers * H * d
    kv, l, b, o, g, c = decode_tag(buf.view(np.uint32), cfg)
    pos = 0
    for s in range(sess.n_sessions):
        for layer in range(cfg.n_layers):
            for which in (0, 1):
                for t in range(int(begins[s]), int(sess.prefix_lens[s])):
                    sl = slice(pos, pos + H * d)
                    assert np.all(kv[sl] == which) and np.all(l[sl] == layer)
                    assert np.all(b[sl] == sess.block_table[s, t // bs]) and np.all(o[sl] == t % bs)
                    assert np.array_equal(g[sl], np.repeat(np.arange(H), d))
                    assert np.array_equal(c[sl], np.tile(np.arange(d), H))
                    pos += H * d
    assert pos == buf.size


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_tail_completes_an_earlier_whole_pack(oracle_mod, dtype):
    """Plane by plane (session, layer, K|V): the rows packed when the session had tail_begin tokens, followed by the
    tail's rows, are the rows of a whole pack at the present length; with tail_begin = 0 the tail IS the whole pack."""
    cfg = small_cfg(dtype, n_layers=3, n_sessions=6, n_blocks=96, prefix_dist=("uniform", 0, 40))
    sess = W.make_sessions(cfg, 31)
    k_pool, v_pool = W.make_pool_host(cfg, sess, 31)
    begins = _tail_begins(sess, np.random.default_rng(31))
    L, row = cfg.n_layers, cfg.n_kv_heads * cfg.head_dim
    P = sess.prefix_lens
    whole = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, P, sess.buf_token_offsets)
    old_off = np.concatenate([[0], np.cumsum(begins)]).astype(np.int64)
    old = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, begins, old_off)      # the cache as it was at length begin
    tail = oracle_mod.kv_pack_tail(k_pool, v_pool, sess.block_table, P, begins)
    tail_off = oracle_mod.tail_offsets(P, begins)
    for s in range(sess.n_sessions):
        Ps, Bs = int(P[s]), int(begins[s])
        for plane in range(2 * L):
            w0 = (int(sess.buf_token_offsets[s]) * 2 * L + plane * Ps) * row
            o0 = (int(old_off[s]) * 2 * L + plane * Bs) * row
            t0 = (int(tail_off[s]) * 2 * L + plane * (Ps - Bs)) * row
            joined = np.concatenate([old[o0:o0 + Bs * row], tail[t0:t0 + (Ps - Bs) * row]])
            assert joined.tobytes() == whole[w0:w0 + Ps * row].tobytes()
    zero = np.zeros_like(begins)
    assert oracle_mod.kv_pack_tail(k_pool, v_pool, sess.block_table, P, zero).tobytes() == whole.tobytes()
    assert oracle_mod.kv_pack_tail(k_pool, v_pool, sess.block_table, P, P.copy()).size == 0


def test_unpack_tail_touches_the_tail_slots_only(oracle_mod):
    """Scattering a tail changes exactly the slots of tokens tail_begin .. P-1; after a whole unpack at the earlier
    length it completes the pools to those of a whole unpack at the present length."""
    cfg = small_cfg("bf16", n_layers=2, n_sessions=5, n_blocks=96, prefix_dist=("uniform", 0, 40))
    sess = W.make_sessions(cfg, 32)
    k_pool, v_pool = W.make_pool_host(cfg, sess, 32)
    begins = _tail_begins(sess, np.random.default_rng(32))
    P, dst = sess.prefix_lens, sess.dst_block_table
    whole = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, P, sess.buf_token_offsets)
    tail = oracle_mod.kv_pack_tail(k_pool, v_pool, sess.block_table, P, begins)
    ks, vs = np.full_like(k_pool, 0x7FC1), np.full_like(v_pool, 0x7FC1)
    oracle_mod.kv_unpack_tail(ks, vs, dst, P, begins, tail)
    bs = cfg.block_size
    touched = np.zeros(k_pool.shape[1:3], dtype=bool)           # [block, slot]
    for s in range(sess.n_sessions):
        for t in range(int(begins[s]), int(P[s])):
            touched[dst[s, t // bs], t % bs] = True
            assert np.array_equal(ks[:, dst[s, t // bs], t % bs], k_pool[:, sess.block_table[s, t // bs], t % bs])
            assert np.array_equal(vs[:, dst[s, t // bs], t % bs], v_pool[:, sess.block_table[s, t // bs], t % bs])
    assert np.all(ks[:, ~touched] == 0x7FC1) and np.all(vs[:, ~touched] == 0x7FC1)
    # earlier whole unpack + tail == present whole unpack
    old_off = np.concatenate([[0], np.cumsum(begins)]).astype(np.int64)
    old = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, begins, old_off)
    k2, v2 = np.full_like(k_pool, 0x7FC1), np.full_like(v_pool, 0x7FC1)
    oracle_mod.kv_unpack(k2, v2, dst, begins, old_off, old)
    oracle_mod.kv_unpack_tail(k2, v2, dst, P, begins, tail)
    k3, v3 = np.full_like(k_pool, 0x7FC1), np.full_like(v_pool, 0x7FC1)
    oracle_mod.kv_unpack(k3, v3, dst, P, sess.buf_token_offsets, whole)
    assert k2.tobytes() == k3.tobytes() and v2.tobytes() == v3.tobytes()


# --------------------------------------------------------------------------------------------------------
# unit-wise copies: single layers of sessions in one pool of slots (Sec. 3.3, priority-based K,V cache)
# --------------------------------------------------------------------------------------------------------
def random_units(rng, n_units, n_slots, bs, max_len, row):
    ub = W.make_units(rng, n_units, n_slots, bs, max_len)
    return ub.unit_lens, ub.unit_table, ub.unit_chunk_rows, ub.n_buf_rows


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_pack_units_tagged_slot_pool(oracle_mod, seed):
    rng = np.random.default_rng(400 + seed)
    cfg = small_cfg("fp32", n_layers=1, n_blocks=60)
    H, d, bs = cfg.n_kv_heads, cfg.head_dim, cfg.block_size
    k_slots, v_slots = tagged_pools(cfg)
    lens, table, chunk_rows, n_rows = random_units(rng, 7, cfg.n_blocks, bs, 21, H * d)
    sentinel = np.float32(-123.0)
    buf = np.full(n_rows * H * d, sentinel, dtype=np.float32)
    oracle_mod.kv_pack_units(k_slots[0], v_slots[0], table, lens, chunk_rows, buf)
    kv, l, b, o, g, c = decode_tag(buf.view(np.uint32), cfg)
    written = np.zeros(n_rows, dtype=bool)
    for u in range(7):
        for which in (0, 1):
            for t in range(int(lens[u])):
                r = int(chunk_rows[u]) + which * int(lens[u]) + t
                sl = slice(r * H * d, (r + 1) * H * d)
                assert np.all(kv[sl] == which) and np.all(b[sl] == table[u, t // bs]) and np.all(o[sl] == t % bs)
                assert np.array_equal(g[sl], np.repeat(np.arange(H), d)) and np.array_equal(c[sl], np.tile(np.arange(d), H))
                written[r] = True
    untouched = buf.reshape(n_rows, H * d)[~written]
    assert np.all(untouched == sentinel)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_unpack_units_round_trips_and_leaves_other_bytes_alone(oracle_mod, dtype):
    rng = np.random.default_rng(77)
    cfg = small_cfg(dtype, n_layers=1, n_blocks=50)
    H, d, bs = cfg.n_kv_heads, cfg.head_dim, cfg.block_size
    lens, table, chunk_rows, n_rows = random_units(rng, 6, cfg.n_blocks, bs, 18, H * d)
    np_dtype = np.uint16 if dtype == "bf16" else np.float32
    buf = rng.integers(1, 60000, size=n_rows * H * d).astype(np_dtype)
    k_slots = np.full((cfg.n_blocks, bs, H, d), 7, dtype=np_dtype)
    v_slots = np.full((cfg.n_blocks, bs, H, d), 9, dtype=np_dtype)
    oracle_mod.kv_unpack_units(k_slots, v_slots, table, lens, chunk_rows, buf)
    owned = np.zeros((cfg.n_blocks, bs), dtype=bool)
    rows = buf.reshape(n_rows, H, d)
    for u in range(6):
        for t in range(int(lens[u])):
            slot, o = table[u, t // bs], t % bs
            owned[slot, o] = True
            assert np.array_equal(k_slots[slot, o], rows[int(chunk_rows[u]) + t])
            assert np.array_equal(v_slots[slot, o], rows[int(chunk_rows[u]) + int(lens[u]) + t])
    assert np.all(k_slots[~owned] == 7) and np.all(v_slots[~owned] == 9)
    back = np.zeros_like(buf)
    oracle_mod.kv_pack_units(k_slots, v_slots, table, lens, chunk_rows, back)
    mask = np.zeros(n_rows, dtype=bool)
    for u in range(6):
        mask[int(chunk_rows[u]): int(chunk_rows[u]) + 2 * int(lens[u])] = True
    assert np.array_equal(back.reshape(n_rows, -1)[mask], buf.reshape(n_rows, -1)[mask])
    assert np.all(back.reshape(n_rows, -1)[~mask] == 0)


def test_units_of_the_lower_layers_equal_the_layer_range_scatter(oracle_mod):
    """A cache of L layers seen as one pool of L * n_blocks slots (slot = layer * n_blocks + block): scattering the
    units (s, l) for l < r_s is the layer-range scatter, session by session."""
    cfg = small_cfg("bf16", n_layers=3, n_sessions=3, prefix_dist=("uniform", 1, 19))
    sess = W.make_sessions(cfg, 5)
    rng = np.random.default_rng(5)
    L, nb, bs, H, d = cfg.n_layers, cfg.n_blocks, cfg.block_size, cfg.n_kv_heads, cfg.head_dim
    total = int(sess.buf_token_offsets[-1])
    buf = rng.integers(1, 60000, size=total * 2 * L * H * d).astype(np.uint16)
    resident = [3, 1, 2]
    # route 1: unit-wise into the flat pool
    k_flat = np.zeros((L * nb, bs, H, d), dtype=np.uint16)
    v_flat = np.zeros_like(k_flat)
    units = [(s, l) for s in range(3) for l in range(resident[s])]
    lens = np.array([sess.prefix_lens[s] for s, _ in units], dtype=np.int32)
    table = np.stack([np.where(sess.block_table[s] >= 0, sess.block_table[s] + l * nb, 0) for s, l in units]).astype(np.int32)
    chunk_rows = np.array([oracle_mod.unit_chunk_rows(sess.buf_token_offsets, sess.prefix_lens, L, s, l) for s, l in units],
                          dtype=np.int64)
    oracle_mod.kv_unpack_units(k_flat, v_flat, table, lens, chunk_rows, buf)
    # route 2: the layer-range scatter of the L-layer cache, one session at a time
    k_pool = np.zeros((L, nb, bs, H, d), dtype=np.uint16)
    v_pool = np.zeros_like(k_pool)
    for s in range(3):
        lens_s = np.where(np.arange(3) == s, sess.prefix_lens, 0).astype(np.int32)   # other sessions: nothing to move
        # offsets stay those of the whole buffer, so the chunks are found where they are
        oracle_mod.kv_unpack_layers(k_pool, v_pool, sess.block_table, lens_s, sess.buf_token_offsets, buf, 0, resident[s])
    assert np.array_equal(k_flat.reshape(L, nb, bs, H, d), k_pool) and np.array_equal(v_flat.reshape(L, nb, bs, H, d), v_pool)
    assert k_pool.any()
