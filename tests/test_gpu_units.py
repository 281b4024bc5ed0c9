"""symph_kv_pack_units / symph_kv_unpack_units (single layers of sessions in one pool of slots) against the byte-copy
oracle, and the residency pool of symph_pool.h driving them: the lower layers of several announced sessions are moved
in with one launch, memory pressure from the framework overwrites the later layers and leaves the rest intact."""
import numpy as np
import pytest
import torch

import paper_2412_16434_amd as S
import workloads as W
from gpu_util import DEV, to_dev, to_host

pytestmark = pytest.mark.gpu


def _random_bits(rng, shape, np_dtype):
    if np_dtype == np.uint16:
        return rng.integers(1, 0x7F00, size=shape).astype(np.uint16)
    return rng.standard_normal(shape).astype(np.float32)


def _dev_units(ub: W.UnitBatch):
    return tuple(torch.from_numpy(a).to(DEV) for a in (ub.unit_table, ub.unit_lens, ub.unit_token_offsets, ub.unit_chunk_rows))


@pytest.mark.parametrize("kw", [
    dict(n_units=9, n_slots=400, bs=16, H=8, d=128, max_len=500, dtype="bf16"),           # model rows (2 KiB), ragged lengths
    dict(n_units=70, n_slots=3000, bs=16, H=8, d=128, max_len=600, dtype="bf16"),         # many units: the other planes-per-lane choice
    dict(n_units=1, n_slots=300, bs=16, H=8, d=128, max_len=4000, min_len=4000, dtype="bf16"),
    dict(n_units=5, n_slots=200, bs=8, H=2, d=64, max_len=90, dtype="fp32"),
    dict(n_units=6, n_slots=300, bs=4, H=3, d=20, max_len=50, dtype="fp32"),              # rows that are no power of two
    dict(n_units=6, n_slots=300, bs=4, H=1, d=6, max_len=50, dtype="bf16"),               # 12-byte rows: 4-byte vectors
    dict(n_units=4, n_slots=64, bs=16, H=8, d=128, max_len=0, dtype="bf16"),              # nothing to move
])
def test_units_match_the_oracle(oracle_mod, kw):
    rng = np.random.default_rng(900 + kw["n_units"])
    np_dtype = np.uint16 if kw["dtype"] == "bf16" else np.float32
    bs, H, d = kw["bs"], kw["H"], kw["d"]
    ub = W.make_units(rng, kw["n_units"], kw["n_slots"], bs, kw["max_len"], kw.get("min_len", 0))
    k_slots = _random_bits(rng, (kw["n_slots"], bs, H, d), np_dtype)
    v_slots = _random_bits(rng, (kw["n_slots"], bs, H, d), np_dtype)
    buf0 = _random_bits(rng, ub.n_buf_rows * H * d, np_dtype)

    slots = S.KVCache(to_dev(k_slots)[None], to_dev(v_slots)[None])
    table, lens, offs, rows = _dev_units(ub)
    # gather
    ref = buf0.copy()
    oracle_mod.kv_pack_units(k_slots, v_slots, ub.unit_table, ub.unit_lens, ub.unit_chunk_rows, ref)
    buf = to_dev(buf0)
    S.kv_pack_units(slots, table, lens, offs, rows, ub.total_tokens, buf)
    torch.cuda.synchronize()
    assert to_host(buf).tobytes() == ref.tobytes(), "pack_units differs from the oracle"
    # scatter of other data into the same slots
    src = _random_bits(rng, buf0.shape, np_dtype)
    k_ref, v_ref = k_slots.copy(), v_slots.copy()
    oracle_mod.kv_unpack_units(k_ref, v_ref, ub.unit_table, ub.unit_lens, ub.unit_chunk_rows, src)
    S.kv_unpack_units(slots, table, lens, offs, rows, ub.total_tokens, to_dev(src))
    torch.cuda.synchronize()
    assert to_host(slots.k_pool[0]).tobytes() == k_ref.tobytes() and to_host(slots.v_pool[0]).tobytes() == v_ref.tobytes()


def test_units_that_cannot_be_placed_are_skipped():
    """A slot number outside the pool, a negative chunk row and a chunk that passes the end of the buffer: those units
    (or blocks) are left out, everything else moves, nothing out of range is touched."""
    rng = np.random.default_rng(17)
    bs, H, d, n_slots = 16, 8, 128, 200
    ub = W.make_units(rng, 6, n_slots, bs, 300, 100)
    k_slots = _random_bits(rng, (n_slots, bs, H, d), np.uint16)
    v_slots = _random_bits(rng, (n_slots, bs, H, d), np.uint16)
    sentinel = W.SENTINEL16
    table, chunk_rows = ub.unit_table.copy(), ub.unit_chunk_rows.copy()
    table[0, 1] = n_slots + 5          # second block of unit 0: not a slot
    table[1, 0] = -3                   # first block of unit 1
    chunk_rows[2] = -1                 # unit 2 has no place
    chunk_rows[3] = ub.n_buf_rows      # unit 3 would start behind the buffer
    buf = torch.full((ub.n_buf_rows * H * d,), 0, dtype=torch.int16, device=DEV).view(torch.bfloat16)
    buf.view(torch.int16).fill_(int(np.int16(sentinel)))
    slots = S.KVCache(to_dev(k_slots)[None], to_dev(v_slots)[None])
    S.kv_pack_units(slots, torch.from_numpy(table).to(DEV), torch.from_numpy(ub.unit_lens).to(DEV),
                    torch.from_numpy(ub.unit_token_offsets).to(DEV), torch.from_numpy(chunk_rows).to(DEV),
                    ub.total_tokens, buf)
    torch.cuda.synchronize()
    got = to_host(buf).reshape(ub.n_buf_rows, H, d)
    want = np.full_like(got, sentinel)
    for u in range(6):
        if u in (2, 3):
            continue
        P = int(ub.unit_lens[u])
        for t in range(P):
            slot = table[u, t // bs]
            if 0 <= slot < n_slots:
                want[chunk_rows[u] + t] = k_slots[slot, t % bs]
                want[chunk_rows[u] + P + t] = v_slots[slot, t % bs]
    assert got.tobytes() == want.tobytes()


def test_lower_layers_of_two_sessions_through_the_pool(oracle_mod):
    """Sec. 3.3's scenario at model row size: two announced sessions, room for about one.  The pool decides, ONE
    unpack_units launch moves the lower layers of both in, the framework then takes slots (later layers go first) and
    scribbles over what it took; the units that stayed resident still read back bit for bit."""
    L, bs, H, d = 8, 16, 8, 128
    cfg = W.WorkloadConfig(name="units", index=81, dtype="bf16", n_layers=L, n_q_heads=32, n_kv_heads=H, head_dim=d,
                           block_size=bs, n_blocks=512, n_sessions=2, prefix_dist=("uniform", 300, 700),
                           new_dist=("const", 1), sigma=1.0, scale=0.1)
    sess = W.make_sessions(cfg, 3)
    rng = np.random.default_rng(3)
    P = [int(x) for x in sess.prefix_lens]
    blocks = [-(-p // bs) for p in P]
    total = int(sess.buf_token_offsets[-1])
    whole = _random_bits(rng, total * 2 * L * H * d, np.uint16)             # the sessions' migration buffer (host copy)
    n_slots = max(blocks) * L + 3                                           # all of the larger one, hardly more
    pool = S.KvPool(L, n_slots, bs)
    for s in range(2):
        pool.advise(10 + s, P[s])
    loads = [(sid - 10, layer, sl) for kind, sid, layer, sl in pool.settle() if kind == S.KvPool.LOAD]
    r = [pool.resident_layers(10), pool.resident_layers(11)]
    assert 0 < r[0] < L and 0 < r[1] < L and abs(r[0] - r[1]) <= 1          # the lower layers of both

    def unit_arrays(units):
        stride = max(blocks) + 1
        table = np.full((len(units), stride), -1, dtype=np.int32)
        for u, (s, layer, sl) in enumerate(units):
            table[u, : len(sl)] = sl
        lens = np.array([P[s] for s, _, _ in units], dtype=np.int32)
        rows = np.array([oracle_mod.unit_chunk_rows(sess.buf_token_offsets, sess.prefix_lens, L, s, layer)
                         for s, layer, _ in units], dtype=np.int64)
        offs = np.concatenate([[0], np.cumsum(lens.astype(np.int64))]).astype(np.int64)
        return table, lens, offs, rows

    k0 = np.full((n_slots, bs, H, d), W.SENTINEL16, dtype=np.uint16)
    slots = S.KVCache(to_dev(k0)[None], to_dev(k0)[None])
    d_whole = to_dev(whole)
    table, lens, offs, rows = unit_arrays(loads)
    S.kv_unpack_units(slots, *(torch.from_numpy(a).to(DEV) for a in (table, lens, offs, rows)), int(offs[-1]), d_whole)
    torch.cuda.synchronize()
    k_ref, v_ref = k0.copy(), k0.copy()
    oracle_mod.kv_unpack_units(k_ref, v_ref, table, lens, rows, whole)
    assert to_host(slots.k_pool[0]).tobytes() == k_ref.tobytes() and to_host(slots.v_pool[0]).tobytes() == v_ref.tobytes()

    # memory pressure: the framework takes more than is free and overwrites what it got
    free = pool.counts()[0]
    taken = pool.framework_take(free + blocks[0] + 1)
    idx = torch.tensor(taken, device=DEV, dtype=torch.long)
    slots.k_pool[0][idx] = 1.0
    slots.v_pool[0][idx] = 2.0
    torch.cuda.synchronize()
    evicted = [(sid - 10, layer) for kind, sid, layer, _ in pool.settle() if kind == S.KvPool.EVICTED]
    top = max(r) - 1
    assert evicted and all(layer >= top - 1 for _, layer in evicted)         # later layers went first
    held = [(s, layer, pool.table(10 + s, layer)) for s in range(2) for layer in range(pool.resident_layers(10 + s))]
    assert held and not (set(taken) & {x for *_, sl in held for x in sl})
    table, lens, offs, rows = unit_arrays(held)
    back = torch.zeros_like(d_whole)
    S.kv_pack_units(slots, *(torch.from_numpy(a).to(DEV) for a in (table, lens, offs, rows)), int(offs[-1]), back)
    torch.cuda.synchronize()
    got = to_host(back).reshape(-1, H * d)
    src = whole.reshape(-1, H * d)
    mask = np.zeros(got.shape[0], dtype=bool)
    for u in range(len(held)):
        mask[rows[u]: rows[u] + 2 * lens[u]] = True
    assert got[mask].tobytes() == src[mask].tobytes() and not got[~mask].any()
    pool.close()
