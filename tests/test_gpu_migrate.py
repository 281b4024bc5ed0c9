"""symph_kv_pack / symph_kv_unpack against the CPU oracle: bit-exact, element by element on scaled-down versions
of the five workloads and on edge cases; sampled rows plus whole-pool properties at the full sizes."""
import numpy as np
import pytest
import torch

import paper_2412_16434_amd as S
import workloads as W
from gpu_util import DEV, DeviceSessions, gpu_pack, gpu_unpack, to_dev, to_host

pytestmark = pytest.mark.gpu


def sentinel_like(a: np.ndarray) -> np.ndarray:
    out = np.empty_like(a)
    if a.dtype == np.uint16:
        out[...] = W.SENTINEL16
    else:
        out.view(np.uint32)[...] = W.values.SENTINEL32
    return out


def run_case(oracle_mod, cfg, seed=None):
    """pack == oracle; unpack into a sentinel pool == oracle's pool, every byte; round trips."""
    sess = W.make_sessions(cfg, seed)
    k_pool, v_pool = W.make_pool_host(cfg, sess, seed)
    ref_buf = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)

    ds = DeviceSessions(sess)
    cache = S.KVCache(to_dev(k_pool), to_dev(v_pool))
    buf = gpu_pack(cache, ds)
    torch.cuda.synchronize()
    got = to_host(buf)
    assert got.tobytes() == ref_buf.tobytes(), "pack differs from the oracle"
    # pack must not write to the pools
    assert to_host(cache.k_pool).tobytes() == k_pool.tobytes() and to_host(cache.v_pool).tobytes() == v_pool.tobytes()

    # unpack through the destination table into sentinel pools, oracle and GPU side by side
    ks, vs = sentinel_like(k_pool), sentinel_like(v_pool)
    oracle_mod.kv_unpack(ks, vs, sess.dst_block_table, sess.prefix_lens, sess.buf_token_offsets, ref_buf)
    dcache = S.KVCache(to_dev(sentinel_like(k_pool)), to_dev(sentinel_like(v_pool)))
    gpu_unpack(dcache, ds, buf, dst=True)
    torch.cuda.synchronize()
    assert to_host(dcache.k_pool).tobytes() == ks.tobytes(), "unpack: K pool differs from the oracle"
    assert to_host(dcache.v_pool).tobytes() == vs.tobytes(), "unpack: V pool differs from the oracle"
    # resume test: packing what was unpacked gives the buffer back
    again = gpu_pack(dcache, ds, dst=True)
    torch.cuda.synchronize()
    assert torch.equal(again.view(torch.int16) if again.dtype == torch.bfloat16 else again,
                       buf.view(torch.int16) if buf.dtype == torch.bfloat16 else buf)
    return sess


SCALED = {
    "tiny_fp32": dict(),
    "llama8b": dict(n_layers=3, n_sessions=5, prefix_scale=0.05, new_scale=0.2, n_blocks=512),
    "llama70b_long": dict(n_layers=5, prefix_scale=1 / 64, new_scale=1 / 8, n_blocks=128),
    "many_short": dict(n_layers=2, n_sessions=40, prefix_scale=0.1, n_blocks=1024),
    "mixed_resume_incoming": dict(n_layers=4, n_sessions=3, prefix_scale=1 / 16, n_blocks=128),
}


@pytest.mark.parametrize("name", sorted(SCALED))
def test_pack_unpack_scaled_configs(oracle_mod, name):
    cfg = W.get_config(name)
    if SCALED[name]:
        cfg = W.scaled_config(cfg, **SCALED[name])
    run_case(oracle_mod, cfg)


def _cfg(**kw):
    base = dict(name="edge", index=20, dtype="bf16", n_layers=2, n_q_heads=8, n_kv_heads=2, head_dim=64, block_size=16,
                n_blocks=64, n_sessions=4, prefix_dist=("uniform", 1, 100), new_dist=("const", 1), sigma=1.0, scale=0.1)
    base.update(kw)
    return W.WorkloadConfig(**base)


@pytest.mark.parametrize("kw", [
    dict(prefix_dist=("const", 1)),                                   # one token per session
    dict(prefix_dist=("const", 16), n_sessions=3),                    # exactly one full block
    dict(prefix_dist=("const", 17), n_sessions=3),                    # one full block + one slot
    dict(prefix_dist=("uniform", 0, 40), n_sessions=9),               # zero-length sessions mixed in
    dict(n_layers=1, n_sessions=1, prefix_dist=("const", 500), n_blocks=80),
    dict(n_layers=7, block_size=8, n_blocks=256, prefix_dist=("uniform", 1, 60)),   # odd layer count, other block size
    dict(n_layers=3, n_kv_heads=1, head_dim=64, block_size=32, n_blocks=64, prefix_dist=("uniform", 1, 200)),
    dict(dtype="fp32", n_kv_heads=3, head_dim=20, block_size=4, n_blocks=128, prefix_dist=("uniform", 1, 50)),  # 240 B rows
    dict(dtype="bf16", n_kv_heads=1, head_dim=6, block_size=4, n_blocks=128, prefix_dist=("uniform", 1, 50)),   # 12 B rows: 4-byte path
])
def test_pack_unpack_edge_cases(oracle_mod, kw):
    run_case(oracle_mod, _cfg(**kw), seed=77)


@pytest.mark.parametrize("tokens", [1, 15, 16, 17, 31, 33, 47, 100])
def test_workgroup_to_token_mappings(oracle_mod, tokens):
    """The mappings of workgroups to the token space (XCD-contiguous for the gather, identity for the scatter) on the
    Llama row shape (2 KiB rows, two rows per workgroup), for workgroup counts below, at and between multiples of 8."""
    run_case(oracle_mod, _cfg(n_kv_heads=8, head_dim=128, n_sessions=1, prefix_dist=("const", tokens), n_blocks=32),
             seed=tokens)


def test_all_sessions_empty_is_a_no_op(oracle_mod):
    cfg = _cfg(prefix_dist=("const", 0))
    sess = W.make_sessions(cfg, 1)
    k_pool, v_pool = W.make_pool_host(cfg, sess, 1)
    ds = DeviceSessions(sess)
    cache = S.KVCache(to_dev(k_pool), to_dev(v_pool))
    buf = torch.zeros(16, dtype=torch.bfloat16, device=DEV)
    S.kv_pack(cache, ds.table, ds.prefix_lens, ds.offsets, 0, buf)
    S.kv_unpack(cache, ds.table, ds.prefix_lens, ds.offsets, 0, buf)
    torch.cuda.synchronize()
    assert not buf.any() and to_host(cache.k_pool).tobytes() == k_pool.tobytes()


def test_invalid_block_ids_are_skipped_not_dereferenced(oracle_mod):
    """Ids outside [0, n_blocks) must not be touched: the rows they name stay as they were in the buffer."""
    cfg = _cfg(n_sessions=2, prefix_dist=("const", 40))
    sess = W.make_sessions(cfg, 3)
    k_pool, v_pool = W.make_pool_host(cfg, sess, 3)
    ref = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)
    bad = sess.block_table.copy()
    bad[1, 1] = cfg.n_blocks + 5
    bad[0, 2] = -3
    cache = S.KVCache(to_dev(k_pool), to_dev(v_pool))
    ds = DeviceSessions(sess)
    ds.table = torch.from_numpy(bad).to(DEV)
    buf = torch.full((ref.size,), -1, dtype=torch.int16, device=DEV).view(torch.bfloat16)
    S.kv_pack(cache, ds.table, ds.prefix_lens, ds.offsets, sess.total_prefix_tokens, buf)
    torch.cuda.synchronize()
    got = to_host(buf)
    row = cfg.row_elems
    for s in range(2):
        for layer in range(cfg.n_layers):
            for kv in range(2):
                for t in range(40):
                    _, be = oracle_mod.kv_locate(cfg.layer_elems, cfg.block_elems, cfg.n_layers, 16, cfg.n_kv_heads,
                                                 cfg.head_dim, sess.block_table, sess.prefix_lens,
                                                 sess.buf_token_offsets, s, layer, kv, t)
                    skipped = (s == 1 and t // 16 == 1) or (s == 0 and t // 16 == 2)
                    expect = np.full(row, 0xFFFF, np.uint16) if skipped else ref[be: be + row]
                    assert np.array_equal(got[be: be + row], expect)


def test_strided_cache_layout(oracle_mod):
    """Block-major allocation [n_blocks][L][2][bs][H][d] described through the stride fields."""
    cfg = _cfg(n_layers=3, n_sessions=3, prefix_dist=("uniform", 5, 90))
    sess = W.make_sessions(cfg, 9)
    k_pool, v_pool = W.make_pool_host(cfg, sess, 9)          # [L][nb][bs][H][d]
    ref = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)
    fused = np.stack([k_pool, v_pool], axis=0).transpose(2, 1, 0, 3, 4, 5).copy()     # [nb][L][2][bs][H][d]
    ft = to_dev(fused)
    kview = ft[:, :, 0].permute(1, 0, 2, 3, 4)               # [L][nb][bs][H][d] view with strides
    vview = ft[:, :, 1].permute(1, 0, 2, 3, 4)
    cache = S.KVCache(kview, vview)
    ds = DeviceSessions(sess)
    buf = gpu_pack(cache, ds)
    torch.cuda.synchronize()
    assert to_host(buf).tobytes() == ref.tobytes()


def test_pack_on_side_stream_and_host_staging(oracle_mod):
    """a4: pack on one stream, device->pinned-host copy ordered after it on a side stream, and back."""
    cfg = W.scaled_config(W.get_config("llama8b"), n_layers=4, n_sessions=6, prefix_scale=0.1, n_blocks=1024)
    sess = W.make_sessions(cfg)
    k_pool, v_pool = W.make_pool_host(cfg, sess)
    ref = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)
    ds = DeviceSessions(sess)
    cache = S.KVCache(to_dev(k_pool), to_dev(v_pool))
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    ev = torch.cuda.Event()
    nbytes = ref.nbytes
    host = torch.empty(ref.size, dtype=torch.int16, pin_memory=True)
    torch.cuda.synchronize()
    buf = gpu_pack(cache, ds, stream=main)
    S.stage_to_host(host, buf, nbytes, main, side, ev)
    side.synchronize()
    assert host.numpy().view(np.uint16).tobytes() == ref.tobytes()
    # and back: host -> device on the side stream, unpack waits for it on the main stream
    dcache = S.KVCache(to_dev(sentinel_like(k_pool)), to_dev(sentinel_like(v_pool)))
    buf2 = torch.zeros_like(buf)
    torch.cuda.synchronize()
    ev2 = torch.cuda.Event()
    S.stage_to_device(buf2, host, nbytes, main, side, ev2)
    gpu_unpack(dcache, ds, buf2, dst=True, stream=main)
    torch.cuda.synchronize()
    ks, vs = sentinel_like(k_pool), sentinel_like(v_pool)
    oracle_mod.kv_unpack(ks, vs, sess.dst_block_table, sess.prefix_lens, sess.buf_token_offsets, ref)
    assert to_host(dcache.k_pool).tobytes() == ks.tobytes() and to_host(dcache.v_pool).tobytes() == vs.tobytes()


def test_buffer_in_mapped_pinned_host_memory(oracle_mod):
    """The buffer argument may be pinned host memory that the runtime maps for the device at the same address: unpack
    then reads it over PCIe, pack writes it, and no staging copy in HBM is needed."""
    import ctypes
    cfg = W.scaled_config(W.get_config("llama8b"), n_layers=3, n_sessions=5, prefix_scale=0.05, new_scale=0.2, n_blocks=512)
    sess = W.make_sessions(cfg)
    k_pool, v_pool = W.make_pool_host(cfg, sess)
    ref_buf = oracle_mod.kv_pack(k_pool, v_pool, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)
    host = torch.zeros(ref_buf.size, dtype=torch.int16, pin_memory=True)
    mapped = ctypes.c_void_p(0)
    rc = ctypes.CDLL("libamdhip64.so").hipHostGetDevicePointer(ctypes.byref(mapped), ctypes.c_void_p(host.data_ptr()), 0)
    if rc != 0 or mapped.value != host.data_ptr():
        pytest.skip("pinned host memory is not mapped for the device at its host address here")
    ds = DeviceSessions(sess)
    cache = S.KVCache(to_dev(k_pool), to_dev(v_pool))
    hbuf = host.view(torch.bfloat16)
    S.kv_pack(cache, ds.table, ds.prefix_lens, ds.offsets, sess.total_prefix_tokens, hbuf)
    torch.cuda.synchronize()
    assert host.numpy().view(np.uint16).tobytes() == ref_buf.tobytes()
    ks, vs = sentinel_like(k_pool), sentinel_like(v_pool)
    oracle_mod.kv_unpack(ks, vs, sess.dst_block_table, sess.prefix_lens, sess.buf_token_offsets, ref_buf)
    dcache = S.KVCache(to_dev(sentinel_like(k_pool)), to_dev(sentinel_like(v_pool)))
    S.kv_unpack(dcache, ds.dst_table, ds.prefix_lens, ds.offsets, sess.total_prefix_tokens, hbuf)
    torch.cuda.synchronize()
    assert to_host(dcache.k_pool).tobytes() == ks.tobytes() and to_host(dcache.v_pool).tobytes() == vs.tobytes()


def test_device_copy_matches_source():
    src = torch.randint(-2 ** 31, 2 ** 31 - 1, (1 << 22,), dtype=torch.int32, device=DEV)
    for n_bytes in (16, 4096, (1 << 24) - 16, 1 << 24):
        dst = torch.zeros_like(src)
        S.device_copy(dst, src, n_bytes)
        torch.cuda.synchronize()
        assert torch.equal(dst[: n_bytes // 4], src[: n_bytes // 4]) and not dst[n_bytes // 4:].any()


def test_mfma_reference_counts_its_work_and_leaves_the_sink_alone():
    sink = torch.full((4,), 7.0, dtype=torch.float32, device=DEV)
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    flops = S.mfma_reference(16, sink)
    torch.cuda.synchronize()
    # 2 workgroups per CU x 4 waves x 32 instructions per iteration x 2*32*32*16 operations each
    assert flops == 2 * n_cu * 4 * 16 * 32 * 2 * 32 * 32 * 16
    assert torch.equal(sink.cpu(), torch.full((4,), 7.0))


# ---------------------------------------------------------------------------------------------------------
# full sizes: counter-filled device pools, EVERY row of the buffer and of the destination blocks against the oracle's
# index function, whole-pool properties for everything else
# ---------------------------------------------------------------------------------------------------------
ROWS_PER_SLICE = 1 << 15


def _full_size_case(oracle_mod, cfg):
    sess = W.make_sessions(cfg)
    L, nb, bs = cfg.n_layers, cfg.n_blocks, cfg.block_size
    shape = (L, nb, bs, cfg.n_kv_heads, cfg.head_dim)
    k_pool = torch.empty(shape, dtype=torch.bfloat16, device=DEV)
    v_pool = torch.empty(shape, dtype=torch.bfloat16, device=DEV)
    sent = np.array([W.SENTINEL16], dtype=np.uint16).view(np.int16)[0]
    k_pool.view(torch.int16).fill_(int(sent))
    v_pool.view(torch.int16).fill_(int(sent))
    src_blocks = sess.owned_blocks()
    W.fill_pool_blocks_device(k_pool, v_pool, cfg, src_blocks)
    cache = S.KVCache(k_pool, v_pool)
    ds = DeviceSessions(sess)
    buf = gpu_pack(cache, ds)
    torch.cuda.synchronize()
    assert buf.numel() * 2 == sess.payload_bytes()

    # The oracle's index function for every row of the buffer (source table, destination table).  A pool element holds
    # counter(seed, K|V, its own element offset), so the expected bits of a buffer row follow from the offset of the
    # row it is a copy of, and a row of a destination block must hold what its buffer row holds.
    row = cfg.row_elems
    geo = (cfg.layer_elems, cfg.block_elems, L, bs, cfg.n_kv_heads, cfg.head_dim)
    pe_src, kv = oracle_mod.kv_row_map(*geo, sess.block_table, sess.prefix_lens, sess.buf_token_offsets)
    pe_dst, kv2 = oracle_mod.kv_row_map(*geo, sess.dst_block_table, sess.prefix_lens, sess.buf_token_offsets)
    n_rows = pe_src.size
    assert n_rows * row == buf.numel() and np.array_equal(kv, kv2) and pe_src.min() >= 0 and pe_dst.min() >= 0
    cols = torch.arange(row, dtype=torch.int64, device=DEV)
    buf_rows = buf.view(torch.int16).view(n_rows, row)
    pools_flat = (k_pool.view(torch.int16).view(-1), v_pool.view(torch.int16).view(-1))

    def for_every_row(check):
        """check(slice of rows, salt, source offsets, destination offsets, expected bits [n][row]) over the whole buffer."""
        for r0 in range(0, n_rows, ROWS_PER_SLICE):
            r1 = min(n_rows, r0 + ROWS_PER_SLICE)
            for salt in (0, 1):
                pick = np.nonzero(kv[r0:r1] == salt)[0]
                if pick.size == 0:
                    continue
                rows = torch.from_numpy(pick + r0).to(DEV)
                src = torch.from_numpy(pe_src[r0:r1][pick]).to(DEV)
                dst = torch.from_numpy(pe_dst[r0:r1][pick]).to(DEV)
                expect = W.counter_bits_device(cfg.seed, salt, src[:, None] + cols[None, :])
                check(rows, salt, src, dst, expect)

    # (1) pack: every row of the buffer
    def check_pack(rows, salt, src, dst, expect):
        assert torch.equal(buf_rows[rows], expect), "pack: a buffer row differs from the row the oracle names"
    for_every_row(check_pack)

    # (2) unpack into the fresh destination blocks of the same pool: every destination row holds its buffer row, and
    #     every source row still holds what it held
    gpu_unpack(cache, ds, buf, dst=True)
    torch.cuda.synchronize()

    def check_unpack(rows, salt, src, dst, expect):
        flat = pools_flat[salt]
        assert torch.equal(flat[dst[:, None] + cols[None, :]], expect), "unpack: a destination row differs"
        assert torch.equal(flat[src[:, None] + cols[None, :]], expect), "unpack: a source row changed"
    for_every_row(check_unpack)

    # (3) whole pool: exactly the source and destination blocks hold data, everything else is still sentinel,
    #     and the unused tail slots of every source and destination last block are still sentinel
    dst_blocks = sess.owned_blocks(dst=True)
    owned = np.zeros(nb, dtype=bool)
    owned[src_blocks] = True
    owned[dst_blocks] = True
    owned_t = torch.from_numpy(owned).to(DEV)
    for pool in (k_pool, v_pool):
        for layer in range(L):
            touched = (pool[layer].view(torch.int16).view(nb, -1) != int(sent)).any(dim=1)
            assert torch.equal(touched, owned_t), f"layer {layer}: blocks written outside the tables"
    nblk = sess.blocks_per_session()
    for s in range(sess.n_sessions):
        tail = int(sess.prefix_lens[s]) % bs
        if tail:
            last = int(sess.dst_block_table[s, nblk[s] - 1])
            for pool in (k_pool, v_pool):
                assert bool((pool[:, last, tail:].view(torch.int16) == int(sent)).all())

    # (4) resume: packing from the destination table gives the identical buffer
    again = gpu_pack(cache, ds, dst=True)
    torch.cuda.synchronize()
    assert torch.equal(again.view(torch.int16), buf.view(torch.int16))
    print(f"[migrate parity] {cfg.name}: {n_rows} buffer rows and {n_rows} destination rows of {row} elements compared, "
          f"{L * nb * 2} pool blocks scanned", flush=True)


@pytest.mark.parametrize("name", ["llama8b", "llama70b_long", "many_short", "mixed_resume_incoming"])
def test_pack_unpack_full_size(oracle_mod, name):
    _full_size_case(oracle_mod, W.get_config(name))
    torch.cuda.empty_cache()


def test_debug_check_tables_names_the_first_session_that_breaks_the_contract():
    """The optional validator: clean tables pass; an id outside the cache, a table row too narrow for its length, a
    negative length and (destination tables only) a block named twice are reported with the session they occur in."""
    cfg = W.WorkloadConfig(name="chk", index=70, dtype="bf16", n_layers=1, n_q_heads=2, n_kv_heads=2, head_dim=16,
                           block_size=16, n_blocks=64, n_sessions=5, prefix_dist=("uniform", 20, 90),
                           new_dist=("const", 1), sigma=1.0, scale=0.1)
    sess = W.make_sessions(cfg, 2)
    pool = torch.zeros((1, cfg.n_blocks, cfg.block_size, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device=DEV)
    cache = S.KVCache(pool, pool.clone())
    lens = torch.from_numpy(sess.prefix_lens).to(DEV)

    def run(table, lens_t=lens, dst=True):
        return S.debug_check_tables(cache, torch.from_numpy(table).to(DEV), lens_t, dst)

    good = sess.block_table.copy()
    assert run(good) == -1 and run(good, dst=False) == -1
    bad = good.copy(); bad[3, 1] = cfg.n_blocks                     # not a block of the cache
    assert run(bad) == 3 and run(bad, dst=False) == 3
    bad = good.copy(); bad[2, 0] = -1
    assert run(bad) == 2
    bad = good.copy(); bad[4, 0] = good[1, 0]                       # two writers for one block
    assert run(bad) == 4 and run(bad, dst=False) == -1              # legal in a source table (shared prefix)
    bad = good.copy(); bad[1, 1] = good[1, 0]                       # twice inside one session
    assert run(bad) == 1
    narrow = np.ascontiguousarray(good[:, :2])                      # 32 tokens per row at most
    first_long = int(np.argmax(sess.prefix_lens > 32))
    assert run(narrow) == first_long
    neg = sess.prefix_lens.copy(); neg[0] = -5
    assert run(good, torch.from_numpy(neg).to(DEV)) == 0
    bad = good.copy(); bad[2, 4] = 10 ** 6                          # beyond the session's blocks: ignored
    assert run(bad) == -1
