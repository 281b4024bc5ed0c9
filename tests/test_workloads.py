"""The seeded input generators: determinism, stated recipes, host/device bit agreement."""
import numpy as np
import pytest
import torch

import workloads as W


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 65504.0, 1e-30], np.float32)])
    ours = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    assert np.array_equal(W.bf16_bits_to_f32(ours), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_counter_bits_host_equals_torch_and_spreads():
    idx = np.concatenate([np.arange(0, 5000), np.arange(2 ** 32 - 100, 2 ** 32 + 100), np.arange(2 ** 36, 2 ** 36 + 1000)])
    for salt in (0, 1):
        h = W.counter_bits_host(1001, salt, idx)
        d = W.counter_bits_device(1001, salt, torch.from_numpy(idx)).numpy().view(np.uint16)
        assert np.array_equal(h, d)
    a = W.counter_bits_host(1001, 0, idx)
    b = W.counter_bits_host(1001, 1, idx)
    assert np.mean(a == b) < 0.01 and len(np.unique(a)) > 4000


def test_device_fill_equals_host_counter_pool():
    cfg = W.scaled_config(W.get_config("llama8b"), n_layers=2, n_sessions=3, prefix_scale=0.01, new_scale=0.1, n_blocks=64)
    sess = W.make_sessions(cfg)
    kh, vh = W.make_pool_host(cfg, sess, kind="counter")
    shape = kh.shape
    kt = torch.zeros(shape, dtype=torch.int16)
    vt = torch.zeros(shape, dtype=torch.int16)
    blocks = sess.owned_blocks()
    W.fill_pool_blocks_device(kt, vt, cfg, blocks, max_chunk_elems=1 << 16)
    assert np.array_equal(kt.numpy().view(np.uint16)[:, blocks], kh[:, blocks])
    assert np.array_equal(vt.numpy().view(np.uint16)[:, blocks], vh[:, blocks])
    others = np.setdiff1d(np.arange(cfg.n_blocks), blocks)
    assert not kt[:, others].any()


@pytest.mark.parametrize("idx", range(5))
def test_config_recipes(idx):
    cfg = W.get_config(idx)
    sess = W.make_sessions(cfg)
    again = W.make_sessions(cfg)
    assert np.array_equal(sess.block_table, again.block_table) and np.array_equal(sess.new_lens, again.new_lens)
    P, N = sess.prefix_lens, sess.new_lens
    if cfg.name == "tiny_fp32":
        assert (P[0], N[0]) == (256, 32) and len(set(sess.block_table[0])) == 16 and sess.block_table.max() < 48
    if cfg.name == "llama8b":
        assert P.min() >= 1024 and P.max() <= 8192 and N.min() >= 16 and N.max() <= 1024 and len(P) == 16
    if cfg.name == "llama70b_long":
        assert (P[0], N[0]) == (32768, 512) and sess.payload_bytes() == 10 * 2 ** 30
    if cfg.name == "many_short":
        assert len(P) == 256 and np.all(P % 16 != 0) and P.min() >= 16 and P.max() <= 4096 and np.all(N == 64)
        assert 300 < P.mean() < 900
    if cfg.name == "mixed_resume":
        assert len(P) == 128 and np.sum(N == 1) >= 96 and np.sum(N > 1) <= 32 and N.max() <= 2048
        assert P.min() >= 512 and P.max() <= 16384
    # tables: distinct blocks, source and destination disjoint
    src = sess.owned_blocks()
    assert len(np.unique(src)) == len(src) and src.min() >= 0 and src.max() < cfg.n_blocks
    if sess.dst_block_table is not None:
        dst = sess.owned_blocks(dst=True)
        assert len(np.unique(dst)) == len(dst) and not np.intersect1d(src, dst).size
    assert sess.buf_token_offsets[-1] == P.sum() and sess.cu_new_lens[-1] == N.sum()


def test_attn_inputs_sentinel_outside_valid_slots():
    cfg = W.scaled_config(W.get_config("many_short"), n_layers=1, n_sessions=6, prefix_scale=0.05, n_blocks=128)
    sess = W.make_sessions(cfg)
    k_pool, v_pool, q, k_new, v_new = W.make_attn_inputs(cfg, sess)
    valid = np.zeros(k_pool.shape[:2], dtype=bool)
    for s in range(sess.n_sessions):
        for t in range(int(sess.prefix_lens[s])):
            valid[sess.block_table[s, t // 16], t % 16] = True
    for pool in (k_pool, v_pool):
        is_sent = np.all(pool == W.SENTINEL16, axis=(2, 3))
        assert np.array_equal(is_sent, ~valid)
    assert q.shape == (sess.total_new_tokens, 32, 128) and k_new.shape == (sess.total_new_tokens, 8, 128)
    std = W.bf16_bits_to_f32(q).std()
    assert 0.9 < std < 1.1
