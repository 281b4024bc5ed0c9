"""Tensor values for the workloads: seeded Gaussian draws and a counter-based bit generator.

Nothing here gathers, scatters or attends: pools are filled block by block (a block id is just a row
index of the pool array), never through a token -> slot mapping.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np

from .configs import WorkloadConfig
from .sessions import SessionBatch

# bf16 quiet-NaN pattern used for every pool slot that no valid token owns: a kernel that reads such a
# slot into its arithmetic produces NaN, and a scatter that writes one shows up as a changed sentinel.
SENTINEL16 = 0x7FC1
SENTINEL32 = 0x7FC00001

_M32 = 0xFFFFFFFF


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even) and return the 16-bit patterns.  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---------------------------------------------------------------------------------------------------------
# counter-based bits: identical on numpy int64 and torch int64 (only the low 32 bits of products are kept)
# ---------------------------------------------------------------------------------------------------------
def _mix32(x):
    """A 32-bit avalanche mixer (multiply / xor-shift rounds) on non-negative values held in int64."""
    x = x ^ (x >> 16)
    x = (x * 0x7FEB352D) & _M32
    x = x ^ (x >> 15)
    x = (x * 0x846CA68B) & _M32
    x = x ^ (x >> 16)
    return x


def _counter16(seed: int, salt: int, idx):
    lo = idx & _M32
    hi = (idx >> 32) & _M32
    key = (seed * 0x9E3779B1 + salt * 0x85EBCA6B + 0x27D4EB2F) & _M32
    h = _mix32((hi + key) & _M32)
    return _mix32(lo ^ h) & 0xFFFF


def counter_bits_host(seed: int, salt: int, idx: np.ndarray) -> np.ndarray:
    """16-bit pattern for each element index (int64 array) under (seed, salt); numpy."""
    return _counter16(int(seed), int(salt), np.asarray(idx, dtype=np.int64)).astype(np.uint16)


def counter_bits_device(seed: int, salt: int, idx):
    """Same function on a torch int64 tensor (any device); returns int16 holding the same bit patterns."""
    import torch
    v = _counter16(int(seed), int(salt), idx.to(torch.int64))
    # map [0, 65536) onto int16's two's complement without changing bits
    v = torch.where(v >= 32768, v - 65536, v)
    return v.to(torch.int16)


def pool_elem_index(cfg: WorkloadConfig, layer, block, slot=0, col=0):
    """Element index inside the dense [L][n_blocks][bs][H_kv*d] K pool (or V pool)."""
    return ((np.asarray(layer, dtype=np.int64) * cfg.n_blocks + np.asarray(block, dtype=np.int64)) * cfg.block_size
            + np.asarray(slot, dtype=np.int64)) * cfg.row_elems + np.asarray(col, dtype=np.int64)


# ---------------------------------------------------------------------------------------------------------
# host pools (small cases, and the one attention layer of the large ones)
# ---------------------------------------------------------------------------------------------------------
def _np_dtype(cfg: WorkloadConfig):
    return np.uint16 if cfg.dtype == "bf16" else np.float32


def _draw(rng: np.random.Generator, shape, cfg: WorkloadConfig) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if cfg.sigma != 1.0:
        x *= np.float32(cfg.sigma)
    return f32_to_bf16_bits(x).reshape(shape) if cfg.dtype == "bf16" else x


def _sentinel_fill(a: np.ndarray, cfg: WorkloadConfig) -> None:
    if cfg.dtype == "bf16":
        a[...] = SENTINEL16
    else:
        a.view(np.uint32)[...] = SENTINEL32


def make_pool_host(cfg: WorkloadConfig, sess: SessionBatch, seed: Optional[int] = None, *, kind: str = "rng",
                   n_layers: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """K and V pools ``[L][n_blocks][bs][H_kv][d]`` on the host (bf16 bit patterns as uint16, or float32).

    kind="rng": every slot of every block is an N(0, sigma) draw (unowned blocks too, so a misdirected read
    returns plausible but wrong numbers).  kind="counter": every slot holds the counter-based pattern of its
    own element index, the same bits ``fill_pool_blocks_device`` writes.
    """
    L = cfg.n_layers if n_layers is None else n_layers
    shape = (L, cfg.n_blocks, cfg.block_size, cfg.n_kv_heads, cfg.head_dim)
    seed = (cfg.seed if seed is None else seed)
    if kind == "rng":
        rng = np.random.default_rng(seed + 7)
        return _draw(rng, shape, cfg), _draw(rng, shape, cfg)
    if kind == "counter":
        if cfg.dtype != "bf16":
            raise ValueError("counter pools are 16-bit")
        idx = np.arange(int(np.prod(shape)), dtype=np.int64)
        return (counter_bits_host(seed, 0, idx).reshape(shape), counter_bits_host(seed, 1, idx).reshape(shape))
    raise ValueError(kind)


def make_attn_inputs(cfg: WorkloadConfig, sess: SessionBatch, seed: Optional[int] = None):
    """Inputs of one attention layer: (k_pool, v_pool, q, k_new, v_new).

    Pools are ``[n_blocks][bs][H_kv][d]``: owned blocks hold N(0, sigma) draws, every other slot (unowned
    blocks, and the unused tail slots of a session's partially filled last block) holds the NaN sentinel.
    q is ``[T][H_q][d]``; k_new, v_new are ``[T][H_kv][d]`` with T = sum of new-turn lengths.
    """
    seed = (cfg.seed if seed is None else seed)
    rng = np.random.default_rng(seed + 13)
    bs = cfg.block_size
    pshape = (cfg.n_blocks, bs, cfg.n_kv_heads, cfg.head_dim)
    k_pool = np.empty(pshape, dtype=_np_dtype(cfg))
    v_pool = np.empty(pshape, dtype=_np_dtype(cfg))
    _sentinel_fill(k_pool, cfg)
    _sentinel_fill(v_pool, cfg)
    nblk = sess.blocks_per_session()
    for s in range(sess.n_sessions):
        ids = sess.block_table[s, : nblk[s]]
        if ids.size == 0:
            continue
        bshape = (ids.size, bs, cfg.n_kv_heads, cfg.head_dim)
        k_pool[ids] = _draw(rng, bshape, cfg)
        v_pool[ids] = _draw(rng, bshape, cfg)
        tail = int(sess.prefix_lens[s]) % bs
        if tail:
            _sentinel_fill(k_pool[ids[-1], tail:], cfg)
            _sentinel_fill(v_pool[ids[-1], tail:], cfg)
    T = sess.total_new_tokens
    q = _draw(rng, (T, cfg.n_q_heads, cfg.head_dim), cfg)
    k_new = _draw(rng, (T, cfg.n_kv_heads, cfg.head_dim), cfg)
    v_new = _draw(rng, (T, cfg.n_kv_heads, cfg.head_dim), cfg)
    return k_pool, v_pool, q, k_new, v_new


# ---------------------------------------------------------------------------------------------------------
# device pools (multi-layer pools too large to draw on the host)
# ---------------------------------------------------------------------------------------------------------
def fill_pool_blocks_device(k_pool, v_pool, cfg: WorkloadConfig, blocks: np.ndarray, seed: Optional[int] = None,
                            max_chunk_elems: int = 1 << 27) -> None:
    """Write the counter-based pattern into ``blocks`` of every layer of two torch pools (in place).

    ``k_pool`` / ``v_pool``: 16-bit tensors of shape ``[L][n_blocks][bs][H_kv][d]`` on any device.
    Element e of the K pool gets ``counter(seed, 0, e)``, of the V pool ``counter(seed, 1, e)``.
    """
    import torch
    seed = (cfg.seed if seed is None else seed)
    L = k_pool.shape[0]
    dev = k_pool.device
    be = cfg.block_elems
    blocks_t = torch.as_tensor(np.asarray(blocks, dtype=np.int64), device=dev)
    within = torch.arange(be, dtype=torch.int64, device=dev)
    per_chunk = max(1, max_chunk_elems // be)
    for salt, pool in ((0, k_pool), (1, v_pool)):
        flat = pool.view(torch.int16).view(L, cfg.n_blocks, be)
        for layer in range(L):
            for c0 in range(0, blocks_t.numel(), per_chunk):
                b = blocks_t[c0: c0 + per_chunk]
                idx = ((layer * cfg.n_blocks + b) * be)[:, None] + within[None, :]
                flat[layer].index_copy_(0, b, counter_bits_device(seed, salt, idx))


def make_attn_inputs_device(cfg: WorkloadConfig, sess: SessionBatch, device, seed: Optional[int] = None):
    """The inputs of one attention layer drawn ON the device, for timing runs whose pools are too large to draw on the
    host in reasonable time: (k_pool, v_pool, q, k_new, v_new) as torch bf16 tensors of the shapes of
    ``make_attn_inputs``, every element an N(0, sigma) draw of a seeded torch generator (all blocks hold finite values;
    there is no sentinel).  Lengths and block tables are those of ``sess``."""
    import torch
    if cfg.dtype != "bf16":
        raise ValueError("device-drawn inputs are bf16")
    gen = torch.Generator(device=device)
    gen.manual_seed((cfg.seed if seed is None else seed) + 13)

    def draw(shape):
        out = torch.empty(shape, dtype=torch.bfloat16, device=device)
        step = max(1, (1 << 28) // max(1, int(np.prod(shape[1:]))))        # fp32 staging of at most 1 GiB at a time
        for a in range(0, shape[0], step):
            b = min(shape[0], a + step)
            x = torch.randn((b - a,) + tuple(shape[1:]), generator=gen, device=device, dtype=torch.float32)
            out[a:b] = (x * cfg.sigma).to(torch.bfloat16)
        return out
    pshape = (cfg.n_blocks, cfg.block_size, cfg.n_kv_heads, cfg.head_dim)
    T = sess.total_new_tokens
    return (draw(pshape), draw(pshape), draw((T, cfg.n_q_heads, cfg.head_dim)),
            draw((T, cfg.n_kv_heads, cfg.head_dim)), draw((T, cfg.n_kv_heads, cfg.head_dim)))
