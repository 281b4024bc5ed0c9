"""Session lengths and block tables for a workload config (host, numpy, seeded)."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

from .configs import WorkloadConfig


@dataclass
class SessionBatch:
    cfg: WorkloadConfig
    prefix_lens: np.ndarray          # int32 [S]   cached tokens per session
    new_lens: np.ndarray             # int32 [S]   tokens of the new turn
    block_table: np.ndarray          # int32 [S, table_stride]   physical block ids, -1 beyond the session's blocks
    dst_block_table: Optional[np.ndarray]  # int32 [S, table_stride]  a disjoint "free list" assignment, or None
    buf_token_offsets: np.ndarray    # int64 [S+1]  exclusive prefix sum of prefix_lens
    cu_new_lens: np.ndarray          # int32 [S+1]  exclusive prefix sum of new_lens

    @property
    def n_sessions(self) -> int:
        return int(self.prefix_lens.shape[0])

    @property
    def table_stride(self) -> int:
        return int(self.block_table.shape[1])

    @property
    def total_prefix_tokens(self) -> int:
        return int(self.buf_token_offsets[-1])

    @property
    def total_new_tokens(self) -> int:
        return int(self.cu_new_lens[-1])

    @property
    def max_prefix_len(self) -> int:
        return int(self.prefix_lens.max()) if self.n_sessions else 0

    @property
    def max_new_len(self) -> int:
        return int(self.new_lens.max()) if self.n_sessions else 0

    def blocks_per_session(self) -> np.ndarray:
        bs = self.cfg.block_size
        return (self.prefix_lens.astype(np.int64) + bs - 1) // bs

    def owned_blocks(self, dst: bool = False) -> np.ndarray:
        """All physical block ids listed for valid tokens (source or destination table), flattened."""
        tab = self.dst_block_table if dst else self.block_table
        nb = self.blocks_per_session()
        return np.concatenate([tab[s, : nb[s]] for s in range(self.n_sessions)]) if self.n_sessions else \
            np.zeros(0, np.int32)

    def table_with_room_for_the_new_turn(self, seed: int = 0) -> np.ndarray:
        """The block table extended so that it also covers positions P_s .. P_s + N_s - 1: the extra blocks are
        drawn (seeded, without replacement) from the blocks that no source or destination table lists."""
        bs = self.cfg.block_size
        need = (self.prefix_lens.astype(np.int64) + self.new_lens + bs - 1) // bs
        have = self.blocks_per_session()
        used = np.zeros(self.cfg.n_blocks, dtype=bool)
        used[self.owned_blocks()] = True
        if self.dst_block_table is not None:
            used[self.owned_blocks(dst=True)] = True
        free = np.random.default_rng(7000 + seed).permutation(np.nonzero(~used)[0]).astype(np.int32)
        extra = int(np.sum(need - have))
        if extra > free.size:
            raise ValueError("pool too small to extend the tables")
        table = np.full((self.n_sessions, max(int(need.max()) if need.size else 1, 1)), -1, dtype=np.int32)
        at = 0
        for s in range(self.n_sessions):
            table[s, : have[s]] = self.block_table[s, : have[s]]
            n = int(need[s] - have[s])
            table[s, have[s]: have[s] + n] = free[at: at + n]
            at += n
        return table

    def payload_bytes(self) -> int:
        """Bytes of the migration buffer: K and V of every layer for every cached token."""
        return self.total_prefix_tokens * self.cfg.kv_bytes_per_token()

    def attn_flops(self) -> float:
        """4 * H_q * d * sum_s N_s * (P_s + (N_s + 1) / 2): QK^T and PV over the visible region only."""
        n = self.new_lens.astype(np.float64)
        p = self.prefix_lens.astype(np.float64)
        return float(4.0 * self.cfg.n_q_heads * self.cfg.head_dim * np.sum(n * (p + (n + 1.0) / 2.0)))

    def attn_bytes(self) -> int:
        """One pass over the cached K,V of one layer plus Q, O, K_new, V_new."""
        c = self.cfg
        kv = self.total_prefix_tokens * 2 * c.row_elems * c.elem_bytes
        qo = self.total_new_tokens * (2 * c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim * c.elem_bytes
        return int(kv + qo)


def _draw_lengths(dist, n, rng: np.random.Generator, block_size: int) -> np.ndarray:
    kind = dist[0]
    if kind == "const":
        return np.full(n, dist[1], dtype=np.int32)
    if kind == "uniform":
        return rng.integers(dist[1], dist[2] + 1, size=n).astype(np.int32)
    if kind == "geometric":
        _, mean, lo, hi = dist
        p = np.clip(rng.geometric(1.0 / mean, size=n), lo, hi).astype(np.int64)
        # every last block partially filled
        full = (p % block_size) == 0
        p = np.where(full, np.where(p >= hi, p - 1, p + 1), p)
        return p.astype(np.int32)
    if kind == "lognormal":
        _, median, sigma, lo, hi = dist
        v = np.rint(np.exp(rng.normal(np.log(median), sigma, size=n)))
        return np.clip(v, lo, hi).astype(np.int32)
    if kind == "mixed":
        _, n_decode, median, sigma, lo, hi = dist
        n_decode = min(n_decode, n)
        out = np.ones(n, dtype=np.int32)
        order = rng.permutation(n)
        prefill_rows = np.sort(order[n_decode:])
        v = np.rint(np.exp(rng.normal(np.log(median), sigma, size=prefill_rows.shape[0])))
        out[prefill_rows] = np.clip(v, lo, hi).astype(np.int32)
        return out
    raise ValueError(f"unknown length distribution {kind!r}")


def make_sessions(cfg: WorkloadConfig, seed: Optional[int] = None, new_lens: Optional[np.ndarray] = None) -> SessionBatch:
    """Draw lengths, then hand every session consecutive slices of one seeded permutation of the pool.
    ``new_lens``: new-turn lengths to use in place of the drawn ones (same draws otherwise).

    A session's blocks are therefore a uniform sample without replacement of the whole pool, listed in
    random order (fragmented); the destination table (the "fresh free list") takes the next slices of
    the same permutation, so it shares no block with any source table.
    """
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    S, bs = cfg.n_sessions, cfg.block_size
    prefix = _draw_lengths(cfg.prefix_dist, S, rng, bs)
    new = _draw_lengths(cfg.new_dist, S, rng, bs)
    if new_lens is not None:
        new = np.asarray(new_lens, dtype=np.int32).reshape(S)
    nblk = (prefix.astype(np.int64) + bs - 1) // bs
    total_blk = int(nblk.sum())
    need = total_blk * (2 if cfg.fresh_tables else 1)
    if need > cfg.n_blocks:
        raise ValueError(f"{cfg.name}: {need} blocks needed, pool has {cfg.n_blocks}")
    perm = rng.permutation(cfg.n_blocks).astype(np.int32)
    stride = max(1, int(nblk.max()) if S else 1)
    table = np.full((S, stride), -1, dtype=np.int32)
    dst = np.full((S, stride), -1, dtype=np.int32) if cfg.fresh_tables else None
    at = 0
    for s in range(S):
        table[s, : nblk[s]] = perm[at: at + nblk[s]]
        at += int(nblk[s])
    if dst is not None:
        for s in range(S):
            dst[s, : nblk[s]] = perm[at: at + nblk[s]]
            at += int(nblk[s])
    off = np.zeros(S + 1, dtype=np.int64)
    off[1:] = np.cumsum(prefix.astype(np.int64))
    cu = np.zeros(S + 1, dtype=np.int32)
    cu[1:] = np.cumsum(new.astype(np.int64)).astype(np.int32)
    return SessionBatch(cfg, prefix, new, table, dst, off, cu)


@dataclass
class UnitBatch:
    """Single layers of sessions ("units") that live in one pool of slots and in chunks of a larger buffer."""
    unit_lens: np.ndarray          # int32 [U] tokens per unit
    unit_table: np.ndarray         # int32 [U][stride] slot of every block, unused entries negative
    unit_chunk_rows: np.ndarray    # int64 [U] first row (K rows, then as many V rows) in the buffer
    unit_token_offsets: np.ndarray # int64 [U+1] exclusive prefix sum of unit_lens
    n_buf_rows: int

    @property
    def n_units(self) -> int:
        return int(self.unit_lens.shape[0])

    @property
    def total_tokens(self) -> int:
        return int(self.unit_token_offsets[-1])


def make_units(rng: np.random.Generator, n_units: int, n_slots: int, block_size: int, max_len: int, min_len: int = 0,
               max_gap_rows: int = 3) -> UnitBatch:
    """Units of random length with disjoint random slot tables; their chunks lie in random order, with random gaps,
    in one buffer of ``n_buf_rows`` rows."""
    lens = rng.integers(min_len, max_len + 1, size=n_units).astype(np.int32)
    nbs = -(-lens // block_size)
    if int(nbs.sum()) > n_slots:
        raise ValueError("pool too small for these units")
    perm = rng.permutation(n_slots)[: int(nbs.sum())].astype(np.int32)
    stride = max(int(nbs.max()) if n_units else 0, 1) + 1
    table = np.full((n_units, stride), -7, dtype=np.int32)
    at = 0
    for u in range(n_units):
        table[u, : nbs[u]] = perm[at: at + nbs[u]]
        at += int(nbs[u])
    chunk_rows = np.zeros(n_units, dtype=np.int64)
    row_at = 2
    for u in rng.permutation(n_units):
        chunk_rows[u] = row_at
        row_at += 2 * int(lens[u]) + int(rng.integers(0, max_gap_rows + 1))
    offsets = np.concatenate([[0], np.cumsum(lens.astype(np.int64))]).astype(np.int64)
    return UnitBatch(lens, table, chunk_rows, offsets, row_at + 1)
