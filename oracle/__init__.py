"""ctypes front-end of the CPU oracle (``symph_oracle.c``).

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the benchmark's CPU-baseline leg may import
this; the product package never does, and this module never imports the product package.

Arrays are numpy: bf16 tensors travel as ``uint16`` bit patterns, fp32 tensors as ``float32``.  A K or V pool
is a C-contiguous array ``[L][n_blocks][bs][H_kv][d]`` (or ``[n_blocks][bs][H_kv][d]`` for a single layer).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "symph_oracle.c")
# ORACLE_LIBRARY_PATH: load another build of the same source (the sanitizer job sets it in its child process)
_LIB = os.environ.get("ORACLE_LIBRARY_PATH") or os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2, OpenMP on the outermost loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", tmp, _SRC,
                               "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = C.CDLL(_LIB)
        i32, i64, vp, f32 = C.c_int32, C.c_int64, C.c_void_p, C.c_float
        lib.oracle_num_threads.restype = C.c_int
        lib.oracle_kv_buffer_bytes.restype = i64
        lib.oracle_kv_buffer_bytes.argtypes = [i32, i32, i32, i32, i64]
        lib.oracle_kv_locate.restype = None
        lib.oracle_kv_locate.argtypes = [i64, i64, i32, i32, i32, i32, vp, i32, vp, vp, i32, i32, i32, i32, vp, vp]
        lib.oracle_kv_row_map.restype = None
        lib.oracle_kv_row_map.argtypes = [i64, i64, i32, i32, i32, i32, vp, i32, vp, vp, i32, vp, vp]
        for fn in (lib.oracle_kv_pack, lib.oracle_kv_unpack):
            fn.restype = C.c_int
            fn.argtypes = [vp, vp, i64, i64, i32, i32, i32, i32, i32, vp, i32, vp, vp, i32, vp]
        for fn in (lib.oracle_kv_pack_layers, lib.oracle_kv_unpack_layers):
            fn.restype = C.c_int
            fn.argtypes = [vp, vp, i64, i64, i32, i32, i32, i32, i32, vp, i32, vp, vp, i32, vp, i32, i32]
        lib.oracle_kv_copy_batch_layers.restype = C.c_int
        lib.oracle_kv_copy_batch_layers.argtypes = [i32, vp, vp, i64, i64, i32, i32, i32, i32, i32, vp, i32, vp, vp, i32, vp,
                                                    i32, i32]
        for fn in (lib.oracle_kv_pack_tail, lib.oracle_kv_unpack_tail):
            fn.restype = C.c_int
            fn.argtypes = [vp, vp, i64, i64, i32, i32, i32, i32, i32, vp, i32, vp, vp, vp, i32, vp]
        for fn in (lib.oracle_kv_pack_units, lib.oracle_kv_unpack_units):
            fn.restype = C.c_int
            fn.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp, i32, vp, vp, i32, vp]
        lib.oracle_kv_append.restype = C.c_int
        lib.oracle_kv_append.argtypes = [vp, vp, i64, i64, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, i32, i32]
        lib.oracle_prefix_prefill_attn.restype = C.c_int
        lib.oracle_prefix_prefill_attn.argtypes = [vp, vp, i64, i64, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp,
                                                   i32, i32, i32, f32, vp, i32, vp]
        lib.oracle_attn_row_weights.restype = C.c_int
        lib.oracle_attn_row_weights.argtypes = [vp, vp, i64, i64, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp,
                                                i32, i32, f32, i32, i32, i32, vp, vp]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _check(a: np.ndarray, dtype=None, name="array") -> np.ndarray:
    if not isinstance(a, np.ndarray) or not a.flags.c_contiguous:
        raise ValueError(f"{name} must be a C-contiguous numpy array")
    if dtype is not None and a.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {a.dtype}")
    return a


def _pool_geometry(k_pool: np.ndarray, v_pool: np.ndarray) -> Tuple[int, int, int, int, int, int, int, int]:
    """(L, n_blocks, bs, H_kv, d, elem_bytes, layer_stride, block_stride) of dense pools."""
    _check(k_pool, name="k_pool")
    _check(v_pool, name="v_pool")
    if k_pool.shape != v_pool.shape or k_pool.dtype != v_pool.dtype:
        raise ValueError("K and V pools must agree in shape and dtype")
    if k_pool.dtype not in (np.uint16, np.float32):
        raise ValueError("pools are uint16 (bf16 bits) or float32")
    shape = k_pool.shape if k_pool.ndim == 5 else (1,) + tuple(k_pool.shape)
    if len(shape) != 5:
        raise ValueError("pool must be [L][n_blocks][bs][H_kv][d] or [n_blocks][bs][H_kv][d]")
    L, nb, bs, hkv, d = (int(x) for x in shape)
    block_stride = bs * hkv * d
    return L, nb, bs, hkv, d, k_pool.dtype.itemsize, nb * block_stride, block_stride


def kv_buffer_bytes(n_layers: int, n_kv_heads: int, head_dim: int, elem_bytes: int, total_tokens: int) -> int:
    return int(_load().oracle_kv_buffer_bytes(n_layers, n_kv_heads, head_dim, elem_bytes, total_tokens))


def kv_locate(layer_stride: int, block_stride: int, n_layers: int, block_size: int, n_kv_heads: int, head_dim: int,
              table: np.ndarray, prefix_lens: np.ndarray, offsets: np.ndarray, s: int, l: int, kv: int, t: int
              ) -> Tuple[int, int]:
    """(pool element offset, buffer element offset) of one token row."""
    table = _check(table, np.int32, "table")
    prefix_lens = _check(prefix_lens, np.int32, "prefix_lens")
    offsets = _check(offsets, np.int64, "offsets")
    pe, be = C.c_int64(), C.c_int64()
    _load().oracle_kv_locate(layer_stride, block_stride, n_layers, block_size, n_kv_heads, head_dim, _ptr(table),
                             table.shape[1], _ptr(prefix_lens), _ptr(offsets), s, l, kv, t, C.byref(pe), C.byref(be))
    return int(pe.value), int(be.value)


def kv_row_map(layer_stride: int, block_stride: int, n_layers: int, block_size: int, n_kv_heads: int, head_dim: int,
               table: np.ndarray, prefix_lens: np.ndarray, offsets: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """For every row of the migration buffer, in buffer order: (element offset of its source row inside its pool,
    0 for K / 1 for V).  ``oracle_kv_locate`` for every (session, layer, K|V, token), as two arrays."""
    table = _check(table, np.int32, "table")
    prefix_lens = _check(prefix_lens, np.int32, "prefix_lens")
    offsets = _check(offsets, np.int64, "offsets")
    S = prefix_lens.shape[0]
    n_rows = int(offsets[S]) * 2 * n_layers
    pool_elem = np.full(n_rows, -1, dtype=np.int64)
    kv = np.full(n_rows, 255, dtype=np.uint8)
    _load().oracle_kv_row_map(layer_stride, block_stride, n_layers, block_size, n_kv_heads, head_dim, _ptr(table),
                              table.shape[1], _ptr(prefix_lens), _ptr(offsets), S, _ptr(pool_elem), _ptr(kv))
    return pool_elem, kv


def kv_pack(k_pool: np.ndarray, v_pool: np.ndarray, table: np.ndarray, prefix_lens: np.ndarray,
            offsets: np.ndarray) -> np.ndarray:
    """Gather every session's cached K,V into a new migration buffer (1-D array of the pool dtype)."""
    L, nb, bs, hkv, d, eb, ls, bst = _pool_geometry(k_pool, v_pool)
    table = _check(table, np.int32, "table")
    prefix_lens = _check(prefix_lens, np.int32, "prefix_lens")
    offsets = _check(offsets, np.int64, "offsets")
    S = prefix_lens.shape[0]
    n_elems = int(offsets[S]) * 2 * L * hkv * d
    buf = np.zeros(n_elems, dtype=k_pool.dtype)
    rc = _load().oracle_kv_pack(_ptr(k_pool), _ptr(v_pool), ls, bst, L, bs, hkv, d, eb, _ptr(table), table.shape[1],
                                _ptr(prefix_lens), _ptr(offsets), S, _ptr(buf))
    if rc != 0:
        raise RuntimeError("oracle_kv_pack failed")
    return buf


def kv_unpack(k_pool: np.ndarray, v_pool: np.ndarray, table: np.ndarray, prefix_lens: np.ndarray,
              offsets: np.ndarray, buf: np.ndarray) -> None:
    """Scatter a migration buffer into the pools (modified in place) through ``table``."""
    L, nb, bs, hkv, d, eb, ls, bst = _pool_geometry(k_pool, v_pool)
    table = _check(table, np.int32, "table")
    prefix_lens = _check(prefix_lens, np.int32, "prefix_lens")
    offsets = _check(offsets, np.int64, "offsets")
    buf = _check(buf, k_pool.dtype, "buf")
    S = prefix_lens.shape[0]
    if buf.size != int(offsets[S]) * 2 * L * hkv * d:
        raise ValueError("buffer size does not match the sessions")
    rc = _load().oracle_kv_unpack(_ptr(k_pool), _ptr(v_pool), ls, bst, L, bs, hkv, d, eb, _ptr(table),
                                  table.shape[1], _ptr(prefix_lens), _ptr(offsets), S, _ptr(buf))
    if rc != 0:
        raise RuntimeError("oracle_kv_unpack failed")


def tail_offsets(prefix_lens: np.ndarray, tail_begin: np.ndarray) -> np.ndarray:
    """Exclusive prefix sum (int64, S+1 entries) of the tail lengths prefix_lens - tail_begin."""
    t = prefix_lens.astype(np.int64) - tail_begin.astype(np.int64)
    return np.concatenate([[0], np.cumsum(t)]).astype(np.int64)


def kv_pack_tail(k_pool: np.ndarray, v_pool: np.ndarray, table: np.ndarray, prefix_lens: np.ndarray,
                 tail_begin: np.ndarray) -> np.ndarray:
    """Gather tokens ``tail_begin[s] .. prefix_lens[s]-1`` of every session, all layers (Sec. 3.3 write-back of what a
    turn added).  Returns the buffer: layout of a migration buffer for sessions of the tail lengths."""
    L, nb, bs, hkv, d, eb, ls, bst = _pool_geometry(k_pool, v_pool)
    table = _check(table, np.int32, "table")
    prefix_lens = _check(prefix_lens, np.int32, "prefix_lens")
    tail_begin = _check(tail_begin, np.int32, "tail_begin")
    S = prefix_lens.shape[0]
    offsets = tail_offsets(prefix_lens, tail_begin)
    buf = np.zeros(int(offsets[S]) * 2 * L * hkv * d, dtype=k_pool.dtype)
    rc = _load().oracle_kv_pack_tail(_ptr(k_pool), _ptr(v_pool), ls, bst, L, bs, hkv, d, eb, _ptr(table),
                                     table.shape[1], _ptr(prefix_lens), _ptr(tail_begin), _ptr(offsets), S, _ptr(buf))
    if rc != 0:
        raise RuntimeError("oracle_kv_pack_tail failed")
    return buf


def kv_unpack_tail(k_pool: np.ndarray, v_pool: np.ndarray, table: np.ndarray, prefix_lens: np.ndarray,
                   tail_begin: np.ndarray, buf: np.ndarray) -> None:
    """Scatter a tail buffer (see ``kv_pack_tail``) into the pools, in place; nothing but the tails' slots changes."""
    L, nb, bs, hkv, d, eb, ls, bst = _pool_geometry(k_pool, v_pool)
    table = _check(table, np.int32, "table")
    prefix_lens = _check(prefix_lens, np.int32, "prefix_lens")
    tail_begin = _check(tail_begin, np.int32, "tail_begin")
    buf = _check(buf, k_pool.dtype, "buf")
    S = prefix_lens.shape[0]
    offsets = tail_offsets(prefix_lens, tail_begin)
    if buf.size != int(offsets[S]) * 2 * L * hkv * d:
        raise ValueError("buffer size does not match the tails")
    rc = _load().oracle_kv_unpack_tail(_ptr(k_pool), _ptr(v_pool), ls, bst, L, bs, hkv, d, eb, _ptr(table),
                                       table.shape[1], _ptr(prefix_lens), _ptr(tail_begin), _ptr(offsets), S, _ptr(buf))
    if rc != 0:
        raise RuntimeError("oracle_kv_unpack_tail failed")


def unit_chunk_rows(offsets: np.ndarray, prefix_lens: np.ndarray, n_layers: int, s: int, layer: int) -> int:
    """Row of a whole migration buffer at which the K rows of layer ``layer`` of session ``s`` begin."""
    return int(offsets[s]) * 2 * n_layers + 2 * layer * int(prefix_lens[s])


def _units_args(k_slots, v_slots, table, unit_lens, chunk_rows, buf):
    L, n_slots, bs, hkv, d, eb, _, bst = _pool_geometry(k_slots, v_slots)
    if L != 1:
        raise ValueError("the slot pool is [n_slots][bs][H_kv][d]")
    table = _check(table, np.int32, "table")
    unit_lens = _check(unit_lens, np.int32, "unit_lens")
    chunk_rows = _check(chunk_rows, np.int64, "chunk_rows")
    buf = _check(buf, k_slots.dtype, "buf")
    U = unit_lens.shape[0]
    row = hkv * d
    for u in range(U):      # the oracle checks its inputs on the host: every row inside the buffer, every slot in the pool
        if chunk_rows[u] < 0 or (int(chunk_rows[u]) + 2 * int(unit_lens[u])) * row > buf.size:
            raise ValueError("a unit lies outside the buffer")
        nb = -(-int(unit_lens[u]) // bs)
        if nb > table.shape[1] or (nb and (table[u, :nb].min() < 0 or table[u, :nb].max() >= n_slots)):
            raise ValueError("a unit's table names a slot outside the pool")
    return (_ptr(k_slots), _ptr(v_slots), bst, bs, hkv, d, eb, _ptr(table), table.shape[1], _ptr(unit_lens),
            _ptr(chunk_rows), U, _ptr(buf))


def kv_pack_units(k_slots: np.ndarray, v_slots: np.ndarray, table: np.ndarray, unit_lens: np.ndarray,
                  chunk_rows: np.ndarray, buf: np.ndarray) -> None:
    """Gather single layers of sessions ("units", Sec. 3.3 priority-based K,V cache) from one pool of slots
    ``[n_slots][bs][H_kv][d]`` into their chunks of ``buf`` (modified in place; nothing else in it changes)."""
    if _load().oracle_kv_pack_units(*_units_args(k_slots, v_slots, table, unit_lens, chunk_rows, buf)) != 0:
        raise RuntimeError("oracle_kv_pack_units failed")


def kv_unpack_units(k_slots: np.ndarray, v_slots: np.ndarray, table: np.ndarray, unit_lens: np.ndarray,
                    chunk_rows: np.ndarray, buf: np.ndarray) -> None:
    """Scatter the units' chunks of ``buf`` into their slots (pool modified in place; nothing else in it changes)."""
    if _load().oracle_kv_unpack_units(*_units_args(k_slots, v_slots, table, unit_lens, chunk_rows, buf)) != 0:
        raise RuntimeError("oracle_kv_unpack_units failed")


def kv_pack_layers(k_pool: np.ndarray, v_pool: np.ndarray, table: np.ndarray, prefix_lens: np.ndarray,
                   offsets: np.ndarray, buf: np.ndarray, layer_begin: int, layer_end: int) -> None:
    """Gather layers ``layer_begin .. layer_end-1`` only into ``buf`` (whole-cache layout, modified in place)."""
    L, nb, bs, hkv, d, eb, ls, bst = _pool_geometry(k_pool, v_pool)
    table = _check(table, np.int32, "table")
    prefix_lens = _check(prefix_lens, np.int32, "prefix_lens")
    offsets = _check(offsets, np.int64, "offsets")
    buf = _check(buf, k_pool.dtype, "buf")
    S = prefix_lens.shape[0]
    if buf.size != int(offsets[S]) * 2 * L * hkv * d:
        raise ValueError("buffer size does not match the sessions")
    rc = _load().oracle_kv_pack_layers(_ptr(k_pool), _ptr(v_pool), ls, bst, L, bs, hkv, d, eb, _ptr(table),
                                       table.shape[1], _ptr(prefix_lens), _ptr(offsets), S, _ptr(buf),
                                       int(layer_begin), int(layer_end))
    if rc != 0:
        raise RuntimeError("oracle_kv_pack_layers failed")


def kv_unpack_layers(k_pool: np.ndarray, v_pool: np.ndarray, table: np.ndarray, prefix_lens: np.ndarray,
                     offsets: np.ndarray, buf: np.ndarray, layer_begin: int, layer_end: int) -> None:
    """Scatter layers ``layer_begin .. layer_end-1`` only of a migration buffer into the pools (in place)."""
    L, nb, bs, hkv, d, eb, ls, bst = _pool_geometry(k_pool, v_pool)
    table = _check(table, np.int32, "table")
    prefix_lens = _check(prefix_lens, np.int32, "prefix_lens")
    offsets = _check(offsets, np.int64, "offsets")
    buf = _check(buf, k_pool.dtype, "buf")
    S = prefix_lens.shape[0]
    if buf.size != int(offsets[S]) * 2 * L * hkv * d:
        raise ValueError("buffer size does not match the sessions")
    rc = _load().oracle_kv_unpack_layers(_ptr(k_pool), _ptr(v_pool), ls, bst, L, bs, hkv, d, eb, _ptr(table),
                                         table.shape[1], _ptr(prefix_lens), _ptr(offsets), S, _ptr(buf),
                                         int(layer_begin), int(layer_end))
    if rc != 0:
        raise RuntimeError("oracle_kv_unpack_layers failed")


def _batch_layers(to_buffer, k_pool, v_pool, table, prefix_lens, offsets, buf, layer_begin, layer_end):
    L, nb, bs, hkv, d, eb, ls, bst = _pool_geometry(k_pool, v_pool)
    table = _check(table, np.int32, "table")
    prefix_lens = _check(prefix_lens, np.int32, "prefix_lens")
    offsets = _check(offsets, np.int64, "offsets")
    buf = _check(buf, k_pool.dtype, "buf")
    S = prefix_lens.shape[0]
    if buf.size != int(offsets[S]) * 2 * L * hkv * d:
        raise ValueError("buffer size does not match the sessions")
    rc = _load().oracle_kv_copy_batch_layers(1 if to_buffer else 0, _ptr(k_pool), _ptr(v_pool), ls, bst, L, bs, hkv, d, eb,
                                             _ptr(table), table.shape[1], _ptr(prefix_lens), _ptr(offsets), S, _ptr(buf),
                                             int(layer_begin), int(layer_end))
    if rc != 0:
        raise RuntimeError("oracle_kv_copy_batch_layers failed")


def kv_pack_batch_layers(k_pool: np.ndarray, v_pool: np.ndarray, table: np.ndarray, prefix_lens: np.ndarray,
                         offsets: np.ndarray, buf: np.ndarray, layer_begin: int, layer_end: int) -> None:
    """Gather layers ``layer_begin .. layer_end-1`` into ``buf`` laid out layer -> session -> K|V -> token (in place):
    layer l of the whole batch is the contiguous piece of 2 * total rows that starts at row l * 2 * total."""
    _batch_layers(True, k_pool, v_pool, table, prefix_lens, offsets, buf, layer_begin, layer_end)


def kv_unpack_batch_layers(k_pool: np.ndarray, v_pool: np.ndarray, table: np.ndarray, prefix_lens: np.ndarray,
                           offsets: np.ndarray, buf: np.ndarray, layer_begin: int, layer_end: int) -> None:
    """Scatter layers ``layer_begin .. layer_end-1`` of a layer-major buffer into the pools (in place)."""
    _batch_layers(False, k_pool, v_pool, table, prefix_lens, offsets, buf, layer_begin, layer_end)


def kv_append(k_pool: np.ndarray, v_pool: np.ndarray, layer: int, k_new: np.ndarray, v_new: np.ndarray,
              cu_new_lens: np.ndarray, prefix_lens: np.ndarray, table: np.ndarray) -> None:
    """Write the new turn's K,V rows of one layer into the pools (in place) behind each session's prefix."""
    L, nb, bs, hkv, d, eb, ls, bst = _pool_geometry(k_pool, v_pool)
    k_new = _check(k_new, k_pool.dtype, "k_new")
    v_new = _check(v_new, k_pool.dtype, "v_new")
    cu_new_lens = _check(cu_new_lens, np.int32, "cu_new_lens")
    prefix_lens = _check(prefix_lens, np.int32, "prefix_lens")
    table = _check(table, np.int32, "table")
    if k_new.shape != v_new.shape or k_new.shape[1:] != (hkv, d) or int(cu_new_lens[-1]) != k_new.shape[0]:
        raise ValueError("k_new / v_new shapes do not match the pool or cu_new_lens")
    rc = _load().oracle_kv_append(_ptr(k_pool), _ptr(v_pool), ls, bst, L, bs, hkv, d, eb, int(layer), _ptr(k_new),
                                  _ptr(v_new), _ptr(cu_new_lens), _ptr(prefix_lens), _ptr(table), table.shape[1],
                                  prefix_lens.shape[0])
    if rc != 0:
        raise RuntimeError("oracle_kv_append failed")


def _attn_args(k_pool, v_pool, q, k_new, v_new, cu_new_lens, prefix_lens, table):
    L, nb, bs, hkv, d, eb, ls, bst = _pool_geometry(k_pool, v_pool)
    for a, n in ((q, "q"), (k_new, "k_new"), (v_new, "v_new")):
        _check(a, k_pool.dtype, n)
    cu_new_lens = _check(cu_new_lens, np.int32, "cu_new_lens")
    prefix_lens = _check(prefix_lens, np.int32, "prefix_lens")
    table = _check(table, np.int32, "table")
    T, hq, dq = q.shape
    if dq != d or k_new.shape != (T, hkv, d) or v_new.shape != (T, hkv, d):
        raise ValueError("q / k_new / v_new shapes do not match the pool")
    if int(cu_new_lens[-1]) != T:
        raise ValueError("cu_new_lens[-1] must equal the number of query rows")
    return L, bs, hkv, d, eb, ls, bst, T, hq


def prefix_prefill_attn(k_pool: np.ndarray, v_pool: np.ndarray, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray,
                        cu_new_lens: np.ndarray, prefix_lens: np.ndarray, table: np.ndarray, scale: float,
                        layer: int = 0, token_subset: Optional[Sequence[int]] = None) -> np.ndarray:
    """fp64 softmax attention of the new turn over [cached prefix ; causal new tokens]: ``[T][H_q][d]`` float64.

    With ``token_subset`` only those global token rows are computed (all heads); other rows are NaN.
    """
    L, bs, hkv, d, eb, ls, bst, T, hq = _attn_args(k_pool, v_pool, q, k_new, v_new, cu_new_lens, prefix_lens, table)
    out = np.full((T, hq, d), np.nan, dtype=np.float64)
    sub = None
    n_sub = 0
    if token_subset is not None:
        sub = np.ascontiguousarray(np.asarray(token_subset, dtype=np.int32))
        n_sub = int(sub.size)
    rc = _load().oracle_prefix_prefill_attn(
        _ptr(k_pool), _ptr(v_pool), ls, bst, layer, bs, hkv, d, 1 if eb == 2 else 0, _ptr(q), _ptr(k_new),
        _ptr(v_new), _ptr(cu_new_lens), _ptr(prefix_lens), _ptr(table), table.shape[1], prefix_lens.shape[0], hq,
        np.float32(scale), _ptr(sub), n_sub, _ptr(out))
    if rc != 0:
        raise RuntimeError("oracle_prefix_prefill_attn: bad argument")
    return out


def attn_row_weights(k_pool, v_pool, q, k_new, v_new, cu_new_lens, prefix_lens, table, scale: float, s: int, i: int,
                     h: int, layer: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Softmax weights (length P_s + i + 1) and output row (length d) of one query row."""
    L, bs, hkv, d, eb, ls, bst, T, hq = _attn_args(k_pool, v_pool, q, k_new, v_new, cu_new_lens, prefix_lens, table)
    w = np.zeros(int(prefix_lens[s]) + i + 1, dtype=np.float64)
    o = np.zeros(d, dtype=np.float64)
    _load().oracle_attn_row_weights(
        _ptr(k_pool), _ptr(v_pool), ls, bst, layer, bs, hkv, d, 1 if eb == 2 else 0, _ptr(q), _ptr(k_new),
        _ptr(v_new), _ptr(cu_new_lens), _ptr(prefix_lens), _ptr(table), table.shape[1], hq, np.float32(scale), s, i,
        h, _ptr(w), _ptr(o))
    return w, o
