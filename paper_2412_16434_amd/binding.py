"""ctypes binding of libsymph.so: same names as the C entry points, torch tensors in, status checked."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
# SYMPH_LIBRARY_PATH: development override to load an experimental build of the same library
_LIB_PATH = os.environ.get("SYMPH_LIBRARY_PATH") or os.path.join(_HERE, "libsymph.so")
_lib = None

SYMPH_BF16, SYMPH_FP32 = 0, 1

EXPORTED_SYMBOLS = (
    "symph_kv_buffer_bytes", "symph_kv_pack", "symph_kv_unpack", "symph_kv_pack_layers", "symph_kv_unpack_layers",
    "symph_kv_pack_batch_layers", "symph_kv_unpack_batch_layers", "symph_stage_batch_layers_to_host",
    "symph_stage_batch_layers_to_device", "symph_kv_pack_tail", "symph_kv_unpack_tail", "symph_kv_pack_units", "symph_kv_unpack_units", "symph_kv_append",
    "symph_prefix_prefill_attn", "symph_prefix_prefill_attn_workspace_bytes", "symph_prefix_prefill_attn_tuned",
    "symph_prefix_prefill_attn_workspace_bytes_tuned", "symph_prefix_prefill_attn_static", "symph_debug_attn_flags", "symph_stage_to_host",
    "symph_stage_to_device", "symph_stage_layer_to_host", "symph_stage_layer_to_device", "symph_device_copy",
    "symph_mfma_reference", "symph_debug_check_tables",
    "symph_status_string",
    # symph_pool.h (host code only)
    "symph_pool_create", "symph_pool_destroy", "symph_pool_advise", "symph_pool_drop", "symph_pool_claim",
    "symph_pool_framework_take", "symph_pool_framework_give", "symph_pool_settle", "symph_pool_resident_layers",
    "symph_pool_unit_slots", "symph_pool_table", "symph_pool_counts",
)


class SymphError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class _CacheStruct(C.Structure):
    _fields_ = [("k_base", C.c_void_p), ("v_base", C.c_void_p), ("layer_stride", C.c_int64),
                ("block_stride", C.c_int64), ("n_layers", C.c_int32), ("n_blocks", C.c_int32),
                ("block_size", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("dtype", C.c_int32)]


class AttnTuning(C.Structure):
    """symph_attn_tuning: a field left 0 keeps the library's default."""
    _fields_ = [("slots", C.c_int32), ("c_min", C.c_int32), ("coarse", C.c_int32), ("decode", C.c_int32),
                ("decode_wgs", C.c_int32), ("reserved", C.c_int32 * 3)]


class _PoolChange(C.Structure):
    _fields_ = [("session", C.c_int64), ("layer", C.c_int32), ("kind", C.c_int32), ("n_slots", C.c_int32),
                ("slot_begin", C.c_int32)]


PoolChange = _PoolChange


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libsymph.so (built in-tree by ``paper_2412_16434_amd/build.py``). Raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2412_16434_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    i32, i64, vp, f32 = C.c_int32, C.c_int64, C.c_void_p, C.c_float
    cp = C.POINTER(_CacheStruct)
    lib.symph_kv_buffer_bytes.restype = i64
    lib.symph_kv_buffer_bytes.argtypes = [cp, i64]
    for fn in (lib.symph_kv_pack, lib.symph_kv_unpack):
        fn.restype = i32
        fn.argtypes = [cp, vp, i32, vp, vp, i32, i64, vp, i64, vp]
    for fn in (lib.symph_kv_pack_layers, lib.symph_kv_unpack_layers, lib.symph_kv_pack_batch_layers,
               lib.symph_kv_unpack_batch_layers):
        fn.restype = i32
        fn.argtypes = [cp, i32, i32, vp, i32, vp, vp, i32, i64, vp, i64, vp]
    for fn in (lib.symph_stage_batch_layers_to_host, lib.symph_stage_batch_layers_to_device):
        fn.restype = i32
        fn.argtypes = [vp, vp, cp, i32, i32, i64, vp, vp, vp]
    for fn in (lib.symph_kv_pack_tail, lib.symph_kv_unpack_tail):
        fn.restype = i32
        fn.argtypes = [cp, vp, i32, vp, vp, vp, i32, i64, vp, i64, vp]
    for fn in (lib.symph_kv_pack_units, lib.symph_kv_unpack_units):
        fn.restype = i32
        fn.argtypes = [cp, vp, i32, vp, vp, vp, i32, i64, vp, i64, vp]
    for fn in (lib.symph_stage_layer_to_host, lib.symph_stage_layer_to_device):
        fn.restype = i32
        fn.argtypes = [vp, vp, cp, i32, vp, vp, i32, vp, vp, vp]
    lib.symph_kv_append.restype = i32
    lib.symph_kv_append.argtypes = [cp, i32, vp, vp, vp, vp, vp, i32, i32, i32, vp]
    lib.symph_prefix_prefill_attn.restype = i32
    lib.symph_prefix_prefill_attn.argtypes = [cp, i32, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, f32,
                                              vp, i64, vp]
    lib.symph_prefix_prefill_attn_workspace_bytes.restype = i64
    lib.symph_prefix_prefill_attn_workspace_bytes.argtypes = [cp, i32, i32, i32, i32, i32]
    tp = C.POINTER(AttnTuning)
    lib.symph_prefix_prefill_attn_tuned.restype = i32
    lib.symph_prefix_prefill_attn_tuned.argtypes = lib.symph_prefix_prefill_attn.argtypes + [tp]
    lib.symph_prefix_prefill_attn_workspace_bytes_tuned.restype = i64
    lib.symph_prefix_prefill_attn_workspace_bytes_tuned.argtypes = [cp, i32, i32, i32, i32, i32, tp]
    lib.symph_prefix_prefill_attn_static.restype = i32
    lib.symph_prefix_prefill_attn_static.argtypes = lib.symph_prefix_prefill_attn.argtypes[:16] + [vp]
    lib.symph_debug_attn_flags.restype = i32
    lib.symph_debug_attn_flags.argtypes = [vp, vp, C.POINTER(i32)]
    for fn in (lib.symph_stage_to_host, lib.symph_stage_to_device):
        fn.restype = i32
        fn.argtypes = [vp, vp, i64, vp, vp, vp]
    lib.symph_device_copy.restype = i32
    lib.symph_device_copy.argtypes = [vp, vp, i64, vp]
    lib.symph_mfma_reference.restype = i32
    lib.symph_mfma_reference.argtypes = [i32, C.POINTER(C.c_int64), vp, vp]
    lib.symph_debug_check_tables.restype = i32
    lib.symph_debug_check_tables.argtypes = [cp, vp, i32, vp, i32, i32, vp, C.POINTER(i32)]
    lib.symph_status_string.restype = C.c_char_p
    lib.symph_status_string.argtypes = [i32]
    ip = C.POINTER(i32)
    lib.symph_pool_create.restype = i32
    lib.symph_pool_create.argtypes = [i32, i32, i32, C.POINTER(vp)]
    lib.symph_pool_destroy.restype = None
    lib.symph_pool_destroy.argtypes = [vp]
    lib.symph_pool_advise.restype = i32
    lib.symph_pool_advise.argtypes = [vp, i64, i32]
    lib.symph_pool_drop.restype = i32
    lib.symph_pool_drop.argtypes = [vp, i64]
    lib.symph_pool_claim.restype = i32
    lib.symph_pool_claim.argtypes = [vp, i64, ip, i32, ip]
    lib.symph_pool_framework_take.restype = i32
    lib.symph_pool_framework_take.argtypes = [vp, i32, ip]
    lib.symph_pool_framework_give.restype = i32
    lib.symph_pool_framework_give.argtypes = [vp, i32, ip]
    lib.symph_pool_settle.restype = i32
    lib.symph_pool_settle.argtypes = [vp, C.POINTER(_PoolChange), i32, ip, i32, ip, ip]
    lib.symph_pool_resident_layers.restype = i32
    lib.symph_pool_resident_layers.argtypes = [vp, i64]
    lib.symph_pool_unit_slots.restype = i32
    lib.symph_pool_unit_slots.argtypes = [vp, i64]
    lib.symph_pool_table.restype = i32
    lib.symph_pool_table.argtypes = [vp, i64, i32, ip, i32]
    lib.symph_pool_counts.restype = i32
    lib.symph_pool_counts.argtypes = [vp, ip, ip, ip]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().symph_status_string(int(status)).decode()


@dataclass
class KVCache:
    """A paged K,V cache in device memory: two torch tensors ``[L][n_blocks][bs][H_kv][d]`` (bf16 or fp32)."""
    k_pool: "object"
    v_pool: "object"

    def __post_init__(self):
        import torch
        k, v = self.k_pool, self.v_pool
        if k.dim() != 5 or k.shape != v.shape or k.dtype != v.dtype:
            raise ValueError("pools must be two [L][n_blocks][bs][H_kv][d] tensors of one dtype")
        if k.dtype not in (torch.bfloat16, torch.float32):
            raise ValueError("cache dtype must be bfloat16 or float32")
        if k.stride()[2:] != (k.shape[3] * k.shape[4], k.shape[4], 1) or v.stride() != k.stride():
            raise ValueError("token, head and dim axes must be dense")

    @property
    def dtype_code(self) -> int:
        import torch
        return SYMPH_BF16 if self.k_pool.dtype == torch.bfloat16 else SYMPH_FP32

    def struct(self) -> _CacheStruct:
        k = self.k_pool
        return _CacheStruct(k.data_ptr(), self.v_pool.data_ptr(), k.stride(0), k.stride(1), k.shape[0], k.shape[1],
                            k.shape[2], k.shape[3], k.shape[4], self.dtype_code)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _dev(t, name: str, dtype=None, allow_none: bool = False, pinned_ok: bool = False):
    """Check what the C side cannot see: the tensor is on the GPU (or, for buffers, pinned host memory), contiguous and
    of the element type the entry point reads it as.  Returns its data pointer."""
    if t is None:
        if allow_none:
            return None
        raise ValueError(f"{name} is required")
    if not (t.is_cuda or (pinned_ok and t.is_pinned())):
        raise ValueError(f"{name} must be a device tensor" + (" or pinned host memory" if pinned_ok else ""))
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, not {t.dtype}")
    return t.data_ptr()


def _table(t, name: str = "block_table"):
    """(pointer, row stride in entries) of an int32 [n_sessions][stride] block table on the device; (None, 0) if absent."""
    import torch
    if t is None:
        return None, 0
    if t.dim() != 2:
        raise ValueError(f"{name} must be a 2-D int32 tensor [n_sessions][max_blocks]")
    return _dev(t, name, torch.int32), t.shape[1]


def _lens(t, name: str):
    import torch
    return _dev(t, name, torch.int32)


def _offsets(t, name: str):
    import torch
    return _dev(t, name, torch.int64)


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _event_ptr(event) -> int:
    """hipEvent_t of a torch.cuda.Event (torch creates the handle on the first record)."""
    if isinstance(event, int):
        return event
    if not event.cuda_event:
        event.record()
    return event.cuda_event


def _check(status: int, where: str) -> None:
    if status != 0:
        raise SymphError(status, where)


def kv_buffer_bytes(cache: KVCache, total_tokens: int) -> int:
    st = cache.struct()
    n = load_library().symph_kv_buffer_bytes(C.byref(st), int(total_tokens))
    if n < 0:
        raise SymphError(-1, "symph_kv_buffer_bytes")
    return int(n)


def _migrate(fn_name: str, cache: KVCache, head_args, block_table, prefix_lens, mid, offsets, total_tokens, buf, stream):
    """Shared marshalling of the pack / unpack family: (cache, [layer range], table, stride, lens, [extra], offsets, n,
    total, buf, bytes, stream)."""
    st = cache.struct()
    tp, stride = _table(block_table)
    _check(getattr(load_library(), fn_name)(
        C.byref(st), *head_args, tp, stride, _lens(prefix_lens, "prefix_lens"), *mid, _offsets(offsets, "offsets"),
        prefix_lens.shape[0], int(total_tokens), _dev(buf, "buf", pinned_ok=True), buf.numel() * buf.element_size(),
        _stream_ptr(stream)), fn_name)


def kv_pack(cache: KVCache, block_table, prefix_lens, buf_token_offsets, total_tokens: int, buf, stream=None) -> None:
    """Gather into ``buf`` (any dtype, 1-D device tensor of at least kv_buffer_bytes bytes)."""
    _migrate("symph_kv_pack", cache, (), block_table, prefix_lens, (), buf_token_offsets, total_tokens, buf, stream)


def kv_unpack(cache: KVCache, dst_block_table, prefix_lens, buf_token_offsets, total_tokens: int, buf,
              stream=None) -> None:
    _migrate("symph_kv_unpack", cache, (), dst_block_table, prefix_lens, (), buf_token_offsets, total_tokens, buf,
             stream)


def kv_pack_layers(cache: KVCache, layer_begin: int, layer_end: int, block_table, prefix_lens, buf_token_offsets,
                   total_tokens: int, buf, stream=None) -> None:
    """Gather layers ``layer_begin .. layer_end-1`` only into ``buf`` (whole-cache layout)."""
    _migrate("symph_kv_pack_layers", cache, (int(layer_begin), int(layer_end)), block_table, prefix_lens, (),
             buf_token_offsets, total_tokens, buf, stream)


def kv_unpack_layers(cache: KVCache, layer_begin: int, layer_end: int, dst_block_table, prefix_lens,
                     buf_token_offsets, total_tokens: int, buf, stream=None) -> None:
    _migrate("symph_kv_unpack_layers", cache, (int(layer_begin), int(layer_end)), dst_block_table, prefix_lens, (),
             buf_token_offsets, total_tokens, buf, stream)


def kv_pack_batch_layers(cache: KVCache, layer_begin: int, layer_end: int, block_table, prefix_lens, buf_token_offsets,
                         total_tokens: int, buf, stream=None) -> None:
    """Gather layers ``layer_begin .. layer_end-1`` into ``buf`` laid out layer -> session -> K|V -> token."""
    _migrate("symph_kv_pack_batch_layers", cache, (int(layer_begin), int(layer_end)), block_table, prefix_lens, (),
             buf_token_offsets, total_tokens, buf, stream)


def kv_unpack_batch_layers(cache: KVCache, layer_begin: int, layer_end: int, dst_block_table, prefix_lens,
                           buf_token_offsets, total_tokens: int, buf, stream=None) -> None:
    _migrate("symph_kv_unpack_batch_layers", cache, (int(layer_begin), int(layer_end)), dst_block_table, prefix_lens, (),
             buf_token_offsets, total_tokens, buf, stream)


def stage_batch_layers_to_host(h_pinned, d_buf, cache: KVCache, layer_begin: int, layer_end: int, total_tokens: int,
                               producer_stream, side_stream, event) -> None:
    """One copy of the layers' contiguous piece of a layer-major buffer, device -> pinned host, on ``side_stream``."""
    st = cache.struct()
    _check(load_library().symph_stage_batch_layers_to_host(
        _ptr(h_pinned), _ptr(d_buf), C.byref(st), int(layer_begin), int(layer_end), int(total_tokens),
        _stream_ptr(producer_stream), _stream_ptr(side_stream), _event_ptr(event)), "symph_stage_batch_layers_to_host")


def stage_batch_layers_to_device(d_buf, h_pinned, cache: KVCache, layer_begin: int, layer_end: int, total_tokens: int,
                                 consumer_stream, side_stream, event) -> None:
    st = cache.struct()
    _check(load_library().symph_stage_batch_layers_to_device(
        _ptr(d_buf), _ptr(h_pinned), C.byref(st), int(layer_begin), int(layer_end), int(total_tokens),
        _stream_ptr(consumer_stream), _stream_ptr(side_stream), _event_ptr(event)), "symph_stage_batch_layers_to_device")


def _units(fn_name, slots: KVCache, unit_table, unit_lens, unit_token_offsets, unit_chunk_rows, total_unit_tokens, buf,
           stream):
    st = slots.struct()
    tp, stride = _table(unit_table, "unit_table")
    _check(getattr(load_library(), fn_name)(
        C.byref(st), tp, stride, _lens(unit_lens, "unit_lens"), _offsets(unit_token_offsets, "unit_token_offsets"),
        _offsets(unit_chunk_rows, "unit_chunk_rows"), unit_lens.shape[0], int(total_unit_tokens),
        _dev(buf, "buf", pinned_ok=True), buf.numel() * buf.element_size(), _stream_ptr(stream)), fn_name)


def kv_pack_units(slots: KVCache, unit_table, unit_lens, unit_token_offsets, unit_chunk_rows, total_unit_tokens: int,
                  buf, stream=None) -> None:
    """Gather single layers of sessions from one pool of slots (a one-layer KVCache) into their chunks of ``buf``."""
    _units("symph_kv_pack_units", slots, unit_table, unit_lens, unit_token_offsets, unit_chunk_rows, total_unit_tokens,
           buf, stream)


def kv_unpack_units(slots: KVCache, unit_table, unit_lens, unit_token_offsets, unit_chunk_rows, total_unit_tokens: int,
                    buf, stream=None) -> None:
    _units("symph_kv_unpack_units", slots, unit_table, unit_lens, unit_token_offsets, unit_chunk_rows,
           total_unit_tokens, buf, stream)


def debug_check_tables(cache: KVCache, block_table, lens, is_destination: bool, stream=None) -> int:
    """-1 if the table and lengths keep the contract the kernels rely on, else the first offending session."""
    st = cache.struct()
    bad = C.c_int32(-1)
    tp, stride = _table(block_table)
    rc = load_library().symph_debug_check_tables(
        C.byref(st), tp, stride, _lens(lens, "lens"), lens.shape[0], 1 if is_destination else 0, _stream_ptr(stream),
        C.byref(bad))
    if rc != 0 and bad.value < 0:
        _check(rc, "symph_debug_check_tables")
    return bad.value


def kv_pack_tail(cache: KVCache, block_table, prefix_lens, tail_begin, tail_offsets, total_tail_tokens: int, buf,
                 stream=None) -> None:
    """Gather tokens ``tail_begin[s] .. prefix_lens[s]-1`` of every session (all layers) into ``buf``."""
    _migrate("symph_kv_pack_tail", cache, (), block_table, prefix_lens, (_lens(tail_begin, "tail_begin"),),
             tail_offsets, total_tail_tokens, buf, stream)


def kv_unpack_tail(cache: KVCache, dst_block_table, prefix_lens, tail_begin, tail_offsets, total_tail_tokens: int, buf,
                   stream=None) -> None:
    """Scatter a tail buffer (see ``kv_pack_tail``) into the cache through ``dst_block_table``."""
    _migrate("symph_kv_unpack_tail", cache, (), dst_block_table, prefix_lens, (_lens(tail_begin, "tail_begin"),),
             tail_offsets, total_tail_tokens, buf, stream)


def kv_append(cache: KVCache, layer: int, k_new, v_new, cu_new_lens, prefix_lens, block_table, stream=None) -> None:
    """Write the new turn's K,V rows of ``layer`` into the paged cache behind each session's prefix."""
    st = cache.struct()
    dt = cache.k_pool.dtype
    tp, stride = _table(block_table)
    _check(load_library().symph_kv_append(
        C.byref(st), int(layer), _dev(k_new, "k_new", dt), _dev(v_new, "v_new", dt), _lens(cu_new_lens, "cu_new_lens"),
        _lens(prefix_lens, "prefix_lens"), tp, stride, prefix_lens.shape[0], k_new.shape[0], _stream_ptr(stream)),
        "symph_kv_append")


def _tuning_ref(tuning):
    return None if tuning is None else C.byref(tuning)


def prefix_prefill_attn_workspace_bytes(cache: KVCache, n_sessions: int, n_q_heads: int, total_new_tokens: int,
                                        max_new_len: int, max_prefix_len: int, tuning: Optional[AttnTuning] = None) -> int:
    st = cache.struct()
    lib = load_library()
    if tuning is None:
        n = lib.symph_prefix_prefill_attn_workspace_bytes(C.byref(st), n_sessions, n_q_heads, total_new_tokens,
                                                          max_new_len, max_prefix_len)
    else:
        n = lib.symph_prefix_prefill_attn_workspace_bytes_tuned(C.byref(st), n_sessions, n_q_heads, total_new_tokens,
                                                                max_new_len, max_prefix_len, C.byref(tuning))
    if n < 0:
        raise SymphError(-1, "symph_prefix_prefill_attn_workspace_bytes")
    return int(n)


def _attn_args(cache: KVCache, layer, q, k_new, v_new, out, cu_new_lens, prefix_lens, block_table, max_new_len,
               max_prefix_len, scale):
    """The argument list the attention entry points share, up to and including ``scale``."""
    dt = cache.k_pool.dtype
    if q.dim() != 3 or out.shape != q.shape or k_new.dim() != 3 or v_new.shape != k_new.shape:
        raise ValueError("q / out must be [T][H_q][d] and k_new / v_new [T][H_kv][d]")
    tp, stride = _table(block_table)
    return [int(layer), _dev(q, "q", dt), _dev(k_new, "k_new", dt), _dev(v_new, "v_new", dt), _dev(out, "out", dt),
            _lens(cu_new_lens, "cu_new_lens"), _lens(prefix_lens, "prefix_lens"), tp, stride, prefix_lens.shape[0],
            q.shape[1], q.shape[0], int(max_new_len), int(max_prefix_len), float(scale)]


def prefix_prefill_attn(cache: KVCache, layer: int, q, k_new, v_new, out, cu_new_lens, prefix_lens, block_table,
                        max_new_len: int, max_prefix_len: int, scale: float, workspace=None, stream=None,
                        tuning: Optional[AttnTuning] = None) -> None:
    """out[T][H_q][d] <- attention of the new turn over [cached prefix ; causal new tokens] for one layer."""
    st = cache.struct()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    args = _attn_args(cache, layer, q, k_new, v_new, out, cu_new_lens, prefix_lens, block_table, max_new_len,
                      max_prefix_len, scale)
    args += [_dev(workspace, "workspace", allow_none=True), ws_bytes, _stream_ptr(stream)]
    lib = load_library()
    if tuning is None:
        _check(lib.symph_prefix_prefill_attn(C.byref(st), *args), "symph_prefix_prefill_attn")
    else:
        _check(lib.symph_prefix_prefill_attn_tuned(C.byref(st), *args, C.byref(tuning)),
               "symph_prefix_prefill_attn_tuned")


def prefix_prefill_attn_static(cache: KVCache, layer: int, q, k_new, v_new, out, cu_new_lens, prefix_lens, block_table,
                               max_new_len: int, max_prefix_len: int, scale: float, stream=None) -> None:
    """The same attention without a workspace argument: the library's fixed scratch array is used (nothing allocated)."""
    st = cache.struct()
    args = _attn_args(cache, layer, q, k_new, v_new, out, cu_new_lens, prefix_lens, block_table, max_new_len,
                      max_prefix_len, scale)
    _check(load_library().symph_prefix_prefill_attn_static(C.byref(st), *args, _stream_ptr(stream)),
           "symph_prefix_prefill_attn_static")


def debug_attn_flags(workspace, stream=None) -> int:
    """Flags of the device-side scheduler of the last attention call on ``workspace`` (synchronises the stream)."""
    flags = C.c_int32(0)
    _check(load_library().symph_debug_attn_flags(_dev(workspace, "workspace", allow_none=True), _stream_ptr(stream),
                                                 C.byref(flags)), "symph_debug_attn_flags")
    return flags.value


def stage_to_host(h_pinned, d_buf, nbytes: int, producer_stream, side_stream, event) -> None:
    _check(load_library().symph_stage_to_host(_ptr(h_pinned), _ptr(d_buf), int(nbytes), _stream_ptr(producer_stream),
                                              _stream_ptr(side_stream), _event_ptr(event)), "symph_stage_to_host")


def stage_to_device(d_buf, h_pinned, nbytes: int, consumer_stream, side_stream, event) -> None:
    _check(load_library().symph_stage_to_device(_ptr(d_buf), _ptr(h_pinned), int(nbytes),
                                                _stream_ptr(consumer_stream), _stream_ptr(side_stream),
                                                _event_ptr(event)), "symph_stage_to_device")


def stage_layer_to_host(h_pinned, d_buf, cache: KVCache, layer: int, h_prefix_lens, h_buf_token_offsets,
                        producer_stream, side_stream, event) -> None:
    """``h_prefix_lens`` (int32) and ``h_buf_token_offsets`` (int64) are HOST tensors (CPU, contiguous)."""
    st = cache.struct()
    _check(load_library().symph_stage_layer_to_host(
        _ptr(h_pinned), _ptr(d_buf), C.byref(st), int(layer), _ptr(h_prefix_lens), _ptr(h_buf_token_offsets),
        h_prefix_lens.shape[0], _stream_ptr(producer_stream), _stream_ptr(side_stream), _event_ptr(event)),
        "symph_stage_layer_to_host")


def stage_layer_to_device(d_buf, h_pinned, cache: KVCache, layer: int, h_prefix_lens, h_buf_token_offsets,
                          consumer_stream, side_stream, event) -> None:
    st = cache.struct()
    _check(load_library().symph_stage_layer_to_device(
        _ptr(d_buf), _ptr(h_pinned), C.byref(st), int(layer), _ptr(h_prefix_lens), _ptr(h_buf_token_offsets),
        h_prefix_lens.shape[0], _stream_ptr(consumer_stream), _stream_ptr(side_stream), _event_ptr(event)),
        "symph_stage_layer_to_device")


def mfma_reference(iters: int, sink, stream=None) -> int:
    """Launch the MFMA-only reference kernel; returns the floating-point operations of the launch."""
    flops = C.c_int64(0)
    _check(load_library().symph_mfma_reference(int(iters), C.byref(flops), _ptr(sink), _stream_ptr(stream)),
           "symph_mfma_reference")
    return int(flops.value)


def device_copy(dst, src, nbytes: int, stream=None) -> None:
    _check(load_library().symph_device_copy(_ptr(dst), _ptr(src), int(nbytes), _stream_ptr(stream)),
           "symph_device_copy")


class KvPool:
    """The pool object of ``include/symph_pool.h`` (host code): which layers of which announced sessions hold slots lent
    by the framework.  Every method is one C call plus marshalling; failures raise SymphError and change nothing."""

    EVICTED, LOAD = 0, 1

    def __init__(self, n_layers: int, n_slots: int, block_size: int):
        self._lib = load_library()
        self._h = C.c_void_p()
        self.n_layers, self.n_slots, self.block_size = n_layers, n_slots, block_size
        st = self._lib.symph_pool_create(n_layers, n_slots, block_size, C.byref(self._h))
        if st != 0:
            raise SymphError(st, "symph_pool_create")

    @property
    def handle(self):
        """The symph_pool* as a ctypes void pointer, for callers that drive the C entry points with arrays of their own
        (``PoolChange`` is the change record)."""
        return self._h

    def close(self):
        if self._h:
            self._lib.symph_pool_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int, where: str) -> int:
        if st < 0:
            raise SymphError(st, where)
        return st

    def advise(self, session: int, n_tokens: int) -> None:
        self._check(self._lib.symph_pool_advise(self._h, session, n_tokens), "symph_pool_advise")

    def drop(self, session: int) -> None:
        self._check(self._lib.symph_pool_drop(self._h, session), "symph_pool_drop")

    def resident_layers(self, session: int) -> int:
        return self._check(self._lib.symph_pool_resident_layers(self._h, session), "symph_pool_resident_layers")

    def counts(self) -> tuple[int, int, int]:
        f, l, w = C.c_int32(), C.c_int32(), C.c_int32()
        self._check(self._lib.symph_pool_counts(self._h, C.byref(f), C.byref(l), C.byref(w)), "symph_pool_counts")
        return f.value, l.value, w.value

    def unit_slots(self, session: int) -> int:
        """Slots one layer of the session takes."""
        return self._check(self._lib.symph_pool_unit_slots(self._h, session), "symph_pool_unit_slots")

    def table(self, session: int, layer: int) -> list[int]:
        cap = self.unit_slots(session)
        buf = (C.c_int32 * max(cap, 1))()
        n = self._check(self._lib.symph_pool_table(self._h, session, layer, buf, cap), "symph_pool_table")
        return list(buf[:n])

    def claim(self, session: int) -> list[list[int]]:
        """Tables of the resident layers, which now belong to the framework."""
        b = self.unit_slots(session)
        cap = b * self.resident_layers(session)
        buf = (C.c_int32 * max(cap, 1))()
        r = C.c_int32()
        self._check(self._lib.symph_pool_claim(self._h, session, buf, cap, C.byref(r)), "symph_pool_claim")
        return [list(buf[i * b:(i + 1) * b]) for i in range(r.value)]

    def framework_take(self, n: int) -> list[int]:
        buf = (C.c_int32 * max(n, 1))()
        self._check(self._lib.symph_pool_framework_take(self._h, n, buf), "symph_pool_framework_take")
        return list(buf[:n])

    def framework_give(self, slots) -> None:
        n = len(slots)
        buf = (C.c_int32 * max(n, 1))(*slots)
        self._check(self._lib.symph_pool_framework_give(self._h, n, buf), "symph_pool_framework_give")

    def settle(self) -> list[tuple[int, int, int, list[int]]]:
        """[(kind, session, layer, slots)] — evictions first (slots empty), then loads, the most important first."""
        nc, ns = C.c_int32(), C.c_int32()
        st = self._lib.symph_pool_settle(self._h, None, 0, None, 0, C.byref(nc), C.byref(ns))
        if st == 0:
            return []
        if st != -4:
            raise SymphError(st, "symph_pool_settle")
        changes = (_PoolChange * max(nc.value, 1))()
        slots = (C.c_int32 * max(ns.value, 1))()
        self._check(self._lib.symph_pool_settle(self._h, changes, nc.value, slots, ns.value, C.byref(nc), C.byref(ns)),
                    "symph_pool_settle")
        out = []
        for c in changes[:nc.value]:
            own = list(slots[c.slot_begin:c.slot_begin + c.n_slots]) if c.kind == self.LOAD else []
            out.append((c.kind, c.session, c.layer, own))
        return out
