"""The C-ABI library: every entry point declared in include/symph.h is exported, and host-side validation
rejects bad arguments before anything touches a GPU (these run without one)."""
import ctypes as C
import os
import re

import paper_2412_16434_amd as S
from paper_2412_16434_amd.binding import _CacheStruct

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(symph_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = S.load_library()
    names = declared_symbols()
    assert len(names) >= 9
    for n in names:
        assert hasattr(lib, n), f"{n} declared in symph.h but not exported"
    assert sorted(S.EXPORTED_SYMBOLS) == names


def _cache(**kw):
    base = dict(k_base=0x1000, v_base=0x2000, layer_stride=1 << 20, block_stride=16 * 8 * 128, n_layers=2, n_blocks=8,
                block_size=16, n_kv_heads=8, head_dim=128, dtype=0)
    base.update(kw)
    return _CacheStruct(**base)


def test_buffer_bytes_closed_form():
    lib = S.load_library()
    c = _cache(n_layers=80)
    assert lib.symph_kv_buffer_bytes(C.byref(c), 32768) == 10 * 2 ** 30      # Sec. 1: ~10 GB at 32K for 70B
    assert lib.symph_kv_buffer_bytes(C.byref(c), 0) == 0
    assert lib.symph_kv_buffer_bytes(C.byref(c), -1) < 0
    assert lib.symph_kv_buffer_bytes(None, 5) < 0


def test_host_validation_rejects_without_launching():
    lib = S.load_library()
    EINVAL, EUNSUP, EWS = -1, -2, -4
    good = _cache()
    # empty work is fine and launches nothing
    assert lib.symph_kv_pack(C.byref(good), None, 0, None, None, 0, 0, None, 0, None) == 0
    assert lib.symph_kv_unpack(C.byref(good), 0x10, 4, 0x10, 0x10, 3, 0, None, 0, None) == 0
    # null cache / bad shapes
    assert lib.symph_kv_pack(None, 0x10, 4, 0x10, 0x10, 1, 16, 0x100, 1 << 30, None) == EINVAL
    assert lib.symph_kv_pack(C.byref(_cache(n_layers=0)), 0x10, 4, 0x10, 0x10, 1, 16, 0x100, 1 << 30, None) == EINVAL
    assert lib.symph_kv_pack(C.byref(_cache(block_stride=100)), 0x10, 4, 0x10, 0x10, 1, 16, 0x100, 1 << 30, None) == EINVAL
    assert lib.symph_kv_pack(C.byref(_cache(dtype=7)), 0x10, 4, 0x10, 0x10, 1, 16, 0x100, 1 << 30, None) == EUNSUP
    # null device arrays, buffer too small
    assert lib.symph_kv_pack(C.byref(good), None, 4, 0x10, 0x10, 1, 16, 0x100, 1 << 30, None) == EINVAL
    assert lib.symph_kv_pack(C.byref(good), 0x10, 4, 0x10, 0x10, 1, 16, 0x100, 100, None) == EWS
    # attention: layer out of range, heads not divisible, bad scale, unsupported head_dim
    def attn(cache, layer=0, hq=32, scale=0.1, T=4, maxn=4, maxp=16, ts=1):
        return lib.symph_prefix_prefill_attn(C.byref(cache), layer, 0x10, 0x10, 0x10, 0x10, 0x10, 0x10, 0x10, ts, 1,
                                             hq, T, maxn, maxp, scale, None, 0, None)
    assert attn(good, layer=2) == EINVAL
    assert attn(good, hq=12) == EINVAL
    assert attn(good, scale=0.0) == EINVAL
    assert attn(good, scale=float("nan")) == EINVAL
    assert attn(good, maxp=64, ts=1) == EINVAL          # table too narrow for the stated prefix
    assert attn(_cache(head_dim=80, block_stride=16 * 8 * 80)) == EUNSUP
    assert lib.symph_prefix_prefill_attn(C.byref(good), 0, None, None, None, None, None, None, None, 0, 0, 32, 0, 0, 0,
                                         0.1, None, 0, None) == 0
    # staging / copy argument checks
    assert lib.symph_stage_to_host(None, 0x10, 16, None, 0x20, 0x30) == EINVAL
    assert lib.symph_stage_to_host(0x10, 0x10, 16, 0x20, 0x20, 0x30) == EINVAL     # side stream == producer
    assert lib.symph_stage_to_device(0x10, 0x10, 0, None, None, None) == 0
    # layer ranges
    assert lib.symph_kv_pack_layers(C.byref(good), 1, 1, 0x10, 4, 0x10, 0x10, 1, 16, 0x100, 1 << 30, None) == 0   # empty
    assert lib.symph_kv_pack_layers(C.byref(good), -1, 1, 0x10, 4, 0x10, 0x10, 1, 16, 0x100, 1 << 30, None) == EINVAL
    assert lib.symph_kv_unpack_layers(C.byref(good), 0, 3, 0x10, 4, 0x10, 0x10, 1, 16, 0x100, 1 << 30, None) == EINVAL
    assert lib.symph_kv_unpack_layers(C.byref(good), 2, 1, 0x10, 4, 0x10, 0x10, 1, 16, 0x100, 1 << 30, None) == EINVAL
    assert lib.symph_stage_layer_to_host(0x10, 0x10, C.byref(good), 2, 0x10, 0x10, 1, 0x20, 0x30, 0x40) == EINVAL  # layer
    assert lib.symph_stage_layer_to_device(0x10, 0x10, C.byref(good), 0, 0x10, 0x10, 1, 0x20, 0x20, 0x40) == EINVAL
    assert lib.symph_stage_layer_to_device(0x10, 0x10, C.byref(good), 0, None, None, 0, None, None, None) == 0
    assert lib.symph_kv_append(C.byref(good), 2, 0x10, 0x10, 0x10, 0x10, 0x10, 4, 1, 8, None) == EINVAL           # layer
    assert lib.symph_kv_append(C.byref(good), 0, None, 0x10, 0x10, 0x10, 0x10, 4, 1, 8, None) == EINVAL
    assert lib.symph_kv_append(C.byref(good), 0, None, None, None, None, None, 0, 0, 0, None) == 0
    assert lib.symph_device_copy(0x10, 0x20, 24, None) == EUNSUP
    assert lib.symph_device_copy(0x18, 0x20, 32, None) == EUNSUP
    assert lib.symph_kv_pack_tail(C.byref(good), 0x10, 4, 0x10, None, 0x10, 1, 8, 0x10, 1 << 20, None) == EINVAL      # no tail_begin
    assert lib.symph_kv_unpack_tail(C.byref(good), 0x10, 4, 0x10, 0x10, 0x10, 1, 8, 0x10, 16, None) == EWS        # buffer too small
    assert lib.symph_kv_pack_tail(C.byref(good), None, 0, None, None, None, 0, 0, None, 0, None) == 0
    assert lib.symph_kv_unpack_units(C.byref(good), 0x10, 4, 0x10, 0x10, 0x10, 1, 8, 0x10, 1 << 20, None) == EINVAL   # a layer axis
    one = _cache(n_layers=1)
    assert lib.symph_kv_unpack_units(C.byref(one), 0x10, 4, 0x10, 0x10, None, 1, 8, 0x10, 1 << 20, None) == EINVAL    # no chunk rows
    assert lib.symph_kv_pack_units(C.byref(one), 0x10, 4, 0x10, 0x10, 0x10, 1, 8, 0x10, 16, None) == EWS              # buffer too small
    assert lib.symph_kv_pack_units(C.byref(one), None, 0, None, None, None, 0, 0, None, 0, None) == 0
    assert lib.symph_debug_check_tables(None, 0x10, 4, 0x10, 1, 0, None, None) == EINVAL
    assert lib.symph_debug_check_tables(C.byref(good), None, 4, 0x10, 1, 0, None, None) == EINVAL
    assert lib.symph_debug_check_tables(C.byref(good), None, 0, None, 0, 1, None, None) == 0
    assert lib.symph_mfma_reference(0, None, 0x10, None) == EINVAL
    assert lib.symph_mfma_reference(8, None, None, None) == EINVAL
    assert S.status_string(0) == "ok" and "unsupported" in S.status_string(-2)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in (r.stdout + r.stderr)
