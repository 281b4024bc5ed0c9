"""bench.py --write-traffic-summary on synthetic counter files: the summary must describe the full-size launches of the
gather and the scatter (whatever instantiations the library uses for them) scaled by the copy kernel's readings, and
bench.py must read the same figures back.  No GPU needed."""
import argparse
import csv
import importlib.util
import os

import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _write(d, counter, rows):
    os.makedirs(d, exist_ok=True)
    with open(os.path.join(d, "x_counter_collection.csv"), "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Grid_Size", "Kernel_Name", "Counter_Name", "Counter_Value"])
        for grid, name, value in rows:
            w.writerow([grid, name, counter, value])


def test_summary_takes_the_full_size_launches(tmp_path):
    bench = _bench()
    cfg = W.get_config("llama8b")
    payload = W.make_sessions(cfg).payload_bytes()
    V4 = "unsigned int __vector(4)"
    names = {
        "copy": f"void symph::device_copy_kernel<1>({V4}*, {V4} const*, long)",
        "pack": f"void symph::kv_migrate_rows_kernel<{V4}, true, 2, 1, 3>(symph::MigrateParams)",
        "pack_other": f"void symph::kv_migrate_kernel<{V4}, true, 1, 3, true>(symph::MigrateParams)",
        "unpack": f"void symph::kv_migrate_kernel<{V4}, false, 2, 3, true>(symph::MigrateParams)",
        "attn": "void symph::attn_mfma_kernel<4, 4>(symph::MfmaParams)",
    }
    unit_f, unit_w = 2048.0, 1024.0   # bytes per count of the made-up machine
    full = payload / unit_f
    fetch = [(1000, names["copy"], full)] * 3
    fetch += [(900, names["pack"], full * 1.01)] * 3 + [(90, names["pack"], full / 40)] * 12   # full size + write-backs
    fetch += [(50, names["pack_other"], full / 100)] * 5                                      # another instantiation
    fetch += [(800, names["unpack"], full)] * 3 + [(400, names["unpack"], full / 2)] * 12
    fetch += [(70, names["attn"], 1.0e5)] * 3
    write = [(g, n, v * unit_f / unit_w) for g, n, v in fetch]
    _write(str(tmp_path / "f"), "FETCH_SIZE", fetch)
    _write(str(tmp_path / "w"), "WRITE_SIZE", write)
    args = argparse.Namespace(config="llama8b", write_traffic_summary=[str(tmp_path / "f"), str(tmp_path / "w")])
    path = bench.write_traffic_summary(args, out_dir=str(tmp_path))
    text = open(path).read()
    line = [l for l in text.splitlines() if l.startswith("traffic_bytes_per_launch:")][0]
    got = {k: float(v) for k, v in (item.split("=") for item in line.split(":", 1)[1].split())}
    assert abs(got["kv_pack"] / (2.02 * payload) - 1) < 1e-3      # the three full-size launches only
    assert abs(got["kv_unpack"] / (2.0 * payload) - 1) < 1e-3
    assert abs(got["attn_mfma"] / (2 * 1.0e5 * unit_f) - 1) < 1e-3
    # and the reader used for roofline.traffic sees the same numbers
    old = bench.PROFILES
    try:
        bench.PROFILES = str(tmp_path)
        assert bench.measured_traffic("llama8b") == got
    finally:
        bench.PROFILES = old


def test_committed_summary_is_plausible():
    """The committed summary of the benchmark workload: pack and unpack move their algorithmic bytes (within 2 %),
    attention at most 1.5 x its own."""
    bench = _bench()
    sess = W.make_sessions(W.get_config("llama8b"))
    t = bench.measured_traffic("llama8b")
    assert set(t) >= {"kv_pack", "kv_unpack", "attn_mfma"}
    assert abs(t["kv_pack"] / (2.0 * sess.payload_bytes()) - 1) < 0.02
    assert abs(t["kv_unpack"] / (2.0 * sess.payload_bytes()) - 1) < 0.02
    assert 0.9 < t["attn_mfma"] / sess.attn_bytes() < 1.5
