"""The step that turns rocprofv3 output into profiles/ and the staleness rule of bench.py's counter figures, on small
hand-made CSVs (no GPU, no profiler): kernel names are matched through bench.py's own table, counters are scaled by
the copy probe, and figures stamped with another source hash are left out of the benchmark line."""
import csv
import json
import os
import subprocess
import sys

from conftest import ROOT

sys.path.insert(0, ROOT)
import bench  # noqa: E402


def _write(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w", newline="") as fh:
        w = csv.writer(fh, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(header)
        w.writerows(rows)


def _counter_rows(kernel, name, values):
    head = ["Correlation_Id", "Dispatch_Id", "Agent_Id", "Queue_Id", "Process_Id", "Thread_Id", "Grid_Size", "Kernel_Id", "Kernel_Name",
            "Workgroup_Size", "LDS_Block_Size", "Scratch_Size", "VGPR_Count", "Accum_VGPR_Count", "SGPR_Count", "Counter_Name",
            "Counter_Value", "Start_Timestamp", "End_Timestamp"]
    return head, [[i, i, "Agent 1", 1, 1, 1, 1024, 1, kernel, 256, 0, 0, 16, 0, 32, name, v, 0, 1] for i, v in enumerate(values)]


def test_summaries_and_counter_file(tmp_path):
    n = 1 << 28
    full = "void fbsr::round_tiles<1, 1, 2>(float const*, void*, int, unsigned long, unsigned long, unsigned int)"
    qat = "void fbsr::qat_tiles<fbsr::FixedCodec<1, 3>, 4>(unsigned char*, unsigned short const*)"
    line = {"config": {"elements": n}, "steps": 3, "roofline": {"avg_launch_ms": 0.2, "achieved": 6700.0},
            "per_launch": {"e4m3_N2_srff": {"ms": 0.2, "gb_s": 6710.9, "gelem_s": 1342.0, "kernel": "fbsr::round_tiles<1, 1, 2>", "elements": n}},
            "paths": {"qat_adamw_e4m3_N3_src": {"ms": 0.27, "gb_s": 5965.2, "kernel": bench.PATH_KERNELS["qat_adamw_e4m3_N3_src"],
                                                 "elements": n // 2, "launches": 2}}}
    (tmp_path / "bench.json").write_text("noise before the line\n" + json.dumps(line) + "\n")
    # one launch per step of the headline kernel after a slow warm-up step; the path's two timed launches after three
    # slower ones of its warm-up: only the last (steps, launches) of each count
    spans = [(full, 0, 900000), (full, 1000000, 1190000), (full, 2000000, 2200000), (full, 3000000, 3210000)]
    spans += [(qat, 4000000 + 1000000 * i, 4000000 + 1000000 * i + d) for i, d in enumerate((400000, 350000, 300000, 260000, 280000))]
    _write(str(tmp_path / "kt" / "kt_kernel_trace.csv"),
           ["Kind", "Agent_Id", "Queue_Id", "Stream_Id", "Thread_Id", "Dispatch_Id", "Kernel_Id", "Kernel_Name", "Correlation_Id",
            "Start_Timestamp", "End_Timestamp"],
           [["KERNEL_DISPATCH", "Agent 1", 1, 0, 1, i + 1, 1, k, i + 1, a, b] for i, (k, a, b) in enumerate(spans)])
    copy = "__amd_rocclr_copyBuffer"
    for folder, name, scale in (("fetch", "FETCH_SIZE", 0.5), ("write", "WRITE_SIZE", 1.0)):
        rows = []
        head, r = _counter_rows(copy, name, [4.0 * n / 1024 * scale] * 2)
        rows += r
        rows += _counter_rows(full, name, [(4.0 if name == "FETCH_SIZE" else 1.0) * n / 1024 * scale] * 3)[1]
        rows += _counter_rows(qat, name, [(7.0 if name == "FETCH_SIZE" else 5.0) * (n // 2) / 1024 * scale] * 3)[1]
        _write(str(tmp_path / folder / ("x_counter_collection.csv")), head, rows)
    rows = []
    for name, per_wave in (("SQ_WAVES", 1.0), ("SQ_INSTS_VALU", 439.5), ("SQ_INSTS_SALU", 42.0), ("SQ_INSTS_LDS", 18.0)):
        head, r = _counter_rows(qat, name, [262144.0 * per_wave] * 2)
        rows += r
    _write(str(tmp_path / "sq" / "sq_counter_collection.csv"), head, rows)
    head, r = _counter_rows(qat, "VALUBusy", [77.0, 78.0])
    _write(str(tmp_path / "busy" / "b_counter_collection.csv"), head, r)
    out = tmp_path / "profiles"
    subprocess.check_call([sys.executable, "-m", "paper_2504_20634_amd.profile_summary", "--bench-json", str(tmp_path / "bench.json"),
                           "--kt", str(tmp_path / "kt"), "--fetch", str(tmp_path / "fetch"), "--write", str(tmp_path / "write"),
                           "--sq", str(tmp_path / "sq"), "--busy", str(tmp_path / "busy"), "--out", str(out)], cwd=ROOT)
    figures = json.loads((out / "kernel_counters.json").read_text())
    assert figures["sources_sha256"] == bench.kernel_sources_hash()
    assert figures["headline_traffic_bytes_2p28"] == 5 * n          # the probe's scale brings both counters back to bytes
    assert figures["traffic_bytes"]["qat_adamw_e4m3_N3_src"] == 12 * (n // 2)
    assert figures["valu_per_elem"]["qat_adamw_e4m3_N3_src"] == round(439.5 * 262144 * 64 / (n // 2), 1)
    assert figures["valu_busy_pct"]["qat_adamw_e4m3_N3_src"] == 77.5
    trace = (out / "bench_2p28_kernel_trace.md").read_text()
    assert "round_tiles<1, 1, 2> | 4 | 3 | 200.0 | 190.0 | 210.0" in trace
    assert "| 5 | 2 | 270.0 | 260.0 | 280.0" in trace and "qat_adamw_e4m3_N3_src" in trace
    assert "1.00000" in (out / "kernels_2p28_hbm_traffic.md").read_text()


def test_counter_figures_of_other_sources_are_left_out(tmp_path, monkeypatch):
    good = {"sources_sha256": bench.kernel_sources_hash(), "headline_traffic_bytes_2p28": 123}
    path = tmp_path / "kernel_counters.json"
    monkeypatch.setattr(bench, "COUNTERS_JSON", str(path))
    assert bench.load_counters()[0] == {}                            # no file
    path.write_text(json.dumps(good))
    figures, note = bench.load_counters()
    assert figures["headline_traffic_bytes_2p28"] == 123 and "stale" not in note
    path.write_text(json.dumps(dict(good, sources_sha256="0" * 64)))
    figures, note = bench.load_counters()
    assert figures == {} and "stale" in note
    path.write_text("{ not json")
    assert bench.load_counters()[0] == {}


def test_every_bench_path_names_a_kernel_of_the_library():
    """bench.py's path -> kernel table against the kernels the built library holds (by demangled symbol)."""
    lib = os.path.join(ROOT, "paper_2504_20634_amd", "libfbsr.so")
    names = subprocess.run(["nm", "-C", "--defined-only", lib], stdout=subprocess.PIPE, check=True).stdout.decode()
    for path, kernel in bench.PATH_KERNELS.items():
        assert kernel + "(" in names, (path, kernel)
