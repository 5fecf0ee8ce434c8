"""Host-side checks of the module that turns rocprofv3 CSVs into the summaries under
profiles/: the counter scale factors, the per-launch traffic figure bench.py reports as
roofline.traffic, its staleness rule, and the kernel naming.  The CSVs are made up here,
with round numbers, so that every expected value can be worked out by hand."""
import csv
import json

import pytest

from paper_2510_27656_amd import profiling

UNPACK = "void flmoe::dispatch_unpack_kernel<false, false>(flmoe::Dims, flmoe::Tables, int)"
FABRIC_D = "void flmoe::fabric_copy_kernel<false, 0, true>(flmoe::Dims, flmoe::Tables, flmoe::FabricArgs, int)"
FABRIC_C = "void flmoe::fabric_copy_kernel<true, 1, false>(flmoe::Dims, flmoe::Tables, flmoe::FabricArgs, int)"
COPY = "flmoe::plain_copy_kernel(unsigned int*, unsigned int const*, unsigned long)"


def write_counters(path, counter, per_kernel):
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Kernel_Name", "Counter_Name", "Counter_Value"])
        for name, values in per_kernel.items():
            for v in values:
                w.writerow([name, counter, v])


def test_kernel_labels_tell_the_two_fabric_launches_apart():
    assert profiling.kernel_label(UNPACK) == "dispatch_unpack_kernel"
    assert profiling.kernel_label(FABRIC_D) == "fabric_copy_kernel(dispatch)"
    assert profiling.kernel_label(FABRIC_C) == "fabric_copy_kernel(combine)"
    assert profiling.kernel_label("void flmoe::fabric_private_kernel<false, true>(int)") \
        == "fabric_copy_kernel(dispatch, private slots)"


def test_traffic_is_scaled_by_the_copy_kernel_and_tied_to_the_build(tmp_path, monkeypatch):
    monkeypatch.setattr(profiling, "PROFILES", str(tmp_path))
    # a copy of 1 MiB that the fetch counter reads as 512 KiB (x2) and the write counter as 1024 KiB (x1)
    fetch, write, log = tmp_path / "f.csv", tmp_path / "w.csv", tmp_path / "log"
    write_counters(fetch, "FETCH_SIZE", {COPY: [512, 512], UNPACK: [100, 300, 200, 200, 100, 300]})
    write_counters(write, "WRITE_SIZE", {COPY: [1024, 1024], UNPACK: [50, 150, 100, 100, 50, 150]})
    log.write_text("noise\n" + json.dumps({
        "copy_bytes": 1 << 20, "steps": 3, "library_build_id": "abc",
        "algorithmic_bytes": {"dispatch_unpack_kernel": 2 * 500 * 1024}}) + "\n")
    profiling.traffic("wl", str(fetch), str(write), str(log))
    stored = json.load(open(tmp_path / "hbm_traffic.json"))
    # per launch: fetch 200 KiB x 2 + write 100 KiB x 1 = 500 KiB; six dispatches in three steps = two
    # launches per step, so the step's 1000 KiB of algorithmic bytes are 500 KiB per launch
    assert stored["wl"] == {"library_build_id": "abc", "kernels": {"dispatch_unpack_kernel": 500 * 1024}}
    text = (tmp_path / "hbm_traffic_wl.md").read_text()
    assert "2.0000 (fetch) and 1.0000 (write)" in text and "| 1.000 |" in text
    # the figure is handed out only for the build it was measured with
    assert profiling.stored_traffic("wl", "dispatch_unpack_kernel", "abc") == (500 * 1024, None)
    value, note = profiling.stored_traffic("wl", "dispatch_unpack_kernel", "other")
    assert value is None and "abc" in note and "other" in note
    assert profiling.stored_traffic("absent", "dispatch_unpack_kernel", "abc")[0] is None
    # a second workload is added to the same file, the first stays
    profiling.traffic("wl", str(fetch), str(write), str(log), tag="push")
    assert set(json.load(open(tmp_path / "hbm_traffic.json"))) == {"wl", "wl_push"}


def test_stored_traffic_without_a_file(tmp_path, monkeypatch):
    monkeypatch.setattr(profiling, "PROFILES", str(tmp_path))
    value, note = profiling.stored_traffic("dsv3_decode", "dispatch_unpack_kernel", "abc")
    assert value is None and "missing" in note


def test_counter_summary_averages_per_kernel(tmp_path):
    src, out = tmp_path / "c.csv", tmp_path / "c.md"
    with open(src, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Kernel_Name", "Counter_Name", "Counter_Value"])
        for v in (10, 30):
            w.writerow([UNPACK, "SQ_WAVES", v])
        w.writerow([UNPACK, "SQ_BUSY_CYCLES", 7])
        w.writerow(["some_other_kernel(int)", "SQ_WAVES", 99])
    profiling.counters(str(src), str(out), "t", "cmd")
    lines = out.read_text().splitlines()
    row = [l for l in lines if l.startswith("| dispatch_unpack_kernel")]
    assert row == ["| dispatch_unpack_kernel<false, false> | 2 | 7 | 20 |"]       # columns sorted by counter name
    assert not any("some_other_kernel" in l for l in lines)
