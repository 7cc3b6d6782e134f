"""bench.py's reading of the tracked counter file: figures only for the kernel and workload they were taken on."""
import json
import os
import sys
import types

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def _lib(format_id):
    return types.SimpleNamespace(FORMAT_ID=format_id)


def test_counters_are_for_the_format_the_library_writes():
    doc = json.load(open(bench.COUNTERS_FILE))
    assert bench.load_counters(_lib(doc["format_id"])) == doc["kernels"]
    assert bench.load_counters(_lib(doc["format_id"] + 1)) == {}


def test_traffic_and_issue_rates_of_the_headline_kernel():
    doc = json.load(open(bench.COUNTERS_FILE))
    k = doc["kernels"]
    key = "dc_decode_kernel<256,int8>|config3_32layers_64KiB"
    raw = 6476005376
    t = bench.measured_traffic(k, key)
    # blob read + buffer written, within 2 % of the algorithmic bytes of a ratio-1.11 blob
    assert 0.98 < t / (raw * (1 + 1 / 1.1106)) < 1.02
    r = bench.issue_rates(k, key, raw, 2.27)
    assert r["bound"] == "alu" and r["unit"] == "T lane-ops/s"
    assert abs(r["lane_ops_per_decoded_byte"] - k[key]["valu_insts"] * 64 / raw) < 0.01
    # the peak follows from the kernel's mix of two-cycle and four-cycle instructions
    cpi = k[key]["valu_cycles_per_instruction"]
    assert 2.0 < cpi < 4.0
    assert abs(r["frac"] - k[key]["valu_insts"] * 64 / 2.27e-3 / (256 * 4 * 64 * 2.4e9 / cpi)) < 1e-3
    assert abs(bench.alu_peak_lane_ops() - 256 * 4 * 16 * 2.4e9) < 1.0  # four cycles where no mix is recorded
    assert 0 < r["lds_cycles_lost_to_bank_conflicts"] < 1


def test_no_figures_for_a_kernel_or_workload_without_a_counter_run():
    k = json.load(open(bench.COUNTERS_FILE))["kernels"]
    assert bench.measured_traffic(k, "dc_decode_kernel<256,int8>|config3_4layers_64KiB") is None
    assert bench.issue_rates(k, "dc_decode_kernel<256,int8,tANS>|config3_32layers_64KiB", 1, 1.0) is None
    assert bench.issue_rates({}, "anything", 1, 1.0) is None
    # a kernel with traffic readings but no instruction count has no issue rate
    assert bench.issue_rates(k, "dc_decode_kernel<256,int8>|config2_layer_x1_64KiB", 1, 1.0) is None
