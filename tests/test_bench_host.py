"""Host-side logic of bench.py that needs no GPU: the one-GPU guard, the work model that the roofline
figures are divided by, and the parsing of the rocprofv3 counter files."""
import csv
import json
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from gear_inputs import get_workload  # noqa: E402
from gear_inputs.pageviews import PageViewBatch  # noqa: E402

NS = "gear::(anonymous namespace)::"   # as the kernels' names come out of the profiler


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_work_model_counts_what_a_step_has_to_move():
    """A batch small enough to count by hand (Section 1, third point: groups of M per image)."""
    wl = get_workload("tiny").scaled(M=2)                      # d 16, D 64, fp32 everywhere, layers (64, 1)
    model = bench.WorkModel(wl, [wl.in_features, 64], [64, 1])
    # three views: images [5, 5, 7], [], [7]; users 1, 1, 2; urls 3, 4, 4
    b = PageViewBatch(user_id=np.array([1, 1, 2], np.int32), url_id=np.array([3, 4, 4], np.int32),
                      img_off=np.array([0, 3, 3, 4], np.int32), img_id=np.array([5, 5, 7, 7], np.int32),
                      label=np.zeros(3, np.float32))
    w = model.step(b)
    B, nnz, d, D, F = 3, 4, 16, 64, 96
    assert w["fwd_gemm_l0"] == ("mfma", 2.0 * B * 64 * F) == w["wgrad_gemm_l0"] == w["wgrad_gemm"]
    # dLoss/dx is made by two products: the embedding slots (2 d columns), then the DFV slot (D columns)
    assert w["dgrad_gemm_emb"] == ("mfma", 2.0 * B * 64 * 2 * d) and w["dgrad_gemm_l0"] == ("mfma", 2.0 * B * 64 * D)
    assert "fwd_gemm_l1" not in w                                # the logit layer is not a matrix product here
    # gather: ids and offsets, each distinct row once (2 users, 2 urls, 2 images), x written once
    assert w["gather_pool"] == ("hbm", 12.0 * B + 4.0 * nnz + 4 * d * 4 + 2 * D * 4 + B * F * 4)
    # accumulate, first step (all counters 0): both images close one group of M = 2 and leave nothing:
    # no accumulator row read, none written, two emissions; dx rows of the two views that have images
    assert w["accumulate"] == ("hbm", 40.0 * 2 + 8.0 * nnz + 2 * D * 4 + 0 + 0 + 2 * D * 4.0)
    # second step, image 5 once more: its counter is 2 (phase 0), one gradient stays in its accumulator
    b2 = PageViewBatch(user_id=np.array([1], np.int32), url_id=np.array([3], np.int32), img_off=np.array([0, 1], np.int32),
                       img_id=np.array([5], np.int32), label=np.zeros(1, np.float32))
    w2 = model.step(b2)
    assert w2["accumulate"] == ("hbm", 40.0 * 1 + 8.0 * 1 + 1 * D * 4 + 0 + 1 * D * 4.0 + 0)
    # third step, image 5 again: phase 1 -> its accumulator row is read, the group closes, nothing stays
    w3 = model.step(b2)
    assert w3["accumulate"] == ("hbm", 40.0 * 1 + 8.0 * 1 + 1 * D * 4 + 1 * D * 4.0 + 1 * D * 4.0 + 1 * D * 4.0)


def _counter_csv(path, counter, rows):
    with open(path, "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"])
        w.writeheader()
        for i, (name, value) in enumerate(rows):
            w.writerow({"Dispatch_Id": i, "Kernel_Name": name, "Counter_Name": counter, "Counter_Value": value})


def test_counter_files_become_bytes_per_launch(tmp_path, monkeypatch):
    """Two steps' worth of dispatches; the refresh copy of known size calibrates each counter."""
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(tmp_path / "traffic.json"))
    monkeypatch.setattr(bench, "TRAFFIC_SUMMARY", str(tmp_path / "traffic.txt"))
    ns = "void gear::(anonymous namespace)::"
    step = [("k_gather_pool<float, unsigned short, unsigned short>(int)", 10.0), ("k_gemm_nt_dma<0, %sNtWide>(x)" % NS, 20.0),
            ("k_gemm_nt_dma<0, %sNtWide>(x)" % NS, 30.0), ("k_gemm_nt_dma<4, %sNtWide>(x)" % NS, 40.0), ("k_gemm_nt_dma<3, %sNtNarrow>(x)" % NS, 50.0),
            ("k_embedding_chunks<float>(x)", 5.0), ("k_embedding_spans<float>(x)", 7.0),
            ("k_gemm_nt_dma<3, %sNtWide>(x)" % NS, 60.0), ("k_gemm_tn_dma_batch(x)", 70.0), ("k_accumulate<unsigned short>(x)", 80.0)]
    rows = [(ns + n, v) for n, v in step] + [(ns + n, v + 2.0) for n, v in step] + [(ns + "k_refresh(x)", 1000.0)]
    _counter_csv(tmp_path / "f.csv", "FETCH_SIZE", rows)
    _counter_csv(tmp_path / "w.csv", "WRITE_SIZE", [(n, 2 * v) for n, v in rows])
    bench.record_traffic(str(tmp_path / "f.csv"), str(tmp_path / "w.csv"), refresh_bytes=4000)
    rec = json.load(open(tmp_path / "traffic.json"))
    assert rec["calibration"] == {"fetch_bytes_per_count": 4.0, "write_bytes_per_count": 2.0}
    k = rec["kernels"]
    # launches of one kernel inside a step are told apart by their order: fwd l0 is the first NT<0>, the
    # embedding slots of dLoss/dx the first NT<3>
    assert k["fwd_gemm_l0"]["fetch_bytes"] == 4.0 * 21.0 and k["fwd_gemm_l1"]["fetch_bytes"] == 4.0 * 31.0
    assert k["dgrad_gemm_emb"]["fetch_bytes"] == 4.0 * 51.0 and k["dgrad_gemm_l0"]["fetch_bytes"] == 4.0 * 61.0
    assert k["wgrad_gemm"]["write_bytes"] == 2.0 * 142.0
    assert k["accumulate"]["bytes"] == 4.0 * 81.0 + 2.0 * 162.0 and k["accumulate"]["launches"] == 2
    # a span of two launches is the sum of both
    assert k["embedding_update"]["fetch_bytes"] == 4.0 * (6.0 + 8.0)
    assert "accumulate" in open(tmp_path / "traffic.txt").read()
    # a record is only reported while the kernel's source is the one it was taken on
    assert bench.recorded_traffic("accumulate") == k["accumulate"]["bytes"]
    rec["kernels"]["accumulate"]["source_hash"] = "0" * 16
    json.dump(rec, open(tmp_path / "traffic.json", "w"))
    assert bench.recorded_traffic("accumulate") is None and bench.recorded_traffic("gather_pool") is not None


def test_mfma_counters_become_occupancy(tmp_path, monkeypatch):
    """busy cycles over all SIMDs against the cycles on the device (the counter sums the XCDs)."""
    monkeypatch.setattr(bench, "MFMA_SUMMARY", str(tmp_path / "mfma.txt"))
    ns = "void gear::(anonymous namespace)::"
    names = ["k_gemm_nt_dma<0, %sNtWide>(x)" % NS, "k_gemm_nt_dma<0, %sNtWide>(x)" % NS, "k_gemm_nt_dma<4, %sNtWide>(x)" % NS, "k_gemm_nt_dma<3, %sNtNarrow>(x)" % NS, "k_gemm_nt_dma<3, %sNtWide>(x)" % NS,
             "k_gemm_tn_dma_batch(x)"]
    with open(tmp_path / "m.csv", "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"])
        w.writeheader()
        for i, n in enumerate(names):
            w.writerow({"Dispatch_Id": i, "Kernel_Name": ns + n, "Counter_Name": "SQ_VALU_MFMA_BUSY_CYCLES", "Counter_Value": 1024.0 * 100 * (i + 1)})
            w.writerow({"Dispatch_Id": i, "Kernel_Name": ns + n, "Counter_Name": "GRBM_GUI_ACTIVE", "Counter_Value": 8.0 * 1000})
    bench.record_mfma(str(tmp_path / "m.csv"))
    table = {l.split()[0]: l.split() for l in open(tmp_path / "mfma.txt") if not l.startswith("#")}
    assert float(table["fwd_gemm_l0"][4]) == 0.1 and float(table["fwd_gemm_l1"][4]) == 0.2
    assert float(table["wgrad_gemm"][4]) == 0.6 and table["dgrad_gemm_l0"][1] == "1"
