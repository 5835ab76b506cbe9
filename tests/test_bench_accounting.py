"""The byte counts and the traffic record behind bench.py's `roofline` object, checked without a GPU."""
import json
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from paper_2209_06800_amd import inputs  # noqa: E402


def test_gather_model_bytes_worked_by_hand():
    # 3 edges, 2 owned rows, 5 fp32 columns, GCN: per edge a 20-byte row, a 4-byte id and a 4-byte factor;
    # per owned row its own 20-byte row, a 20-byte output row and 12 bytes of row pointers and factor
    assert bench.gather_model_bytes(3, 2, 5, 4, True) == 3 * (20 + 4 + 4) + 2 * (20 + 20 + 12)
    # GIN has no per-edge factor; bf16 rows in, bf16 rows out
    assert bench.gather_model_bytes(3, 2, 8, 2, False, out_bytes=2) == 3 * (16 + 4) + 2 * (16 + 16 + 12)


def test_compulsory_bytes_worked_by_hand():
    # a perfect cache: each of the 2 + 4 table rows once, ids and factors once, the output once
    assert bench.compulsory_bytes(7, 2, 4, 5, 4, True) == 6 * 20 + 7 * 8 + 2 * (20 + 12)


def test_compulsory_never_exceeds_gather_model_on_the_configs():
    for cfg in (1, 2):
        w = inputs.config(cfg)
        lo, hi = int(w.bounds[w.part_id]), int(w.bounds[w.part_id + 1])
        nnz = int(w.row_ptr[hi] - w.row_ptr[lo])
        cols = w.col[w.row_ptr[lo]:w.row_ptr[hi]]
        num_halo = int(np.unique(cols[(cols < lo) | (cols >= hi)]).size)
        esz = 2 if w.dtype == "bf16" else 4
        gcn = w.layers[0].mode == "gcn"
        g = bench.gather_model_bytes(nnz, hi - lo, w.dim, esz, gcn)
        c = bench.compulsory_bytes(nnz, hi - lo, num_halo, w.dim, esz, gcn)
        assert 0 < c <= g


def test_traffic_record_is_complete_and_tied_to_a_commit():
    with open(os.path.join(ROOT, "profiles", "measured_traffic.json")) as f:
        rec = json.load(f)
    assert isinstance(rec["commit"], str) and len(rec["commit"]) >= 7
    want = {"cfg2_rmat20_gcn64_p4": 1, "cfg3_rmat22_gin128_bf16_p8": 1, "cfg4_powerlaw233k_gcn602": 1, "cfg5_rmat2.4M_gcn2layer_p8": 2}
    for name, layers in want.items():
        for layer in range(layers):
            e = rec["workloads"][name][f"layer{layer}"]
            # the bytes of the launch = main kernel + fix-up kernel = reads + writes, and the summary they come from exists
            assert abs(e["bytes"] - (e["main_kernel_bytes"] + e["fixup_kernel_bytes"])) <= 2        # averages, rounded
            assert abs(e["main_kernel_bytes"] - (e["read_bytes"] + e["write_bytes"])) <= 2
            assert os.path.exists(os.path.join(ROOT, e["profile"]))
            # the two ways of counting (DRAM-destined requests, FETCH_SIZE + WRITE_SIZE) agree within 1 %
            assert abs(e["fetch_size_write_size_bytes"] - e["main_kernel_bytes"]) <= 0.01 * e["main_kernel_bytes"]
            # what the summary divides: never above the HBM peak
            assert e["bytes"] / (e["avg_ns"] * 1e-9) <= 8e12
            m = bench.measured_traffic(name, layer)
            assert m == {"bytes": e["bytes"], "commit": rec["commit"], "profile": e["profile"]}
    assert bench.measured_traffic("no_such_workload", 0) is None
    assert bench.measured_traffic("cfg4_powerlaw233k_gcn602", 7) is None


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr or "--gpus 1" in r.stderr
