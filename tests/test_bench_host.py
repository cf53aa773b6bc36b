"""Host-side logic of bench.py that needs no GPU: the single-GPU guard and the byte and flop
counts the roofline figures are built from (checked against hand-computed values of the
workloads: 4*d*sizeof bytes per row and head, 4 bytes per edge and 8 per row of the CSR once,
256 flop per edge)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from sga_inputs import WORKLOADS  # noqa: E402
import paper_2502_01659_amd as sga  # noqa: E402


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in (p.stdout + p.stderr) or "single" in (p.stdout + p.stderr).lower()


@pytest.mark.parametrize("name,nnz,alg_bytes", [
    ("cfg1_sliding_4k", 265_184, 4 * 64 * 4 * 4096 + 4 * 265_184 + 8 * 4097),
    ("cfg2_longformer_64k", 18_919_024, 4 * 64 * 4 * 65536 * 8 + 4 * 18_919_024 + 8 * 65537),
    ("cfg3_dilated_1m", 135_257_984, 4 * 64 * 2 * (1 << 20) * 4),
    ("cfg4_bigbird_1m", 671_014_912, 4 * 64 * 2 * (1 << 20) * 4 + 4 * 671_014_912 + 8 * ((1 << 20) + 1)),
    ("cfg5_sliding_160m", 5_279_999_728, 4 * 64 * 2 * 160_000_000),
])
def test_algorithmic_bytes_of_the_workloads(name, nnz, alg_bytes):
    wl = WORKLOADS[name]
    assert sga.mask_nnz(wl.mask) == nnz
    assert bench.algorithmic_bytes(wl, nnz) == alg_bytes
    assert bench.FLOPS_PER_EDGE == 4 * wl.d


def test_gather_aware_bytes():
    """BigBird-style mask: each of the nb - G non-global block rows fetches its R random key
    blocks (K and V) for itself, and the global rows pass over K and V once more per head."""
    wl = WORKLOADS["cfg4_bigbird_1m"]
    nnz = sga.mask_nnz(wl.mask)
    nb = (1 << 20) // 64
    extra_per_head = (nb - 2) * 3 * 64 * 64 * 2 * 2 + 2 * (1 << 20) * 64 * 2
    assert bench.gather_aware_bytes(wl, nnz) == bench.algorithmic_bytes(wl, nnz) + 4 * extra_per_head
    for name in ("cfg2_longformer_64k", "cfg3_dilated_1m"):
        w = WORKLOADS[name]
        n = sga.mask_nnz(w.mask)
        assert bench.gather_aware_bytes(w, n) == bench.algorithmic_bytes(w, n)


def test_roofline_record_fields():
    wl = WORKLOADS["cfg2_longformer_64k"]
    nnz = sga.mask_nnz(wl.mask)
    r = bench.roofline_of(wl, nnz, 0.5, 0.6, "auto", "tile_attend_kernel")
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 157.3
    assert abs(r["achieved"] - 256 * nnz * 8 / 0.5e-3 / 1e12) < 1e-9
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12
    # forward level: the same flops over the whole call, and the call's algorithmic bytes
    assert abs(r["forward"]["achieved"] - 256 * nnz * 8 / 0.6e-3 / 1e12) < 1e-9
    assert r["forward"]["algorithmic_bytes"] == bench.algorithmic_bytes(wl, nnz)
    r = bench.roofline_of(WORKLOADS["cfg5_sliding_160m"], 5_279_999_728, 15.0, 15.0, "auto", "k")
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["achieved"] - 81.92e9 / 15e-3 / 1e9) < 1e-6
    # explicit fp16 workload: the dominant kernel's figure counts the tensors only (the tile
    # kernel never reads col_idx); the forward-level one counts col_idx and row_ptr unless the
    # graph was prepared
    w4 = WORKLOADS["cfg4_bigbird_1m"]
    n4 = sga.mask_nnz(w4.mask)
    tensors = 4 * 64 * 2 * (1 << 20) * 4
    r = bench.roofline_of(w4, n4, 1.0, 2.0, "auto", "tile_attend_kernel")
    assert abs(r["achieved"] - tensors / 1e-3 / 1e9) < 1e-6
    assert abs(r["forward"]["achieved"] - bench.algorithmic_bytes(w4, n4) / 2e-3 / 1e9) < 1e-6
    r = bench.roofline_of(w4, n4, 1.0, 1.25, "auto", "tile_attend_kernel", prepared=True)
    assert abs(r["forward"]["achieved"] - tensors / 1.25e-3 / 1e9) < 1e-6


def test_traffic_summary_from_counter_files(tmp_path, monkeypatch):
    """The per-forward traffic record is computed from rocprofv3 counter files: synthetic csv
    files with known values go in, scaled per-kernel bytes come out."""
    import json
    head = ('"Correlation_Id","Dispatch_Id","Agent_Id","Queue_Id","Process_Id","Thread_Id","Grid_Size",'
            '"Kernel_Id","Kernel_Name","Workgroup_Size","LDS_Block_Size","Scratch_Size","VGPR_Count",'
            '"Accum_VGPR_Count","SGPR_Count","Counter_Name","Counter_Value","Start_Timestamp","End_Timestamp"\n')

    def write(sub, counter, rows):
        d = tmp_path / sub
        d.mkdir()
        with open(d / "x_counter_collection.csv", "w") as f:
            f.write(head)
            for i, (name, val) in enumerate(rows):
                f.write(f'{i},{i},"Agent 1",1,1,1,64,1,"{name}",256,0,0,8,0,8,"{counter}",{val},0,1\n')

    copy = "__amd_rocclr_copyBuffer"
    attend = "void sga::(anonymous namespace)::tile_attend_kernel<__half, 1>(args)"
    analyze = "sga::(anonymous namespace)::tile_analyze_kernel(args)"
    write("fetch_copy", "FETCH_SIZE", [(copy, 524288.0)] * 2)            # shows half of 1 GiB
    write("write_copy", "WRITE_SIZE", [(copy, 1048576.0)] * 2)
    write("fetch_cfg4_bigbird_1m", "FETCH_SIZE", [(analyze, 100.0), (attend, 1000.0)] * 3)
    write("write_cfg4_bigbird_1m", "WRITE_SIZE", [(analyze, 10.0), (attend, 50.0)] * 3)
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(tmp_path / "t.json"))
    bench.traffic_summary(str(tmp_path), "cfg4_bigbird_1m", False)
    rec = json.load(open(tmp_path / "t.json"))["cfg4_bigbird_1m"]
    assert rec["dominant_kernel"] == "tile_attend_kernel<half>"
    assert rec["dominant_kernel_bytes"] == int(1000 * 1024 * 2.0 + 50 * 1024)
    assert rec["forward_bytes"] == int(1100 * 1024 * 2.0 + 60 * 1024)
    assert bench.measured_traffic("cfg4_bigbird_1m") == (rec["dominant_kernel_bytes"], rec["forward_bytes"])
    assert bench.measured_traffic("cfg4_bigbird_1m", prepared=True) == (None, None)
