"""profile_report.py on small hand-written rocprofv3 CSV files (no GPU, no profiler): the counters are scaled by what
the calibration copy reads, the matrix-core table is derived as documented, and the traffic table gets the bytes of
the named kernel's largest launch together with the digest of the kernel sources the run recorded."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

HEAD = ('"Correlation_Id","Dispatch_Id","Agent_Id","Queue_Id","Process_Id","Thread_Id","Grid_Size","Kernel_Id","Kernel_Name",'
        '"Workgroup_Size","LDS_Block_Size","Scratch_Size","VGPR_Count","Accum_VGPR_Count","SGPR_Count","Counter_Name",'
        '"Counter_Value","Start_Timestamp","End_Timestamp"\n')


def row(i, grid, kernel, counter, value, t0=1000, t1=3000):
    return '%d,%d,"Agent 1",1,1,1,%d,7,"%s",256,0,0,8,0,16,"%s",%f,%d,%d\n' % (i, i, grid, kernel, counter, value, t0, t1)


def test_report_from_hand_written_csv(tmp_path):
    name = "unit_test_profile"
    out = os.path.join(ROOT, "gpurun_out", "prof_" + name)
    os.makedirs(out, exist_ok=True)
    gate = "void hmoe::ffn_tile_fit_kernel<true, 4, false>(hmoe::TiledCtx, unsigned short const*, unsigned short*)"
    files = {
        "trace.log": json.dumps({"config": {"workload": "stress/prefill16384"}, "value": 1.0, "unit": "tokens/s", "ms_per_step": 2.0,
                                 "roofline": {"bound": "mfma", "frac": 0.4}, "phases": {}}) + "\n",
        "trace_kernel_stats.csv": '"Name","Calls","TotalDurationNs","AverageNs","Percentage","MinNs","MaxNs","StdDev"\n'
                                  '"%s",4,4000,1000.0,80.0,900,1100,1.0\n' % gate,
        # the copy reads half of what it moved on FETCH_SIZE and all of it on WRITE_SIZE: factors 2 and 1
        "fetch_counter_collection.csv": HEAD + row(1, 131072, "__amd_rocclr_copyBuffer", "FETCH_SIZE", 524288.0)
        + row(2, 1000, gate, "FETCH_SIZE", 100.0) + row(3, 2000, gate, "FETCH_SIZE", 1000.0) + row(4, 2000, gate, "FETCH_SIZE", 3000.0),
        "write_counter_collection.csv": HEAD + row(1, 131072, "__amd_rocclr_copyBuffer", "WRITE_SIZE", 1048576.0)
        + row(2, 1000, gate, "WRITE_SIZE", 50.0) + row(3, 2000, gate, "WRITE_SIZE", 500.0) + row(4, 2000, gate, "WRITE_SIZE", 500.0),
        # 8 dies x 1000 cycles in 2000 ns -> 0.5 GHz; 1024 SIMDs x 400 busy cycles -> MFMA busy 0.4; 512 x 1e6 flop
        "sq_counter_collection.csv": HEAD + "".join(row(5, 2000, gate, c, v) for c, v in (
            ("GRBM_GUI_ACTIVE", 8000.0), ("SQ_VALU_MFMA_BUSY_CYCLES", 409600.0), ("SQ_INSTS_VALU_MFMA_MOPS_BF16", 1.0e6),
            ("SQ_ACTIVE_INST_VALU", 10.0), ("SQ_ACTIVE_INST_LDS", 5.0), ("SQ_LDS_BANK_CONFLICT", 0.0))),
        "kernel_sources.txt": "0123456789abcdef\n",
    }
    for f, text in files.items():
        with open(os.path.join(out, f), "w") as fh:
            fh.write(text)
    traffic = os.path.join(ROOT, "profiles", "traffic.json")
    with open(traffic) as fh:
        before = fh.read()
    try:
        run = subprocess.run([sys.executable, os.path.join(ROOT, "profile_report.py"), name, "--report-only", "--sq", "--traffic",
                              "unit/test=ffn_tile_fit_kernel<true", "--", "--workload", "stress"], capture_output=True, text=True, cwd=ROOT)
        assert run.returncode == 0, run.stderr
        with open(os.path.join(ROOT, "profiles", name + ".md")) as fh:
            md = fh.read()
        with open(traffic) as fh:
            table = json.load(fh)
    finally:
        with open(traffic, "w") as fh:
            fh.write(before)
        md_path = os.path.join(ROOT, "profiles", name + ".md")
        if os.path.exists(md_path):
            os.remove(md_path)
    assert "scaled by 2.000 and 1.000" in md
    # largest grid (2000): fetch mean 2000 KiB x 2 + write 500 KiB = 4500 KiB
    assert table["unit/test"] == {"bytes": 4500 * 1024, "kernel": "ffn_tile_fit_kernel<true, 4, false>", "grid": 2000,
                                  "sources": "0123456789abcdef", "profile": "profiles/%s.md" % name}
    line = [l for l in md.splitlines() if l.startswith("| `ffn_tile_fit_kernel<true, 4, false>` | 2000 | 1 |")][-1]
    cells = [c.strip() for c in line.split("|")]
    assert cells[5] == "1000" and cells[6] == "0.50" and cells[7] == "0.400" and cells[8] == "0.0005"
