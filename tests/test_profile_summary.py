"""The rocprofv3 CSV summariser on small hand-made CSV files (CPU only)."""
import json
import subprocess
import sys

HEAD = '"Correlation_Id","Dispatch_Id","Agent_Id","Queue_Id","Process_Id","Thread_Id","Grid_Size","Kernel_Id","Kernel_Name","Workgroup_Size","LDS_Block_Size","Scratch_Size","VGPR_Count","Accum_VGPR_Count","SGPR_Count","Counter_Name","Counter_Value","Start_Timestamp","End_Timestamp"\n'


def _row(kernel, counter, value):
    return '1,1,"Agent 1",1,1,1,65536,1,"%s",256,0,0,64,0,32,"%s",%s,0,1\n' % (kernel, counter, value)


def _write(path, counter, att, comb, copy):
    att_name = "void (anonymous namespace)::attention_kernel<128, 1>((anonymous namespace)::AttnParams)"
    comb_name = "void (anonymous namespace)::combine_kernel<128>((anonymous namespace)::AttnParams, unsigned int)"
    path.mkdir()
    with open(path / "out_counter_collection.csv", "w") as f:
        f.write(HEAD)
        for v in att:
            f.write(_row(att_name, counter, v))
        for v in comb:
            f.write(_row(comb_name, counter, v))
        f.write(_row("__amd_rocclr_copyBuffer", counter, 7.0))          # a small upload: not the calibration copy
        f.write(_row("__amd_rocclr_copyBuffer", counter, copy))
        f.write(_row("some_other_kernel", counter, 1e9))


def test_traffic_scaling_and_json(tmp_path):
    # FETCH_SIZE reads half of the copy's 262144 KiB -> scale 2; WRITE_SIZE reads all of it -> scale 1
    _write(tmp_path / "fetch", "FETCH_SIZE", att=[1000.0, 3000.0], comb=[100.0], copy=131072.0)
    _write(tmp_path / "write", "WRITE_SIZE", att=[500.0, 500.0], comb=[50.0], copy=262144.0)
    out = tmp_path / "t.json"
    res = subprocess.run([sys.executable, "-m", "paper_2512_07350_amd.profile_summary", "traffic", str(tmp_path / "fetch"),
                          str(tmp_path / "write"), "--workload", "w", "--json", str(out), "--algorithmic-bytes", "123"],
                         capture_output=True, text=True, check=True)
    assert "scale 2.0000" in res.stdout and "scale 1.0000" in res.stdout
    doc = json.loads(out.read_text())["records"][0]
    assert len(doc["attention_source_sha256"]) == 64
    att = doc["kernels"]["attention_kernel<128,1>"]
    assert att["launches"] == 2 and att["fetch_bytes"] == 2000 * 1024 * 2 and att["write_bytes"] == 500 * 1024
    comb = doc["kernels"]["combine_kernel<128>"]
    # per call: attention + (merge launches / attention launches) x merge
    want = att["fetch_bytes"] + att["write_bytes"] + (comb["fetch_bytes"] + comb["write_bytes"]) * 1 / 2
    assert doc["attention_bytes_per_launch"] == int(want)
    assert doc["workload"] == "w" and doc["algorithmic_bytes_per_launch"] == 123
    # a second summary of the same workload replaces the record; another workload is appended
    for name in ("w", "w2"):
        subprocess.run([sys.executable, "-m", "paper_2512_07350_amd.profile_summary", "traffic", str(tmp_path / "fetch"),
                        str(tmp_path / "write"), "--workload", name, "--json", str(out)], capture_output=True, text=True, check=True)
    assert [r["workload"] for r in json.loads(out.read_text())["records"]] == ["w", "w2"]


def test_stats_table(tmp_path):
    (tmp_path / "s").mkdir()
    with open(tmp_path / "s" / "bench_kernel_stats.csv", "w") as f:
        f.write('"Name","Calls","TotalDurationNs","AverageNs","Percentage","MinNs","MaxNs","StdDev"\n')
        f.write('"void (anonymous namespace)::attention_kernel<128, 1>((anonymous namespace)::AttnParams)",4,400000,100000.0,80.0,90000,110000,1.0\n')
        f.write('"void at::native::something<float>(int)",10,100000,10000.0,20.0,1,2,1.0\n')
    res = subprocess.run([sys.executable, "-m", "paper_2512_07350_amd.profile_summary", "stats", str(tmp_path / "s")],
                         capture_output=True, text=True, check=True)
    lines = [l for l in res.stdout.splitlines() if l.startswith("| `")]
    assert lines == ["| `attention_kernel<128,1>` | 4 | 0.400 | 100.00 | 80.00 | 90.00 | 110.00 |"]
