"""The rocprofv3 CSV summariser (paper_2604_26666_amd/counters.py) on small synthetic files: the copy-based
scale of FETCH_SIZE / WRITE_SIZE, the consecutive-run listing of a kernel trace, and the traffic file
that bench.py quotes (which must name the kernel build it was measured on)."""
import io
import json

from paper_2604_26666_amd import counters

HEAD_C = '"Correlation_Id","Dispatch_Id","Agent_Id","Queue_Id","Process_Id","Thread_Id","Grid_Size","Kernel_Id","Kernel_Name","Workgroup_Size","LDS_Block_Size","Scratch_Size","VGPR_Count","Accum_VGPR_Count","SGPR_Count","Counter_Name","Counter_Value","Start_Timestamp","End_Timestamp"\n'
HEAD_T = '"Kind","Agent_Id","Queue_Id","Stream_Id","Thread_Id","Dispatch_Id","Kernel_Id","Kernel_Name","Correlation_Id","Start_Timestamp","End_Timestamp","LDS_Block_Size","Scratch_Size","VGPR_Count","Accum_VGPR_Count","SGPR_Count","Workgroup_Size_X","Workgroup_Size_Y","Workgroup_Size_Z","Grid_Size_X","Grid_Size_Y","Grid_Size_Z"\n'


def counter_csv(path, counter, gemm_vals, copy_vals):
    rows, t = [], 1000
    for i, v in enumerate([12.0] + list(gemm_vals)):          # a small copy first (an upload), then the GEMMs
        name = "__amd_rocclr_copyBuffer" if i == 0 else "void fact::gemm_kernel<256, 256, 2, 2, false, 64, 2, false>(fact::GemmArgs)"
        rows.append(f'{i+1},{i+1},"Agent 1",1,1,1,{1024 if i == 0 else 262144},8,"{name}",256,0,0,8,0,32,"{counter}",{v},{t},{t+500}\n')
        t += 1000
    for j, v in enumerate(copy_vals):
        k = len(rows) + 1
        rows.append(f'{k},{k},"Agent 1",1,1,1,131072,9,"__amd_rocclr_copyBuffer",512,0,0,8,0,32,"{counter}",{v},{t},{t+400000}\n')
        t += 500000
    path.write_text(HEAD_C + "".join(rows))


def test_copy_scale_and_traffic_file(tmp_path):
    f, w, probe, out = tmp_path / "f.csv", tmp_path / "w.csv", tmp_path / "probe.txt", tmp_path / "t.json"
    counter_csv(f, "FETCH_SIZE", [786000.0, 787000.0, 788000.0], [524288.0] * 3)        # the counter reports half the bytes read
    counter_csv(w, "WRITE_SIZE", [131072.0] * 3, [1048576.0] * 3)
    probe.write_text('noise\n{"traffic_probe": true, "gemm_launches": 3, "copies": 3, "copy_bytes": 1073741824, "n": 8192, "kernel_tag": "cfg0.tb0.v999"}\n')
    gr = counters.groups(counters.read(str(f)))
    assert abs(counters.copy_scale(gr, "FETCH_SIZE") - 2048.0) < 1e-9
    counters.traffic_json(str(f), str(w), str(probe), str(out))
    doc = json.loads(out.read_text())
    assert doc["n"] == 8192 and doc["kernel_tag"] == "cfg0.tb0.v999"
    assert abs(doc["FETCH_SIZE"]["bytes"] - 787000.0 * 2048.0) < 1.0
    assert abs(doc["WRITE_SIZE"]["bytes"] - 131072.0 * 1024.0) < 1.0
    assert abs(doc["bytes_per_launch"] - (787000.0 * 2048.0 + 131072.0 * 1024.0)) < 2.0
    buf = io.StringIO()
    counters.summarise([str(f)], out=buf)
    text = buf.getvalue()
    assert "gemm_kernel<256, 256, 2, 2, false, 64, 2, false>" in text and "1611.78 MB" in text        # 787000 KiB x 2048 B


def test_runs_lists_consecutive_launches(tmp_path):
    p = tmp_path / "trace.csv"
    rows, t = [], 0
    def add(name, gx, n, dur):
        nonlocal t
        for _ in range(n):
            rows.append(f'"KERNEL_DISPATCH","Agent 1",1,1,1,{len(rows)+1},7,"{name}",{len(rows)+1},{t},{t+dur},0,0,8,0,32,256,1,1,{gx},1,1\n')
            t += dur + 100
    add("void fact::gemm_kernel<128, 128, 2, 2, true, 64, 2, false>(fact::GemmArgs)", 4096, 30, 9000)
    add("other_kernel", 64, 3, 100)
    add("void fact::gemm_kernel<128, 128, 2, 2, true, 64, 2, false>(fact::GemmArgs)", 4096, 25, 11000)    # the same kernel again: a second run
    p.write_text(HEAD_T + "".join(rows))
    buf = io.StringIO()
    counters.runs(str(p), 20, out=buf)
    lines = [l for l in buf.getvalue().splitlines() if l]
    assert len(lines) == 2
    assert "launches 30" in lines[0] and "second_half_avg_us 9.00" in lines[0]
    assert "launches 25" in lines[1] and "second_half_avg_us 11.00" in lines[1]


def test_bench_quotes_the_traffic_file_only_for_the_kernel_it_describes(tmp_path, monkeypatch):
    import bench
    f = tmp_path / "traffic.json"
    f.write_text(json.dumps({"n": 8192, "kernel_tag": "cfg0.tb0.v7", "bytes_per_launch": 1.5e9}))
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(f))
    value, source = bench.measured_traffic(8192, "cfg0.tb0.v7")
    assert value == 1.5e9 and "not this run" in source
    value, source = bench.measured_traffic(8192, "cfg0.tb0.v8")           # another build of the kernel: no figure
    assert value is None and "another kernel" in source
    value, source = bench.measured_traffic(4096, "cfg0.tb0.v7")
    assert value is None
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(tmp_path / "missing.json"))
    assert bench.measured_traffic(8192, "cfg0.tb0.v7") == (None, None)
