"""Host-side pieces of the measurement: the profiler-output condenser and the traffic files bench.py reads."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from benchprobe import pmc_summary  # noqa: E402

HDR = ('"Correlation_Id","Dispatch_Id","Agent_Id","Queue_Id","Process_Id","Thread_Id","Grid_Size","Kernel_Id","Kernel_Name",'
       '"Workgroup_Size","LDS_Block_Size","Scratch_Size","VGPR_Count","Accum_VGPR_Count","SGPR_Count","Counter_Name","Counter_Value",'
       '"Start_Timestamp","End_Timestamp"\n')


def _row(i, kernel, counter, value):
    return '%d,%d,"Agent 1",1,7,7,512,7,"%s",256,0,0,8,0,32,"%s",%f,100,200\n' % (i, i, kernel, counter, value)


def test_pmc_summary_scales_counters_by_the_copy_of_known_size(tmp_path):
    """FETCH_SIZE reads half the bytes on this device and WRITE_SIZE all of them: both factors come from the copy kernel's
    rows of the same run, and the traffic file carries the hash of the attention kernel's sources."""
    attn = "void kvq::k_decode_split<2, false>(kvq::AttnParams)"
    copy = "benchprobe::k_probe_copy(HIP_vector_type<unsigned int, 4u>*, HIP_vector_type<unsigned int, 4u> const*, unsigned long)"
    for name, counter, attn_v, copy_v in (("fetch", "FETCH_SIZE", 1000.0, 524288.0), ("write", "WRITE_SIZE", 10.0, 1048576.0)):
        d = tmp_path / name / "vm"
        d.mkdir(parents=True)
        with open(d / "1_counter_collection.csv", "w") as f:
            f.write(HDR)
            f.write(_row(1, attn, counter, attn_v))
            f.write(_row(2, attn, counter, attn_v + 2.0))
            f.write(_row(3, copy, counter, copy_v))
    d = tmp_path / "trace" / "vm"
    d.mkdir(parents=True)
    with open(d / "1_kernel_stats.csv", "w") as f:
        f.write('"Name","Calls","TotalDurationNs","AverageNs","Percentage","MinNs","MaxNs","StdDev"\n')
        f.write('"%s",2,220000,110000.0,90.0,109000,111000,1.0\n' % attn)
    out, traffic = tmp_path / "summary.txt", tmp_path / "traffic.txt"
    r = subprocess.run([sys.executable, os.path.join(ROOT, "benchprobe", "pmc_summary.py"), "--dirs", str(tmp_path / "trace"),
                        str(tmp_path / "fetch"), str(tmp_path / "write"), "--kernel", "k_", "--out", str(out),
                        "--traffic-kernel", "k_decode_split<2, false>", "--traffic-out", str(traffic)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    text = out.read_text()
    assert "k_decode_split<2, false>" in text and "110.00" in text and "k_probe_copy" in text
    kv = dict(l.strip().split("=", 1) for l in traffic.read_text().splitlines() if "=" in l and not l.startswith("#"))
    assert abs(float(kv["fetch_factor"]) - 2.0) < 1e-3 and abs(float(kv["write_factor"]) - 1.0) < 1e-3   # (1e-4 rounding of the printed factor)
    want = (1001.0 * 2.0 + 11.0 * 1.0) * 1024.0
    assert abs(float(kv["traffic_bytes_per_launch"]) - want) <= 2.0
    assert kv["sources_sha256"] == pmc_summary.sources_sha256()


def test_committed_traffic_files_belong_to_the_attention_kernel_in_this_tree():
    """bench.py prints roofline.traffic only while the attention kernel's sources hash to the value in the profile: a
    kernel change without new --pmc runs would silently drop the figure, so it fails here first."""
    now = pmc_summary.sources_sha256()
    for cfg in (4, 5):
        path = os.path.join(ROOT, "profiles", "k_decode_split_cfg%d_traffic.txt" % cfg)
        kv = dict(l.strip().split("=", 1) for l in open(path) if "=" in l and not l.startswith("#"))
        assert kv["sources_sha256"] == now, "%s was taken from other sources: run the --pmc commands of the profile again" % path
        assert 0.99 < float(kv["traffic_bytes_per_launch"]) / {4: 707951104.0, 5: 2546136064.0}[cfg] < 1.02
