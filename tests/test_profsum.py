"""The profile summariser (paper_2503_08640_amd/profsum.py) on small hand-written rocprofv3-style CSVs: kernel
names are shortened, launches of one kernel are grouped by duration, the traffic figures scale each counter by the
256 MiB calibration copy and tell the prefill launches apart by their template arguments, and bench.py drops the
stored traffic when the kernel sources no longer match the digest it was measured at."""
import json
import os
import types

from paper_2503_08640_amd import profsum as ps

PRE = "void (anonymous namespace)::attn_prefill64_kernel<4, 2, false, true, false, false>(AttnParams)"
QRY = "void (anonymous namespace)::attn_prefill64_kernel<4, 2, true, false, false, false>(AttnParams)"
MRG = "void (anonymous namespace)::prefill_merge_kernel(AttnParams, int, int)"
DEC = "void (anonymous namespace)::decode_group_kernel<false>(AttnParams)"
DMG = "void (anonymous namespace)::decode_group_merge_kernel(AttnParams)"
COPY = "__amd_rocclr_copyBuffer"
HEAD = ('"Correlation_Id","Dispatch_Id","Agent_Id","Queue_Id","Process_Id","Thread_Id","Grid_Size","Kernel_Id","Kernel_Name",'
        '"Workgroup_Size","LDS_Block_Size","Scratch_Size","VGPR_Count","Accum_VGPR_Count","SGPR_Count","Counter_Name",'
        '"Counter_Value","Start_Timestamp","End_Timestamp"')


def counter_csv(path, counter, rows):
    """rows: (dispatch, kernel, grid, value, start, end)"""
    with open(path, "w") as f:
        f.write(HEAD + "\n")
        for d, k, g, v, t0, t1 in rows:
            f.write(f'{d},{d},"Agent 1",1,1,1,{g},1,"{k}",256,0,0,8,0,32,"{counter}",{v},{t0},{t1}\n')


def test_names_and_duration_groups():
    assert ps.short_name(PRE) == "attn_prefill64_kernel<4,2,false,true,false,false>"
    assert ps.short_name(MRG) == "prefill_merge_kernel"
    assert len(ps.short_name("x" * 200)) == 64
    groups = ps.clusters({1: 100.0, 2: 110.0, 3: 400.0, 4: 390.0, 5: 1000.0})
    assert [sorted(g) for g in groups] == [[1, 2], [3, 4], [5]]
    assert ps.clusters({}) == []


def test_traffic_scales_by_the_copy_and_groups_by_template_arguments(tmp_path):
    fetch, write, out = tmp_path / "f.csv", tmp_path / "w.csv", tmp_path / "t.json"
    # FETCH_SIZE reads half the KiB of the copy, WRITE_SIZE all of it; small copies (uploads) must not be taken for it
    counter_csv(fetch, "FETCH_SIZE", [(1, COPY, 512, 4.0, 0, 10), (2, COPY, 131072, 131072.0, 0, 10), (3, PRE, 65536, 1000.0, 0, 10),
                                      (4, PRE, 65536, 3000.0, 0, 10), (5, QRY, 65536, 500.0, 0, 10), (6, MRG, 4096, 20.0, 0, 10),
                                      (7, DEC, 110592, 100.0, 0, 10), (8, DMG, 512, 10.0, 0, 10)])
    counter_csv(write, "WRITE_SIZE", [(1, COPY, 512, 4.0, 0, 10), (2, COPY, 131072, 262144.0, 0, 10), (3, PRE, 65536, 700.0, 0, 10),
                                      (4, PRE, 65536, 700.0, 0, 10), (5, QRY, 65536, 30.0, 0, 10), (6, MRG, 4096, 8.0, 0, 10),
                                      (7, DEC, 110592, 12.0, 0, 10), (8, DMG, 512, 1.0, 0, 10)])
    args = types.SimpleNamespace(fetch=str(fetch), write=str(write), out=str(out), commit="abc1234")
    assert ps.cmd_traffic(args) == 0
    rec = json.load(open(out))
    assert rec["git_commit"] == "abc1234" and rec["sources_sha256"] == ps.kernel_sources_digest()
    assert abs(rec["fetch_factor"] - 2.0) < 1e-9 and abs(rec["write_factor"] - 1.0) < 1e-9
    assert rec["preencode"]["bytes_per_launch"] == int((2000.0 * 2.0 + 700.0) * 1024)          # mean of the two launches
    assert rec["query_prefill"]["bytes_per_launch"] == int(((500.0 + 20.0) * 2.0 + 38.0) * 1024)  # prefill + its merge
    assert rec["decode_step"]["bytes_per_launch"] == int(((100.0 + 10.0) * 2.0 + 13.0) * 1024)   # group kernel + merge, not twice


def test_source_digest_follows_the_kernel_sources(tmp_path, monkeypatch):
    before = ps.kernel_sources_digest()
    assert before == ps.kernel_sources_digest() and len(before) == 64
    src = tmp_path / "csrc"
    src.mkdir()
    (src / "a.hip").write_text("x")
    (src / "notes.txt").write_text("ignored")
    monkeypatch.setattr(ps, "ROOT", str(tmp_path))
    d1 = ps.kernel_sources_digest()
    (src / "notes.txt").write_text("still ignored")
    assert ps.kernel_sources_digest() == d1
    (src / "a.hip").write_text("y")
    assert ps.kernel_sources_digest() != d1


def test_committed_traffic_record_names_what_it_was_measured_at():
    path = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles", "hbm_traffic.json")
    rec = json.load(open(path))
    assert len(rec["sources_sha256"]) == 64 and rec["git_commit"]
    for key in ("preencode", "query_prefill", "decode_step"):
        assert rec[key]["bytes_per_launch"] > 0


def test_bench_reports_no_traffic_when_the_sources_changed(monkeypatch):
    import bench
    traffic, at = bench.load_traffic()
    assert at is not None and set(at) == {"git_commit", "sources_sha256", "current"}
    assert at["current"] == (at["sources_sha256"] == ps.kernel_sources_digest())
    assert bool(traffic) == at["current"]
    monkeypatch.setattr(ps, "kernel_sources_digest", lambda: "0" * 64)
    traffic, at = bench.load_traffic()
    assert traffic == {} and at["current"] is False
