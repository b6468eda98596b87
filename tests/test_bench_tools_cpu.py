"""Host-side checks of the measurement tooling (no GPU): bench.py's argument contract, the traffic
figure it reads from the committed profile summary, and the rocprofv3 CSV summariser."""
import csv
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""          # no JSON line that could be mistaken for a measurement


def test_bench_without_a_gpu_fails_loudly():
    import torch
    if torch.cuda.is_available():
        return
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True)
    assert r.returncode == 3 and "no CPU fallback" in r.stderr and r.stdout.strip() == ""


def test_traffic_figures_come_from_the_committed_summaries_with_their_commit():
    import bench
    for fname, algorithmic in (("decode_retrieval_c3_llama8b_128k_b4.txt", 2 * 4 * 8 * 131072 * 128 * 2),
                               ("prefill_c4_64k_chunked.txt", None)):
        nbytes, source = bench.profiled_traffic(fname)
        assert nbytes and nbytes > 0
        assert fname in source and "@" in source and "not measured in this run" in source
        commit = source.split("@")[1].split()[0]
        assert len(commit) >= 7 and all(ch in "0123456789abcdef" for ch in commit)
        if algorithmic:                    # the decode launch reads its K and V once: within 1 % of the algorithmic bytes
            assert algorithmic <= nbytes <= 1.01 * algorithmic
    assert bench.profiled_traffic("no_such_summary.txt") == (None, None)


def test_every_profile_summary_names_its_command_and_runs_committed_files_only():
    pdir = os.path.join(ROOT, "profiles")
    names = sorted(os.listdir(pdir))
    assert names, "profiles/ is empty"
    tracked = set(subprocess.run(["git", "ls-files"], cwd=ROOT, capture_output=True, text=True).stdout.split())
    for name in names:
        text = open(os.path.join(pdir, name)).read()
        assert len(text) < 40000, name + " is not a short summary"
        cmds = [l for l in text.splitlines() if "rocprofv3" in l and " -- " in l]
        assert cmds, name + " names no rocprofv3 command"
        for l in cmds:
            prog = l.split(" -- ", 1)[1].split()
            assert prog[0] == "python3" and prog[1].endswith(".py"), l     # the program itself follows "--"
            if tracked:
                assert prog[1] in tracked, prog[1] + " is not a committed file"


def test_profile_summary_tables(tmp_path):
    from paper_2508_12407_amd import profile_summary as ps
    d = tmp_path / "run" / "host"
    d.mkdir(parents=True)
    with open(d / "1_kernel_trace.csv", "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Kind", "Kernel_Name", "Start_Timestamp", "End_Timestamp", "LDS_Block_Size", "Workgroup_Size_X",
                    "Grid_Size_X", "Grid_Size_Y", "Grid_Size_Z"])
        for i, (name, dur, gx) in enumerate([("void zz_a(int)", 1000, 256), ("void zz_a(int)", 3000, 256), ("void zz_a(int)", 500, 512),
                                             ("zz_b()", 10000, 64)]):
            w.writerow(["KERNEL_DISPATCH", name, 100000 * i, 100000 * i + dur, 1024, 256, gx, 1, 1])
    out = ps.kernels(str(tmp_path / "run"), top=5).splitlines()
    rows = [l.split() for l in out[1:-1]]
    assert out[-1] == "GPU time of all dispatches: 0.015 ms"               # 14.5 us, three decimals
    assert rows[0][0] == "zz_b()" and rows[0][-6:-2] == ["1", "10.00", "10.00", "10.00"]   # sorted by total time
    a256 = [r for r in rows if r[0] == "zz_a(int)" and "(256," in " ".join(r)][0]
    assert a256[-6:-2] == ["2", "2.00", "1.00", "3.00"]                       # calls, average, minimum, maximum
    with open(d / "1_counter_collection.csv", "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Kernel_Name", "Grid_Size", "Counter_Name", "Counter_Value"])
        w.writerow(["zz_a(int)", 256, "FETCH_SIZE", 10.0])
        w.writerow(["zz_a(int)", 256, "FETCH_SIZE", 30.0])
        w.writerow(["other()", 256, "FETCH_SIZE", 99.0])
    out = ps.counters(str(tmp_path / "run"), "zz_|copyBuffer").splitlines()
    assert len(out) == 2 and out[1].split()[-4:] == ["2", "20.0", "10.0", "30.0"]
