"""bench.py's command-line contract that can be checked without a GPU."""

import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_of_the_headline_workload():
    sys.path.insert(0, ROOT)
    import bench
    # bf16 in + 4-bit codes + 16-bit metadata per block of 32: 2.5625 B per element
    assert bench.algorithmic_bytes(16384, 3072) == 128974848
    assert bench.algorithmic_bytes(16384, 3072, 16) == 16384 * 3072 * 2 + 16384 * 3072 // 2 + 16384 * 192 * 2
    assert bench.HBM_PEAK_GBS == 8000.0


def test_profile_summary_turns_counter_csvs_into_the_traffic_figure(tmp_path):
    sys.path.insert(0, ROOT)
    from paper_2603_02883_amd import profile_summary as ps
    head = "void fb4::" + ps.HEADLINE + "(unsigned char const*)"
    copy = "__amd_rocclr_copyBuffer"

    def write(sub, counter, rows):
        d = tmp_path / sub / "vm"
        d.mkdir(parents=True)
        with open(d / "1_counter_collection.csv", "w") as f:
            f.write("Kernel_Name,Counter_Name,Counter_Value\n")
            for k, v in rows:
                f.write('"%s",%s,%s\n' % (k, counter, v))

    # the copy moves 98,304 KiB each way; FETCH_SIZE reads half of it (its unit is 2 KiB here), WRITE_SIZE all of it
    write("fetch", "FETCH_SIZE", [(copy, 49152.0), (copy, 12.0), (head, 49200.0), (head, 49204.0)])
    write("write", "WRITE_SIZE", [(copy, 98304.0), (head, 27648.0), (head, 27648.0)])
    d = tmp_path / "kt" / "vm"
    d.mkdir(parents=True)
    with open(d / "1_kernel_stats.csv", "w") as f:
        f.write("Name,Calls,TotalDurationNs,AverageNs,Percentage,MinNs,MaxNs,StdDev\n")
        f.write('"%s",200,4700000,23500.0,99.0,23100,25000,100\n' % head)
    lines = ps.summarize(str(tmp_path))
    out = tmp_path / "summary.txt"
    out.write_text("# header\n" + "\n".join(lines) + "\n")
    got = ps.read_summary(str(out))
    assert got["kernel"] == "fb4::" + ps.HEADLINE
    assert float(got["read_factor"]) == 2.0 and float(got["write_factor"]) == 1.0
    assert int(got["traffic_bytes_per_launch"]) == int(round((49202.0 * 2.0 + 27648.0) * 1024))
    assert got["kernel_trace_average_ns"] == "23500.0"
    assert ps.read_summary(str(tmp_path / "missing.txt")) == {}


def test_pruning_study_is_consistent():
    # bench.py --pruning-study on a small sample: the union over a wavefront's blocks can only keep more dialects
    # alive than a block alone, all 32 are alive at the start, and at least the best one at the end
    import bench
    r = bench.pruning_study(n_wavefronts=4)["pruning_study"]
    a, u = r["alive_dialects_per_block_after_8_16_24_32_elements"], r["alive_in_wavefront_union_after_8_16_24_32_elements"]
    assert r["blocks"] == 256 and all(1.0 <= x <= y <= 32.0 for x, y in zip(a, u))
    assert a == sorted(a, reverse=True) and u == sorted(u, reverse=True)
    assert 0.0 < r["work_fraction_per_block_pruning"] <= r["work_fraction_wavefront_union"] <= 1.0
