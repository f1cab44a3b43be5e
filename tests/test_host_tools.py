"""Host-side tools that need no GPU: bench.py's refusal of more than one GPU, and the summariser of
rocprofv3 CSV output."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_refuses_a_multi_rank_launch():
    env = dict(os.environ, WORLD_SIZE="2", RANK="0")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode == 2 and "one GPU" in r.stderr


def test_profile_summaries(tmp_path):
    from paper_2310_00837_amd import prof
    trace = tmp_path / "x_kernel_trace.csv"
    trace.write_text(
        '"Kind","Kernel_Name","Start_Timestamp","End_Timestamp","Workgroup_Size_X","Grid_Size_X"\n'
        '"KERNEL_DISPATCH","void helios::(anonymous namespace)::gather_rows_kernel<32, 1, 1>(helios::(anonymous namespace)::GatherArgs)",1000,5000,256,524288\n'
        '"KERNEL_DISPATCH","void helios::(anonymous namespace)::gather_rows_kernel<32, 1, 1>(helios::(anonymous namespace)::GatherArgs)",9000,15000,256,1048576\n'
        '"KERNEL_DISPATCH","void helios::(anonymous namespace)::gather_rows_kernel<32, 1, 4>(helios::(anonymous namespace)::GatherArgs)",20000,110000,256,11264\n'
        '"KERNEL_DISPATCH","(anonymous namespace)::missq_submit_kernel((anonymous namespace)::SubmitArgs)",0,7000,256,4096\n'
        '"KERNEL_DISPATCH","void at::native::some_torch_kernel()",0,1000000,256,256\n')
    lines = prof.trace(str(tmp_path), "x").splitlines()
    assert len(lines) == 4                                     # header + three kernels of this library
    hbm = [ln for ln in lines if ln.startswith("gather_rows_kernel<32, 1, 1>")][0].split()
    assert hbm[-6:-1] == ["2048-4096", "2", "5.00", "4.00", "6.00"]  # workgroups (range), calls, avg, min, max (us)
    assert any(ln.startswith("missq_submit_kernel") and " 16 " in ln for ln in lines)
    # one line per kernel and grid size: grids seen fewer than five times share a line
    rows = ['"KERNEL_DISPATCH","void helios::(anonymous namespace)::batch_compact_kernel(helios::CompactGang)",%d,%d,256,%d\n'
            % (100 * k, 100 * k + (40 if k < 6 else 90), 256 * (51 if k < 6 else 204 if k < 12 else 7 + k)) for k in range(14)]
    trace.write_text('"Kind","Kernel_Name","Start_Timestamp","End_Timestamp","Workgroup_Size_X","Grid_Size_X"\n' + "".join(rows))
    by_grid = [ln.split() for ln in prof.trace(str(tmp_path), "x", by_grid=True).splitlines()[1:]]
    assert [ln[-6:-4] for ln in by_grid] == [["51", "6"], ["204", "6"], ["19-20", "2"]]
    assert by_grid[2][1:3] == ["(other", "grids)"] and by_grid[0][-4] == "0.04" and by_grid[1][-4] == "0.09"
    assert len(prof.trace(str(tmp_path), "x").splitlines()) == 2
    pmc = tmp_path / "x_counter_collection.csv"
    pmc.write_text(
        '"Kernel_Name","Counter_Name","Counter_Value","Grid_Size","Workgroup_Size"\n'
        '"helios::(anonymous namespace)::calibration_copy_kernel(a)","FETCH_SIZE",524288.0,2097152,256\n'
        '"helios::(anonymous namespace)::calibration_copy_kernel(a)","FETCH_SIZE",524290.0,2097152,256\n'
        '"helios::(anonymous namespace)::calibration_copy_kernel(a)","WRITE_SIZE",7.0,2097152,256\n')
    out = prof.pmc(str(tmp_path), "x", "FETCH_SIZE").splitlines()
    assert len(out) == 2 and out[1].split()[-3:] == ["8192", "2", "524289.0"]
