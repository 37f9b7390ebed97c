"""Host logic of the measurement side (no GPU): the profile condenser on small synthetic CSV files in
rocprofv3's column layout, and bench.py's reader of the committed HBM-traffic summary."""
import io
import os
import sys
from contextlib import redirect_stdout

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
import profsum  # noqa: E402


def run(fn, *args):
    buf = io.StringIO()
    with redirect_stdout(buf):
        fn(*args)
    return buf.getvalue()


def test_kernel_names_are_shortened():
    assert profsum.short("void itq3s::gemv_kernel<1, 3, true, 0, false, false, 1>(itq3s::GemvArgs)") == "gemv_kernel<1, 3, true, 0, false, false, 1>"
    assert profsum.short("_ZN5itq3s11gemm_kernelENS_8GemmArgsEiii") == "gemm_kernel"
    assert profsum.ours("__amd_rocclr_copyBuffer") and not profsum.ours("at::native::vectorized_elementwise_kernel")


def test_pmc_summary_scales_by_the_calibration_copy(tmp_path):
    p = tmp_path / "c.csv"
    rows = ["Kernel_Name,Grid_Size,Counter_Name,Counter_Value"]
    rows += ["__amd_rocclr_copyBuffer,131072,FETCH_SIZE,524288.0"] * 3  # the counter shows half of the 1 GiB read
    rows += ['"void itq3s::gemv_kernel<1, 2, false, 0, false, false, 1>(itq3s::GemvArgs)",131072,FETCH_SIZE,%.1f' % v for v in (29000.0, 29100.0)]
    rows += ["some_other_kernel,64,FETCH_SIZE,1.0"]
    p.write_text("\n".join(rows) + "\n")
    out = run(profsum.pmc, str(p), 1048576.0)
    assert "factor 2.0000" in out
    line = [l for l in out.splitlines() if l.startswith("gemv_kernel")][0].split()
    assert line[-3:] == ["2", "29050.0", "58100.0"]
    assert "some_other_kernel" not in out


def test_gaps_separate_in_replay_dispatches_from_isolated_ones(tmp_path):
    p = tmp_path / "t.csv"
    name = '"void itq3s::gemv_kernel<1, 2, false, 0, false, false, 1>(itq3s::GemvArgs)"'
    rows = ["Kernel_Name,Grid_Size,Start_Timestamp,End_Timestamp"]
    t = 0
    for i in range(12):  # back to back, 100 ns apart: inside a replayed step
        rows.append("%s,131072,%d,%d" % (name, t, t + 7000))
        t += 7100
    t += 1_000_000
    rows.append("%s,131072,%d,%d" % (name, t, t + 9000))  # on its own
    p.write_text("\n".join(rows) + "\n")
    out = run(profsum.gaps, str(p))
    replay = [l for l in out.splitlines() if l.startswith("gemv_kernel")][0].split()
    assert replay[-3:] == ["11", "7000.0", "100.0"]
    assert "launched on its own" in out and "2 calls avg 8000.0 ns" in out  # the first dispatch of the run and the late one


def test_bench_reads_the_committed_traffic_summary():
    t = bench.measured_traffic("llama70b_decode")
    assert t is not None and t["source"] == os.path.join("profiles", "gemv_llama70b_decode.hbm_traffic.txt")
    # 320 launches of 83.68 MB algorithmic: the measured mean lies within a few per cent above it
    alg = 83681280
    assert alg <= t["bytes_per_launch"] <= 1.05 * alg
    assert t["write_bytes"] == (2 * 32 + 40 + 224) * 1024 // 4
    assert bench.measured_traffic("no-such-workload") is None


def test_algorithmic_bytes():
    assert bench.packed_bytes(2048, 2048) == 128 * 8 * 1600
    assert bench.packed_bytes(17, 256) == 2 * 1600  # storage pads to 16 rows
    assert bench.alg_bytes(8192, 8192, 1) == 512 * 32 * 1600 + 8192 * 2 + 8192 * 4
