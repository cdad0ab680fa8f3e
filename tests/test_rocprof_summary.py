"""The profiler-summary helper on small hand-made inputs (no GPU, no profiler): the calibration by
the copy kernel, the per-launch and per-step traffic sums, and the kernel-trace table."""
import sqlite3

from paper_2605_11186_amd import rocprof_summary as rs


def _csv(path, rows):
    path.write_text("Kernel_Name,Counter_Name,Counter_Value\n" +
                    "".join(f'"{k}",X,{v}\n' for k, v in rows))


def test_traffic_is_scaled_by_the_copy_kernel_and_summed_per_step(tmp_path):
    # the copy of 1 GiB reads 524288 counter units and writes 1048576: scales 2.0 and 1.0 to KiB
    gemm = "void (anonymous namespace)::cats_gemm_skinny_bf16<2, 8, 1, 2, true>(GemmArgs)"
    acc = "(anonymous namespace)::cats_accept(int const*)"
    pack = "(anonymous namespace)::cats_pack_matrix_kernel(unsigned short const*)"
    fetch = [("__amd_rocclr_copyBuffer", 524288.0)] + [(gemm, 50000.0)] * 6 + [(acc, 0.0)] * 2 + [(pack, 1000.0)]
    write = [("__amd_rocclr_copyBuffer", 1048576.0)] + [(gemm, 10000.0)] * 6 + [(acc, 1.0)] * 2 + [(pack, 1000.0)]
    _csv(tmp_path / "f.csv", fetch)
    _csv(tmp_path / "w.csv", write)
    text = rs.traffic(str(tmp_path / "f.csv"), str(tmp_path / "w.csv"))
    per_launch = (50000.0 * 2.0 + 10000.0 * 1.0) * 1024
    assert f"gemm_traffic_bytes_per_launch: {int(per_launch)}" in text
    # two steps (two accept dispatches): three GEMM launches and one accept per step; the one-time
    # weight re-tiling is not part of a step
    assert f"step_traffic_bytes: {int(3 * per_launch + 1.0 * 1024)}" in text
    assert "fetch x2.0000, write x1.0000" in text


def test_kernel_trace_table(tmp_path):
    db = tmp_path / "t.db"
    con = sqlite3.connect(db)
    con.execute("create table kernels (name text, start integer, end integer)")
    rows = [("void (anonymous namespace)::cats_gemm_skinny_bf16<2, 8, 1, 2, true>(GemmArgs)", 0, 20000),
            ("void (anonymous namespace)::cats_gemm_skinny_bf16<2, 8, 1, 2, true>(GemmArgs)", 30000, 60000),
            ("(anonymous namespace)::cats_accept(int const*)", 70000, 75000)]
    con.executemany("insert into kernels values (?, ?, ?)", rows)
    con.commit()
    con.close()
    text = rs.kernel_trace(str(db))
    line = next(l for l in text.splitlines() if "cats_gemm" in l)
    assert line.split()[-6:] == ["2", "0.050", "25.00", "20.00", "30.00", "90.91"]
    assert "1 verify steps in the trace" in text and "0.055 ms per step" in text
