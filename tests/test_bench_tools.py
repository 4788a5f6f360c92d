"""The reducers bench.py offers for profiler output (`--stats-from`, `--counters-from`): plain text in, tables out.
No GPU involved."""
import importlib.util
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


TRACE = '''"Kind","Agent_Id","Queue_Id","Kernel_Name","Start_Timestamp","End_Timestamp","Grid_Size_X"
"KERNEL_DISPATCH",1,1,"void eclip::conv_gemm_kernel<eclip::bf16_t, 128>(eclip::GemmDev)",1000,11000,4096
"KERNEL_DISPATCH",1,1,"eclip::(anonymous namespace)::probe_kernel(unsigned int*)",12000,13000,512
"KERNEL_DISPATCH",1,1,"void eclip::conv_gemm_kernel<eclip::bf16_t, 128>(eclip::GemmDev)",14000,24000,4096
"KERNEL_DISPATCH",1,1,"void eclip::conv_gemm_kernel<eclip::bf16_t, 128>(eclip::GemmDev)",24000,36000,4096
"KERNEL_DISPATCH",1,1,"void eclip::conv_gemm_kernel<eclip::bf16_t, 128>(eclip::GemmDev)",36000,5036000,4096
"KERNEL_DISPATCH",1,1,"void eclip::(anonymous namespace)::row_kernel<eclip::bf16_t, 8, 4, 64, false>(eclip::RowArgs)",5036000,5041000,96
"KERNEL_DISPATCH",1,1,"eclip::(anonymous namespace)::probe_kernel(unsigned int*)",5042000,5043000,512
'''


def test_stats_from_pools_instantiations_drops_stamps_of_a_dry_queue_and_finds_the_marked_pass(tmp_path, capsys):
    p = tmp_path / "kt.csv"
    p.write_text(TRACE)
    _bench().stats_from(str(p))
    out = capsys.readouterr().out
    whole, marked = out.split("# per-layer timing pass")
    # whole process: 4 dispatches of the GEMM kernel, one of them (5 ms for a 10 us kernel) left out of the mean
    assert "probe_kernel" not in whole
    row = next(l for l in whole.splitlines() if l.startswith("conv_gemm_kernel")).split()
    assert row[1:3] == ["4", "1"]
    assert abs(float(row[3]) - (10 + 10 + 12) / 3) < 6e-3          # printed with two decimals
    # between the two probe_kernel marks: 3 GEMM dispatches (one outlier) and the row kernel
    rows = {l.split()[0]: l.split() for l in marked.splitlines() if l and not l.startswith(("#", "kernel", " ("))}
    assert rows["conv_gemm_kernel"][1:3] == ["3", "1"]
    assert abs(float(rows["conv_gemm_kernel"][3]) - 11.0) < 6e-3
    assert rows["row_kernel"][1] == "1" and abs(float(rows["row_kernel"][3]) - 5.0) < 6e-3
    assert "probe_kernel" not in rows


COUNTERS = '''"Dispatch_Id","Kernel_Name","Counter_Name","Counter_Value"
1,"void eclip::conv_gemm_kernel<eclip::bf16_t, 256, 256>(eclip::GemmDev)","SQ_INSTS_MFMA",100
2,"void eclip::conv_gemm_kernel<eclip::bf16_t, 256, 256>(eclip::GemmDev)","SQ_INSTS_MFMA",300
3,"void eclip::conv_gemm_kernel<eclip::bf16_t, 96, 64>(eclip::GemmDev)","SQ_INSTS_MFMA",50
1,"void eclip::conv_gemm_kernel<eclip::bf16_t, 256, 256>(eclip::GemmDev)","SQ_INSTS_VALU",500
'''


def test_counters_from_keeps_tile_shapes_apart_and_averages_per_dispatch(tmp_path, capsys):
    p = tmp_path / "cc.csv"
    p.write_text(COUNTERS)
    _bench().counters_from([str(p)])
    lines = capsys.readouterr().out.splitlines()
    i = lines.index("conv_gemm_kernel<bf16_t, 256, 256>")
    assert "SQ_INSTS_MFMA" in lines[i + 1] and "dispatches      2" in lines[i + 1] and lines[i + 1].rstrip().endswith("mean 200")
    assert "SQ_INSTS_VALU" in lines[i + 2] and lines[i + 2].rstrip().endswith("mean 500")
    j = lines.index("conv_gemm_kernel<bf16_t, 96, 64>")
    assert lines[j + 1].rstrip().endswith("mean 50")
