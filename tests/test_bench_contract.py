"""The benchmark's command-line contract, as far as it can be checked without a GPU, and its JSON line on one."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    """This build runs on one GPU; asking for more must end with a message that says so, not with a number."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_product_path_does_not_import_the_oracle():
    """The oracle is test infrastructure: the package never imports it, and bench.py only in its CPU-baseline leg."""
    pkg = os.path.join(ROOT, "paper_2512_17077_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "hcsa_oracle" not in text, f
    bench = open(os.path.join(ROOT, "bench.py")).read()
    lo, hi = bench.index("def cpu_baseline"), bench.index("def gqa_union_bytes")
    assert lo < hi < bench.index("def main")
    at = [i for i in range(len(bench)) if bench.startswith("import oracle", i)]
    assert at and all(lo < i < hi for i in at)       # the baseline leg and the child process it starts, nowhere else


def test_ceilings_program_compiles_for_gfx950(tmp_path):
    """ceilings.py builds ceilings.hip on the GPU machine at run time; keep it compiling (no GPU needed for that)."""
    import shutil
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not installed")
    out = tmp_path / "ceilings.o"
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                        "-Wno-inline-asm", "-c", os.path.join(ROOT, "ceilings.hip"), "-o", str(out)],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    assert out.stat().st_size > 0


def test_traffic_tool_reads_a_counter_run(tmp_path):
    """bench_traffic.read_run on a hand-made counter file: the copy probe is found, only launches after it count,
    and a kernel's figure is the mean of its last three launches."""
    sys.path.insert(0, ROOT)
    import bench_traffic
    header = ("Correlation_Id,Dispatch_Id,Agent_Id,Queue_Id,Process_Id,Thread_Id,Grid_Size,Kernel_Id,Kernel_Name,Workgroup_Size,"
              "LDS_Block_Size,Scratch_Size,VGPR_Count,Accum_VGPR_Count,SGPR_Count,Counter_Name,Counter_Value,Start_Timestamp,"
              "End_Timestamp")
    add = "void at::native::vectorized_elementwise_kernel<4, at::native::CUDAFunctorOnSelf_add<int>, std::array<char*, 2ul> >(int)"
    ker = "void dllm::score_kernel<2, 128, 1>(char const*, char const*)"
    rows = [(1, ker, 1024, 256, 999.0),            # set-up launch, before the probe: ignored
            (2, add, 1 << 26, 256, 524288.0),
            (3, ker, 1024, 256, 500.0),            # warm-up
            (4, ker, 1024, 256, 100.0), (5, ker, 1024, 256, 110.0), (6, ker, 1024, 256, 120.0),
            (7, "void dllm::topk_reg_kernel<8, 512>(float const*)", 2048, 512, 7.0)]
    d = tmp_path / "FETCH_SIZE" / "select_reuse"
    d.mkdir(parents=True)
    with open(d / "p_counter_collection.csv", "w") as f:
        f.write(header + "\n")
        for i, name, grid, wg, val in rows:
            f.write(f'{i},{i},"Agent 1",1,1,1,{grid},1,"{name}",{wg},0,0,8,0,32,"FETCH_SIZE",{val},0,1\n')
    probe, per = bench_traffic.read_run(str(d), "FETCH_SIZE")
    assert probe == 524288.0
    assert per["score_kernel<2, 128, 1>"] == ("4 x 256", 110.0)
    assert per["topk_reg_kernel<8, 512>"] == ("4 x 512", 7.0)


def test_traffic_file_and_summary_agree_and_cover_the_roofline_kernels():
    """bench.py takes roofline.traffic from profiles/hbm_traffic.json; the summary beside it (the table the
    reader sees) must state the same figures, and every kernel a roofline names must be in the file."""
    sys.path.insert(0, ROOT)
    import bench
    data = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic.json")))
    md = open(os.path.join(ROOT, "profiles", "hbm_traffic_pmc.md")).read()
    rows = [[c.strip() for c in line.split("|")[1:-1]] for line in md.splitlines() if line.startswith("| ") and "---" not in line][1:]
    seen = set()
    for call, kernel, fetch, write, read_mb, write_mb, _ in rows:
        name = kernel[:kernel.rindex("(")].strip()
        t = data["calls"][call][name]
        assert abs(float(fetch) - t["fetch_kib"]) <= 0.5 and abs(float(write) - t["write_kib"]) <= 0.5
        assert abs(float(read_mb) - t["read_bytes"] / 1e6) <= 0.05 and abs(float(write_mb) - t["write_bytes"] / 1e6) <= 0.05
        # the scaling: KiB x 1024 x (known probe bytes / probe counter)
        assert abs(t["read_bytes"] - t["fetch_kib"] * 1024 * data["factor"]["FETCH_SIZE"]) <= 1024
        seen.add((call, name))
    assert len(seen) == sum(len(v) for v in data["calls"].values())
    traffic = bench.load_traffic()
    assert traffic == data["calls"]
    for call, kernel in (("dense_refresh", "attend_dense_bf16_kernel"), ("attend_reuse", "attend_sparse_multi_bf16_kernel"),
                         ("select_reuse", "score_kernel"), ("select_mixed", "select_fused_kernel")):
        total = bench.traffic_of(traffic, call, kernel)
        assert total is not None and total > 0
    # the figures are measured traffic of these workloads: within a few percent of the algorithmic bytes
    from paper_2512_17077_amd import synth
    w3 = synth.config(3)
    assert 0.95 < bench.traffic_of(traffic, "attend_reuse", "attend_sparse_multi") / w3.attend_sparse_bytes() < 1.05
    assert 0.95 < bench.traffic_of(traffic, "select_reuse", "score_kernel") / w3.select_bytes() < 1.05
    assert 0.98 < bench.traffic_of(traffic, "select_mixed", "select_fused_kernel") / synth.config(5).select_bytes() < 1.02


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_the_contract_keys():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "5", "--warmup", "2", "--no-cpu-baseline"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 5 and out["warmup"] == 2 and out["vs_baseline"] is None
    assert "workload" in out["config"]
    roof = out["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-12
    assert 0.0 < out["roofline_reuse"]["frac"] < 1.0 and 0.0 < out["roofline_select"]["frac"] < 1.0
    assert roof["traffic"] is not None and out["roofline_reuse"]["traffic"] is not None
    assert set(out["small_config_call_us"]) == {"select_c1", "attend_c1", "select_c2", "attend_c2"}
    assert all(v > 0 for v in out["reuse_select_options_gbps"].values())
    assert out["call_ms_mean_min_median_warm"] is not None and len(out["call_ms_mean_min_median"]["attend_reuse"]) == 3
    mixed = out["mixed_attend"]
    assert mixed["reuse_part_bytes_gqa_union"] < mixed["reuse_part_bytes_per_head"]
    assert mixed["refresh_part_read_bytes_counter"] is not None
    assert out["config"]["step"] == ["select_reuse", "attend_reuse", "dense_refresh", "select_mixed", "attend_mixed"]
