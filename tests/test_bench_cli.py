"""CPU-only checks of bench.py's command line: what it must refuse, and that it never falls back to a CPU path."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          cwd=ROOT, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    for n in ("2", "8"):
        p = run("--gpus", n)
        assert p.returncode != 0
        assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_without_a_gpu_there_is_no_result_line():
    import torch
    if torch.cuda.is_available():
        return                      # on a GPU machine the real benchmark would start: covered by the GPU tiers
    p = run("--steps", "1", "--warmup", "0")
    assert p.returncode != 0
    assert "needs a GPU" in p.stderr and p.stdout.strip() == ""


def test_unknown_workload_and_mode_are_refused():
    assert run("--mode", "everything").returncode != 0
    import torch
    if not torch.cuda.is_available():
        return
    assert run("--workload", "nonsense", "--steps", "1").returncode != 0


def test_product_and_oracle_share_nothing():
    """The package never names the oracle, the oracle never names the package, and bench.py reaches the oracle
    only inside its cpu_baseline leg; the one shared module, synth.py, holds no arithmetic of the method."""
    import ast
    import re
    pkg = os.path.join(ROOT, "paper_2412_21124_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"\boracle\b", text.replace("CPU oracle", "").replace("the oracle", "")) or f == "synth.py", f
                assert "import oracle" not in text and "from oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2412_21124_amd" not in text and "normtest.h" not in text and "libnormtest.so" not in text, f
    assert "oracle" not in open(os.path.join(ROOT, "include", "normtest.h")).read()
    tree = ast.parse(open(os.path.join(ROOT, "bench.py")).read())
    for node in tree.body:                                   # module level: no oracle import
        if isinstance(node, (ast.Import, ast.ImportFrom)):
            names = [a.name for a in node.names] + [getattr(node, "module", "") or ""]
            assert not any(n.split(".")[0] == "oracle" for n in names)
    users = [fn.name for fn in ast.walk(tree) if isinstance(fn, ast.FunctionDef)
             and any(isinstance(n, ast.Import) and any(a.name == "oracle" for a in n.names) for n in ast.walk(fn))]
    assert users == ["cpu_baseline"]
    synth = open(os.path.join(pkg, "synth.py")).read()
    for word in ("beta1 *", "sqrt(v", "weight_decay *", "eta *", "ceil("):
        assert word not in synth, word


def test_traffic_is_quoted_from_the_tracked_profile_or_absent(tmp_path):
    """roofline.traffic is never a constant in bench.py: it is the figure the tracked counter profile holds for the
    kernel source as it stands, and null once the source differs from the profiled one."""
    import json
    sys.path.insert(0, ROOT)
    import bench
    src = tmp_path / "kernel.hip"
    src.write_text("// kernel v1\n")
    prof = tmp_path / "traffic.json"
    prof.write_text(json.dumps({"kernel_source_sha256": bench.kernel_source_sha256(str(src)),
                                "entries": {"flat_1p5b/full": {"hbm_bytes_per_step": 60010000000.0}}}))
    assert bench.traffic_from_profile("flat_1p5b", "full", str(prof), str(src)) == 60010000000.0
    assert bench.traffic_from_profile("flat_1p5b", "stats", str(prof), str(src)) is None    # not profiled
    src.write_text("// kernel v2\n")                                                         # the kernel changed
    assert bench.traffic_from_profile("flat_1p5b", "full", str(prof), str(src)) is None
    assert bench.traffic_from_profile("flat_1p5b", "full", str(tmp_path / "missing.json"), str(src)) is None
    # no byte count is written into bench.py itself
    text = open(os.path.join(ROOT, "bench.py")).read()
    assert "6.0010e10" not in text and "60010000000" not in text and "MEASURED_TRAFFIC" not in text


def test_tracked_traffic_profile_is_well_formed():
    """If profiles/traffic.json is there, the value bench.py would print is the file's own, for every entry."""
    import json
    sys.path.insert(0, ROOT)
    import bench
    if not os.path.exists(bench.TRAFFIC_FILE):
        return
    prof = json.load(open(bench.TRAFFIC_FILE))
    assert set(prof) >= {"kernel_source_sha256", "entries", "calibration"}
    current = prof["kernel_source_sha256"] == bench.kernel_source_sha256()
    for key, entry in prof["entries"].items():
        wl, mode = key.split("/")
        got = bench.traffic_from_profile(wl, mode)
        assert got == (float(entry["hbm_bytes_per_step"]) if current else None), key
        assert entry["hbm_bytes_per_step"] == entry["fetch_bytes"] + entry["write_bytes"]


def test_row_sweep_workloads_are_parsed_on_the_host():
    """rows:J:d is J bf16 rows with the headline's recipe, rows:J:d:f32 the same with fp32 rows; anything else in the
    fourth field is refused."""
    import pytest
    import torch
    sys.path.insert(0, ROOT)
    import bench
    wl = bench.make_workload("rows:12:5000", "cpu", 1.0)
    assert (wl.name, wl.J, wl.d, wl.grads.dtype) == ("rows_J12", 12, 5000, torch.bfloat16)
    wf = bench.make_workload("rows:12:5000:f32", "cpu", 1.0)
    assert (wf.name, wf.J, wf.d, wf.grads.dtype) == ("rows_J12_f32", 12, 5000, torch.float32)
    assert wf.hyper == wl.hyper
    for bad in ("rows:12:5000:f16", "rows:12", "rows:12:5000:f32:x"):
        with pytest.raises(SystemExit):
            bench.make_workload(bad, "cpu", 1.0)
