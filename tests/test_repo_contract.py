"""Structure checks that need no GPU: the benchmark's command-line contract, the byte counts its
rooflines are priced with, and the separation between the product path and the CPU oracle."""
import ast
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _imported_modules(path):
    tree = ast.parse(open(path).read())
    found = set()
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            found.update(alias.name for alias in node.names)
        elif isinstance(node, ast.ImportFrom):
            found.add(("." * node.level) + (node.module or ""))
    return found


def test_bench_refuses_more_than_one_gpu():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, cwd=ROOT)
    assert run.returncode != 0
    assert "one GPU" in run.stderr
    assert run.stdout.strip() == ""          # no benchmark line on the refusal path


def test_algorithmic_bytes_of_the_bandwidth_bound_kernels():
    sys.path.insert(0, ROOT)
    import bench
    # quantizer, per element: bf16 in + half a byte of codes + one mask bit; per row: one fp32 scale
    rows, cols = 16384, 2048
    assert bench.algorithmic_bytes_quantize(rows, cols) == rows * (cols * 2 + cols // 2 + cols // 8 + 4)
    # masked inverse transform: bf16 gradient in, one mask bit, bf16 out
    assert bench.algorithmic_bytes_backward(rows, cols) == rows * (cols * 2 + cols // 8 + cols * 2)


def test_traffic_constants_of_the_benchmark_are_those_of_the_committed_profile():
    """bench.py reports measured HBM-side traffic from constants; they must be the table of the
    rocprofv3 summary under profiles/, so that a re-measurement updates one place and fails here
    until the other follows."""
    import re
    sys.path.insert(0, ROOT)
    import bench
    text = open(os.path.join(ROOT, "profiles", "bench_step_mlp_up_1p6b_hbm_traffic.md")).read()
    table = {}
    for key, read, write in re.findall(r"^\| `(\w+)` \| ([0-9.]+) \| ([0-9.]+) \|$", text, flags=re.M):
        table[key] = (float(read), float(write))
    assert set(table) == set(bench.MEASURED_TRAFFIC_MIB) == set(bench.STEP_KERNELS)
    for key, pair in bench.MEASURED_TRAFFIC_MIB.items():
        assert table[key] == pair, key


def test_the_product_never_imports_the_oracle_and_the_oracle_never_imports_the_product():
    package = os.path.join(ROOT, "paper_2502_05003_amd")
    for name in os.listdir(package):
        if name.endswith(".py"):
            mods = _imported_modules(os.path.join(package, name))
            assert not any(m.lstrip(".").split(".")[0] == "oracle" for m in mods), name
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith(".py"):
            mods = _imported_modules(os.path.join(ROOT, "oracle", name))
            assert not any("paper_2502_05003_amd" in m or m == "torch" for m in mods), name
    # the HIP sources and the oracle's C file share no header
    csrc = os.path.join(package, "csrc")
    for name in os.listdir(csrc):
        text = open(os.path.join(csrc, name)).read()
        assert "oracle" not in text, name
    oracle_c = open(os.path.join(ROOT, "oracle", "quest_oracle.c")).read()
    assert "quest.h" not in oracle_c and "csrc" not in oracle_c


def test_bench_reaches_the_oracle_only_in_its_cpu_baseline_leg():
    tree = ast.parse(open(os.path.join(ROOT, "bench.py")).read())
    for node in tree.body:
        if isinstance(node, ast.FunctionDef):
            uses = any(isinstance(n, ast.ImportFrom) and (n.module or "").startswith("oracle")
                       for n in ast.walk(node))
            assert uses == (node.name == "cpu_baseline"), node.name
        else:
            assert not (isinstance(node, (ast.Import, ast.ImportFrom)) and "oracle" in ast.dump(node))


def test_binding_has_no_fallback_when_the_library_is_missing(tmp_path, monkeypatch):
    import pytest

    from paper_2502_05003_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libquest.so"))
    with pytest.raises(FileNotFoundError):
        binding.quest_alpha_star(4)
