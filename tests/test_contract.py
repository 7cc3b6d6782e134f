"""Host-side contract of the repository's entry points: one GPU only, no silent fallback, the product
never reaches into the oracle, and the oracle never into the product."""
import ast
import os
import shutil
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(args, cwd=ROOT, env=None):
    return subprocess.run([sys.executable] + args, cwd=cwd, env=env, capture_output=True, text=True, timeout=120)


def test_bench_refuses_more_than_one_gpu():
    r = run(["bench.py", "--gpus", "2", "--steps", "1", "--warmup", "0"])
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_package_without_its_library_fails_at_import(tmp_path):
    """A copy of the package with no built library beside it: importing it raises and names the build step;
    nothing falls back to a CPU path."""
    dst = tmp_path / "paper_2502_15443_amd"
    shutil.copytree(os.path.join(ROOT, "paper_2502_15443_amd"), dst,
                    ignore=shutil.ignore_patterns("*.so", "__pycache__", "csrc", "_build"))
    env = dict(os.environ, PYTHONPATH=str(tmp_path))
    r = run(["-c", "import paper_2502_15443_amd"], cwd=str(tmp_path), env=env)
    assert r.returncode != 0
    assert "ImportError" in r.stderr and "libdc_mi355x.so is missing" in r.stderr and "no fallback" in r.stderr


def imported_modules(path):
    tree = ast.parse(open(path).read(), path)
    names = set()
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            names.update(a.name.split(".")[0] for a in node.names)
        elif isinstance(node, ast.ImportFrom) and node.module and node.level == 0:
            names.add(node.module.split(".")[0])
    return names


def python_files(folder):
    for base, dirs, files in os.walk(os.path.join(ROOT, folder)):
        dirs[:] = [d for d in dirs if d != "__pycache__"]
        for f in files:
            if f.endswith(".py"):
                yield os.path.join(base, f)


def test_product_and_oracle_do_not_import_each_other():
    for f in python_files("paper_2502_15443_amd"):
        assert "oracle" not in imported_modules(f), f
    for f in python_files("oracle"):
        assert "paper_2502_15443_amd" not in imported_modules(f), f
    for f in python_files("synth"):
        mods = imported_modules(f)
        assert "oracle" not in mods and "paper_2502_15443_amd" not in mods, f


def test_native_sources_of_product_and_oracle_share_no_file():
    """The C oracle includes only the C library; the library's sources include nothing from the oracle."""
    def includes(path):
        return [ln.split()[1].strip('<>"') for ln in open(path) if ln.lstrip().startswith("#include")]
    csrc = os.path.join(ROOT, "paper_2502_15443_amd", "csrc")
    for f in os.listdir(csrc):
        for inc in includes(os.path.join(csrc, f)):
            assert "oracle" not in inc and "orc_" not in inc, (f, inc)
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".c", ".h")):
            for inc in includes(os.path.join(ROOT, "oracle", f)):
                assert inc in {"stdint.h", "stddef.h", "stdlib.h", "string.h", "stdio.h", "math.h", "limits.h"} \
                    or inc.startswith("dc_oracle"), (f, inc)


def test_the_bench_imports_the_oracle_only_in_its_cpu_baseline_leg():
    src = open(os.path.join(ROOT, "bench.py")).read()
    tree = ast.parse(src)
    lines = [n.lineno for n in ast.walk(tree)
             if (isinstance(n, ast.Import) and any(a.name.startswith("oracle") for a in n.names))
             or (isinstance(n, ast.ImportFrom) and (n.module or "").startswith("oracle"))]
    assert len(lines) == 1
    fn = [n for n in ast.walk(tree) if isinstance(n, ast.FunctionDef) and n.lineno <= lines[0] <= n.end_lineno]
    assert [f.name for f in fn] == ["cpu_baseline"], "the oracle import must sit inside the cpu_baseline leg"
    # and that leg is entered from one place, which --no-cpu switches off
    calls = [n for n in ast.walk(tree) if isinstance(n, ast.Call) and getattr(n.func, "id", "") == "cpu_baseline"]
    assert len(calls) == 1
    guard = src.splitlines()[max(0, calls[0].lineno - 3):calls[0].lineno]
    assert any("no_cpu" in ln for ln in guard)


def test_every_bench_flag_the_readme_names_exists():
    """README.md tells a user which flags time which workload; each of them is one bench.py accepts."""
    import re
    readme = open(os.path.join(ROOT, "README.md")).read()
    named = set(re.findall(r"`(--[a-z][a-z0-9-]*)", readme))
    assert {"--workload", "--mix-sweep", "--wg-trace", "--alpha-sweep", "--pair-stats"} <= named
    helptext = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"], capture_output=True, text=True,
                              timeout=120).stdout
    missing = sorted(f for f in named if f not in helptext)
    assert not missing, missing
