"""Host-side checks of the repository's contract with its harness: bench.py refuses more than one GPU with a
message, the entry module offers build() and smoke(), and nothing on the product path reaches into the oracle (the
oracle is test infrastructure: only tests, smoke() and the bench's CPU baseline may import it)."""
import ast
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_several_gpus_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""          # no JSON line that a driver could mistake for a measurement


def test_entry_module_offers_build_and_smoke():
    sys.path.insert(0, ROOT)
    import __graft_entry__ as entry
    assert callable(entry.build) and callable(entry.smoke)


def _imports(path):
    tree = ast.parse(open(path).read())
    names = set()
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            names.update(a.name.split(".")[0] for a in node.names)
        elif isinstance(node, ast.ImportFrom) and node.module:
            names.add(node.module.split(".")[0])
    return names


def test_the_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2503_03588_amd")
    for fn in os.listdir(pkg):
        if fn.endswith(".py"):
            assert "oracle" not in _imports(os.path.join(pkg, fn)), fn


def test_the_oracle_never_imports_the_package():
    orc = os.path.join(ROOT, "oracle")
    for fn in os.listdir(orc):
        if fn.endswith(".py"):
            assert "paper_2503_03588_amd" not in _imports(os.path.join(orc, fn)), fn


def test_the_binding_fails_loudly_without_the_library(tmp_path):
    code = ("import os, sys; sys.path.insert(0, %r); os.environ['POWATTN_LIB'] = %r\n"
            "from paper_2503_03588_amd import binding as pa\n"
            "try:\n    pa.lib()\nexcept RuntimeError as e:\n    print('raised:', e); sys.exit(0)\nsys.exit(1)\n"
            % (ROOT, str(tmp_path / "missing.so")))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "no fallback" in r.stdout
