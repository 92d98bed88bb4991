"""Checks on the test suite itself (CPU only): a module that defines the same top-level
test function twice silently loses the first one - Python rebinds the name and pytest
collects only the last definition."""
import ast
import glob
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def top_level_names(path):
    tree = ast.parse(open(path).read(), filename=path)
    return [(n.name, n.lineno) for n in tree.body
            if isinstance(n, (ast.FunctionDef, ast.AsyncFunctionDef, ast.ClassDef))]


def test_no_module_defines_a_name_twice():
    clashes = []
    for path in sorted(glob.glob(os.path.join(HERE, "*.py"))):
        seen = {}
        for name, line in top_level_names(path):
            if name in seen:
                clashes.append("%s: %s at lines %d and %d" % (os.path.basename(path), name, seen[name], line))
            seen[name] = line
    assert not clashes, "shadowed definitions:\n" + "\n".join(clashes)


def test_every_gpu_module_is_marked():
    # a GPU test without the marker would run (and fail) in the CPU-only pass
    for path in sorted(glob.glob(os.path.join(HERE, "test_gpu_*.py")) + glob.glob(os.path.join(HERE, "test_zz_*.py"))):
        text = open(path).read()
        assert "pytestmark = pytest.mark.gpu" in text or "@pytest.mark.gpu" in text, os.path.basename(path)
