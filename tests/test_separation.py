"""The product path and the oracle share nothing: checked on the sources (no GPU needed)."""
import ast
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _imports(path):
    tree = ast.parse(open(path).read(), path)
    names = set()
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            names.update(a.name for a in node.names)
        elif isinstance(node, ast.ImportFrom) and node.module:
            names.add(("." * node.level) + node.module)
    return names


def _py_files(folder):
    for base, _, files in os.walk(os.path.join(ROOT, folder)):
        if "__pycache__" in base:
            continue
        for f in files:
            if f.endswith(".py"):
                yield os.path.join(base, f)


def test_the_package_never_imports_the_oracle_or_the_tests():
    for path in _py_files("paper_2604_06483_amd"):
        for name in _imports(path):
            top = name.lstrip(".").split(".")[0]
            assert top not in ("oracle", "tests"), (path, name)


def test_the_oracle_imports_nothing_of_the_product():
    for path in _py_files("oracle"):
        for name in _imports(path):
            top = name.lstrip(".").split(".")[0]
            assert top not in ("paper_2604_06483_amd", "torch", "ctypes"), (path, name)


def test_device_sources_do_not_mention_the_oracle():
    csrc = os.path.join(ROOT, "paper_2604_06483_amd", "csrc")
    for f in sorted(os.listdir(csrc)) + ["../../include/ll.h"]:
        text = open(os.path.join(csrc, f)).read()
        assert not re.search(r"\boracle\b", text, re.I), f


_WORK = re.compile(r"""(?<![A-Za-z0-9])_work(/|["'])""")     # the folder as a path piece, not "ll_workspace_bytes"


def test_nothing_committed_reaches_into_the_working_folder():
    for folder in ("paper_2604_06483_amd", "oracle", "tests"):
        for path in _py_files(folder):
            if os.path.abspath(path) == os.path.abspath(__file__):
                continue
            assert not _WORK.search(open(path).read()), path
    for f in ("bench.py", "__graft_entry__.py"):
        assert not _WORK.search(open(os.path.join(ROOT, f)).read()), f
