"""Host-side checks of how the pieces may depend on each other: the product path never touches the
oracle, fails loudly without its library, and the benchmark refuses more than one GPU."""
import os
import re
import subprocess
import sys

import pytest

import paper_2507_02957_amd as csat

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _sources(folder, exts):
    for base, _, files in os.walk(os.path.join(ROOT, folder)):
        for f in files:
            if f.endswith(exts):
                yield os.path.join(base, f)


def test_product_path_does_not_use_the_oracle_or_a_cpu_fallback():
    for path in _sources("paper_2507_02957_amd", (".py", ".h", ".hip")):
        text = open(path).read()
        assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f"{path} imports the oracle"
        assert "csat_oracle" not in text, f"{path} names the oracle module"
    # the oracle and the input generators do not load the library either
    for path in list(_sources("oracle", (".py",))) + [os.path.join(ROOT, "csat_inputs.py")]:
        text = open(path).read()
        assert "paper_2507_02957_amd" not in text and "libcsat" not in text, f"{path} refers to the HIP path"
    # the input generators hold none of the method's arithmetic: no softmax, no thresholding, no ISTA step
    gen = open(os.path.join(ROOT, "csat_inputs.py")).read()
    gen = re.sub(r'"""(?:.|\n)*?"""', "", gen)          # code only, not the docstrings
    for word in ("softmax", "soft_threshold", "ista(", "np.exp("):
        assert word not in gen, f"csat_inputs.py contains {word!r}"


def test_missing_library_raises(monkeypatch):
    monkeypatch.setattr(csat, "_lib", None)
    monkeypatch.setattr(csat, "LIB_PATH", os.path.join(ROOT, "paper_2507_02957_amd", "no_such_library.so"))
    with pytest.raises(FileNotFoundError):
        csat.load_library()


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def test_every_header_declaration_has_a_binding():
    header = open(os.path.join(ROOT, "include", "csat.h")).read()
    declared = set(re.findall(r"\b(csat_[a-z0-9_]+)\s*\(", header))
    assert declared == set(csat.EXPORTS), declared ^ set(csat.EXPORTS)
    for name in declared - {"csat_create", "csat_destroy", "csat_status_string"}:
        assert hasattr(csat, name), f"no Python wrapper for {name}"
