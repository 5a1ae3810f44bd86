"""The product path must not reach into the oracle, the working folder or a CPU fallback."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2605_26632_amd")


def _sources():
    for d, _, files in os.walk(PKG):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                yield os.path.join(d, f)
    yield os.path.join(ROOT, "include", "rtlynx.h")


def test_package_never_references_oracle_or_work_folder():
    for path in _sources():
        text = open(path).read()
        assert not re.search(r"^\s*(from|import)\s+oracle", text, re.M), path
        assert "rtlynx_oracle" not in text and "_work/" not in text, path


def test_binding_has_no_fallback_when_library_is_missing(tmp_path, monkeypatch):
    from paper_2605_26632_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "absent.so"))
    try:
        binding.lib()
    except RuntimeError as e:
        assert "not built" in str(e)
    else:
        raise AssertionError("binding.lib() must raise when librtlynx.so is absent")


def test_oracle_is_only_used_by_tests_smoke_and_cpu_baseline():
    bench = open(os.path.join(ROOT, "bench.py")).read()
    # the only oracle import in bench.py sits inside the cpu_baseline leg
    assert bench.count("import oracle") == 1
    assert bench.index("import oracle") > bench.index("cpu_baseline = None")
