"""The oracle and the HIP path share nothing: the package never imports or links the oracle, the
oracle never imports the package, only the tests, smoke() and bench.py's CPU-baseline leg use the
oracle, and nothing that is part of the repository reads the builder's working folder."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _sources(*dirs, suffixes=(".py", ".h", ".hip", ".cpp", ".c")):
    for d in dirs:
        base = os.path.join(ROOT, d)
        if os.path.isfile(base):
            yield base
            continue
        for dirpath, dirnames, filenames in os.walk(base):
            dirnames[:] = [n for n in dirnames if n not in ("__pycache__", "_build")]
            for f in filenames:
                if f.endswith(suffixes):
                    yield os.path.join(dirpath, f)


def test_package_never_touches_the_oracle():
    for path in _sources("paper_2111_00153_amd", "include", "synth_inputs.py"):
        text = open(path, encoding="utf-8").read()
        assert not re.search(r"import\s+oracle|from\s+oracle|liboracle|rmsmp_oracle|oracle/|oracle\.", text), path


def test_oracle_never_touches_the_package():
    for path in _sources("oracle"):
        text = open(path, encoding="utf-8").read()
        assert "paper_2111_00153_amd" not in text and "librmsmp" not in text and "rmsmp.h" not in text, path


def test_seeded_inputs_hold_no_arithmetic_of_the_method():
    text = open(os.path.join(ROOT, "synth_inputs.py"), encoding="utf-8").read()
    assert "paper_2111_00153_amd" not in text and "ctypes" not in text


def test_bench_uses_the_oracle_only_outside_the_timed_path():
    text = open(os.path.join(ROOT, "bench.py"), encoding="utf-8").read()
    # one guarded import, behind the switch that skips the CPU baseline
    assert len(re.findall(r"^\s*import oracle\b", text, re.M)) == 1
    assert re.search(r"if not args\.no_cpu_baseline:\s*\n\s*import oracle", text)


def test_nothing_committed_reads_the_working_folder():
    for path in _sources("paper_2111_00153_amd", "include", "oracle", "tests", "bench.py", "__graft_entry__.py", "synth_inputs.py"):
        if os.path.basename(path) == "test_independence.py":
            continue
        assert not re.search(r"_work(/|\b)", open(path, encoding="utf-8").read()), path
