"""bench.py's contract that can be checked without a GPU: more than one GPU is refused with a
message, and the product path does not import the oracle outside the cpu_baseline leg."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr


def test_oracle_is_only_used_by_tests_smoke_and_the_cpu_baseline():
    pkg = os.path.join(ROOT, "paper_2401_06706_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", src, flags=re.M), f
                assert "mcsd_oracle" not in src, f
    bench = open(os.path.join(ROOT, "bench.py")).read()
    # every import of the oracle in bench.py sits inside a function of the cpu-baseline legs
    for m in re.finditer(r"from oracle import", bench):
        head = bench[:m.start()]
        fn = re.findall(r"^def (\w+)\(", head, flags=re.M)[-1]
        assert fn in ("cpu_baseline", "bench_draft_sample", "bench_kv_commit"), fn


def test_no_committed_file_reads_the_scratch_folder():
    for dirpath, dirs, files in os.walk(ROOT):
        dirs[:] = [d for d in dirs if d not in (".git", "_work", "gpurun_out", "__pycache__", ".pytest_cache")]
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".c")) and f != "test_bench_contract.py":
                src = open(os.path.join(dirpath, f), errors="ignore").read()
                assert not re.search(r"(^|[^A-Za-z0-9])_work(/|\\b)", src), os.path.join(dirpath, f)
