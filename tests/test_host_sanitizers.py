"""The host side of the library (argument validation, tail plan, planner formulas, scheduler
set-up) under AddressSanitizer + UndefinedBehaviorSanitizer: a copy of the package is built with
the sanitizers on the host code only and the host-side ABI tests run against it in a child process
with the ASan runtime preloaded.  No GPU is touched (every call returns before device work)."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _asan_runtime():
    clang = "/opt/rocm/llvm/bin/clang"
    if not os.path.exists(clang):
        return None
    path = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    rt = _asan_runtime()
    if rt is None or not os.path.exists("/opt/rocm/bin/hipcc"):
        pytest.skip("no hipcc / ASan runtime here")
    tree = tmp_path / "tree"
    for name in ("tests", "synth", "oracle", "include", "paper_2511_12056_amd"):
        shutil.copytree(os.path.join(ROOT, name), tree / name,
                        ignore=shutil.ignore_patterns("*.so", "__pycache__", "test_host_sanitizers.py"))
    build = ("import importlib.util, sys; s = importlib.util.spec_from_file_location('b', sys.argv[1]); "
             "m = importlib.util.module_from_spec(s); s.loader.exec_module(m); m.build_library(host_sanitizers=True)")
    subprocess.run([sys.executable, "-c", build, str(tree / "paper_2511_12056_amd" / "build.py")], check=True, timeout=600)
    preload = os.environ.get("LD_PRELOAD", "")           # the ASan runtime must come first; whatever is there stays
    env = dict(os.environ, LD_PRELOAD=rt + (":" + preload if preload else ""), ASAN_OPTIONS="detect_leaks=0:halt_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    res = subprocess.run([sys.executable, "-m", "pytest", "tests/test_abi_host.py", "tests/test_planner_parity.py",
                          "-x", "-q", "-p", "no:cacheprovider"], cwd=str(tree), env=env, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert "passed" in res.stdout and "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr
