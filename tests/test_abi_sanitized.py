"""The boundary's host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

Every translation unit's host side -- argument validation, workspace arithmetic, error reporting -- is built with both
sanitizers and without any device code, and tests/test_abi.py (every rejected-argument case, the symbol list, the
workspace formulas) runs against that build in a child process with the sanitizer runtime preloaded.  A sanitizer report
fails the run: UBSan halts on the first error, ASan aborts."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _build_module():
    # loaded by path: the check must not depend on a regular build being importable
    spec = importlib.util.spec_from_file_location("_bbm_build", os.path.join(ROOT, "paper_2409_15097_amd", "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_abi_checks_pass_under_host_sanitizers(tmp_path):
    build = _build_module()
    lib = build.build_host_sanitized(str(tmp_path / "hostsan"))
    symbols = subprocess.run(["nm", lib], stdout=subprocess.PIPE, text=True, check=True).stdout
    assert "__asan_report" in symbols and "__ubsan_handle" in symbols          # really instrumented
    env = dict(os.environ)
    env["LD_PRELOAD"] = ":".join(x for x in (build.sanitizer_runtime(), env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"                      # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["BBM_LIBRARY"] = lib
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_abi.py"), "-q", "-x", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "AddressSanitizer" not in r.stdout and "runtime error:" not in r.stdout, r.stdout[-4000:]
    assert " passed" in r.stdout
