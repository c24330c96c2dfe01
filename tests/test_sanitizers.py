"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer, on the CPU.

* the C oracle: built with gcc's sanitizers, and its whole pin suite (tests/test_oracle_*.py) run
  against that build in a child process that has gcc's libasan preloaded;
* the C-ABI library: its host pass (validation, planners, argument marshalling) built with the HIP
  compiler's sanitizers, device code as always, and tests/test_abi.py (code that returns before
  any launch) and tests/test_host_planners.py (every planner and launch table, up to the launch
  that fails for want of a device) run against that build in a child process that has the
  compiler's ASan runtime preloaded.  No GPU is involved.
Any report of either sanitizer ends the child with a non-zero status."""
import glob
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _child_env(runtime, **more):
    env = dict(os.environ)
    pre = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = runtime + (":" + pre if pre else "")
    # the interpreter itself is not instrumented: no leak report at exit, no complaint about the
    # order of the preloaded libraries
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(more)
    return env


def test_oracle_pin_suite_under_asan_and_ubsan(tmp_path):
    sys.path.insert(0, ROOT)
    import oracle
    lib = oracle.build_sanitized(str(tmp_path))
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    assert os.path.isabs(runtime) and os.path.exists(runtime), runtime
    files = sorted(glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py")))
    assert len(files) >= 10
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files],
                       cwd=ROOT, env=_child_env(runtime, AWQ_ORACLE_LIBRARY=lib),
                       capture_output=True, text=True, timeout=1200)
    assert p.returncode == 0, (p.stdout[-3000:], p.stderr[-3000:])
    assert " passed" in p.stdout


def test_c_abi_validation_layer_under_asan_and_ubsan(tmp_path):
    sys.path.insert(0, ROOT)
    from paper_2306_00978_amd import build as hip_build
    lib = hip_build.build(sanitize_host_into=str(tmp_path))
    runtime = hip_build.sanitizer_runtime()
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_abi.py"),
                        os.path.join(ROOT, "tests", "test_host_planners.py")],
                       cwd=ROOT, env=_child_env(runtime, AWQ_MI355X_LIBRARY=lib),
                       capture_output=True, text=True, timeout=1200)
    assert p.returncode == 0, (p.stdout[-3000:], p.stderr[-3000:])
    assert " passed" in p.stdout
