"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, no GPU code runs):
the C oracle while its pins run, and the C-ABI library's argument validation and host routines
while the host ABI tests run.  Each runs in a child process with the sanitizer runtime preloaded;
any report aborts the child."""
import glob
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(files, env_extra, runtime):
    env = dict(os.environ)
    env.update(env_extra)
    pre = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = runtime + (":" + pre if pre else "")
    # python itself is not instrumented: no leak check at exit, and the runtime need not come first
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0:protect_shadow_gap=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "passed" in r.stdout


def test_oracle_pins_under_address_and_undefined_behaviour_sanitizers():
    runtime = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    assert os.path.isabs(runtime) and os.path.exists(runtime)
    _run(["tests/test_oracle_pins.py", "tests/test_focal_selection.py"], {"FASTOCR_ORACLE_SANITIZE": "1"}, runtime)


def test_abi_validation_under_address_and_undefined_behaviour_sanitizers():
    from paper_2605_17447_amd._build import build
    lib = build(host_sanitize=True)
    found = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    assert found, "clang's AddressSanitizer runtime not found"
    _run(["tests/test_abi_host.py"], {"FASTOCR_LIB": lib}, found[0])
