"""CPU sanitizer leg: the oracle and the host side of the C ABI (argument validation and call sequencing) rebuilt with
AddressSanitizer + UndefinedBehaviorSanitizer and driven by the existing tests in a child process.  Nothing here touches a
GPU: the HIP library's kernels are replaced by counting stand-ins (tests/hostcheck/launcher_stubs.cpp), and only host code
is instrumented."""
import glob
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TESTS = os.path.join(ROOT, "tests")


def child_env(runtime, **extra):
    """the child's environment: the sanitizer runtime appended to whatever is preloaded already (it must be loaded before
    the instrumented library; python itself is not instrumented, so leak checking and the link-order check are off)"""
    env = dict(os.environ)
    pre = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = (pre + ":" if pre else "") + runtime
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env.update(extra)
    return env


def run_child(args, env, timeout):
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + args, cwd=ROOT, env=env,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=timeout)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout, r.stdout[-4000:]
    return r.stdout


@pytest.mark.timeout(900)
def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gcc_asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    if not os.path.isabs(gcc_asan) or not os.path.exists(gcc_asan):
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    from oracle import build as oracle_build
    lib = oracle_build.build_sanitized(str(tmp_path / "libquartet_ref_san.so"))
    out = run_child([os.path.join(TESTS, f) for f in ("test_oracle_pins.py", "test_oracle_blocks.py", "test_oracle_mxfp8.py",
                                                      "test_oracle_table1.py")],
                    child_env(gcc_asan, QUARTET_REF_LIB=lib), 800)
    assert " passed" in out


@pytest.mark.timeout(600)
def test_abi_argument_checks_pass_under_sanitizers_with_the_kernels_stubbed_out(tmp_path):
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc is not installed")
    rts = glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not rts:
        pytest.skip("clang's AddressSanitizer runtime is not installed")
    csrc = os.path.join(ROOT, "paper_2505_14669_amd", "csrc")
    lib = str(tmp_path / "libquartet.so")
    # sanitizers on the host pass only (each -fsanitize directly after -Xarch_host); api.hip has no kernels of its own
    cmd = ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-I", csrc,
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all",
           os.path.join(csrc, "api.hip"), os.path.join(TESTS, "hostcheck", "launcher_stubs.cpp"), "-o", lib]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-3000:]
    shutil.copy(os.path.join(ROOT, "paper_2505_14669_amd", "binding.py"), str(tmp_path / "binding.py"))
    out = run_child([os.path.join(TESTS, "test_abi_host.py")], child_env(rts[0], QUARTET_HOSTCHECK_DIR=str(tmp_path)), 500)
    assert " passed" in out
