"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only; GPU sanitizers are not used).

Two legs, each in a child process with the sanitizer runtime preloaded:
  * the oracle, rebuilt with g++ -fsanitize=address,undefined, runs its hand-worked Algorithm 1 cases, the
    permutation pins and the tiny-layer (config 1) pins;
  * the HIP library, rebuilt with the sanitizers on its host side only, runs the C-ABI tests: the table
    validator, workspace sizing and every argument-error path.
A sanitizer report aborts the child (-fno-sanitize-recover, ASan's default), so a clean run is rc 0."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_pytest(files, env_extra, preload):
    env = dict(os.environ)
    env.update(env_extra)
    env["LD_PRELOAD"] = preload + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"       # the interpreter's own allocations are not ours
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-s", "-p", "no:cacheprovider", *files], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=900)
    tail = "\n".join((r.stdout + r.stderr).splitlines()[-6:])
    print(tail)
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "failed" not in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_oracle_under_asan_and_ubsan(tmp_path):
    import oracle
    lib = oracle.build_sanitized(str(tmp_path / "libbm_oracle_san.so"))
    rt = subprocess.run(["g++", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    if not os.path.isabs(rt):
        pytest.skip("g++ has no AddressSanitizer runtime here")
    _run_pytest(["tests/test_oracle_remap.py", "tests/test_oracle_layer.py", "tests/test_oracle_gates.py",
                 "tests/test_oracle_psi.py", "tests/test_oracle_profiling.py"], {"BM_ORACLE_LIBRARY": lib}, rt)


def test_library_host_side_under_asan_and_ubsan(tmp_path):
    from paper_2511_10054_amd.build import HIPCC, HOST_SANITIZE, build_library
    rts = glob.glob(os.path.join(os.path.dirname(os.path.dirname(os.path.realpath(HIPCC))),
                                 "llvm", "lib", "clang", "*", "lib", "linux", "libclang_rt.asan-x86_64.so"))
    if not rts:
        pytest.skip("no clang AddressSanitizer runtime beside hipcc")
    lib = build_library(extra=HOST_SANITIZE, lib=str(tmp_path / "libbuddymoe_san.so"), objdir=str(tmp_path / "obj"),
                        link_extra=["-fsanitize=address", "-fsanitize=undefined", "-shared-libasan"])
    _run_pytest(["tests/test_abi.py"], {"BUDDYMOE_LIBRARY": lib}, rts[0])
