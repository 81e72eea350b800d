"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the policy core and the oracle
are rebuilt with -fsanitize=address,undefined (errors abort) and the CPU suites that exercise them
are run again, in a child process, against those builds.  GPU code is not involved."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
SUITES = ["tests/test_policy_cpu.py", "tests/test_swap_profile_cpu.py", "tests/test_oracle_pins.py",
          "tests/test_serving_cpu.py"]


def test_policy_core_and_oracle_are_clean_under_asan_and_ubsan(tmp_path):
    import oracle
    from paper_2503_13773_amd.build import build_policy_library
    pol = build_policy_library(out=str(tmp_path / "libkvc_policy_san.so"), extra_flags=SAN)
    ora = oracle.build(force=True, out=str(tmp_path / "libkvc_oracle_san.so"), extra_flags=SAN)
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    assert os.path.isabs(asan) and os.path.exists(asan), "gcc has no libasan.so"
    env = dict(os.environ)
    env["KVC_POLICY_LIBRARY"], env["KVC_ORACLE_LIBRARY"] = pol, ora
    # the sanitizer runtime has to be in the process before the libraries are loaded with dlopen
    env["LD_PRELOAD"] = " ".join(x for x in (os.environ.get("LD_PRELOAD", ""), asan) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *SUITES],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "AddressSanitizer" not in r.stdout + r.stderr and "runtime error:" not in r.stdout + r.stderr, tail
    assert " passed" in r.stdout
