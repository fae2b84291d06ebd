"""AddressSanitizer + UndefinedBehaviorSanitizer over the host C of this repository: the CPU
oracle and the library's host-side controller / payload geometry, built together with a small C
driver into one sanitized executable (no Python in that process) and run on ragged, empty,
odd-tail and one-element cases with output buffers of exactly the reported sizes."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_oracle_and_host_abi_under_asan_ubsan(tmp_path):
    exe = tmp_path / "sanitize_driver"
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fno-omit-frame-pointer", "-fno-fast-math", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fopenmp", "-Wall", "-Wextra",
           "-I", os.path.join(ROOT, "include"),
           os.path.join(HERE, "sanitize_driver.c"),
           os.path.join(ROOT, "oracle", "nsml_oracle.c"),
           os.path.join(ROOT, "paper_2506_16235_amd", "csrc", "nsml_ctl.c"),
           "-o", str(exe), "-lm"]
    subprocess.check_call(cmd)
    env = dict(os.environ)
    # link order is not checked: a library preloaded by the environment may come first
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "2"
    p = subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stdout + p.stderr
    assert "clean" in p.stdout
