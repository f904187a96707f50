"""Sanitizer passes over host code (no GPU needed).

The CPU oracle: oracle/plogp_oracle.c and a small driver are compiled with AddressSanitizer
and UndefinedBehaviorSanitizer into one program that calls every entry point on small tables
and grids (empty candidate lists, every strategy id, refused arguments).

The library's host side: its sources and a driver are compiled by hipcc with the same
sanitizers on the host pass only; the driver goes through the argument checks and the grid
preparation of the C ABI and lays out the launch plan of twenty thousand random shapes.

Any finding aborts the program."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "sanitize_oracle"
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-mfma", "-ffp-contract=off", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-o", str(exe), os.path.join(ROOT, "tests", "native", "sanitize_oracle.c"),
           os.path.join(ROOT, "oracle", "plogp_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["OMP_NUM_THREADS"] = "2"
    res = subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=300)
    sys.stdout.write(res.stdout)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr
    assert "checksum" in res.stdout


def test_library_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        import pytest
        pytest.skip("no hipcc")
    exe = tmp_path / "sanitize_host"
    csrc = os.path.join(ROOT, "paper_cs_0408034_amd", "csrc")
    host_san = "-Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined -Xarch_host -fno-sanitize-recover=all"
    cmd = ([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-ffp-contract=off",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
           + host_san.split() + ["-o", str(exe), os.path.join(ROOT, "tests", "native", "sanitize_host.hip")]
           + [os.path.join(csrc, f) for f in ("plogp_api.hip", "plogp_kernels.hip", "plogp_cutover.hip",
                                               "plogp_robust.hip", "plogp_profile.hip")])
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0"
    res = subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=600)
    sys.stdout.write(res.stdout)
    assert res.returncode == 0, res.stdout + res.stderr[-3000:]
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-3000:]
    assert "plans laid out" in res.stdout
