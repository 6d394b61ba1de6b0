"""The host side of the library (schedule builder, argument checks) under AddressSanitizer and UBSan.
Host code only: the GPU pass is compiled without sanitizers and no device call is made."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_schedule_and_validation_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "schedule_fuzz")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address,undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", exe, os.path.join(ROOT, "tests", "host", "schedule_fuzz.cpp"),
           os.path.join(ROOT, "paper_2409_19134_amd", "csrc", "spd_api.hip")]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0 and run.stdout.strip().endswith("ok 400"), run.stdout[-3000:]


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_device_tables_under_asan_ubsan(tmp_path):
    """What the kernels read of a schedule (items linked into pieces, split rows, slot bookkeeping), built on the host
    for random views in both mappings: every item reached once, every token and slot covered once, flags and row
    addresses as the kernels expect them."""
    exe = str(tmp_path / "device_tables_fuzz")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-x", "hip",
           "-Xarch_host", "-fsanitize=address,undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", exe, os.path.join(ROOT, "tests", "host", "device_tables_fuzz.cpp")]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0 and run.stdout.strip().endswith("ok 600"), run.stdout[-3000:]


def test_schedule_key_and_growth_rule_under_asan_ubsan(tmp_path):
    """The key a schedule is remembered by (what is part of it, what is not) and the rule by which a schedule serves
    a view whose lengths have all grown by the same 1..64 tokens: plain C++, no GPU."""
    exe = str(tmp_path / "schedule_key_fuzz")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-o", exe, os.path.join(ROOT, "tests", "host", "schedule_key_fuzz.cpp")]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0 and run.stdout.strip().endswith("ok 2000"), run.stdout[-3000:]


def test_oracle_under_asan_ubsan(tmp_path):
    """The C oracle itself: small random inputs in every storage mode, with AddressSanitizer and UBSan."""
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-o", exe, os.path.join(ROOT, "tests", "host", "oracle_sanitize.c"), "-lm"]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1", OMP_NUM_THREADS="4")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0 and run.stdout.strip().endswith("ok 60"), run.stdout[-3000:]


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_no_kernel_spills_registers(tmp_path):
    """Every kernel instance fits its register budget: a spill in the streaming kernel (which has happened after an
    innocent-looking refactoring) costs several percent of bandwidth without failing any parity test."""
    import importlib.util
    import re
    spec = importlib.util.spec_from_file_location("spd_build", os.path.join(ROOT, "paper_2409_19134_amd", "build.py"))
    build = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(build)
    cmd = [HIPCC, *build.HIPCC_FLAGS, "-Rpass-analysis=kernel-resource-usage", "-o", str(tmp_path / "lib.so"),
           os.path.join(ROOT, "paper_2409_19134_amd", "csrc", "spd_api.hip")]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-3000:]
    spills = [int(x) for x in re.findall(r"VGPRs Spill: (\d+)", res.stdout)]
    scratch = [int(x) for x in re.findall(r"ScratchSize \[bytes/lane\]: (\d+)", res.stdout)]
    assert len(spills) >= 40 and len(scratch) == len(spills)          # every kernel instance reported
    assert max(spills) == 0 and max(scratch) == 0
