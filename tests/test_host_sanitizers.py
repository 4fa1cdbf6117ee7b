"""Host code of the library under AddressSanitizer and UBSan (CPU only).

Second test: tests/native/host_order.cpp links the same host code against a CPU stand-in for the
HIP runtime (tests/native/fake_hip.cpp: streams that run only when pumped, in random orders that
stream and event semantics allow) and checks that no copy into reused pages overtakes a queued kernel
that reads them, that no kernel overtakes its adapter's copy or its batch image, and that batch
objects are not reused under queued kernels (the ordering that evict / load / batch reuse need).

tests/native/host_sanitize.cpp drives the allocator and the batch translation of a placement-only
pool through random histories and checks the invariants of Sec. III-C (tables ascending, pairwise
disjoint, page counts, busy / exists / not-found answers, stable grouping).  It is compiled together
with plora_pool.cpp by the host compiler with -fsanitize=address,undefined; the kernel launchers are
stubbed, no GPU call is made.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir("/opt/rocm/include"), reason="needs g++ and the HIP headers")
def test_allocator_and_translation_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"),
           "-I" + os.path.join(ROOT, "paper_2512_20210_amd", "csrc"),
           os.path.join(ROOT, "tests", "native", "host_sanitize.cpp"),
           os.path.join(ROOT, "paper_2512_20210_amd", "csrc", "plora_pool.cpp"),
           "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-o", exe]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300, env=env)
    assert r.returncode == 0 and "host sanitize run OK" in r.stdout, r.stdout[-3000:]


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir("/opt/rocm/include"), reason="needs g++ and the HIP headers")
def test_copy_and_kernel_ordering_against_a_cpu_stand_in_runtime(tmp_path):
    exe = str(tmp_path / "host_order")
    nat = os.path.join(ROOT, "tests", "native")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"),
           "-I" + os.path.join(ROOT, "paper_2512_20210_amd", "csrc"), "-I" + nat,
           os.path.join(nat, "host_order.cpp"), os.path.join(nat, "fake_hip.cpp"),
           os.path.join(ROOT, "paper_2512_20210_amd", "csrc", "plora_pool.cpp"), "-o", exe]  # no HIP library: the stand-in defines the calls
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300, env=env)
    assert r.returncode == 0 and "host order run OK" in r.stdout, r.stdout[-3000:]


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_predictor_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "predictor_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-I" + os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "native", "predictor_sanitize.cpp"),
           os.path.join(ROOT, "paper_2512_20210_amd", "csrc", "plora_predictor.cpp"), "-pthread", "-o", exe]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300, env=env)
    assert r.returncode == 0 and "predictor sanitize run OK" in r.stdout, r.stdout[-3000:]
