"""AddressSanitizer + UBSan over the HOST side of libmoonwalk, on the CPU.

Every translation unit is compiled host-only (no device code) with the sanitizers, linked against a stand-in for
the HIP runtime (tests/sanitizer/fake_hip.cpp: zeroed host memory for device memory, launches checked and
dropped) and driven through the C ABI by tests/sanitizer/abi_driver.cpp: argument validation, then whole calls of
every entry point on small networks of every kind, and an allocator that gives out at every possible point of a
setup. A heap overflow in a pointer table, a leak on an error path, a signed overflow in a buffer plan or a
misaligned access fails the run. No GPU is involved and no kernel runs."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, " ".join(cmd) + "\n" + r.stdout[-4000:]
    return r.stdout


def test_host_code_under_asan_and_ubsan():
    import __graft_entry__ as entry
    hipcc = entry._hipcc()
    out = os.path.join(ROOT, "_build", "sanitizer")
    os.makedirs(out, exist_ok=True)
    common = ["-O1", "-g", "-std=c++17", "-fPIC", "-fno-omit-frame-pointer"]
    # without the function-type check: in a host-only build it swallows every launch made through a pointer to a
    # kernel (the launch configuration is pushed and the kernel's host stub is never called); the stand-in
    # runtime counts pushed configurations that no launch took up, so this cannot come back unnoticed
    host_san = [f for s in SAN + ["-fno-sanitize=function"] for f in ("-Xarch_host", s)]
    procs = []
    for src in entry.SOURCES:
        obj = os.path.join(out, src.replace(".hip", ".o"))
        cmd = [hipcc, "--offload-arch=gfx950", "--cuda-host-only", "-ffp-contract=off"] + common + host_san + \
              ["-c", os.path.join(entry.CSRC, src), "-o", obj]
        procs.append((cmd, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs = []
    for cmd, obj, p in procs:
        text, _ = p.communicate()
        assert p.returncode == 0, " ".join(cmd) + "\n" + text[-4000:]
        objs.append(obj)
    # a host-only object still names its (absent) device code object: give every such name a definition
    names = sorted({line.split()[-1] for line in _run(["nm", "-u"] + objs).splitlines() if "__hip_fatbin_" in line})
    stub = os.path.join(out, "fatbin_stubs.cpp")
    with open(stub, "w") as f:
        f.write("".join(f'extern "C" const char {n}[8] = {{0}};\n' for n in names))
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "llvm", "bin", "clang++")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang++"
    exe = os.path.join(out, "abi_driver")
    sdir = os.path.join(ROOT, "tests", "sanitizer")
    _run([clang] + common + SAN + ["-I/opt/rocm/include", "-D__HIP_PLATFORM_AMD__", os.path.join(sdir, "fake_hip.cpp"), os.path.join(sdir, "abi_driver.cpp"), stub] + objs + ["-o", exe, "-lpthread", "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout[-6000:]
    assert "abi_driver: ok" in r.stdout
    assert "runtime error" not in r.stdout and "AddressSanitizer" not in r.stdout and "LeakSanitizer" not in r.stdout, r.stdout[-6000:]
