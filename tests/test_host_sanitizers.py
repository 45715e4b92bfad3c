"""The library's host side (argument validation, the plan of a client step, message bounds, the
sizing of the decode plan, clean-up) built for the CPU alone with AddressSanitizer and
UndefinedBehaviorSanitizer, the HIP runtime replaced by a stand-in whose "device" memory is heap
blocks of the requested sizes, and driven through the C ABI by a small program.  No GPU."""
import os
import re
import subprocess

from paper_1805_08768_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "host_sanitize")
HIPCC = "/opt/rocm/bin/hipcc"
CLANGXX = "/opt/rocm/lib/llvm/bin/clang++"
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    assert r.returncode == 0, "%s\n%s\n%s" % (" ".join(cmd), r.stdout[-3000:], r.stderr[-3000:])
    return r


def test_host_side_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    obj = str(tmp_path / "sbc_host.o")
    host_flags = [f for s in SAN for f in ("-Xarch_host", s)]
    run([HIPCC, "--cuda-host-only", "-O1", "-g", "-std=c++17", "-fPIC", *host_flags, "-c",
         os.path.join(ROOT, "paper_1805_08768_amd", "csrc", "sbc_lib.hip"), "-o", obj])
    # the registration code refers to the device code object, which a host-only build does not have
    syms = run(["nm", obj]).stdout
    fatbin = re.findall(r"\bU (__hip_fatbin\w*)", syms)
    exe = str(tmp_path / "driver")
    run([CLANGXX, "-O1", "-g", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"), "-I", "/opt/rocm/include",
         "-D__HIP_PLATFORM_AMD__", os.path.join(HERE, "driver.cpp"), os.path.join(HERE, "hip_stub.cpp"), obj,
         *["-Wl,--defsym,%s=0" % s for s in fatbin], "-o", exe])
    sizes = tmp_path / "sizes.txt"
    sizes.write_text("\n".join(str(n) for n in synth.numels(synth.resnet50_shapes())))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)
    r = run([exe, str(sizes)], env=env)
    assert "host checks passed" in r.stdout, r.stdout[-2000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
