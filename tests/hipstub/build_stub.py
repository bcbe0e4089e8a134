"""Builds the library's HOST code against the stand-in HIP runtime (hipstub.cpp) with
AddressSanitizer and UBSan, without any device code: `hipcc --cuda-host-only`. The result is a
directory holding a copy of the Python binding next to a `liblop.so` whose kernels do nothing,
so that plan construction, weight packing, the per-band scheduler, graph capture, the queries
and the teardown can run on a machine without a GPU under the sanitizers.

Test infrastructure only (used by tests/test_host_under_stub.py).
"""
import os
import re
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
PKG = os.path.join(ROOT, "paper_2507_05829_amd")
CSRC = os.path.join(PKG, "csrc")
LLVM = "/opt/rocm/llvm/bin"
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
       "-shared-libasan"]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("failed: %s\n%s\n%s" % (" ".join(cmd), r.stdout, r.stderr))
    return r.stdout


def asan_runtime() -> str:
    return _run([os.path.join(LLVM, "clang++"), "-print-file-name=libclang_rt.asan-x86_64.so"]).strip()


def build(out_dir: str) -> str:
    """Returns the directory to put on sys.path (it holds the package copy)."""
    from paper_2507_05829_amd.build import SOURCES
    pkg = os.path.join(out_dir, "paper_2507_05829_amd")
    os.makedirs(pkg, exist_ok=True)
    clang = os.path.join(LLVM, "clang++")
    stub = os.path.join(pkg, "libhipstub.so")
    _run([clang, "-O1", "-g", "-std=c++17", "-fPIC", "-shared", *SAN, "-I", "/opt/rocm/include",
          os.path.join(HERE, "hipstub.cpp"), "-o", stub])
    objs = []
    for src in SOURCES:
        obj = os.path.join(out_dir, src + ".o")
        _run(["/opt/rocm/bin/hipcc", "--offload-arch=gfx950", "--cuda-host-only", "-O1", "-g", "-std=c++17",
              "-fPIC", *SAN, "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include"),
              "-I", CSRC, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    # the host objects refer to the device code object they would embed: give them empty ones
    syms = set()
    for obj in objs:
        syms.update(re.findall(r"\bU (__hip_fatbin_\w+)", _run(["nm", obj])))
    fat = os.path.join(out_dir, "fatbin_symbols.c")
    with open(fat, "w") as f:
        for s in sorted(syms):
            f.write("char %s[64] __attribute__((aligned(4096)));\n" % s)
    fat_o = fat + ".o"
    _run([os.path.join(LLVM, "clang"), "-fPIC", "-c", fat, "-o", fat_o])
    _run([clang, "-shared", "-fPIC", *SAN, *objs, fat_o, "-L", pkg, "-lhipstub", "-Wl,-rpath,$ORIGIN",
          "-o", os.path.join(pkg, "liblop.so")])
    for name in ("lop.py", "__init__.py"):
        shutil.copy(os.path.join(PKG, name), os.path.join(pkg, name))
    return out_dir
